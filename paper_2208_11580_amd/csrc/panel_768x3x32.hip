// Panel kernel variant: 768 threads, 3 owned indices per thread, blocks of 32 steps.
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL(768, 3, 32)
}
