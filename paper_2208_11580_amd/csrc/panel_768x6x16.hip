// Panel kernel variant: 768 threads, 6 owned indices per thread, blocks of 16 steps.
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL(768, 6, 16)
}
