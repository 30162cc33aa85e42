// Panel kernel variant: 1024 threads, 2 owned indices per thread, blocks of 32 steps.
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL(1024, 2, 32)
}
