// Panel kernel variant: 256 threads, 1 owned indices per thread, blocks of 64 steps.
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL(256, 1, 64)
}
