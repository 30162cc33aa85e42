// Panel kernel variant: 1024 threads, 2 owned indices per thread, blocks of 48 steps
// (32 block vectors in registers, 16 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL(1024, 2, 32, 16)
}
