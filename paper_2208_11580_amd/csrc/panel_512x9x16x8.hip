// Panel kernel variant: 512 threads, 9 owned indices per thread, blocks of 24 steps
// (16 block vectors in registers, 8 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL(512, 9, 16, 8)
}
