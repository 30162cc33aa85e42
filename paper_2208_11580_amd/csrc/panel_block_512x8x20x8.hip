// Panel kernel variant for block pruning (blocks of 4): 512 threads, 8 owned indices per thread, blocks of 28 steps
// (20 block vectors in registers, 8 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(512, 8, 20, 8)
}
