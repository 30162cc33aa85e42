// Panel kernel variant for block pruning (blocks of 4): 256 threads, 1 owned indices per thread,
// blocks of 64 steps (64 block vectors in registers, 0 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(256, 1, 64, 0)
}
