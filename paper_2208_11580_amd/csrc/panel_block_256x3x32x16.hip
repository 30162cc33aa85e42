// Panel kernel variant for block pruning (blocks of 4): 256 threads, 3 owned indices per thread,
// blocks of 48 steps (32 block vectors in registers, 16 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(256, 3, 32, 16)
}
