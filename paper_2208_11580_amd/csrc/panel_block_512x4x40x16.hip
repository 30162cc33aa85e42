// Panel kernel variant for block pruning (blocks of 4): 512 threads, 4 owned indices per thread,
// blocks of 56 steps (40 block vectors in registers, 16 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(512, 4, 40, 16)
}
