// Panel kernel variant for block pruning (blocks of 4): 512 threads, 3 owned indices per thread,
// blocks of 64 steps (48 block vectors in registers, 16 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(512, 3, 48, 16)
}
