// Panel kernel variant for block pruning (blocks of 4): 768 threads, 6 owned indices per thread,
// blocks of 24 steps (16 block vectors in registers, 8 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(768, 6, 16, 8)
}
