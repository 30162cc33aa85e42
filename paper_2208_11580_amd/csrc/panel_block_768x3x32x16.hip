// Panel kernel variant for block pruning (blocks of 4): 768 threads, 3 owned indices per thread,
// blocks of 48 steps (32 block vectors in registers, 16 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(768, 3, 32, 16)
}
