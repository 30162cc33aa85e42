// Panel kernel variant for block pruning (blocks of 4): 768 threads, 4 owned indices per thread,
// blocks of 36 steps (24 block vectors in registers, 12 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(768, 4, 24, 12)
}
