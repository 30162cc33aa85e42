// Panel kernel variant for block pruning (blocks of 4): 512 threads, 6 owned indices per thread, blocks of 40 steps
// (28 block vectors in registers, 12 in LDS).
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL_BLOCK(512, 6, 28, 12)
}
