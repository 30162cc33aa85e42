// Panel kernel variant: 256 threads, 3 owned indices per thread, blocks of 48 steps
// (32 block vectors in registers, 16 in LDS).  Small enough that three workgroups share a CU:
// used when there are more rows than CUs, so that the rows' step latencies overlap.
#include "panel_impl.h"

namespace obc_blocked {
OBC_DEFINE_PANEL(256, 3, 32, 16)
}
