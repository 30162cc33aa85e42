// Declarations shared by the blocked row solver's translation units: workspace layout, kernel
// argument blocks, and the per-variant panel launchers (one translation unit per variant so that
// the heavily unrolled panel kernels compile in parallel).
#pragma once

#include "rows_common.h"

namespace obc_blocked {

using namespace obc_rows;

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BMAX = 64;       // largest block; leading dimension of the per-row U / pivot arrays
constexpr int FT = 128;        // flush tile edge
constexpr int FLD = FT + 4;    // padded LDS row of the flush operand tiles

// Layout of a row's private matrix after its first flush ("row-quad" layout): element (i, j) is at
// float index ((i / 4) * ld + j) * 4 + i % 4, i.e. four consecutive rows of a column sit together.
// It matches the MFMA accumulator layout (a lane holds four consecutive rows of one column: one
// 16-byte store) and it makes both ways the panel reads the symmetric matrix -- along a row and
// along a column -- cost the same 16-byte granularity instead of 4 bytes vs one cache line.
__host__ __device__ inline size_t quad_index(int i, int j, int ld)
{
    return ((size_t)(i >> 2) * ld + j) * 4 + (i & 3);
}

struct BlockedWs {
    float *Abuf[2];     // R x d x d each
    float *U;           // R x BMAX x ldu
    int ldu;            // leading dimension of U: d rounded up to a multiple of 4 (16-byte rows)
    float *invd;        // R x BMAX
    int *piv;           // R x BMAX  (compact index of each pivot of the current block)
    int *map;           // R x d     (new compact index -> old compact index)
    double *w;          // R x d     (compact)
    double *diag;       // R x d
    int *orig;          // R x d     compact -> original index; ~index for an already-pruned weight
    int *m;             // R   live size
    int *done;          // R   steps done (including up-front eliminations)
    int *total;         // R   steps to do
    int *ndead;         // R   up-front eliminations
    int *nb;            // R   steps done in the last panel
    uint8_t *blk;       // R x d  N:M counters (d / M used)
    // bulk elimination of already-pruned indices, BMAX at a time (rows_blocked.hip)
    float *G;           // R x BMAX x ldu  rows of the matrix at the block's pivots
    double *Mb;         // R x BMAX x BMAX the pivots' principal submatrix, then its Cholesky factor
    double *Tb;         // R x BMAX x BMAX inverse of that factor
    int *scal;          // [0] smallest number of up-front eliminations over the rows, [1] the most eliminations any row does
};


struct PanelArgs {
    const float *A_cur;      // matrix buffer the rows are read from
    size_t a_row_stride;     // elements between two rows' matrices (0: all rows share H^-1)
    int ld;                  // leading dimension of A_cur
    int swz;                 // 0: A_cur is plain row-major (the shared H^-1); 1: row-quad layout
    int d;                   // original width (stride of the per-row state arrays)
    int nm_n, nm_m;
    const float *delta, *offset;
    int maxq;
    int outliers;            // OBQ: restrict the choice to outliers while there are any
    BlockedWs ws;
    int32_t *order;
    float *loss;
    int32_t *codes;
    float *W_out;
    float *trace;
    int out_ld;
    int *status;
};

// launchers defined in panel_<T>x<EPT>x<BR>x<BL>.hip (pruning and OBQ) and
// panel_block_<T>x<EPT>x<BR>x<BL>.hip (block pruning, blocks of 4): T threads, EPT owned indices per thread,
// blocks of BR + BL steps (BR vectors in registers, BL in LDS).  Return 0 or -1 (HIP error).
#define OBC_DECLARE_PANEL(T, EPT, BR, BL) \
    int launch_panel_##T##_##EPT##_##BR##_##BL(int mode, int R, size_t lds_nm, hipStream_t st, const PanelArgs &a); \
    int launch_panel_block_##T##_##EPT##_##BR##_##BL(int mode, int R, size_t lds_nm, hipStream_t st, const PanelArgs &a)
OBC_DECLARE_PANEL(256, 1, 64, 0);
OBC_DECLARE_PANEL(256, 3, 32, 16);
OBC_DECLARE_PANEL(1024, 1, 64, 0);
OBC_DECLARE_PANEL(512, 3, 48, 16);
OBC_DECLARE_PANEL(512, 4, 40, 16);
OBC_DECLARE_PANEL(768, 3, 32, 16);
OBC_DECLARE_PANEL(512, 6, 28, 12);
OBC_DECLARE_PANEL(512, 8, 20, 8);
OBC_DECLARE_PANEL(512, 9, 16, 8);

}  // namespace obc_blocked
