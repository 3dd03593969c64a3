// Host-side interface of the 16x16x64 int8 GEMM kernels (static_linear_k64.hip), used by the entry
// points in static_linear.hip.
#pragma once

#include "gemm_tile.h"

namespace sasq {

struct GemmK64Args {
    const int8_t* xq;        // staged activation codes (1 KB blocks of 16 rows x 64 K-bytes)
    const uint8_t* wq;       // weights in the layout `wmode` names
    const float* s;          // activation factor (one, or one per row with `rows`)
    const float* s_w;
    const float* bias;
    uint16_t* y;
    int32_t* acc_out;
    int64_t M, N, K;
};

// wmode: 0 = int8 row-major, 2 = int8 pre-arranged, 3 = int4 pre-arranged (the values of the weight paths in static_linear.hip).
// tile: 0 = 256x256, 1 = 128x256, 2 = 128x128 (two workgroups per CU).  K must be a multiple of 64.
void launch_gemm_k64(const GemmK64Args& a, sasq_dtype dt, int wmode, int tile, bool rows, hipStream_t st);
// Grouped activation factors (a.s points at K / (64 group_tiles) factors, a.acc_out receives the fp32 sums):
// tile 1 = 128x256, 2 = 128x128.  group_tiles = 0: groups of 32 channels (two per K tile; 128x128 tiles).
void launch_gemm_k64_grouped(const GemmK64Args& a, sasq_dtype dt, int wmode, int tile, int group_tiles, hipStream_t st);
// split_tail: hand the tiles of a sparsely filled last round out as 128x256 halves (sets b.split_first / b.split_count)
void launch_gemm_k64_batch(LinBatch& b, int grid, sasq_dtype dt, int wmode, bool split_tail, hipStream_t st);

}  // namespace sasq
