// Tile geometry, LDS stage layout and workgroup-to-tile mapping shared by the MFMA GEMM kernels
// of the SASQ library (gfx950 only).
#pragma once

#include "sasq_device.h"

namespace sasq {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

// s_waitcnt immediates (gfx9 encoding): vmcnt split over bits [3:0] and [15:14]; expcnt and
// lgkmcnt left at "no wait".
constexpr int waitcnt_vm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }
constexpr int kWaitLgkm0 = 0xF | (0x3 << 14) | (0x7 << 4) | (0x0 << 8);

constexpr int kBK = 64;             // contraction bytes per LDS stage and operand row
constexpr int kStages = 4;
constexpr int kGemmThreads = 256;

// Position swizzle of the four 16-byte chunks of an operand row in an LDS stage (and in the
// pre-arranged 1 KB operand blocks in memory): chunk c of row r sits at position c ^ swz64(r).
__device__ __forceinline__ int swz64(int r) { return ((r >> 1) & 3) ^ ((r >> 3) & 1); }

// Tile geometry.  BM x BN is the workgroup tile (256x256, 128x256 or 128x128); the four waves
// form a 2x2 grid, each owning (BM/2) x (BN/2) as MF x NF tiles of 32x32.
template <int BM, int BN>
struct Tile {
    static_assert((BM == 128 || BM == 256) && (BN == 128 || BN == 256) && BM <= BN, "unsupported tile");
    static constexpr int MF = BM / 64, NF = BN / 64;                    // 32x32 tiles per wave along m, n
    static constexpr int XS = BM / 64, WS = BN / 64;                    // 1 KB slabs per wave per stage
    static constexpr int kXBytes = BM * kBK, kWBytes = BN * kBK;        // per stage
    static constexpr int kStageBytes = kXBytes + kWBytes;
    static constexpr int kEpiStride = BN + 16;                          // bytes per staged output row (+16: bank spread)
    static constexpr int kEpiBytes = (BM / 2) * kEpiStride;             // per wave
    static constexpr int kLds = 4 * kEpiBytes > kStages * kStageBytes ? 4 * kEpiBytes : kStages * kStageBytes;
    static constexpr int kWavesPerSimd = (MF * NF * 16 <= 64) ? 2 : 1;  // 128x128 tiles: two workgroups per CU
};

// XCD-aware tile order.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2:
// give every XCD a contiguous range of logical tile ids, and number the tiles so that 32
// consecutive ids (what one XCD's 32 CUs hold at a time) form an 8 (m) x 4 (n) block that shares
// 8 activation row-panels and 4 weight row-panels in that L2.
__device__ __forceinline__ bool tile_of_block(int bid, int tiles_m, int tiles_n, int& tm, int& tn)
{
    constexpr int PN = 4;                              // n-tiles per panel (2..8 measured within noise of each other)
    const int total = tiles_m * tiles_n;
    const int per = (total + 7) >> 3;
    const int logical = (bid & 7) * per + (bid >> 3);
    if (logical >= total) return false;
    const int panel = logical / (tiles_m * PN);
    const int in = logical - panel * tiles_m * PN;
    const int width = min(PN, tiles_n - panel * PN);   // last panel may be narrower
    tm = in / width;
    tn = panel * PN + in % width;
    return true;
}

// The projections of one layer in one launch (their activation pre-passes and their GEMMs).
constexpr int kMaxLinearBatch = SASQ_MAX_BATCH;
struct LinItem {
    const void* x;          // 16-bit activations
    int8_t* xq;             // staged codes (workspace)
    const float* s;
    const uint8_t* wq;
    const float* s_w;
    const float* bias;
    uint16_t* y;
    int M, N, K, tiles_m, tiles_n;
};
struct LinBatch {
    LinItem it[kMaxLinearBatch];
    int first_block[kMaxLinearBatch + 1];
    int count;
    int split_first, split_count;   // 16x16x64 kernel: workgroup ids from split_first on are half tiles (see gemm_k64_batch_kernel)
};

__device__ __forceinline__ int lin_item_of(const LinBatch& b, int block)
{
    int k = 0;
#pragma unroll
    for (int i = 1; i < kMaxLinearBatch; ++i)
        if (i < b.count && block >= b.first_block[i]) k = i;
    return k;
}

}  // namespace sasq
