// int8 GEMM of the static-inference linear (Sec. 3, Eq. 2) on v_mfma_i32_16x16x64_i8, over
// pre-quantized activations, with the dequantizing epilogue.
//
// Same machine shape as the 32x32x32 kernel in static_linear.hip -- workgroup tile BM x BN, four
// waves in a 2x2 arrangement, a ring of four LDS stages of 64 K-bytes filled by direct L2 -> LDS
// loads three to four stages ahead, XOR-swizzled 16-byte chunks, XCD-aware tile order, the
// LDS-staged 128-bit store epilogue -- but the wave's (BM/2) x (BN/2) block is (BM/32) x (BN/32)
// tiles of 16x16 and one MFMA contracts a whole 64-byte stage.  On this part the matrix units are
// power-limited, and the 16x16x64 form sustains about 15 % more than 32x32x32 on the same operand
// codes (a register-only loop reads 4.4-4.5 POP/s against 3.9): it moves half as many accumulator
// values per multiply-add.  Fragment bytes read from LDS per multiply-add are the same.
//
// MFMA operand layout: lane l supplies row l%16 of its operand and the 16 K-bytes 16*(l/16) ..
// +15 of the stage; A = weight tile (rows n), B = activation tile (rows m); the result D[i][j]
// (i <-> n, j <-> m) puts n = 4*(l/16) + v, m = l%16 in register v of lane l, so a lane holds
// four consecutive n of one m.
#include "sasq_device.h"
#include "gemm_tile.h"
#include "gemm_k64.h"

// Instrumented build (the benchmark's libsasq_ts.so, `bench.py --tile-timestamps`; never the product library): thread 0
// of every workgroup of the batched kernel writes s_memtime (shader cycles) and s_memrealtime (100 MHz) at five points
// of its tile into a caller-provided buffer of 16 uint64 per workgroup: [2k], [2k+1] = the stamps of point k; [14] = K,
// [15] = 0 for a whole tile, 1 / 2 for the upper / lower half of a split one.
#ifdef SASQ_GEMM_TIMESTAMPS
namespace sasq { __device__ unsigned long long* g_tile_ts = nullptr; }
#define SASQ_TILE_TS(k)                                                                                   \
    do {                                                                                                  \
        if (sasq::g_tile_ts && threadIdx.x == 0) {                                                        \
            sasq::g_tile_ts[(size_t)blockIdx.x * 16 + 2 * (k)] = __builtin_amdgcn_s_memtime();            \
            sasq::g_tile_ts[(size_t)blockIdx.x * 16 + 2 * (k) + 1] = __builtin_amdgcn_s_memrealtime();    \
        }                                                                                                 \
    } while (0)
#endif
#include "gemm_k64_body.h"
#include <type_traits>

namespace sasq {

template <int DT, int WMODE, int BM, int BN, bool ROWS>
__global__ __launch_bounds__(kGemmThreads)
__attribute__((amdgpu_waves_per_eu(Tile<BM, BN>::kWavesPerSimd, Tile<BM, BN>::kWavesPerSimd)))
void gemm_k64_kernel(const int8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
                     const float* __restrict__ s_ptr, const float* __restrict__ s_w,
                     const float* __restrict__ bias, uint16_t* __restrict__ y,
                     int32_t* __restrict__ acc_out, int M, int N, int K, int tiles_m, int tiles_n)
{
    __shared__ __attribute__((aligned(1024))) char lds[lds_bytes_k64<BM, BN>()];
    int tm, tn;
    if (!tile_of_block((int)blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    gemm_k64_body<DT, WMODE, BM, BN, ROWS>(xq, wq, s_ptr, s_w, bias, y, acc_out, M, N, K, tm, tn, lds);
}

template <int DT, int WMODE, int BM, int BN, int GMODE>
__global__ __launch_bounds__(kGemmThreads)
__attribute__((amdgpu_waves_per_eu(Tile<BM, BN>::kWavesPerSimd, Tile<BM, BN>::kWavesPerSimd)))
void gemm_k64_grouped_kernel(const int8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
                             const float* __restrict__ s_g, const float* __restrict__ s_w,
                             const float* __restrict__ bias, uint16_t* __restrict__ y,
                             int32_t* __restrict__ f_out, int M, int N, int K, int tiles_m, int tiles_n, int group_tiles)
{
    __shared__ __attribute__((aligned(1024))) char lds[lds_bytes_k64<BM, BN>()];
    int tm, tn;
    if (!tile_of_block((int)blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    gemm_k64_body<DT, WMODE, BM, BN, false, GMODE>(xq, wq, s_g, s_w, bias, y, f_out, M, N, K, tm, tn, lds, group_tiles);
}

// Several projections in one launch, 256x256 tiles: each projection owns a run of workgroup ids
// (a multiple of 8, so the XCD-aware tile numbering holds inside it), longest K first.
// The launch's last, partly filled round: when its tiles would occupy fewer than half of the CUs,
// the host hands them out as two 128x256 halves each (workgroup ids from b.split_first on: first
// the upper halves, then the lower ones, in the tiles' own order), so that twice as many CUs
// share the tail and it ends in about 0.6 of a round instead of a whole one.
template <int DT, int WMODE>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_k64_batch_kernel(const LinBatch b)
{
    __shared__ __attribute__((aligned(1024))) char lds[lds_bytes_k64<256, 256>()];
    static_assert(lds_bytes_k64<128, 256>() <= lds_bytes_k64<256, 256>(), "one LDS buffer for both tile shapes");
    int bid = (int)blockIdx.x, half = -1;
    if (bid >= b.split_first) {                                  // a half tile of the tail
        const int j = bid - b.split_first;
        half = j >= b.split_count;
        bid = b.split_first + (half ? j - b.split_count : j);
    }
    const int k = lin_item_of(b, bid);
    const LinItem& it = b.it[k];
    int tm, tn;
    if (!tile_of_block(bid - b.first_block[k], it.tiles_m, it.tiles_n, tm, tn)) return;
#ifdef SASQ_GEMM_TIMESTAMPS
    if (g_tile_ts && threadIdx.x == 0) {
        g_tile_ts[(size_t)blockIdx.x * 16 + 14] = (unsigned long long)it.K;
        g_tile_ts[(size_t)blockIdx.x * 16 + 15] = (unsigned long long)(half + 1);
    }
#endif
    if (half < 0) {
        gemm_k64_body<DT, WMODE, 256, 256, false>(it.xq, it.wq, it.s, it.s_w, it.bias, it.y, nullptr, it.M, it.N, it.K, tm, tn, lds);
    } else {
        if ((2 * tm + half) * 128 >= it.M) return;               // the lower half of a tile that ends within its upper half
        gemm_k64_body<DT, WMODE, 128, 256, false>(it.xq, it.wq, it.s, it.s_w, it.bias, it.y, nullptr, it.M, it.N, it.K, 2 * tm + half, tn, lds);
    }
}

template <int DT, int WMODE, int BM, int BN, bool ROWS>
static void launch_one(const GemmK64Args& a, hipStream_t st)
{
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
    gemm_k64_kernel<DT, WMODE, BM, BN, ROWS><<<grid, kGemmThreads, 0, st>>>(
        a.xq, a.wq, a.s, a.s_w, a.bias, a.y, a.acc_out, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n);
}

template <int DT, int WMODE, bool ROWS>
static void launch_tile(const GemmK64Args& a, int tile, hipStream_t st)
{
    switch (tile) {
        case 0: launch_one<DT, WMODE, 256, 256, ROWS>(a, st); break;
        case 1: launch_one<DT, WMODE, 128, 256, ROWS>(a, st); break;
        default: launch_one<DT, WMODE, 128, 128, ROWS>(a, st); break;
    }
}

template <int DT>
static void launch_dt(const GemmK64Args& a, int wmode, int tile, bool rows, hipStream_t st)
{
    if (wmode == KW_I8B)      { if (rows) launch_tile<DT, KW_I8B, true>(a, tile, st); else launch_tile<DT, KW_I8B, false>(a, tile, st); }
    else if (wmode == KW_I4B) { if (rows) launch_tile<DT, KW_I4B, true>(a, tile, st); else launch_tile<DT, KW_I4B, false>(a, tile, st); }
    else                      { if (rows) launch_tile<DT, KW_I8, true>(a, tile, st);  else launch_tile<DT, KW_I8, false>(a, tile, st); }
}

template <int DT, int WMODE, int BM, int BN>
static void launch_grouped_one(const GemmK64Args& a, int group_tiles, hipStream_t st)
{
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
    if (group_tiles == 0)     // groups of 32 channels: two per K tile
        gemm_k64_grouped_kernel<DT, WMODE, BM, BN, 2><<<grid, kGemmThreads, 0, st>>>(
            a.xq, a.wq, a.s, a.s_w, a.bias, a.y, a.acc_out, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n, 0);
    else
        gemm_k64_grouped_kernel<DT, WMODE, BM, BN, 1><<<grid, kGemmThreads, 0, st>>>(
            a.xq, a.wq, a.s, a.s_w, a.bias, a.y, a.acc_out, (int)a.M, (int)a.N, (int)a.K, tiles_m, tiles_n, group_tiles);
}

template <int DT, int WMODE>
static void launch_grouped_w(const GemmK64Args& a, int tile, int group_tiles, hipStream_t st)
{
    if (tile == 1 && group_tiles != 0) launch_grouped_one<DT, WMODE, 128, 256>(a, group_tiles, st);
    else                               launch_grouped_one<DT, WMODE, 128, 128>(a, group_tiles, st);
}

template <int DT>
static void launch_grouped_dt(const GemmK64Args& a, int wmode, int tile, int group_tiles, hipStream_t st)
{
    if (wmode == KW_I8B)      launch_grouped_w<DT, KW_I8B>(a, tile, group_tiles, st);
    else if (wmode == KW_I4B) launch_grouped_w<DT, KW_I4B>(a, tile, group_tiles, st);
    else                      launch_grouped_w<DT, KW_I8>(a, tile, group_tiles, st);
}

void launch_gemm_k64_grouped(const GemmK64Args& a, sasq_dtype dt, int wmode, int tile, int group_tiles, hipStream_t st)
{
    if (dt == SASQ_F16) launch_grouped_dt<SASQ_F16>(a, wmode, tile, group_tiles, st);
    else                launch_grouped_dt<SASQ_BF16>(a, wmode, tile, group_tiles, st);
}

void launch_gemm_k64(const GemmK64Args& a, sasq_dtype dt, int wmode, int tile, bool rows, hipStream_t st)
{
    if (dt == SASQ_F16) launch_dt<SASQ_F16>(a, wmode, tile, rows, st);
    else                launch_dt<SASQ_BF16>(a, wmode, tile, rows, st);
}

template <int DT>
static void launch_batch_dt(const LinBatch& b, int grid, int wmode, hipStream_t st)
{
    if (wmode == KW_I8B)      gemm_k64_batch_kernel<DT, KW_I8B><<<grid, kGemmThreads, 0, st>>>(b);
    else if (wmode == KW_I4B) gemm_k64_batch_kernel<DT, KW_I4B><<<grid, kGemmThreads, 0, st>>>(b);
    else                      gemm_k64_batch_kernel<DT, KW_I8><<<grid, kGemmThreads, 0, st>>>(b);
}

void launch_gemm_k64_batch(LinBatch& b, int grid, sasq_dtype dt, int wmode, bool split_tail, hipStream_t st)
{
    // Tail of the launch: `grid` workgroup ids in all, 256 resident at a time.
    b.split_first = grid;
    b.split_count = 0;
    const int rem = grid % 256;
    if (split_tail && rem > 0 && rem <= 128 && grid > 256) {
        b.split_first = grid - rem;
        b.split_count = rem;
        grid += rem;
    }
    if (dt == SASQ_F16) launch_batch_dt<SASQ_F16>(b, grid, wmode, st);
    else                launch_batch_dt<SASQ_BF16>(b, grid, wmode, st);
}

}  // namespace sasq

#ifdef SASQ_GEMM_TIMESTAMPS
// Where the batched GEMM's workgroups write their stamps from now on (device memory, 128 bytes per workgroup of the
// launches to come; nullptr: nowhere).  Only the instrumented build exports this.
extern "C" int sasq_ts_set_buffer(void* device_buffer)
{
    return hipMemcpyToSymbol(HIP_SYMBOL(sasq::g_tile_ts), &device_buffer, sizeof(device_buffer)) == hipSuccess ? 0 : 1;
}
#endif
