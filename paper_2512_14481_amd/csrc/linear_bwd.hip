// Backward of the frozen quantized linear with respect to its input (Sec. 4.2: during scale
// training the gradient reaches each quantization factor through the frozen layers):
//     dX[m,k] = sum_n dY[m,n] * Wq[n,k],   Wq[n,k] = round16(fl32(W_int[n,k]) * s_w[n])   (Eq. 2's W_int * S_w)
// as a 16-bit MFMA GEMM with fp32 accumulation for gfx950.  The dequantized weight is prepared
// once (it is frozen) in the GEMM's operand blocks, transposed so that the contraction index n
// runs along operand rows.
#include "sasq_device.h"
#include "gemm_tile.h"
#include "gemm_k64_body.h"
#include <cstdlib>
#include <cstring>
#include <type_traits>

namespace sasq {

constexpr int kBwdCols = kBK / 2;                  // contraction elements per stage row (16-bit)

// Prepared weight layout: the matrix B[k][n] = Wq[n][k] (K rows, N 16-bit columns; rows padded
// to a multiple of 16 and columns to a multiple of 32 with zeros) cut into 1 KB blocks of 16 rows
// x 32 columns, block (kb, nb) at (kb * Npad/32 + nb) * 1024, the 16-byte chunk c (8 columns) of
// row r at 16 * (4r + (c ^ swz64(r))): what one wave's direct load deposits in an LDS stage.
// One thread per chunk; consecutive lanes take consecutive k so the byte reads of W rows coalesce.
__device__ __forceinline__ int64_t bwd_weight_offset(int64_t k, int64_t n, int64_t Npad)
{
    const int r = (int)(k & 15), c = (int)((n >> 3) & 3);
    return ((k >> 4) * (Npad / kBwdCols) + (n >> 5)) * 1024 + ((4 * r + (c ^ swz64(r))) << 4) + ((n & 7) << 1);
}

template <int DT, bool INT4>
__global__ __launch_bounds__(256) void prepare_bwd_weight_kernel(
    const uint8_t* __restrict__ wq, const float* __restrict__ s_w, uint8_t* __restrict__ out,
    int64_t N, int64_t K, int64_t Npad, int64_t Kpad)
{
    using S = Store16<DT>;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t k = t % Kpad, nc = t / Kpad;     // nc: chunk of 8 contraction columns
    if (nc >= Npad / 8) return;
    uint32_t o[4] = {0u, 0u, 0u, 0u};
    if (k < K) {
        uint16_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t n = nc * 8 + e;
            h[e] = 0;
            if (n >= N) continue;
            int w;
            if (INT4) {
                const uint32_t byte = wq[n * (K / 2) + k / 2];
                const uint32_t nib = (k & 1) ? (byte >> 4) : (byte & 15u);
                w = (int)(nib ^ 8u) - 8;
            } else {
                w = (int8_t)wq[n * K + k];
            }
            h[e] = S::enc((float)w * s_w[n]);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (uint32_t)h[2 * e] | ((uint32_t)h[2 * e + 1] << 16);
    }
    *reinterpret_cast<u32x4*>(out + bwd_weight_offset(k, nc * 8, Npad)) = u32x4{o[0], o[1], o[2], o[3]};
}

// Any-shape fallback (contraction length not a multiple of 32, or unaligned rows): one thread per
// output, fp32 accumulation in ascending n.
template <int DT>
__global__ __launch_bounds__(256) void linear_bwd_scalar_kernel(
    const uint16_t* __restrict__ dy, const uint8_t* __restrict__ wt, uint16_t* __restrict__ dx,
    float* __restrict__ acc_out, int64_t M, int64_t N, int64_t K, int64_t Npad)
{
    using S = Store16<DT>;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * K) return;
    const int64_t m = idx / K, k = idx - m * K;
    float acc = 0.0f;
    for (int64_t n = 0; n < N; ++n) {
        const float w = S::one(*reinterpret_cast<const uint16_t*>(wt + bwd_weight_offset(k, n, Npad)));
        acc = acc + S::one(dy[m * N + n]) * w;
    }
    if (acc_out) acc_out[idx] = acc;
    dx[idx] = S::enc(acc);
}

template <int DT> struct Mfma16;
template <> struct Mfma16<SASQ_F16> {
    static __device__ __forceinline__ f32x16 mma(const i32x4& a, const i32x4& b, const f32x16& c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mfma16<SASQ_BF16> {
    static __device__ __forceinline__ f32x16 mma(const i32x4& a, const i32x4& b, const f32x16& c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------------------------------------
// 16-bit MFMA GEMM, dX[M,K] = dY[M,N] . B^T with B the prepared weight.
//
// Same machine shape as the int8 forward GEMM: workgroup tile BM (m) x BN (k), 4 waves 2x2, each
// wave (BM/2) x (BN/2) as 32x32 tiles of v_mfma_f32_32x32x16_{f16,bf16}; a ring of 4 LDS stages
// of 64 contraction bytes (32 elements) per operand row, filled three stages ahead with direct
// 128-bit L2 -> LDS loads dealt out one per MFMA group; fragments of the next contraction substep
// are read from LDS behind the MFMAs of the current one; one workgroup barrier per stage.
// dY is read row-major (16 rows x 64 bytes per wave load), the weight block-wise (1 KB per load).
// The weight tile is the MFMA's A operand, the dY tile its B operand: D[i][j], i <-> k, j <-> m,
// so a lane holds 4 consecutive k per accumulator quad; lane group g of an operand holds
// contraction elements 8g..8g+7 of the 16-element substep, the natural order of a 16-byte chunk.
// The accumulation order inside the matrix unit is the hardware's; results are compared within
// the fp32 accumulation bound, not bit for bit.
// ---------------------------------------------------------------------------------------------
template <int DT, int BM, int BN>
__global__ __launch_bounds__(kGemmThreads)
__attribute__((amdgpu_waves_per_eu(Tile<BM, BN>::kWavesPerSimd, Tile<BM, BN>::kWavesPerSimd)))
void linear_bwd_mfma_kernel(const uint8_t* __restrict__ dy, const uint8_t* __restrict__ wt,
                            uint16_t* __restrict__ dx, float* __restrict__ acc_out,
                            int M, int N, int K, int tiles_m, int tiles_n)
{
    using S = Store16<DT>;
    using T = Tile<BM, BN>;
    constexpr int MF = T::MF, NF = T::NF, XS = T::XS, WS = T::WS;
    __shared__ __attribute__((aligned(1024))) char lds[T::kLds];
    auto stage_ptr = [&](int st, int operand) -> char* { return &lds[st * T::kStageBytes + operand * T::kXBytes]; };

    int tm, tn;
    if (!tile_of_block((int)blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * BM, k0 = tn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int KT = N / kBwdCols;                                   // contraction tiles
    auto eff_tile = [&](int Tk) { return min(max(Tk, 0), KT - 1); };
    auto stage_of = [&](int Tk) { return (Tk < 0 ? 0 : Tk) & 3; };

    // direct loads: load j of wave w fills rows (4j + w)*16 .. +16 of a stage; lane i writes LDS
    // slot i of that 1 KB (row i/4, position i%4) and so fetches logical chunk (i%4) ^ swz64(row)
    const int lrow = lane >> 2;
    const int lchunk = (lane & 3) ^ (((lane >> 3) & 3) ^ ((lane >> 5) & 1));
    const uint8_t* gx[XS];
    const uint8_t* gw[WS];
    const int64_t row_bytes = (int64_t)N * 2;
#pragma unroll
    for (int j = 0; j < XS; ++j)
        gx[j] = dy + (int64_t)min(m0 + (4 * j + wave) * 16 + lrow, M - 1) * row_bytes + lchunk * 16;
#pragma unroll
    for (int j = 0; j < WS; ++j)
        gw[j] = wt + (int64_t)min((k0 >> 4) + 4 * j + wave, (K - 1) >> 4) * KT * 1024 + lane * 16;
    auto dma_x = [&](int Tk, int j) {
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(gx[j] + eff_tile(Tk) * kBK),
                                         (lds_ptr_t)(stage_ptr(stage_of(Tk), 0) + (4 * j + wave) * 1024), 16, 0, 0);
    };
    auto dma_w = [&](int Tk, int j) {
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(gw[j] + eff_tile(Tk) * 1024),
                                         (lds_ptr_t)(stage_ptr(stage_of(Tk), 1) + (4 * j + wave) * 1024), 16, 0, 0);
    };

    // LDS -> MFMA fragments
    const int frow = lane & 31, fgrp = lane >> 5;
    int foff[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) foff[kk] = frow * kBK + (((kk * 2 + fgrp) ^ swz64(frow)) << 4);
    const int xbase = wm * (BM / 2) * kBK, wbase = wn * (BN / 2) * kBK;
    i32x4 fx[2][MF], fw[2][NF];
    auto read_frag = [&](int set, int st, int kk, int idx) {
        if (idx < MF) fx[set][idx] = *reinterpret_cast<const i32x4*>(stage_ptr(st, 0) + xbase + idx * 32 * kBK + foff[kk]);
        else          fw[set][idx - MF] = *reinterpret_cast<const i32x4*>(stage_ptr(st, 1) + wbase + (idx - MF) * 32 * kBK + foff[kk]);
    };

    f32x16 acc[NF][MF];   // [k tile][m tile]; first written by the MFMAs of contraction tile 0

    constexpr int kFrags = MF + NF;
    // group g of substep `set`: MF MFMAs with the group's side items dealt out behind them
    auto group = [&](int set, int g, auto mode_tag, int nitems, auto&& item) {
        constexpr int MODE = decltype(mode_tag)::value;     // 0: pipeline fill, 1: math, 2: math into zero
        if (MODE == 0) {
            for (int k = 0; k < nitems; ++k) item(k);
            __builtin_amdgcn_sched_barrier(0);
            return;
        }
#pragma unroll
        for (int b = 0; b < MF; ++b) {
            if (MODE == 2 && set == 0) {
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                acc[g][b] = Mfma16<DT>::mma(fw[set][g], fx[set][b], zero);
            } else {
                acc[g][b] = Mfma16<DT>::mma(fw[set][g], fx[set][b], acc[g][b]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (b < MF - 1) {
                if (b < nitems) item(b);
            } else {
                for (int k = MF - 1; k < nitems; ++k) item(k);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // Iteration i consumes contraction tile i in two substeps; phase 0 issues the weight loads of
    // tile i+3, phase 1 the dY loads of tile i+4; loads return in issue order, so "tile i+1 has
    // landed" is one vmcnt wait with the number of loads issued after it.
    auto iteration = [&](int i, auto mode_tag) {
        constexpr bool MATH = decltype(mode_tag)::value != 0;
        const int st = i & 3;
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            const int r0 = g * kFrags / NF, nr = MATH ? (g + 1) * kFrags / NF - r0 : 0;
            group(0, g, mode_tag, nr + 1, [&](int k) {
                if (k < nr) { read_frag(1, st, 1, r0 + k); return; }
                if (g < WS) dma_w(i + 3, g);
            });
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(2 * XS + 2 * WS));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            const int r0 = g * kFrags / NF, nr = (i + 1 >= 0) ? (g + 1) * kFrags / NF - r0 : 0;
            group(1, g, mode_tag, nr + 1, [&](int k) {
                if (k < nr) { read_frag(0, (i + 1) & 3, 0, r0 + k); return; }
                if (g < XS) dma_x(i + 4, g);
            });
        }
    };
    using Fill = std::integral_constant<int, 0>;
    using Math = std::integral_constant<int, 1>;
    using Open = std::integral_constant<int, 2>;
    iteration(-4, Fill{});
    iteration(-3, Fill{});
    iteration(-2, Fill{});
    iteration(-1, Fill{});
    iteration(0, Open{});
#pragma unroll 1
    for (int it = 1; it < KT; ++it) iteration(it, Math{});
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // epilogue: D[i][j], i = 8*(v/4) + 4*(lane/32) + v%4 -> k, j = lane%32 -> m.  Each wave rounds
    // its block to 16 bits, stages it through its own LDS region in [m][k] order and writes dX
    // with 128-bit stores.
    char* epi = &lds[wave * T::kEpiBytes];
    const int wk0 = k0 + wn * (BN / 2), wm0 = m0 + wm * (BM / 2);
#pragma unroll
    for (int a = 0; a < NF; ++a)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int kl = a * 32 + 8 * g + 4 * fgrp;
#pragma unroll
            for (int b = 0; b < MF; ++b) {
                const int ml = b * 32 + frow;
                u32x2 pk = {S::pack(acc[a][b][4 * g], acc[a][b][4 * g + 1]), S::pack(acc[a][b][4 * g + 2], acc[a][b][4 * g + 3])};
                *reinterpret_cast<u32x2*>(epi + ml * T::kEpiStride + kl * 2) = pk;
            }
        }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    const bool vec_ok = (K & 7) == 0;
    constexpr int kChunksPerRow = BN / 16;
    constexpr int kRowsPerPass = 64 / kChunksPerRow;
    const int crow = lane / kChunksPerRow, cchunk = lane % kChunksPerRow;
#pragma unroll 4
    for (int p = 0; p < (BM / 2) / kRowsPerPass; ++p) {
        const int ml = p * kRowsPerPass + crow;
        const int m = wm0 + ml, k = wk0 + cchunk * 8;
        if (m >= M || k >= K) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(epi + ml * T::kEpiStride + cchunk * 16);
        uint16_t* dst = dx + (int64_t)m * K + k;
        if (vec_ok && k + 7 < K) {
            *reinterpret_cast<u32x4*>(dst) = v;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (k + e < K) dst[e] = (uint16_t)(v[e >> 1] >> (16 * (e & 1)));
        }
    }
    // inspection output: the fp32 sums before the 16-bit rounding, straight from the registers
    if (acc_out) {
#pragma unroll
        for (int a = 0; a < NF; ++a)
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int b = 0; b < MF; ++b) {
                    const int m = wm0 + b * 32 + frow, k = wk0 + a * 32 + 8 * g + 4 * fgrp;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (m < M && k + e < K) acc_out[(int64_t)m * K + k + e] = acc[a][b][4 * g + e];
                }
    }
}

template <int DT, int BM, int BN>
static void launch_bwd(const void* dy, const void* wt, void* dx, float* acc_out, int64_t M, int64_t N, int64_t K, hipStream_t st)
{
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((K + BN - 1) / BN);
    const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
    linear_bwd_mfma_kernel<DT, BM, BN><<<grid, kGemmThreads, 0, st>>>(
        static_cast<const uint8_t*>(dy), static_cast<const uint8_t*>(wt), static_cast<uint16_t*>(dx), acc_out,
        (int)M, (int)N, (int)K, tiles_m, tiles_n);
}

// The same GEMM on v_mfma_f32_16x16x32_{f16,bf16} through the tile body shared with the int8 forward GEMM
// (gemm_k64_body.h): 16x16 tiles, one MFMA per 64-byte stage row, scalar-addressed direct loads, chunked epilogue.
// The default: a register-only loop of the 16x16x32 form sustains about 18 % more than 32x32x16 on this
// power-limited part (1.97 against 1.67 PFLOP/s for f16).  dY is the body's row-major operand, the prepared
// weight its block operand; K of the body is the contraction length in bytes.
template <int DT, int BM, int BN>
__global__ __launch_bounds__(kGemmThreads)
__attribute__((amdgpu_waves_per_eu(Tile<BM, BN>::kWavesPerSimd, Tile<BM, BN>::kWavesPerSimd)))
void linear_bwd_k32_kernel(const uint8_t* __restrict__ dy, const uint8_t* __restrict__ wt,
                           uint16_t* __restrict__ dx, float* __restrict__ acc_out,
                           int M, int N, int K, int tiles_m, int tiles_n)
{
    __shared__ __attribute__((aligned(1024))) char lds[lds_bytes_k64<BM, BN>()];
    int tm, tn;
    if (!tile_of_block((int)blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    gemm_k64_body<DT, KW_I8B, BM, BN, false, false, 1>(reinterpret_cast<const int8_t*>(dy), wt, nullptr, nullptr, nullptr, dx,
                                                        reinterpret_cast<int32_t*>(acc_out), M, K, N * 2, tm, tn, lds);
}

template <int DT, int BM, int BN>
static void launch_bwd_k32(const void* dy, const void* wt, void* dx, float* acc_out, int64_t M, int64_t N, int64_t K, hipStream_t st)
{
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((K + BN - 1) / BN);
    const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
    linear_bwd_k32_kernel<DT, BM, BN><<<grid, kGemmThreads, 0, st>>>(
        static_cast<const uint8_t*>(dy), static_cast<const uint8_t*>(wt), static_cast<uint16_t*>(dx), acc_out,
        (int)M, (int)N, (int)K, tiles_m, tiles_n);
}

// 256x256 tiles unless they would leave most of the 256 CUs idle for a round; then 128x128
// (two workgroups per CU).  sasq_set_tuning(SASQ_TUNE_BWD_TILE, 1 | 2) forces one of them.
static bool bwd_small_tiles(int64_t M, int64_t K)
{
    if (tuning(SASQ_TUNE_BWD_TILE) == 1) return false;
    if (tuning(SASQ_TUNE_BWD_TILE) == 2) return true;
    const int64_t t256 = ((M + 255) / 256) * ((K + 255) / 256), t128 = ((M + 127) / 128) * ((K + 127) / 128);
    const double c256 = (double)((t256 + 255) / 256), c128 = (double)((t128 + 511) / 512) * 0.5 * 1.42;
    return c128 < c256;
}

static int64_t bwd_kpad(int64_t K) { return (K + 15) / 16 * 16; }
static int64_t bwd_npad(int64_t N) { return (N + kBwdCols - 1) / kBwdCols * kBwdCols; }
constexpr int64_t kBwdMaxProduct = INT64_C(1) << 40;    // elements of any operand or of the output

}  // namespace sasq

using namespace sasq;

extern "C" size_t sasq_bwd_weight_bytes(int64_t N, int64_t K)
{
    if (N <= 0 || K <= 0 || N > 0x3FFFFFFF || K > 0x7FFFFFFF || N > kBwdMaxProduct / K) return 0;
    return (size_t)bwd_kpad(K) * (size_t)bwd_npad(N) * 2;
}

extern "C" int sasq_prepare_bwd_weight(const void* wq, const float* s_w, void* wt, int64_t N, int64_t K,
                                       sasq_wfmt wf, sasq_dtype dt, void* stream)
{
    if (!wq || !s_w || !wt) return SASQ_ERR_NULL;
    if (N <= 0 || K <= 0 || N > 0x3FFFFFFF || K > 0x7FFFFFFF || N > kBwdMaxProduct / K) return SASQ_ERR_SHAPE;
    if (wf != SASQ_W_INT8 && wf != SASQ_W_INT4_PACKED) return SASQ_ERR_UNSUPPORTED;
    if (wf == SASQ_W_INT4_PACKED && (K & 1)) return SASQ_ERR_SHAPE;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    if (!aligned16(wt)) return SASQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    const int64_t Kpad = bwd_kpad(K), Npad = bwd_npad(N);
    const int64_t threads = Kpad * (Npad / 8);
    const int64_t grid = (threads + 255) / 256;
    if (grid > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    const auto* W = static_cast<const uint8_t*>(wq);
    auto* O = static_cast<uint8_t*>(wt);
    const bool i4 = wf == SASQ_W_INT4_PACKED;
    if (dt == SASQ_F16) {
        if (i4) prepare_bwd_weight_kernel<SASQ_F16, true><<<(int)grid, 256, 0, st>>>(W, s_w, O, N, K, Npad, Kpad);
        else    prepare_bwd_weight_kernel<SASQ_F16, false><<<(int)grid, 256, 0, st>>>(W, s_w, O, N, K, Npad, Kpad);
    } else {
        if (i4) prepare_bwd_weight_kernel<SASQ_BF16, true><<<(int)grid, 256, 0, st>>>(W, s_w, O, N, K, Npad, Kpad);
        else    prepare_bwd_weight_kernel<SASQ_BF16, false><<<(int)grid, 256, 0, st>>>(W, s_w, O, N, K, Npad, Kpad);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" int sasq_linear_bwd_input(const void* dy, const void* wt, void* dx, float* acc_out,
                                     int64_t M, int64_t N, int64_t K, sasq_dtype dt, void* stream)
{
    if (!dy || !wt || !dx) return SASQ_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0) return SASQ_ERR_SHAPE;
    if (M > 0x7FFFFFFF || N > 0x3FFFFFFF || K > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    if (M > kBwdMaxProduct / N || M > kBwdMaxProduct / K || N > kBwdMaxProduct / K) return SASQ_ERR_SHAPE;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    if (!aligned16(dy) || !aligned16(wt) || !aligned16(dx)) return SASQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    if (N % kBwdCols) {
        // rows of dY are not whole 64-byte stage rows: scalar kernel
        const int64_t grid = (M * K + 255) / 256;
        if (grid > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
        auto* DY = static_cast<const uint16_t*>(dy);
        auto* WT = static_cast<const uint8_t*>(wt);
        auto* DX = static_cast<uint16_t*>(dx);
        if (dt == SASQ_F16) linear_bwd_scalar_kernel<SASQ_F16><<<(int)grid, 256, 0, st>>>(DY, WT, DX, acc_out, M, N, K, bwd_npad(N));
        else                linear_bwd_scalar_kernel<SASQ_BF16><<<(int)grid, 256, 0, st>>>(DY, WT, DX, acc_out, M, N, K, bwd_npad(N));
        return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
    }
    const bool small = bwd_small_tiles(M, K);
    // the 16x16x32 kernel addresses dY rows with 32-bit byte offsets inside a 256-row tile
    if (tuning(SASQ_TUNE_LINEAR_MFMA) != 1 && N <= (INT64_C(1) << 22)) {
        if (dt == SASQ_F16) {
            if (small) launch_bwd_k32<SASQ_F16, 128, 128>(dy, wt, dx, acc_out, M, N, K, st);
            else       launch_bwd_k32<SASQ_F16, 256, 256>(dy, wt, dx, acc_out, M, N, K, st);
        } else {
            if (small) launch_bwd_k32<SASQ_BF16, 128, 128>(dy, wt, dx, acc_out, M, N, K, st);
            else       launch_bwd_k32<SASQ_BF16, 256, 256>(dy, wt, dx, acc_out, M, N, K, st);
        }
        return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
    }
    if (dt == SASQ_F16) {
        if (small) launch_bwd<SASQ_F16, 128, 128>(dy, wt, dx, acc_out, M, N, K, st);
        else       launch_bwd<SASQ_F16, 256, 256>(dy, wt, dx, acc_out, M, N, K, st);
    } else {
        if (small) launch_bwd<SASQ_BF16, 128, 128>(dy, wt, dx, acc_out, M, N, K, st);
        else       launch_bwd<SASQ_BF16, 256, 256>(dy, wt, dx, acc_out, M, N, K, st);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}
