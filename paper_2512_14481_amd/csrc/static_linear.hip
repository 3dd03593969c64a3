// Static-inference quantized linear (Sec. 3, Eq. 2) for gfx950: activation quantize with the
// fixed scale, int8 MFMA GEMM against frozen per-output-channel weights, dequantizing epilogue.
#include "sasq_device.h"

namespace sasq {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

// s_waitcnt immediates (gfx9 encoding): vmcnt split over bits [3:0] and [15:14]; expcnt and
// lgkmcnt left at "no wait".
constexpr int waitcnt_vm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }
constexpr int kWaitLgkm0 = 0xF | (0x3 << 14) | (0x7 << 4) | (0x0 << 8);

// ---------------------------------------------------------------------------------------------
// Activation quantize pre-pass: xq[m,k] = clamp(round(X[m,k]/s))  (Sec. 3, Eq. 1), int8.
// PERM8: store each aligned group of 8 codes as (k0,k2,k4,k6,k1,k3,k5,k7) -- the K order in
// which packed int4 weights unpack -- instead of natural order.
// ---------------------------------------------------------------------------------------------
template <int DT, bool PERM8>
__global__ __launch_bounds__(256) void quantize_act_kernel(
    const u32x4* __restrict__ x, const float* __restrict__ s_ptr, u32x2* __restrict__ xq,
    int64_t nvec, int64_t n, int bits)
{
    using S = Store16<DT>;
    const QConst k = make_qconst(*s_ptr, bits);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
        u32x4 v = x[i];
        float c[8];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            c[2 * w] = quantize(S::lo(v[w]), k).c;
            c[2 * w + 1] = quantize(S::hi(v[w]), k).c;
        }
        u32x2 o;
        if (PERM8) { o[0] = pack_codes4(c[0], c[2], c[4], c[6]); o[1] = pack_codes4(c[1], c[3], c[5], c[7]); }
        else       { o[0] = pack_codes4(c[0], c[1], c[2], c[3]); o[1] = pack_codes4(c[4], c[5], c[6], c[7]); }
        xq[i] = o;
    }
    if (!PERM8 && blockIdx.x == 0 && threadIdx.x < (unsigned)(n - nvec * 8)) {
        int64_t i = nvec * 8 + threadIdx.x;
        reinterpret_cast<int8_t*>(xq)[i] =
            (int8_t)code_of(quantize(S::one(reinterpret_cast<const uint16_t*>(x)[i]), k));
    }
}

// ---------------------------------------------------------------------------------------------
// Epilogue arithmetic, identical on every path:  y = fl32(fl32(acc) * fl32(s*s_w[n])) (+ bias).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float dequant(int acc, float c, float bias, bool has_bias)
{
    float y = (float)acc * c;
    if (has_bias) y = y + bias;
    return y;
}

// ---------------------------------------------------------------------------------------------
// Scalar kernel for shapes the MFMA kernel does not take (K not a multiple of 64): one thread
// per output element over pre-quantized activations.
// ---------------------------------------------------------------------------------------------
template <int DT, bool INT4>
__global__ __launch_bounds__(256) void linear_scalar_kernel(
    const int8_t* __restrict__ xq, const uint8_t* __restrict__ wq, const float* __restrict__ s_ptr,
    const float* __restrict__ s_w, const float* __restrict__ bias, uint16_t* __restrict__ y,
    int32_t* __restrict__ acc_out, int64_t M, int64_t N, int64_t K)
{
    using S = Store16<DT>;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * N) return;
    const int64_t m = idx / N, n = idx % N;
    const int8_t* xr = xq + m * K;
    int acc = 0;
    if (INT4) {
        const uint8_t* wr = wq + n * (K / 2);
        for (int64_t j = 0; j < K / 2; ++j) {
            int b = wr[j];
            int lo = ((b & 15) ^ 8) - 8, hi = ((b >> 4) ^ 8) - 8;
            acc += (int)xr[2 * j] * lo + (int)xr[2 * j + 1] * hi;
        }
    } else {
        const int8_t* wr = reinterpret_cast<const int8_t*>(wq) + n * K;
        for (int64_t k = 0; k < K; ++k) acc += (int)xr[k] * (int)wr[k];
    }
    const float c = *s_ptr * s_w[n];
    y[idx] = S::enc(dequant(acc, c, bias ? bias[n] : 0.0f, bias != nullptr));
    if (acc_out) acc_out[idx] = acc;
}

// ---------------------------------------------------------------------------------------------
// int8 MFMA GEMM over pre-quantized activations.
//
// Workgroup tile 256 (m) x 256 (n), 4 waves in a 2x2 arrangement, each wave owns a 128x128 block
// as 4x4 tiles of v_mfma_i32_32x32x32_i8 (256 int32 accumulators per lane, 1 wave per SIMD).
//
// K pipeline: a ring of 4 LDS stages of 64 K-bytes each (16 KB per operand per stage, 128 KB in
// all).  Operand tiles go L2 -> LDS with direct 128-bit LDS loads (no VGPR round trip), issued
// one per four MFMAs so the wave never sits in a burst of memory issue, and three stages ahead
// of their use.  Within a stage the fragments of the next K-substep are read from LDS while the
// MFMAs of the current one run; there is one workgroup barrier per stage.
//
// LDS stage layout: row r (an m or n index) holds its 64 K-bytes as four 16-byte chunks; chunk c
// is stored at position c ^ swz64(r), so that the 128-bit fragment reads of consecutive rows at
// one logical chunk fall in distinct banks (rocprof: SQ_LDS_BANK_CONFLICT = 0).
//
// The MFMA pairs byte j of lane-group g in its A operand with byte j of lane-group g in its B
// operand, so any assignment of K indices to (g, j) slots is valid as long as both operands use
// the same one; here slot (g, j) of K-substep kk is k = 32*kk + 16*g + j.  The weight tile is
// the MFMA's A operand and the activation tile its B operand: D[i][j] with i <-> n, j <-> m, so
// a lane holds 4 consecutive n per accumulator quad.
//
// Epilogue: each wave dequantizes its 128x128 block, stages it through its own LDS region as
// 16-bit values in [m][n] order and writes Y with 128-bit stores, 256 contiguous bytes per row.
// ---------------------------------------------------------------------------------------------
constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kStages = 4;
constexpr int kStageBytes = kBM * kBK;              // 16 KB per operand per stage
constexpr int kGemmThreads = 256;
constexpr int kEpiStride = 272;                     // bytes per staged output row: 256 + 16 (bank spread)
constexpr int kEpiBytes = 128 * kEpiStride;         // per wave
constexpr int kGemmLds = 4 * kEpiBytes > kStages * 2 * kStageBytes ? 4 * kEpiBytes : kStages * 2 * kStageBytes;

__device__ __forceinline__ int swz64(int r) { return ((r >> 1) & 3) ^ ((r >> 3) & 1); }

// XCD-aware tile order.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2:
// give every XCD a contiguous range of logical tile ids, and number the tiles so that 32
// consecutive ids (what one XCD's 32 CUs hold at a time) form an 8 (m) x 4 (n) block that shares
// 8 activation row-panels and 4 weight row-panels in that L2.
__device__ __forceinline__ bool tile_of_block(int bid, int tiles_m, int tiles_n, int& tm, int& tn)
{
    const int total = tiles_m * tiles_n;
    const int per = (total + 7) >> 3;
    const int logical = (bid & 7) * per + (bid >> 3);
    if (logical >= total) return false;
    constexpr int PN = 4;                              // n-tiles per panel
    const int panel = logical / (tiles_m * PN);
    const int in = logical - panel * tiles_m * PN;
    const int width = min(PN, tiles_n - panel * PN);   // last panel may be narrower
    tm = in / width;
    tn = panel * PN + in % width;
    return true;
}

template <int DT>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void linear_mfma_kernel(const int8_t* __restrict__ xq, const int8_t* __restrict__ wq,
                        const float* __restrict__ s_ptr, const float* __restrict__ s_w,
                        const float* __restrict__ bias, uint16_t* __restrict__ y,
                        int32_t* __restrict__ acc_out, int M, int N, int K, int tiles_m, int tiles_n)
{
    using S = Store16<DT>;
    __shared__ __attribute__((aligned(1024))) char lds[kGemmLds];
    auto stage_ptr = [&](int st, int operand) -> char* { return &lds[(st * 2 + operand) * kStageBytes]; };

    int tm, tn;
    if (!tile_of_block(blockIdx.x, tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * kBM, n0 = tn * kBN;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    // ---- global -> LDS: load j of wave w fills rows (4j + w)*16 .. +16 of a stage (1 KB) ----
    // Lane i writes LDS slot i of that 1 KB: row i/4, position i%4; it therefore fetches the
    // logical chunk (i%4) ^ swz64(row), and swz64 of these rows depends on the lane only.
    const int lrow = lane >> 2;
    const int lchunk = (lane & 3) ^ (((lane >> 3) & 3) ^ ((lane >> 5) & 1));
    const int8_t* gx[4];
    const int8_t* gw[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = (4 * j + wave) * 16 + lrow;
        const int mr = min(m0 + r, M - 1), nr = min(n0 + r, N - 1);   // rows past the edge re-read the last row
        gx[j] = xq + (int64_t)mr * K + lchunk * 16;
        gw[j] = wq + (int64_t)nr * K + lchunk * 16;
    }
    // load q (0..3: activation slabs, 4..7: weight slabs) of K tile kt into stage st
    auto issue_one = [&](int st, int kt, int q) {
        const int j = q & 3;
        const int slab = (4 * j + wave) * 1024;
        if (q < 4) __builtin_amdgcn_global_load_lds((glb_ptr_t)(gx[j] + kt * kBK), (lds_ptr_t)(stage_ptr(st, 0) + slab), 16, 0, 0);
        else       __builtin_amdgcn_global_load_lds((glb_ptr_t)(gw[j] + kt * kBK), (lds_ptr_t)(stage_ptr(st, 1) + slab), 16, 0, 0);
    };

    // ---- LDS -> registers ----
    const int frow = lane & 31, fgrp = lane >> 5;
    int foff[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) foff[kk] = frow * kBK + (((kk * 2 + fgrp) ^ swz64(frow)) << 4);
    const int xbase = wm * 128 * kBK, wbase = wn * 128 * kBK;
    i32x4 fx[2][4], fw[2][4];
    auto read_x = [&](int set, int st, int kk, int t) {
        fx[set][t] = *reinterpret_cast<const i32x4*>(stage_ptr(st, 0) + xbase + t * 32 * kBK + foff[kk]);
    };
    auto read_w = [&](int set, int st, int kk, int t) {
        fw[set][t] = *reinterpret_cast<const i32x4*>(stage_ptr(st, 1) + wbase + t * 32 * kBK + foff[kk]);
    };

    i32x16 acc[4][4];   // [n tile][m tile]
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    // Loads past the last K tile are clamped to the last tile: they land in stages that are free
    // anyway, keep the loop branch-free and the vmcnt bookkeeping constant.
    const int KT = K / kBK;
    // prologue: tiles 0, 1, 2 and the first half of tile 3
#pragma unroll
    for (int t0 = 0; t0 < 3; ++t0) {
#pragma unroll
        for (int q = 0; q < 8; ++q) issue_one(t0, min(t0, KT - 1), q);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_one(3, min(3, KT - 1), q);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(20));             // tile 0 has landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int t = 0; t < 4; ++t) { read_x(0, 0, 0, t); read_w(0, 0, 0, t); }

    for (int kt = 0; kt < KT; ++kt) {
        const int st = kt & 3;
        const int t3 = min(kt + 3, KT - 1), t4 = min(kt + 4, KT - 1);
        // phase 0: MFMAs of K-substep 0; read substep 1; second half of tile kt+3
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            read_x(1, st, 1, g); read_w(1, st, 1, g);
            issue_one((kt + 3) & 3, t3, 4 + g);
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[g][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[0][g], fx[0][b], acc[g][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        asm volatile("" ::: "memory");
        // Substep-1 fragments are in registers, so this stage may be refilled after the barrier;
        // tile kt+1 has landed for this wave (the 16 newer loads may still be in flight), so after
        // the barrier it is complete for everyone.
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(16));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // phase 1: MFMAs of substep 1; read substep 0 of the next tile; first half of tile kt+4
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            read_x(0, (kt + 1) & 3, 0, g); read_w(0, (kt + 1) & 3, 0, g);
            issue_one(st, t4, g);
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[g][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[1][g], fx[1][b], acc[g][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // drain the clamped tail loads and the last fragment reads before LDS is reused
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ---- epilogue: D[i][j], i = 8*(v/4) + 4*(lane/32) + v%4 -> n, j = lane%32 -> m ----
    const float s = *s_ptr;
    const bool has_bias = bias != nullptr;
    char* epi = &lds[wave * kEpiBytes];
    const int wn0 = n0 + wn * 128, wm0 = m0 + wm * 128;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nl = a * 32 + 8 * g + 4 * fgrp;          // column within the wave's block
            float c[4], bz[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int ne = min(wn0 + nl + e, N - 1);
                c[e] = s * s_w[ne];
                bz[e] = has_bias ? bias[ne] : 0.0f;
            }
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int ml = b * 32 + frow;
                u32x2 pk;
                pk[0] = S::pack(dequant(acc[a][b][4 * g + 0], c[0], bz[0], has_bias),
                                dequant(acc[a][b][4 * g + 1], c[1], bz[1], has_bias));
                pk[1] = S::pack(dequant(acc[a][b][4 * g + 2], c[2], bz[2], has_bias),
                                dequant(acc[a][b][4 * g + 3], c[3], bz[3], has_bias));
                *reinterpret_cast<u32x2*>(epi + ml * kEpiStride + nl * 2) = pk;
                if (acc_out) {
                    const int m = wm0 + ml, n = wn0 + nl;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (m < M && n + e < N) acc_out[(int64_t)m * N + n + e] = acc[a][b][4 * g + e];
                }
            }
        }
    }
    // each wave reads back only what it wrote itself: no workgroup barrier needed
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    const bool vec_ok = (N & 7) == 0;
    const int crow = lane >> 4, cchunk = lane & 15;            // 4 rows x 16 chunks of 16 B per pass
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
        const int ml = it * 4 + crow;
        const int m = wm0 + ml, n = wn0 + cchunk * 8;
        if (m >= M || n >= N) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(epi + ml * kEpiStride + cchunk * 16);
        uint16_t* dst = y + (int64_t)m * N + n;
        if (vec_ok && n + 7 < N) {
            *reinterpret_cast<u32x4*>(dst) = v;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (n + e < N) dst[e] = (uint16_t)(v[e >> 1] >> (16 * (e & 1)));
        }
    }
}

// W4 -> W8 unpack pre-pass (first version of the W4A8 path): natural K order, sign-extended.
__global__ __launch_bounds__(256) void unpack_int4_kernel(const uint8_t* __restrict__ w4,
                                                          int8_t* __restrict__ w8, int64_t nbytes)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nbytes; i += (int64_t)gridDim.x * 256) {
        int b = w4[i];
        w8[2 * i] = (int8_t)(((b & 15) ^ 8) - 8);
        w8[2 * i + 1] = (int8_t)(((b >> 4) ^ 8) - 8);
    }
}

static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace sasq

using namespace sasq;

extern "C" size_t sasq_static_linear_workspace(int64_t M, int64_t N, int64_t K, sasq_wfmt wf)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    size_t bytes = round_up((size_t)M * (size_t)K, 256);              // quantized activations
    if (wf == SASQ_W_INT4_PACKED) bytes += round_up((size_t)N * (size_t)K, 256);   // unpacked weights
    return bytes;
}

extern "C" int sasq_static_linear(const void* x, const float* s, const void* wq, const float* s_w,
                                  const float* bias, void* y, int32_t* acc_out, int8_t* xq_out,
                                  int64_t M, int64_t N, int64_t K, int a_bits, sasq_wfmt wf, sasq_dtype dt,
                                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !s || !wq || !s_w || !y) return SASQ_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0) return SASQ_ERR_SHAPE;
    const int64_t lim = INT64_C(1) << 40;
    if (M > lim / K || N > lim / K || M > lim / N || K > 131071 || M > 0x7FFFFFFF || N > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    if (a_bits < 2 || a_bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (wf != SASQ_W_INT8 && wf != SASQ_W_INT4_PACKED) return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    if (wf == SASQ_W_INT4_PACKED && (K & 1)) return SASQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(wq) || !aligned16(y) || (acc_out && !aligned16(acc_out)) ||
        (xq_out && (reinterpret_cast<uintptr_t>(xq_out) & 7u))) return SASQ_ERR_ALIGN;
    const size_t need = sasq_static_linear_workspace(M, N, K, wf);
    if (!workspace || workspace_bytes < need) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;

    hipStream_t st = as_stream(stream);
    int8_t* xq_ws = static_cast<int8_t*>(workspace);
    int8_t* w8_ws = xq_ws + round_up((size_t)M * (size_t)K, 256);

    // pass 1: quantize the activations with the fixed scale (no reduction over X anywhere)
    const int64_t n = M * K, nvec = n / 8;
    int64_t qb = (nvec + 255) / 256;
    const int qgrid = (int)(qb < 1 ? 1 : (qb > 65536 ? 65536 : qb));
    auto X = static_cast<const u32x4*>(x);
    if (dt == SASQ_F16) quantize_act_kernel<SASQ_F16, false><<<qgrid, 256, 0, st>>>(X, s, reinterpret_cast<u32x2*>(xq_ws), nvec, n, a_bits);
    else                quantize_act_kernel<SASQ_BF16, false><<<qgrid, 256, 0, st>>>(X, s, reinterpret_cast<u32x2*>(xq_ws), nvec, n, a_bits);
    if (xq_out) {
        if (dt == SASQ_F16) quantize_act_kernel<SASQ_F16, false><<<qgrid, 256, 0, st>>>(X, s, reinterpret_cast<u32x2*>(xq_out), nvec, n, a_bits);
        else                quantize_act_kernel<SASQ_BF16, false><<<qgrid, 256, 0, st>>>(X, s, reinterpret_cast<u32x2*>(xq_out), nvec, n, a_bits);
    }

    const int8_t* w8 = static_cast<const int8_t*>(wq);
    const bool mfma_ok = (K % kBK) == 0 && K >= kBK;
    if (wf == SASQ_W_INT4_PACKED && mfma_ok) {
        const int64_t nb = N * (K / 2);
        int64_t ub = (nb + 255) / 256;
        unpack_int4_kernel<<<(int)(ub > 65536 ? 65536 : ub), 256, 0, st>>>(static_cast<const uint8_t*>(wq), w8_ws, nb);
        w8 = w8_ws;
    }

    if (mfma_ok) {
        const int tiles_m = (int)((M + kBM - 1) / kBM), tiles_n = (int)((N + kBN - 1) / kBN);
        const int total = tiles_m * tiles_n;
        const int grid = ((total + 7) / 8) * 8;
        if (dt == SASQ_F16)
            linear_mfma_kernel<SASQ_F16><<<grid, kGemmThreads, 0, st>>>(xq_ws, w8, s, s_w, bias, static_cast<uint16_t*>(y), acc_out, (int)M, (int)N, (int)K, tiles_m, tiles_n);
        else
            linear_mfma_kernel<SASQ_BF16><<<grid, kGemmThreads, 0, st>>>(xq_ws, w8, s, s_w, bias, static_cast<uint16_t*>(y), acc_out, (int)M, (int)N, (int)K, tiles_m, tiles_n);
    } else {
        const int64_t total = M * N;
        const int64_t blocks = (total + 255) / 256;
        if (blocks > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
        auto W = static_cast<const uint8_t*>(wq);
        auto Y = static_cast<uint16_t*>(y);
        if (dt == SASQ_F16) {
            if (wf == SASQ_W_INT8) linear_scalar_kernel<SASQ_F16, false><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s, s_w, bias, Y, acc_out, M, N, K);
            else                   linear_scalar_kernel<SASQ_F16, true><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s, s_w, bias, Y, acc_out, M, N, K);
        } else {
            if (wf == SASQ_W_INT8) linear_scalar_kernel<SASQ_BF16, false><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s, s_w, bias, Y, acc_out, M, N, K);
            else                   linear_scalar_kernel<SASQ_BF16, true><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s, s_w, bias, Y, acc_out, M, N, K);
        }
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}
