// Static-inference quantized linear (Sec. 3, Eq. 2) for gfx950: activation quantize with the
// fixed scale, int8 MFMA GEMM against frozen per-output-channel weights, dequantizing epilogue.
#include "sasq_device.h"
#include "gemm_tile.h"
#include "gemm_k64.h"
#include <cstdlib>
#include <cstring>
#include <type_traits>

namespace sasq {

// ---------------------------------------------------------------------------------------------
// Activation quantize pre-pass: xq[m,k] = clamp(round(X[m,k]/s))  (Sec. 3, Eq. 1), int8.
// PERM8: store each aligned group of 8 codes as (k0,k2,k4,k6,k1,k3,k5,k7) -- the K order in
// which packed int4 weights unpack -- instead of natural order.
// TILED: store in the GEMM's staging layout instead of row-major: the matrix is cut into blocks
// of 16 rows x 64 K-bytes, block (rb, kb) is the 1 KB at ((rb * K/64) + kb) * 1024, and inside a
// block the 16-byte chunk c of row r sits at 16 * (4r + (c ^ swz64(r))) -- byte for byte what one
// wave's direct-to-LDS load deposits, so the GEMM fetches each block as one contiguous 1 KB read
// (full cache lines) instead of sixteen 64-byte row pieces.  Needs K % 64 == 0.
// ---------------------------------------------------------------------------------------------

template <int DT, bool PERM8, bool TILED>
__device__ __forceinline__ void quantize_act_body(
    const u32x4* __restrict__ x, const float* __restrict__ s_ptr, u32x2* __restrict__ xq,
    int64_t nvec, int64_t n, int K, int bits, int block, int nblocks)
{
    using S = Store16<DT>;
    const QConst k = make_qconst(*s_ptr, bits);
    const int kvec = K >> 3;                      // 8-element vectors per row
    for (int64_t i = (int64_t)block * 256 + threadIdx.x; i < nvec; i += (int64_t)nblocks * 256) {
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
        if (TILED) {
            const int64_t m = i / kvec;
            const int k0 = (int)(i - m * kvec) << 3;
            const int r = (int)(m & 15), ch = (k0 & 63) >> 4;
            const int64_t blk = (m >> 4) * (K >> 6) + (k0 >> 6);
            const int64_t off = blk * 1024 + ((4 * r + (ch ^ swz64(r))) << 4) + (k0 & 15);
            *reinterpret_cast<u32x2*>(reinterpret_cast<char*>(xq) + off) = o;
        } else {
            xq[i] = o;
        }
    }
    if (!PERM8 && !TILED && block == 0 && threadIdx.x < (unsigned)(n - nvec * 8)) {
        int64_t i = nvec * 8 + threadIdx.x;
        reinterpret_cast<int8_t*>(xq)[i] =
            (int8_t)code_of(quantize(S::one(reinterpret_cast<const uint16_t*>(x)[i]), k));
    }
}

template <int DT, bool PERM8, bool TILED>
__global__ __launch_bounds__(256) void quantize_act_kernel(
    const u32x4* __restrict__ x, const float* __restrict__ s_ptr, u32x2* __restrict__ xq,
    int64_t nvec, int64_t n, int K, int bits)
{
    quantize_act_body<DT, PERM8, TILED>(x, s_ptr, xq, nvec, n, K, bits, (int)blockIdx.x, (int)gridDim.x);
}

// The activation pre-passes of a layer.  Projections that read the same X (q/k/v, gate/up: one
// activation tensor, one factor each) form one entry: X is loaded once and quantized with every
// member's factor into that member's staging buffer.
constexpr int kMaxQuantShare = 3;
struct QuantItem {
    const void* x;
    int M, K;
    int ns;                                  // members
    const float* s[kMaxQuantShare];
    int8_t* xq[kMaxQuantShare];
};
struct QuantBatch {
    QuantItem it[kMaxLinearBatch];
    int first_block[kMaxLinearBatch + 1];
    int count;
};

// One wave per 1 KB staging block (16 rows x 64 K): lane l quantizes the 16 elements of chunk l%4
// of row l/4 (two 128-bit loads; a row's 64 elements are one full 128-byte line) and the wave
// writes the block as one contiguous, fully coalesced 1 KB.  Walking X linearly instead and
// scattering 8-byte pieces into the blocks writes half cache lines: 43.5 us against 36.2 us for
// the three inputs of the 7B MLP (more blocks in flight per wave were slower: 37.2 us with two,
// 39.5 with four).  NS members share the loads.
template <int DT, bool PERM8, int NS>
__device__ __forceinline__ void quantize_act_blocks_body(const QuantItem& it, int bits, int block, int nblocks)
{
    using S = Store16<DT>;
    const uint16_t* __restrict__ x = static_cast<const uint16_t*>(it.x);
    const int M = it.M, K = it.K, KT = K >> 6;
    const int64_t nblk = (int64_t)((M + 15) >> 4) * KT;
    QConst k[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) k[j] = make_qconst(*it.s[j], bits);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane >> 2, c = lane & 3;
    const int slot = ((4 * r + (c ^ swz64(r))) << 4);            // byte position of this lane's chunk in a block
    for (int64_t g = (int64_t)block * 4 + wave; g < nblk; g += (int64_t)nblocks * 4) {
        const int64_t rb = g / KT;
        const int kb = (int)(g - rb * KT);
        const int64_t m = rb * 16 + r;
        if (m >= M) continue;                                   // rows past M in the last row block stay unwritten (never used)
        const u32x4* p = reinterpret_cast<const u32x4*>(x + m * K + kb * 64 + c * 16);
        u32x4 v[2];
        v[0] = __builtin_nontemporal_load(p);
        v[1] = __builtin_nontemporal_load(p + 1);
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            float cc[16];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    cc[8 * h + 2 * w] = quantize(S::lo(v[h][w]), k[j]).c;
                    cc[8 * h + 2 * w + 1] = quantize(S::hi(v[h][w]), k[j]).c;
                }
            u32x4 o;
            if (PERM8) {
                o[0] = pack_codes4(cc[0], cc[2], cc[4], cc[6]);    o[1] = pack_codes4(cc[1], cc[3], cc[5], cc[7]);
                o[2] = pack_codes4(cc[8], cc[10], cc[12], cc[14]); o[3] = pack_codes4(cc[9], cc[11], cc[13], cc[15]);
            } else {
                o[0] = pack_codes4(cc[0], cc[1], cc[2], cc[3]);    o[1] = pack_codes4(cc[4], cc[5], cc[6], cc[7]);
                o[2] = pack_codes4(cc[8], cc[9], cc[10], cc[11]);  o[3] = pack_codes4(cc[12], cc[13], cc[14], cc[15]);
            }
            *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(it.xq[j]) + g * 1024 + slot) = o;
        }
    }
}

// one tensor, one factor: the pre-pass of a single sasq_static_linear call
template <int DT, bool PERM8>
__global__ __launch_bounds__(256) void quantize_act_blocks_kernel(const QuantItem it, int bits)
{
    quantize_act_blocks_body<DT, PERM8, 1>(it, bits, (int)blockIdx.x, (int)gridDim.x);
}

template <int DT, bool PERM8>
__global__ __launch_bounds__(256) void quantize_act_batch_kernel(const QuantBatch b, int bits)
{
    int k = 0;
#pragma unroll
    for (int i = 1; i < kMaxLinearBatch; ++i)
        if (i < b.count && (int)blockIdx.x >= b.first_block[i]) k = i;
    const QuantItem& it = b.it[k];
    const int block = (int)blockIdx.x - b.first_block[k], nblocks = b.first_block[k + 1] - b.first_block[k];
    if (it.ns == 2)      quantize_act_blocks_body<DT, PERM8, 2>(it, bits, block, nblocks);
    else if (it.ns == 3) quantize_act_blocks_body<DT, PERM8, 3>(it, bits, block, nblocks);
    else                 quantize_act_blocks_body<DT, PERM8, 1>(it, bits, block, nblocks);
}

// Same pre-pass with one factor per group of `group` consecutive channels (Sec. 3, Eq. 3; Eq. 1
// per group): the vector form needs group % 8 == 0 and K % 8 == 0 (a vector never straddles two
// groups), the element form takes any group.
template <int DT, bool PERM8, bool TILED>
__global__ __launch_bounds__(256) void quantize_act_grouped_kernel(
    const u32x4* __restrict__ x, const float* __restrict__ s_g, u32x2* __restrict__ xq,
    int64_t nvec, int K, int group, int bits)
{
    using S = Store16<DT>;
    const int kvec = K >> 3;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
        const int64_t m = i / kvec;
        const int k0 = (int)(i - m * kvec) << 3;
        const QConst k = make_qconst(s_g[k0 / group], bits);
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
        if (TILED) {
            const int r = (int)(m & 15), ch = (k0 & 63) >> 4;
            const int64_t blk = (m >> 4) * (K >> 6) + (k0 >> 6);
            const int64_t off = blk * 1024 + ((4 * r + (ch ^ swz64(r))) << 4) + (k0 & 15);
            *reinterpret_cast<u32x2*>(reinterpret_cast<char*>(xq) + off) = o;
        } else {
            xq[i] = o;
        }
    }
}

template <int DT>
__global__ __launch_bounds__(256) void quantize_act_grouped_elem_kernel(
    const uint16_t* __restrict__ x, const float* __restrict__ s_g, int8_t* __restrict__ xq,
    int64_t n, int K, int group, int bits)
{
    using S = Store16<DT>;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const QConst k = make_qconst(s_g[(int)(i % K) / group], bits);
        xq[i] = (int8_t)code_of(quantize(S::one(x[i]), k));
    }
}

// Dynamic per-token pre-pass (the online step static factors remove, Sec. 3): one workgroup per
// row finds the row's absmax (an integer max of 15-bit magnitudes: exact, order-independent),
// forms s_m = fl32(absmax / Qp) (1 for an all-zero row), then re-reads the row (it is in L2) and
// quantizes it with s_m.  VEC: K % 8 == 0, 128-bit accesses, optional staging layout; otherwise
// element by element, row-major only.
template <int DT, bool PERM8, bool TILED, bool VEC>
__global__ __launch_bounds__(256) void quantize_rows_kernel(
    const uint16_t* __restrict__ x, int8_t* __restrict__ xq, float* __restrict__ s_row, int K, int bits)
{
    using S = Store16<DT>;
    __shared__ uint32_t sh[4];
    const int64_t m = blockIdx.x;
    const uint16_t* row = x + m * K;
    uint32_t mx = 0;
    if (VEC) {
        const u32x4* rv = reinterpret_cast<const u32x4*>(row);
        for (int i = threadIdx.x; i < (K >> 3); i += 256) {
            const u32x4 v = rv[i];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t lo = v[w] & 0x7FFFu, hi = (v[w] >> 16) & 0x7FFFu;
                mx = lo > mx ? lo : mx;
                mx = hi > mx ? hi : mx;
            }
        }
    } else {
        for (int i = threadIdx.x; i < K; i += 256) {
            const uint32_t a = row[i] & 0x7FFFu;
            mx = a > mx ? a : mx;
        }
    }
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = max(max(sh[0], sh[1]), max(sh[2], sh[3]));
    const float sm = mx == 0 ? 1.0f : S::one((uint16_t)mx) / (float)((1 << (bits - 1)) - 1);
    if (threadIdx.x == 0) s_row[m] = sm;
    const QConst k = make_qconst(sm, bits);
    if (VEC) {
        const u32x4* rv = reinterpret_cast<const u32x4*>(row);
        for (int i = threadIdx.x; i < (K >> 3); i += 256) {
            const u32x4 v = rv[i];
            float c[8];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                c[2 * w] = quantize(S::lo(v[w]), k).c;
                c[2 * w + 1] = quantize(S::hi(v[w]), k).c;
            }
            u32x2 o;
            if (PERM8) { o[0] = pack_codes4(c[0], c[2], c[4], c[6]); o[1] = pack_codes4(c[1], c[3], c[5], c[7]); }
            else       { o[0] = pack_codes4(c[0], c[1], c[2], c[3]); o[1] = pack_codes4(c[4], c[5], c[6], c[7]); }
            const int k0 = i << 3;
            if (TILED) {
                const int r = (int)(m & 15), ch = (k0 & 63) >> 4;
                const int64_t blk = (m >> 4) * (K >> 6) + (k0 >> 6);
                const int64_t off = blk * 1024 + ((4 * r + (ch ^ swz64(r))) << 4) + (k0 & 15);
                *reinterpret_cast<u32x2*>(reinterpret_cast<char*>(xq) + off) = o;
            } else {
                *reinterpret_cast<u32x2*>(xq + m * K + k0) = o;
            }
        }
    } else {
        for (int i = threadIdx.x; i < K; i += 256)
            xq[m * K + i] = (int8_t)code_of(quantize(S::one(row[i]), k));
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
template <int DT, bool INT4, bool ROWS = false>
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
    const float c = s_ptr[ROWS ? m : 0] * s_w[n];      // ROWS: one factor per row (dynamic per-token)
    y[idx] = S::enc(dequant(acc, c, bias ? bias[n] : 0.0f, bias != nullptr));
    if (acc_out) acc_out[idx] = acc;
}

// Grouped form (Sec. 3, Eq. 3) for shapes the MFMA kernel does not take: per group an exact int32
// product, folded into fp32 with one fused multiply-add per group in ascending order.
template <int DT, bool INT4>
__global__ __launch_bounds__(256) void linear_grouped_scalar_kernel(
    const int8_t* __restrict__ xq, const uint8_t* __restrict__ wq, const float* __restrict__ s_g,
    const float* __restrict__ s_w, const float* __restrict__ bias, uint16_t* __restrict__ y,
    float* __restrict__ f_out, int64_t M, int64_t N, int64_t K, int64_t group)
{
    using S = Store16<DT>;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= M * N) return;
    const int64_t m = idx / N, n = idx % N;
    const int8_t* xr = xq + m * K;
    float f = 0.0f;
    for (int64_t g0 = 0; g0 < K; g0 += group) {
        int acc = 0;
        for (int64_t k = g0; k < g0 + group; ++k) {
            int w;
            if (INT4) {
                const int b = wq[n * (K / 2) + k / 2];
                w = (((k & 1) ? (b >> 4) : (b & 15)) ^ 8) - 8;
            } else {
                w = reinterpret_cast<const int8_t*>(wq)[n * K + k];
            }
            acc += (int)xr[k] * w;
        }
        f = __builtin_fmaf((float)acc, s_g[g0 / group], f);
    }
    if (f_out) f_out[idx] = f;
    float yv = f * s_w[n];
    if (bias) yv = yv + bias[n];
    y[idx] = S::enc(yv);
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
constexpr int64_t kFusedMaxN = 0;                   // quantize-on-load when N has at most this many columns
constexpr double kCost128x256 = 1.28, kCost128x128 = 1.42;   // time per output element relative to 256x256 tiles

// Operand paths of the GEMM kernel.
//   XMODE 0: activations were quantized by a separate pass; int8 tile goes L2 -> LDS directly.
//   XMODE 1: quantize-on-load: the 16-bit activation tile is loaded into registers, quantized
//            with the fixed scale (Sec. 3, Eq. 1) and written to LDS as int8.
//   WMODE 0: int8 weights, L2 -> LDS directly.
//   WMODE 1: packed int4 weights: loaded into registers and unpacked there.  A nibble moved to
//            the high half of a byte is the int8 value 16*w, so two mask/shift operations turn
//            8 nibbles into 8 bytes; the accumulator is then exactly 16*acc and is shifted back
//            in the epilogue.  The even nibbles of a dword come out before the odd ones, so
//            within every group of 8 consecutive k the byte order is (0,2,4,6,1,3,5,7); the
//            activation bytes are stored in the same order (any K order common to both operands
//            gives the same dot product).
//   WMODE 2: int8 weights pre-arranged by sasq_pack_weight in the same 1 KB blocks of 16 rows x 64
//            K-bytes as the staged activations: each direct load is one contiguous 1 KB.
//   WMODE 3: int4 weights pre-arranged by sasq_pack_weight: they go L2 -> LDS still packed (half
//            the bytes) and are unpacked in registers between the LDS fragment read and the MFMA
//            (4 operations per 32x16 fragment).  A 1 KB block holds 32 rows x 64 k; the 8 bytes of
//            (K-substep kk, lane group g, row r) sit at 512 kk + 256 g + 8 r, which is exactly
//            the order in which the 64 lanes of a fragment read fetch them (conflict-free), and
//            their nibbles are ordered so that the two mask/shift operations per dword yield
//            natural K order (byte b of the first dword: k = b low, k = 4 + b high; second dword
//            likewise for k = 8.., 12..), so the activation bytes stay in natural order.
enum { X_PREQ = 0, X_FUSED = 1 };
enum { W_I8 = 0, W_I4 = 1, W_I8B = 2, W_I4B = 3 };
static_assert(W_I8 == SASQ_W_INT8 && W_I4 == SASQ_W_INT4_PACKED && W_I8B == SASQ_W_INT8_BLOCKED && W_I4B == SASQ_W_INT4_BLOCKED,
              "the weight paths are numbered like the interface's weight formats");

// GROUPED (Sec. 3, Eq. 3): one activation factor per group of `group_tiles` K tiles.  s_ptr then
// points at the G factors; the int32 accumulators cover one group at a time (the first K-substep
// of a group multiplies into a zero accumulator operand) and are folded into fp32 sums at each
// group's end, f = fma(fl32(acc), s_g, f) in ascending group order; the epilogue applies s_w and
// the bias to f.  acc_out then receives f (as float).  Needs tiles with at most 128 accumulators
// per lane (128x256, 128x128), as f takes as many registers again.
// ROWS: one activation factor per row of X (dynamic per-token quantization, the baseline of
// Sec. 3 / Sec. 4.5): s_ptr points at the M factors and the epilogue uses fl32(s_m * s_w[n]).
template <int DT, int XMODE, int WMODE, int BM, int BN, bool GROUPED = false, bool ROWS = false>
__device__ __forceinline__
void linear_mfma_body(const void* __restrict__ xin, const uint8_t* __restrict__ wq,
                      const float* __restrict__ s_ptr, const float* __restrict__ s_w,
                      const float* __restrict__ bias, uint16_t* __restrict__ y,
                      int32_t* __restrict__ acc_out, int M, int N, int K, int a_bits,
                      int tiles_m, int tiles_n, int group_tiles, int bid)
{
    using S = Store16<DT>;
    using T = Tile<BM, BN>;
    static_assert(!GROUPED || (BM == 128 && XMODE == X_PREQ), "grouped factors: 128-row tiles over staged activations");
    static_assert(!ROWS || (!GROUPED && XMODE == X_PREQ), "per-row factors: staged activations");
    constexpr int MF = T::MF, NF = T::NF, XS = T::XS, WS = T::WS;
    __shared__ __attribute__((aligned(1024))) char lds[T::kLds];
    auto stage_ptr = [&](int st, int operand) -> char* { return &lds[st * T::kStageBytes + operand * T::kXBytes]; };

    int tm, tn;
    if (!tile_of_block(bid, tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int KT = K / kBK;
    auto eff_tile = [&](int Tk) { return min(max(Tk, 0), KT - 1); };
    // LDS stage of K tile Tk.  Tiles before the first are directed at tile 0's own stage (an
    // identical rewrite), tiles past the last at the stage they would own (free by then).
    auto stage_of = [&](int Tk) { return (Tk < 0 ? 0 : Tk) & 3; };

    // ---- direct L2 -> LDS path: load j of wave w fills rows (4j + w)*16 .. +16 of a stage ----
    // Lane i writes LDS slot i of that 1 KB: row i/4, position i%4; it therefore fetches the
    // logical chunk (i%4) ^ swz64(row), and swz64 of these rows depends on the lane only.
    const int lrow = lane >> 2;
    const int lchunk = (lane & 3) ^ (((lane >> 3) & 3) ^ ((lane >> 5) & 1));
    const int8_t* gx[XS];
    const int8_t* gw[WS];
    // pre-quantized activations are stored tiled (see quantize_act_kernel): slab j of wave w is the
    // contiguous 1 KB block (row block, K tile); row blocks past the edge re-read the last block
    const int last_rb = (M - 1) >> 4;
#pragma unroll
    for (int j = 0; j < XS; ++j)
        gx[j] = static_cast<const int8_t*>(xin) + (int64_t)min((m0 >> 4) + 4 * j + wave, last_rb) * KT * 1024 + lane * 16;
#pragma unroll
    for (int j = 0; j < WS; ++j) {
        if (WMODE == W_I8B) {          // blocks of 16 rows
            gw[j] = reinterpret_cast<const int8_t*>(wq) + (int64_t)min((n0 >> 4) + 4 * j + wave, (N - 1) >> 4) * KT * 1024 + lane * 16;
        } else if (WMODE == W_I4B) {   // blocks of 32 rows (only the first WS/2 are used)
            gw[j] = reinterpret_cast<const int8_t*>(wq) + (int64_t)min((n0 >> 5) + 4 * j + wave, (N - 1) >> 5) * KT * 1024 + lane * 16;
        } else {
            const int nr = min(n0 + (4 * j + wave) * 16 + lrow, N - 1);
            gw[j] = reinterpret_cast<const int8_t*>(wq) + (int64_t)nr * K + lchunk * 16;
        }
    }
    constexpr int kWTileStep = (WMODE == W_I8B || WMODE == W_I4B) ? 1024 : kBK;   // bytes from one K tile to the next
    auto dma_x = [&](int Tk, int j) {
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(gx[j] + eff_tile(Tk) * 1024),
                                         (lds_ptr_t)(stage_ptr(stage_of(Tk), 0) + (4 * j + wave) * 1024), 16, 0, 0);
    };
    auto dma_w = [&](int Tk, int j) {
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(gw[j] + eff_tile(Tk) * kWTileStep),
                                         (lds_ptr_t)(stage_ptr(stage_of(Tk), 1) + (4 * j + wave) * 1024), 16, 0, 0);
    };

    // ---- register path: thread t owns 16-byte chunk t%4 of rows t/4 + 64j ----
    const int rrow = tid >> 2, rchunk = tid & 3;
    const int rslot = rrow * kBK + ((rchunk ^ swz64(rrow)) << 4);       // swz64(rrow + 64j) == swz64(rrow)
    const QConst qk = make_qconst(*s_ptr, a_bits);
    u32x4 xr[3][2 * XS];   // XMODE 1: three K tiles of 16-bit activations in flight (2 x 128 bit per task)
    u32x2 wr[3][WS];       // WMODE 1: three K tiles of packed int4 weights in flight (64 bit per task)
#pragma unroll
    for (int a = 0; a < 3; ++a) {
#pragma unroll
        for (int b = 0; b < 2 * XS; ++b) xr[a][b] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int b = 0; b < WS; ++b) wr[a][b] = u32x2{0u, 0u};
    }
    const uint16_t* rx[XS];
    const uint8_t* rw[WS];
#pragma unroll
    for (int j = 0; j < XS; ++j)
        rx[j] = static_cast<const uint16_t*>(xin) + (int64_t)min(m0 + rrow + 64 * j, M - 1) * K + rchunk * 16;
#pragma unroll
    for (int j = 0; j < WS; ++j)
        rw[j] = wq + (int64_t)min(n0 + rrow + 64 * j, N - 1) * (K / 2) + rchunk * 8;
    // Register sets are selected with compile-time indices (a run-time index would put the arrays
    // in scratch memory): the K loop is unrolled by 3 and passes set = tile mod 3 as a constant.
    auto regload_x = [&](int Tk, auto set_c) {
        constexpr int set = decltype(set_c)::value;
#pragma unroll
        for (int j = 0; j < XS; ++j) {
            const u32x4* p = reinterpret_cast<const u32x4*>(rx[j] + eff_tile(Tk) * kBK);
            xr[set][2 * j] = p[0];
            xr[set][2 * j + 1] = p[1];
        }
    };
    auto regload_w = [&](int Tk, auto set_c) {
        constexpr int set = decltype(set_c)::value;
#pragma unroll
        for (int j = 0; j < WS; ++j) wr[set][j] = *reinterpret_cast<const u32x2*>(rw[j] + eff_tile(Tk) * (kBK / 2));
    };
    // quantize task j of tile Tk (16 elements) and store the 16 int8 codes
    auto convert_x = [&](int Tk, int j, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        float c[16];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                c[8 * h + 2 * w] = quantize(S::lo(xr[set][2 * j + h][w]), qk).c;
                c[8 * h + 2 * w + 1] = quantize(S::hi(xr[set][2 * j + h][w]), qk).c;
            }
        u32x4 o;
        if (WMODE == W_I4) {
            o[0] = pack_codes4(c[0], c[2], c[4], c[6]);    o[1] = pack_codes4(c[1], c[3], c[5], c[7]);
            o[2] = pack_codes4(c[8], c[10], c[12], c[14]); o[3] = pack_codes4(c[9], c[11], c[13], c[15]);
        } else {
            o[0] = pack_codes4(c[0], c[1], c[2], c[3]);    o[1] = pack_codes4(c[4], c[5], c[6], c[7]);
            o[2] = pack_codes4(c[8], c[9], c[10], c[11]);  o[3] = pack_codes4(c[12], c[13], c[14], c[15]);
        }
        *reinterpret_cast<u32x4*>(stage_ptr(stage_of(Tk), 0) + (rslot + 64 * j * kBK)) = o;
    };
    auto convert_w = [&](int Tk, int j, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        const uint32_t w0 = wr[set][j][0], w1 = wr[set][j][1];
        u32x4 o = {(w0 << 4) & 0xF0F0F0F0u, w0 & 0xF0F0F0F0u, (w1 << 4) & 0xF0F0F0F0u, w1 & 0xF0F0F0F0u};
        *reinterpret_cast<u32x4*>(stage_ptr(stage_of(Tk), 1) + (rslot + 64 * j * kBK)) = o;
    };

    // ---- LDS -> MFMA fragments ----
    const int frow = lane & 31, fgrp = lane >> 5;
    int foff[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) foff[kk] = frow * kBK + (((kk * 2 + fgrp) ^ swz64(frow)) << 4);
    const int xbase = wm * (BM / 2) * kBK, wbase = wn * (BN / 2) * kBK;
    i32x4 fx[2][MF], fw[2][NF];
    // fragment `idx` of a K-substep: the MF activation fragments first, then the NF weight ones
    auto read_frag = [&](int set, int st, int kk, int idx) {
        if (idx < MF) {
            fx[set][idx] = *reinterpret_cast<const i32x4*>(stage_ptr(st, 0) + xbase + idx * 32 * kBK + foff[kk]);
        } else if (WMODE == W_I4B) {
            const u32x2 p = *reinterpret_cast<const u32x2*>(stage_ptr(st, 1) + (wn * (BN / 64) + (idx - MF)) * 1024 + kk * 512 + lane * 8);
            fw[set][idx - MF][0] = (int)p[0];
            fw[set][idx - MF][1] = (int)p[1];
        } else {
            fw[set][idx - MF] = *reinterpret_cast<const i32x4*>(stage_ptr(st, 1) + wbase + (idx - MF) * 32 * kBK + foff[kk]);
        }
    };
    // the MFMA's weight operand: as read, or (pre-arranged int4) unpacked here
    auto wfrag = [&](int set, int g) -> i32x4 {
        if (WMODE == W_I4B) {
            const uint32_t p0 = (uint32_t)fw[set][g][0], p1 = (uint32_t)fw[set][g][1];
            return i32x4{(int)((p0 << 4) & 0xF0F0F0F0u), (int)(p0 & 0xF0F0F0F0u), (int)((p1 << 4) & 0xF0F0F0F0u), (int)(p1 & 0xF0F0F0F0u)};
        }
        return fw[set][g];
    };

    i32x16 acc[NF][MF];   // [n tile][m tile]
    f32x16 fsum[GROUPED ? NF : 1][GROUPED ? MF : 1];   // fp32 sums over groups
#pragma unroll
    for (int a = 0; a < (GROUPED ? NF : 1); ++a)
#pragma unroll
        for (int b = 0; b < (GROUPED ? MF : 1); ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) fsum[a][b][v] = 0.0f;
    // acc is first written by the MFMAs of K tile 0, which multiply into a zero accumulator operand
    // (clearing 256 registers per lane first would cost a microsecond per tile)

    // ---- K pipeline ----
    // Iteration i consumes K tile i in two phases (K-substeps of 32), each NF groups of MF MFMAs.
    // Phase 0 issues the weight loads of tile i+3, phase 1 the activation loads of tile i+4, so
    // the per-wave issue order is W(i+3), X(i+4), W(i+4), ... and every "has landed" condition
    // below is one s_waitcnt vmcnt(n) with n = loads issued later (memory loads return in issue
    // order).  Register-path tiles are converted into LDS ahead of use: X(i+1) half in phase 1
    // of iteration i-1 and half in phase 0 of iteration i, W(i+1) in phase 0 of iteration i.
    // A group's side work is its share of the next substep's fragment reads (activation fragments
    // before weight fragments: the order in which the next phase needs them), then one load.
    // Iterations -4..-1 only fill the pipeline.
    constexpr int nX = XMODE == X_FUSED ? 2 * XS : XS;     // loads per wave per K tile
    constexpr int nW = WMODE == W_I4B ? WS / 2 : WS;
    constexpr int kFrags = MF + NF;
    // Group g of K-substep `set`: MF MFMAs with the group's side work (its share of the next
    // substep's fragment reads, then its loads / conversions) dealt out behind them, item k
    // behind MFMA k.  With one wave per SIMD the matrix pipe only stays busy if whatever is
    // issued between two MFMAs fits in the 32 cycles one of them takes; a clump of a dozen
    // instructions between groups leaves it idle.  Pre-arranged int4 weights are unpacked one
    // group ahead, behind the first MFMA of the previous group, also across the phase boundary
    // when the first weight fragment of the next substep has been read by then (kCross).
    constexpr bool kCross = MF < (NF - 1) * kFrags / NF;
    i32x4 wnext = {0, 0, 0, 0};
    // mode 0: pipeline fill (no math); 1: math; 2: math, and the K tile opens a group of factors
    auto group = [&](int set, int g, auto mode_tag, int nitems, auto&& item) {
        constexpr int MODE = decltype(mode_tag)::value;
        constexpr bool MATH = MODE != 0;
        if (!MATH) {
            for (int k = 0; k < nitems; ++k) item(k);
            __builtin_amdgcn_sched_barrier(0);
            return;
        }
        i32x4 wv = fw[set][g];
        if (WMODE == W_I4B) {
            if (g == 0 && !kCross) wnext = wfrag(set, 0);
            wv = wnext;
        }
#pragma unroll
        for (int b = 0; b < MF; ++b) {
            if (MODE == 2 && set == 0) {
                const i32x16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                acc[g][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv, fx[set][b], zero, 0, 0, 0);
            } else {
                acc[g][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv, fx[set][b], acc[g][b], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (WMODE == W_I4B && b == 0) {
                if (g + 1 < NF) wnext = wfrag(set, g + 1);
                else if (kCross) wnext = wfrag(1 - set, 0);
            }
            if (b < MF - 1) {
                if (b < nitems) item(b);
            } else {
                for (int k = MF - 1; k < nitems; ++k) item(k);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto iteration = [&](int i, auto mode_tag, auto r_tag) {
        constexpr bool MATH = decltype(mode_tag)::value != 0;
        constexpr int R = decltype(r_tag)::value;              // (i + 6) % 3: register set of tile i
        using S0 = std::integral_constant<int, R>;
        using S1 = std::integral_constant<int, (R + 1) % 3>;
        using S2 = std::integral_constant<int, (R + 2) % 3>;
        const int st = i & 3;
        // ---------------- phase 0 ----------------
        if (WMODE == W_I4) __builtin_amdgcn_s_waitcnt(waitcnt_vm(2 * nX + nW));     // W(i+1) registers are here
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            const int r0 = g * kFrags / NF, nr = MATH ? (g + 1) * kFrags / NF - r0 : 0;
            group(0, g, mode_tag, nr + 1, [&](int k) {
                if (k < nr) { read_frag(1, st, 1, r0 + k); return; }
                if (WMODE != W_I4 && g < nW) dma_w(i + 3, g);
                if (WMODE == W_I4) convert_w(i + 1, g, S1{});
                if (XMODE == X_FUSED && g >= XS / 2 && g < XS) convert_x(i + 1, g, S1{});   // second half of X(i+1)
            });
        }
        if (WMODE == W_I4) regload_w(i + 3, S0{});
        asm volatile("" ::: "memory");
        // All LDS writes of this wave for tile i+1 are done, its last fragments of tile i are in
        // registers (so stage i&3 may be refilled), and its direct loads of tile i+1 have landed;
        // after the barrier tile i+1 is complete for everyone.
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(2 * nX + 2 * nW));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // ---------------- phase 1 ----------------
        if (XMODE == X_FUSED) __builtin_amdgcn_s_waitcnt(waitcnt_vm(2 * nW + nX));  // X(i+2) registers are here
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            const int r0 = g * kFrags / NF, nr = (i + 1 >= 0) ? (g + 1) * kFrags / NF - r0 : 0;
            group(1, g, mode_tag, nr + 1, [&](int k) {
                if (k < nr) { read_frag(0, (i + 1) & 3, 0, r0 + k); return; }
                if (XMODE == X_PREQ && g < XS) dma_x(i + 4, g);
                if (XMODE == X_FUSED && g < XS / 2) convert_x(i + 2, g, S2{});              // first half of X(i+2)
            });
        }
        if (XMODE == X_FUSED) regload_x(i + 4, S1{});
    };
    using R0 = std::integral_constant<int, 0>;
    using R1 = std::integral_constant<int, 1>;
    using R2 = std::integral_constant<int, 2>;
    using Fill = std::integral_constant<int, 0>;
    using Math = std::integral_constant<int, 1>;
    using Open = std::integral_constant<int, 2>;
    iteration(-4, Fill{}, R2{});
    iteration(-3, Fill{}, R0{});
    iteration(-2, Fill{}, R1{});
    iteration(-1, Fill{}, R2{});
    if (WMODE == W_I4B && kCross) wnext = wfrag(0, 0);
    // one K tile of math; with grouped factors also the group bookkeeping (all of it uniform)
    int in_group = 0, group_idx = 0;
    constexpr float kAccScale = (WMODE == W_I4 || WMODE == W_I4B) ? 0.0625f : 1.0f;   // int4 accumulators are 16 x acc
    auto step = [&](int i, auto r_tag) {
        if (!GROUPED) { iteration(i, Math{}, r_tag); return; }
        if (in_group == 0) iteration(i, Open{}, r_tag);
        else               iteration(i, Math{}, r_tag);
        if (++in_group == group_tiles) {
            // fl32(16 a) = 16 fl32(a) and s/16 is exact, so the fused multiply-add below rounds
            // exactly like fma(fl32(a), s, f)
            const float sg = s_ptr[group_idx] * kAccScale;
#pragma unroll
            for (int a = 0; a < (GROUPED ? NF : 1); ++a)
#pragma unroll
                for (int b = 0; b < (GROUPED ? MF : 1); ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) fsum[a][b][v] = __builtin_fmaf((float)acc[a][b][v], sg, fsum[a][b][v]);
            in_group = 0;
            ++group_idx;
        }
    };
    // K tile 0 (there always is one) opens the accumulators; the rest in threes for the register sets
    if (GROUPED) step(0, R0{});
    else         iteration(0, Open{}, R0{});
    int it = 1;
#pragma unroll 1
    for (; it + 2 < KT; it += 3) {
        step(it, R1{});
        step(it + 1, R2{});
        step(it + 2, R0{});
    }
    if (it < KT) step(it, R1{});
    if (it + 1 < KT) step(it + 1, R2{});
    // drain the tail loads and the last fragment reads before LDS is reused
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ---- epilogue: D[i][j], i = 8*(v/4) + 4*(lane/32) + v%4 -> n, j = lane%32 -> m ----
    // Each wave dequantizes its (BM/2) x (BN/2) block, stages it through its own LDS region as
    // 16-bit values in [m][n] order and writes Y with 128-bit stores, BN contiguous bytes per row.
    const float s = qk.s;
    const bool has_bias = bias != nullptr;
    char* epi = &lds[wave * T::kEpiBytes];
    const int wn0 = n0 + wn * (BN / 2), wm0 = m0 + wm * (BM / 2);
    constexpr int kAccShift = (WMODE == W_I4 || WMODE == W_I4B) ? 4 : 0;
    // The nest
    // below is straight-line code over all 256 accumulators; what the common call does not need
    // (bias, inspection outputs) is kept out of it: the epilogue is bound by instruction issue and
    // fetch (measured: 9 us of a 60 us tile at K = 4096).
    float srow[MF];                                            // ROWS: the factor of each row this lane holds
#pragma unroll
    for (int b = 0; b < MF; ++b) srow[b] = ROWS ? s_ptr[min(wm0 + b * 32 + frow, M - 1)] : 1.0f;
    const bool cols_inside = wn0 + BN / 2 <= N && (reinterpret_cast<uintptr_t>(s_w) & 15u) == 0 &&
                             (bias == nullptr || (reinterpret_cast<uintptr_t>(bias) & 15u) == 0);
    auto write_tile = [&](auto bias_tag) {
        constexpr bool BIAS = decltype(bias_tag)::value;
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            // this column tile's factors, requested together.  (All 64 up front would save three
            // memory latencies per tile but spill registers to scratch: 15 -> 27 us on a one-iteration tile.)
            float cs[4][4], bs[4][4];
            if (cols_inside) {
                // whole block inside N and 16-byte aligned factor arrays: one 128-bit load per four columns
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int nb = wn0 + a * 32 + 8 * g + 4 * fgrp;
                    const f32x4 sv = *reinterpret_cast<const f32x4*>(s_w + nb);
                    f32x4 bv = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (BIAS) bv = *reinterpret_cast<const f32x4*>(bias + nb);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        cs[g][e] = (GROUPED || ROWS) ? sv[e] : s * sv[e];
                        bs[g][e] = bv[e];
                    }
                }
            } else {
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int ne = min(wn0 + a * 32 + 8 * g + 4 * fgrp + e, N - 1);
                        cs[g][e] = (GROUPED || ROWS) ? s_w[ne] : s * s_w[ne];
                        bs[g][e] = BIAS ? bias[ne] : 0.0f;
                    }
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int nl = a * 32 + 8 * g + 4 * fgrp;      // column within the wave's block
#pragma unroll
                for (int b = 0; b < MF; ++b) {
                    const int ml = b * 32 + frow;
                    float yv[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (GROUPED) {
                            yv[e] = fsum[GROUPED ? a : 0][GROUPED ? b : 0][4 * g + e] * cs[g][e];      // Y = fl32(f * s_w[n])
                            if (BIAS) yv[e] = yv[e] + bs[g][e];
                        } else {
                            const float cc = ROWS ? srow[b] * cs[g][e] : cs[g][e];
                            yv[e] = dequant(acc[a][b][4 * g + e] >> kAccShift, cc, bs[g][e], BIAS);
                        }
                    }
                    u32x2 pk = {S::pack(yv[0], yv[1]), S::pack(yv[2], yv[3])};
                    *reinterpret_cast<u32x2*>(epi + ml * T::kEpiStride + nl * 2) = pk;
                }
            }
        }
    };
    if (has_bias) write_tile(std::true_type{});
    else          write_tile(std::false_type{});
    // each wave reads back only what it wrote itself: no workgroup barrier needed
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    const bool vec_ok = (N & 7) == 0;
    constexpr int kChunksPerRow = BN / 16;                      // 16-byte chunks in a wave-block row
    constexpr int kRowsPerPass = 64 / kChunksPerRow;
    const int crow = lane / kChunksPerRow, cchunk = lane % kChunksPerRow;
    if (vec_ok && wm0 + BM / 2 <= M && wn0 + BN / 2 <= N) {
        // block inside the matrix: no bounds, eight LDS reads in flight, then their eight stores
        const char* src = epi + crow * T::kEpiStride + cchunk * 16;
        char* dst = reinterpret_cast<char*>(y + (int64_t)(wm0 + crow) * N + wn0 + cchunk * 8);
        const int64_t row_step = (int64_t)kRowsPerPass * N * 2;
        constexpr int kPasses = (BM / 2) / kRowsPerPass;
#pragma unroll
        for (int p0 = 0; p0 < kPasses; p0 += 8) {
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = *reinterpret_cast<const u32x4*>(src + (p0 + j) * kRowsPerPass * T::kEpiStride);
#pragma unroll
            for (int j = 0; j < 8; ++j) *reinterpret_cast<u32x4*>(dst + (p0 + j) * row_step) = v[j];
        }
    } else
#pragma unroll 4
    for (int p = 0; p < (BM / 2) / kRowsPerPass; ++p) {
        const int ml = p * kRowsPerPass + crow;
        const int m = wm0 + ml, n = wn0 + cchunk * 8;
        if (m >= M || n >= N) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(epi + ml * T::kEpiStride + cchunk * 16);
        uint16_t* dst = y + (int64_t)m * N + n;
        if (vec_ok && n + 7 < N) {
            *reinterpret_cast<u32x4*>(dst) = v;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (n + e < N) dst[e] = (uint16_t)(v[e >> 1] >> (16 * (e & 1)));
        }
    }
    // inspection output (int32 accumulators, or the fp32 group sums): straight from the registers,
    // after and apart from the common path
    if (acc_out) {
#pragma unroll
        for (int a = 0; a < NF; ++a)
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int b = 0; b < MF; ++b) {
                    const int m = wm0 + b * 32 + frow, n = wn0 + a * 32 + 8 * g + 4 * fgrp;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = GROUPED ? __float_as_int(fsum[GROUPED ? a : 0][GROUPED ? b : 0][4 * g + e])
                                              : (acc[a][b][4 * g + e] >> kAccShift);
                        if (m < M && n + e < N) acc_out[(int64_t)m * N + n + e] = v;
                    }
                }
    }
}

template <int DT, int XMODE, int WMODE, int BM, int BN, bool GROUPED = false, bool ROWS = false>
__global__ __launch_bounds__(kGemmThreads)
__attribute__((amdgpu_waves_per_eu(Tile<BM, BN>::kWavesPerSimd, Tile<BM, BN>::kWavesPerSimd)))
void linear_mfma_kernel(const void* __restrict__ xin, const uint8_t* __restrict__ wq,
                        const float* __restrict__ s_ptr, const float* __restrict__ s_w,
                        const float* __restrict__ bias, uint16_t* __restrict__ y,
                        int32_t* __restrict__ acc_out, int M, int N, int K, int a_bits,
                        int tiles_m, int tiles_n, int group_tiles)
{
    linear_mfma_body<DT, XMODE, WMODE, BM, BN, GROUPED, ROWS>(xin, wq, s_ptr, s_w, bias, y, acc_out, M, N, K, a_bits,
                                                              tiles_m, tiles_n, group_tiles, (int)blockIdx.x);
}

// The GEMMs of several projections in one launch, 256x256 tiles.  Each projection owns a run of
// workgroup ids (a multiple of 8, so the XCD-aware tile numbering holds inside it); the host puts
// the projections with the longest K first, so that the dispatcher, which hands out workgroups in
// id order as CUs fall free, ends the launch with the short tiles: one ramp and one drain for the
// layer, and the partly filled last round of each projection is filled by the next one's tiles.
template <int DT, int WMODE>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void linear_mfma_batch_kernel(const LinBatch b, int a_bits)
{
    const int k = lin_item_of(b, (int)blockIdx.x);
    const LinItem& it = b.it[k];
    linear_mfma_body<DT, X_PREQ, WMODE, 256, 256>(it.xq, it.wq, it.s, it.s_w, it.bias, it.y, nullptr, it.M, it.N, it.K, a_bits,
                                                  it.tiles_m, it.tiles_n, 0, (int)blockIdx.x - b.first_block[k]);
}

static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Which activation path the MFMA kernel takes: 0 = by shape, 1 = separate quantize pass,
// 2 = quantize-on-load (sasq_set_tuning(SASQ_TUNE_LINEAR_PATH, ...)).
static int path_override() { return tuning(SASQ_TUNE_LINEAR_PATH); }

// Quantize-on-load re-quantizes each activation row once per column tile (about 3 VALU
// operations per element on the SIMD that also issues the MFMAs) and doubles the A-side L2
// traffic; the separate pass costs 3 bytes of HBM traffic per element once.  On MI355X the
// separate pass measured faster at every workload shape, down to N = 1024 (4 column tiles:
// 121 us against 150 us at M = K = 8192), so the shape rule currently never fuses; the fused
// kernel stays selectable and is covered by the same parity tests.
static bool choose_fused(int64_t M, int64_t N, int64_t K)
{
    (void)M; (void)K;
    return N <= kFusedMaxN;
}

template <int DT, int XMODE, int WMODE, int BM, int BN, bool GROUPED = false, bool ROWS = false>
static void launch_tiles(const void* xin, const void* wq, const float* s, const float* s_w, const float* bias,
                         void* y, int32_t* acc_out, int64_t M, int64_t N, int64_t K, int a_bits, hipStream_t st,
                         int group_tiles = 0)
{
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    const int grid = ((tiles_m * tiles_n + 7) / 8) * 8;
    linear_mfma_kernel<DT, XMODE, WMODE, BM, BN, GROUPED, ROWS><<<grid, kGemmThreads, 0, st>>>(
        xin, static_cast<const uint8_t*>(wq), s, s_w, bias, static_cast<uint16_t*>(y), acc_out,
        (int)M, (int)N, (int)K, a_bits, tiles_m, tiles_n, group_tiles);
}

// Tile choice.  256x256 tiles are the most efficient per operation but a launch of T tiles takes
// ceil(T / 256) rounds on 256 CUs; problems with few tiles use 128x256 or 128x128 tiles (the
// latter two workgroups per CU) so that the chip is filled.  Relative costs per output element
// (measured) are folded into `cost`.  sasq_set_tuning(SASQ_TUNE_LINEAR_TILE, 1 | 2 | 3) forces one.
static int choose_tile(int64_t M, int64_t N)
{
    if (const int t = tuning(SASQ_TUNE_LINEAR_TILE)) return t - 1;
    auto rounds = [&](int bm, int bn, int slots) {
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        return (double)((tiles + slots - 1) / slots);
    };
    // 256x256: a last round that fills at most half of the CUs is handed out as half tiles and takes about 0.6 of a round
    const int64_t t0 = ((M + 255) / 256) * ((N + 255) / 256);
    const double c0 = (t0 > 256 && t0 % 256 > 0 && t0 % 256 <= 128) ? (double)(t0 / 256) + 0.6 : rounds(256, 256, 256) * 1.00;
    const double c1 = rounds(128, 256, 256) * 0.50 * kCost128x256;
    const double c2 = rounds(128, 128, 512) * 0.50 * kCost128x128;   // two co-resident workgroups share a CU
    if (c0 <= c1 && c0 <= c2) return 0;
    return c1 <= c2 ? 1 : 2;
}

// int8 weights and pre-arranged int4 weights over staged activations run on the 16x16x64 MFMA kernel (static_linear_k64.hip) unless
// sasq_set_tuning(SASQ_TUNE_LINEAR_MFMA, 1) asks for the 32x32x32 one.
static bool use_k64(int xmode, int wmode)
{
    return xmode == X_PREQ && (wmode == W_I8 || wmode == W_I8B || wmode == W_I4B) && tuning(SASQ_TUNE_LINEAR_MFMA) != 1;
}

template <int DT>
static void launch_k64(const void* xq, const void* wq, const float* s, const float* s_w, const float* bias, void* y,
                       int32_t* acc_out, int64_t M, int64_t N, int64_t K, int wmode, bool rows, hipStream_t st)
{
    const int tile = choose_tile(M, N);
    if (tile == 0 && !rows && !acc_out && tuning(SASQ_TUNE_LINEAR_TILE) == 0) {
        // the plain call with 256x256 tiles is a batch of one: it gets the batch kernel's handling of a
        // sparsely filled last round (its tiles handed out as 128x256 halves)
        LinBatch g{};
        g.count = 1;
        LinItem& li = g.it[0];
        li.x = nullptr;
        li.xq = const_cast<int8_t*>(static_cast<const int8_t*>(xq));
        li.s = s; li.wq = static_cast<const uint8_t*>(wq); li.s_w = s_w; li.bias = bias; li.y = static_cast<uint16_t*>(y);
        li.M = (int)M; li.N = (int)N; li.K = (int)K;
        li.tiles_m = (int)((M + 255) / 256); li.tiles_n = (int)((N + 255) / 256);
        const int grid = ((li.tiles_m * li.tiles_n + 7) / 8) * 8;
        for (int i = 0; i < kMaxLinearBatch; ++i) g.first_block[i + 1] = grid;
        launch_gemm_k64_batch(g, grid, (sasq_dtype)DT, wmode, true, st);
        return;
    }
    GemmK64Args a{static_cast<const int8_t*>(xq), static_cast<const uint8_t*>(wq), s, s_w, bias,
                  static_cast<uint16_t*>(y), acc_out, M, N, K};
    launch_gemm_k64(a, (sasq_dtype)DT, wmode, tile, rows, st);
}

template <int DT, int XMODE, int WMODE>
static void launch_mfma(const void* xin, const void* wq, const float* s, const float* s_w, const float* bias,
                        void* y, int32_t* acc_out, int64_t M, int64_t N, int64_t K, int a_bits, hipStream_t st)
{
    if (use_k64(XMODE, WMODE)) { launch_k64<DT>(xin, wq, s, s_w, bias, y, acc_out, M, N, K, WMODE, false, st); return; }
    switch (choose_tile(M, N)) {
        case 0: launch_tiles<DT, XMODE, WMODE, 256, 256>(xin, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
        case 1: launch_tiles<DT, XMODE, WMODE, 128, 256>(xin, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
        default: launch_tiles<DT, XMODE, WMODE, 128, 128>(xin, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
    }
}

// the staged (tiled) activation pre-pass of one tensor: one wave per 1 KB block
template <int DT, bool PERM8>
static void launch_quantize_blocks(const void* x, const float* s, int8_t* xq, int64_t M, int64_t K, int a_bits, hipStream_t st)
{
    QuantItem it{};
    it.x = x;
    it.M = (int)M;
    it.K = (int)K;
    it.ns = 1;
    it.s[0] = s;
    it.xq[0] = xq;
    const int64_t nblk = ((M + 15) / 16) * (K / 64);
    int64_t grid = (nblk + 3) / 4;
    if (grid > 65536) grid = 65536;
    quantize_act_blocks_kernel<DT, PERM8><<<(int)grid, 256, 0, st>>>(it, a_bits);
}

template <int DT>
static void run_linear(const void* x, const float* s, const void* wq, const float* s_w, const float* bias,
                       void* y, int32_t* acc_out, int8_t* xq_out, int64_t M, int64_t N, int64_t K, int a_bits,
                       sasq_wfmt wf, int8_t* xq_ws, hipStream_t st)
{
    const int64_t n = M * K, nvec = n / 8;
    int64_t qb = (nvec + 255) / 256;
    const int qgrid = (int)(qb < 1 ? 1 : (qb > 65536 ? 65536 : qb));
    auto X = static_cast<const u32x4*>(x);
    if (xq_out) quantize_act_kernel<DT, false, false><<<qgrid, 256, 0, st>>>(X, s, reinterpret_cast<u32x2*>(xq_out), nvec, n, (int)K, a_bits);

    const bool mfma_ok = (K % kBK) == 0;
    const bool int4 = wf == SASQ_W_INT4_PACKED;
    if (wf == SASQ_W_INT8_BLOCKED || wf == SASQ_W_INT4_BLOCKED) {
        // pre-arranged weights (K % 64 == 0 was checked by the caller): always the two-pass MFMA path
        launch_quantize_blocks<DT, false>(x, s, xq_ws, M, K, a_bits, st);
        if (wf == SASQ_W_INT8_BLOCKED) launch_mfma<DT, X_PREQ, W_I8B>(xq_ws, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st);
        else                           launch_mfma<DT, X_PREQ, W_I4B>(xq_ws, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st);
    } else if (mfma_ok) {
        const int ov = path_override();
        const bool fused = ov == 2 || (ov == 0 && choose_fused(M, N, K));
        if (fused) {
            if (int4) launch_mfma<DT, X_FUSED, W_I4>(x, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st);
            else      launch_mfma<DT, X_FUSED, W_I8>(x, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st);
        } else {
            // pass 1: quantize the activations once with the fixed scale (no reduction over X anywhere)
            if (int4) {
                launch_quantize_blocks<DT, true>(x, s, xq_ws, M, K, a_bits, st);
                launch_mfma<DT, X_PREQ, W_I4>(xq_ws, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st);
            } else {
                launch_quantize_blocks<DT, false>(x, s, xq_ws, M, K, a_bits, st);
                launch_mfma<DT, X_PREQ, W_I8>(xq_ws, wq, s, s_w, bias, y, acc_out, M, N, K, a_bits, st);
            }
        }
    } else {
        quantize_act_kernel<DT, false, false><<<qgrid, 256, 0, st>>>(X, s, reinterpret_cast<u32x2*>(xq_ws), nvec, n, (int)K, a_bits);
        const int64_t blocks = (M * N + 255) / 256;
        auto W = static_cast<const uint8_t*>(wq);
        auto Y = static_cast<uint16_t*>(y);
        if (int4) linear_scalar_kernel<DT, true><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s, s_w, bias, Y, acc_out, M, N, K);
        else      linear_scalar_kernel<DT, false><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s, s_w, bias, Y, acc_out, M, N, K);
    }
}

// Grouped factors: 128-row tiles only (the fp32 group sums double the accumulator registers).
template <int DT, int WMODE>
static void launch_mfma_grouped(const void* xin, const void* wq, const float* s_g, const float* s_w, const float* bias,
                                void* y, float* f_out, int64_t M, int64_t N, int64_t K, int a_bits, int group_tiles,
                                hipStream_t st)
{
    // 128x128 tiles, two workgroups per CU: the fp32 sums and the accumulators then all fit in
    // VGPRs (no accumulator-register moves in the fold) and one wave's fold overlaps the MFMAs of
    // the other wave on its SIMD; measured 1.3-1.6 x faster than 128x256 tiles at every group size.
    const int tile = tuning(SASQ_TUNE_LINEAR_TILE) == 2 ? 1 : 2;
    auto acc_out = reinterpret_cast<int32_t*>(f_out);
    // group_tiles 0 = groups of 32 channels: the 16x16x64 kernel only
    if constexpr (WMODE != W_I4) if (use_k64(X_PREQ, WMODE) || group_tiles == 0) {
        GemmK64Args a{static_cast<const int8_t*>(xin), static_cast<const uint8_t*>(wq), s_g, s_w, bias,
                      static_cast<uint16_t*>(y), acc_out, M, N, K};
        launch_gemm_k64_grouped(a, (sasq_dtype)DT, WMODE, tile, group_tiles, st);
        return;
    }
    if (tile == 1) launch_tiles<DT, X_PREQ, WMODE, 128, 256, true>(xin, wq, s_g, s_w, bias, y, acc_out, M, N, K, a_bits, st, group_tiles);
    else           launch_tiles<DT, X_PREQ, WMODE, 128, 128, true>(xin, wq, s_g, s_w, bias, y, acc_out, M, N, K, a_bits, st, group_tiles);
}

template <int DT>
static void run_linear_grouped(const void* x, const float* s_g, const void* wq, const float* s_w, const float* bias,
                               void* y, float* f_out, int8_t* xq_out, int64_t M, int64_t N, int64_t K, int64_t group,
                               int a_bits, sasq_wfmt wf, int8_t* xq_ws, hipStream_t st)
{
    const int64_t n = M * K, nvec = n / 8;
    auto grid_of = [](int64_t work) { int64_t b = (work + 255) / 256; return (int)(b < 1 ? 1 : (b > 65536 ? 65536 : b)); };
    const bool vec_ok = (K % 8) == 0 && (group % 8) == 0;
    auto X = static_cast<const u32x4*>(x);
    auto quantize_rowmajor = [&](int8_t* dst) {
        if (vec_ok) quantize_act_grouped_kernel<DT, false, false><<<grid_of(nvec), 256, 0, st>>>(X, s_g, reinterpret_cast<u32x2*>(dst), nvec, (int)K, (int)group, a_bits);
        else        quantize_act_grouped_elem_kernel<DT><<<grid_of(n), 256, 0, st>>>(static_cast<const uint16_t*>(x), s_g, dst, n, (int)K, (int)group, a_bits);
    };
    if (xq_out) quantize_rowmajor(xq_out);
    // groups of 32 channels run on the matrix units too (16x16x64 kernel, int8 and pre-arranged int4 weights)
    const bool half_ok = group == 32 && (K % kBK) == 0 && wf != SASQ_W_INT4_PACKED;
    const bool mfma_ok = ((K % kBK) == 0 && (group % kBK) == 0) || half_ok;
    if (mfma_ok) {
        // row-major packed int4 unpacks in (0,2,4,6,1,3,5,7) order: the activation bytes are stored to match
        if (wf == SASQ_W_INT4_PACKED)
            quantize_act_grouped_kernel<DT, true, true><<<grid_of(nvec), 256, 0, st>>>(X, s_g, reinterpret_cast<u32x2*>(xq_ws), nvec, (int)K, (int)group, a_bits);
        else
            quantize_act_grouped_kernel<DT, false, true><<<grid_of(nvec), 256, 0, st>>>(X, s_g, reinterpret_cast<u32x2*>(xq_ws), nvec, (int)K, (int)group, a_bits);
        const int gt = (int)(group / kBK);
        switch (wf) {
            case SASQ_W_INT8:         launch_mfma_grouped<DT, W_I8>(xq_ws, wq, s_g, s_w, bias, y, f_out, M, N, K, a_bits, gt, st); break;
            case SASQ_W_INT4_PACKED:  launch_mfma_grouped<DT, W_I4>(xq_ws, wq, s_g, s_w, bias, y, f_out, M, N, K, a_bits, gt, st); break;
            case SASQ_W_INT8_BLOCKED: launch_mfma_grouped<DT, W_I8B>(xq_ws, wq, s_g, s_w, bias, y, f_out, M, N, K, a_bits, gt, st); break;
            default:                  launch_mfma_grouped<DT, W_I4B>(xq_ws, wq, s_g, s_w, bias, y, f_out, M, N, K, a_bits, gt, st); break;
        }
    } else {
        quantize_rowmajor(xq_ws);
        const int64_t blocks = (M * N + 255) / 256;
        auto W = static_cast<const uint8_t*>(wq);
        auto Y = static_cast<uint16_t*>(y);
        if (wf == SASQ_W_INT4_PACKED) linear_grouped_scalar_kernel<DT, true><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s_g, s_w, bias, Y, f_out, M, N, K, group);
        else                          linear_grouped_scalar_kernel<DT, false><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s_g, s_w, bias, Y, f_out, M, N, K, group);
    }
}

template <int DT, int WMODE>
static void launch_mfma_rows(const void* xin, const void* wq, const float* s_row, const float* s_w, const float* bias,
                             void* y, int32_t* acc_out, int64_t M, int64_t N, int64_t K, int a_bits, hipStream_t st)
{
    if (use_k64(X_PREQ, WMODE)) { launch_k64<DT>(xin, wq, s_row, s_w, bias, y, acc_out, M, N, K, WMODE, true, st); return; }
    switch (choose_tile(M, N)) {
        case 0: launch_tiles<DT, X_PREQ, WMODE, 256, 256, false, true>(xin, wq, s_row, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
        case 1: launch_tiles<DT, X_PREQ, WMODE, 128, 256, false, true>(xin, wq, s_row, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
        default: launch_tiles<DT, X_PREQ, WMODE, 128, 128, false, true>(xin, wq, s_row, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
    }
}

template <int DT>
static void run_dynamic(const void* x, const void* wq, const float* s_w, const float* bias, void* y, int32_t* acc_out,
                        int8_t* xq_out, float* s_row, int64_t M, int64_t N, int64_t K, int a_bits, sasq_wfmt wf,
                        int8_t* xq_ws, hipStream_t st)
{
    auto X = static_cast<const uint16_t*>(x);
    const bool vec = (K % 8) == 0;
    auto quantize_rowmajor = [&](int8_t* dst) {
        if (vec) quantize_rows_kernel<DT, false, false, true><<<(int)M, 256, 0, st>>>(X, dst, s_row, (int)K, a_bits);
        else     quantize_rows_kernel<DT, false, false, false><<<(int)M, 256, 0, st>>>(X, dst, s_row, (int)K, a_bits);
    };
    if (xq_out) quantize_rowmajor(xq_out);
    if ((K % kBK) == 0) {
        if (wf == SASQ_W_INT4_PACKED) quantize_rows_kernel<DT, true, true, true><<<(int)M, 256, 0, st>>>(X, xq_ws, s_row, (int)K, a_bits);
        else                          quantize_rows_kernel<DT, false, true, true><<<(int)M, 256, 0, st>>>(X, xq_ws, s_row, (int)K, a_bits);
        switch (wf) {
            case SASQ_W_INT8:         launch_mfma_rows<DT, W_I8>(xq_ws, wq, s_row, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
            case SASQ_W_INT4_PACKED:  launch_mfma_rows<DT, W_I4>(xq_ws, wq, s_row, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
            case SASQ_W_INT8_BLOCKED: launch_mfma_rows<DT, W_I8B>(xq_ws, wq, s_row, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
            default:                  launch_mfma_rows<DT, W_I4B>(xq_ws, wq, s_row, s_w, bias, y, acc_out, M, N, K, a_bits, st); break;
        }
    } else {
        quantize_rowmajor(xq_ws);
        const int64_t blocks = (M * N + 255) / 256;
        auto W = static_cast<const uint8_t*>(wq);
        auto Y = static_cast<uint16_t*>(y);
        if (wf == SASQ_W_INT4_PACKED) linear_scalar_kernel<DT, true, true><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s_row, s_w, bias, Y, acc_out, M, N, K);
        else                          linear_scalar_kernel<DT, false, true><<<(int)blocks, 256, 0, st>>>(xq_ws, W, s_row, s_w, bias, Y, acc_out, M, N, K);
    }
}

}  // namespace sasq

using namespace sasq;

extern "C" size_t sasq_static_linear_workspace(int64_t M, int64_t N, int64_t K, sasq_wfmt wf)
{
    (void)N; (void)wf;
    if (M <= 0 || K <= 0) return 0;
    return round_up(round_up((size_t)M, 16) * (size_t)K, 256);   // int8 activation codes of the two-pass path, rows padded to 16
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
    if (wf != SASQ_W_INT8 && wf != SASQ_W_INT4_PACKED && wf != SASQ_W_INT8_BLOCKED && wf != SASQ_W_INT4_BLOCKED)
        return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    if (wf == SASQ_W_INT4_PACKED && (K & 1)) return SASQ_ERR_SHAPE;
    if ((wf == SASQ_W_INT8_BLOCKED || wf == SASQ_W_INT4_BLOCKED) && (K % kBK)) return SASQ_ERR_SHAPE;
    if ((M * N + 255) / 256 > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(wq) || !aligned16(y) || (acc_out && !aligned16(acc_out)) ||
        (xq_out && (reinterpret_cast<uintptr_t>(xq_out) & 7u))) return SASQ_ERR_ALIGN;
    const size_t need = sasq_static_linear_workspace(M, N, K, wf);
    if (!workspace || workspace_bytes < need) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;

    hipStream_t st = as_stream(stream);
    int8_t* xq_ws = static_cast<int8_t*>(workspace);
    if (dt == SASQ_F16) run_linear<SASQ_F16>(x, s, wq, s_w, bias, y, acc_out, xq_out, M, N, K, a_bits, wf, xq_ws, st);
    else                run_linear<SASQ_BF16>(x, s, wq, s_w, bias, y, acc_out, xq_out, M, N, K, a_bits, wf, xq_ws, st);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" int sasq_static_linear_grouped(const void* x, const float* s_g, const void* wq, const float* s_w,
                                          const float* bias, void* y, float* f_out, int8_t* xq_out,
                                          int64_t M, int64_t N, int64_t K, int64_t group, int a_bits,
                                          sasq_wfmt wf, sasq_dtype dt, void* workspace, size_t workspace_bytes,
                                          void* stream)
{
    if (!x || !s_g || !wq || !s_w || !y) return SASQ_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || group <= 0 || K % group) return SASQ_ERR_SHAPE;
    const int64_t lim = INT64_C(1) << 40;
    if (M > lim / K || N > lim / K || M > lim / N || K > 131071 || M > 0x7FFFFFFF || N > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    if (a_bits < 2 || a_bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (wf != SASQ_W_INT8 && wf != SASQ_W_INT4_PACKED && wf != SASQ_W_INT8_BLOCKED && wf != SASQ_W_INT4_BLOCKED)
        return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    if (wf == SASQ_W_INT4_PACKED && (K & 1)) return SASQ_ERR_SHAPE;
    // the pre-arranged formats exist for the MFMA kernels only, which take whole K tiles per group or groups of 32
    if ((wf == SASQ_W_INT8_BLOCKED || wf == SASQ_W_INT4_BLOCKED) && ((K % kBK) || ((group % kBK) && group != 32))) return SASQ_ERR_SHAPE;
    if ((M * N + 255) / 256 > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(wq) || !aligned16(y) || (f_out && !aligned16(f_out)) ||
        (xq_out && (reinterpret_cast<uintptr_t>(xq_out) & 7u))) return SASQ_ERR_ALIGN;
    const size_t need = sasq_static_linear_workspace(M, N, K, wf);
    if (!workspace || workspace_bytes < need) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;

    hipStream_t st = as_stream(stream);
    int8_t* xq_ws = static_cast<int8_t*>(workspace);
    if (dt == SASQ_F16) run_linear_grouped<SASQ_F16>(x, s_g, wq, s_w, bias, y, f_out, xq_out, M, N, K, group, a_bits, wf, xq_ws, st);
    else                run_linear_grouped<SASQ_BF16>(x, s_g, wq, s_w, bias, y, f_out, xq_out, M, N, K, group, a_bits, wf, xq_ws, st);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" size_t sasq_dynamic_linear_workspace(int64_t M, int64_t N, int64_t K, sasq_wfmt wf)
{
    if (M <= 0 || K <= 0) return 0;
    return sasq_static_linear_workspace(M, N, K, wf) + round_up(sizeof(float) * (size_t)M, 256);   // codes + row factors
}

extern "C" int sasq_dynamic_linear(const void* x, const void* wq, const float* s_w, const float* bias, void* y,
                                   int32_t* acc_out, int8_t* xq_out, float* s_row_out,
                                   int64_t M, int64_t N, int64_t K, int a_bits, sasq_wfmt wf, sasq_dtype dt,
                                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !wq || !s_w || !y) return SASQ_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0) return SASQ_ERR_SHAPE;
    const int64_t lim = INT64_C(1) << 40;
    if (M > lim / K || N > lim / K || M > lim / N || K > 131071 || M > 0x7FFFFFFF || N > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    if (a_bits < 2 || a_bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (wf != SASQ_W_INT8 && wf != SASQ_W_INT4_PACKED && wf != SASQ_W_INT8_BLOCKED && wf != SASQ_W_INT4_BLOCKED)
        return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    if (wf == SASQ_W_INT4_PACKED && (K & 1)) return SASQ_ERR_SHAPE;
    if ((wf == SASQ_W_INT8_BLOCKED || wf == SASQ_W_INT4_BLOCKED) && (K % kBK)) return SASQ_ERR_SHAPE;
    if ((M * N + 255) / 256 > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(wq) || !aligned16(y) || (acc_out && !aligned16(acc_out)) ||
        (xq_out && (reinterpret_cast<uintptr_t>(xq_out) & 7u)) || (s_row_out && (reinterpret_cast<uintptr_t>(s_row_out) & 3u)))
        return SASQ_ERR_ALIGN;
    const size_t need = sasq_dynamic_linear_workspace(M, N, K, wf);
    if (!workspace || workspace_bytes < need) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;

    hipStream_t st = as_stream(stream);
    int8_t* xq_ws = static_cast<int8_t*>(workspace);
    float* s_row = s_row_out ? s_row_out
                             : reinterpret_cast<float*>(static_cast<char*>(workspace) + sasq_static_linear_workspace(M, N, K, wf));
    if (dt == SASQ_F16) run_dynamic<SASQ_F16>(x, wq, s_w, bias, y, acc_out, xq_out, s_row, M, N, K, a_bits, wf, xq_ws, st);
    else                run_dynamic<SASQ_BF16>(x, wq, s_w, bias, y, acc_out, xq_out, s_row, M, N, K, a_bits, wf, xq_ws, st);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

// ---- the linears of one layer in two launches ---------------------------------------------------
extern "C" size_t sasq_static_linear_batch_workspace(const sasq_linear_item* items, int count, sasq_wfmt wf)
{
    if (!items || count <= 0 || count > kMaxLinearBatch) return 0;
    size_t total = 0;
    for (int i = 0; i < count; ++i) total += sasq_static_linear_workspace(items[i].M, items[i].N, items[i].K, wf);
    return total;
}

extern "C" int sasq_static_linear_batch(const sasq_linear_item* items, int count, int a_bits, sasq_wfmt wf,
                                        sasq_dtype dt, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!items) return SASQ_ERR_NULL;
    if (count <= 0 || count > kMaxLinearBatch) return SASQ_ERR_SHAPE;
    if (a_bits < 2 || a_bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (wf != SASQ_W_INT8 && wf != SASQ_W_INT4_PACKED && wf != SASQ_W_INT8_BLOCKED && wf != SASQ_W_INT4_BLOCKED)
        return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    const int64_t lim = INT64_C(1) << 40;
    int64_t total_tiles = 0;
    for (int i = 0; i < count; ++i) {
        const sasq_linear_item& it = items[i];
        if (!it.x || !it.s || !it.wq || !it.s_w || !it.y) return SASQ_ERR_NULL;
        if (it.M <= 0 || it.N <= 0 || it.K <= 0 || (it.K % kBK)) return SASQ_ERR_SHAPE;      // MFMA shapes only
        if (it.M > lim / it.K || it.N > lim / it.K || it.M > lim / it.N || it.K > 131071 || it.M > 0x7FFFFFFF || it.N > 0x7FFFFFFF)
            return SASQ_ERR_SHAPE;
        if (!aligned16(it.x) || !aligned16(it.wq) || !aligned16(it.y)) return SASQ_ERR_ALIGN;
        total_tiles += ((it.M + 255) / 256) * ((it.N + 255) / 256) + 8;
    }
    if (total_tiles > 0x7FFFFFF0) return SASQ_ERR_SHAPE;
    if (!workspace || workspace_bytes < sasq_static_linear_batch_workspace(items, count, wf)) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;

    // longest K first (stable), see linear_mfma_batch_kernel
    int order[kMaxLinearBatch];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && items[order[j]].K > items[order[j - 1]].K; --j) { const int tmp = order[j]; order[j] = order[j - 1]; order[j - 1] = tmp; }

    LinBatch g{};
    char* ws = static_cast<char*>(workspace);
    g.count = count;
    g.first_block[0] = 0;
    for (int i = 0; i < count; ++i) {
        const sasq_linear_item& src = items[order[i]];
        LinItem li;
        li.x = src.x;
        li.xq = reinterpret_cast<int8_t*>(ws);
        ws += sasq_static_linear_workspace(src.M, src.N, src.K, wf);
        li.s = src.s;
        li.wq = static_cast<const uint8_t*>(src.wq);
        li.s_w = src.s_w;
        li.bias = src.bias;
        li.y = static_cast<uint16_t*>(src.y);
        li.M = (int)src.M; li.N = (int)src.N; li.K = (int)src.K;
        li.tiles_m = (int)((src.M + 255) / 256);
        li.tiles_n = (int)((src.N + 255) / 256);
        g.it[i] = li;
        g.first_block[i + 1] = g.first_block[i] + ((li.tiles_m * li.tiles_n + 7) / 8) * 8;
    }
    for (int i = count; i < kMaxLinearBatch; ++i) g.first_block[i + 1] = g.first_block[count];

    // the pre-passes: projections on the same X (same pointer, M and K) share one entry
    QuantBatch q{};
    bool taken[kMaxLinearBatch] = {false};
    int64_t total_vec = 0;
    for (int i = 0; i < count; ++i) {
        if (taken[i]) continue;
        QuantItem& e = q.it[q.count++];
        e.x = g.it[i].x;
        e.M = g.it[i].M;
        e.K = g.it[i].K;
        e.ns = 0;
        for (int j = i; j < count && e.ns < kMaxQuantShare; ++j) {
            if (taken[j] || g.it[j].x != e.x || g.it[j].M != e.M || g.it[j].K != e.K) continue;
            taken[j] = true;
            e.s[e.ns] = g.it[j].s;
            e.xq[e.ns] = g.it[j].xq;
            ++e.ns;
        }
        total_vec += ((int64_t)e.M * e.K / 8 + 1) * e.ns;
    }
    const int kQuantBlocks = 4096;
    q.first_block[0] = 0;
    for (int i = 0; i < q.count; ++i) {
        const int64_t nvec = (int64_t)q.it[i].M * q.it[i].K / 8;
        int64_t share = ((nvec + 1) * q.it[i].ns * kQuantBlocks + total_vec - 1) / total_vec;
        const int64_t need = (nvec + 255) / 256;
        if (share > need) share = need;
        if (share < 1) share = 1;
        q.first_block[i + 1] = q.first_block[i] + (int)share;
    }
    for (int i = q.count; i < kMaxLinearBatch; ++i) q.first_block[i + 1] = q.first_block[q.count];

    hipStream_t st = as_stream(stream);
    const int qgrid = q.first_block[q.count], ggrid = g.first_block[count];
    const bool perm8 = wf == SASQ_W_INT4_PACKED;      // row-major packed int4 unpacks in (0,2,4,6,1,3,5,7) order
#define SASQ_LAUNCH_BATCH(DTV)                                                                                          \
    do {                                                                                                                \
        if (perm8) quantize_act_batch_kernel<DTV, true><<<qgrid, 256, 0, st>>>(q, a_bits);                              \
        else       quantize_act_batch_kernel<DTV, false><<<qgrid, 256, 0, st>>>(q, a_bits);                             \
        if (use_k64(X_PREQ, (int)wf)) {          /* the sasq_wfmt values are those of the kernels' weight paths */     \
            launch_gemm_k64_batch(g, ggrid, dt, (int)wf, tuning(SASQ_TUNE_LINEAR_TILE) == 0, st);                       \
        } else switch (wf) {                                                                                            \
            case SASQ_W_INT8:         linear_mfma_batch_kernel<DTV, W_I8><<<ggrid, kGemmThreads, 0, st>>>(g, a_bits); break;   \
            case SASQ_W_INT4_PACKED:  linear_mfma_batch_kernel<DTV, W_I4><<<ggrid, kGemmThreads, 0, st>>>(g, a_bits); break;   \
            case SASQ_W_INT8_BLOCKED: linear_mfma_batch_kernel<DTV, W_I8B><<<ggrid, kGemmThreads, 0, st>>>(g, a_bits); break;  \
            default:                  linear_mfma_batch_kernel<DTV, W_I4B><<<ggrid, kGemmThreads, 0, st>>>(g, a_bits); break;  \
        }                                                                                                               \
    } while (0)
    if (dt == SASQ_F16) SASQ_LAUNCH_BATCH(SASQ_F16);
    else                SASQ_LAUNCH_BATCH(SASQ_BF16);
#undef SASQ_LAUNCH_BATCH
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}
