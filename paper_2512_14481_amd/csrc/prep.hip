// Set-up operations: workspace initialisation, frozen-weight quantization and re-arrangement,
// absmax initial scale.
#include "sasq_device.h"

namespace sasq {

constexpr int kPrepThreads = 256;
constexpr int kMaxAbsmaxBlocks = 2048;

__global__ void fill_zero_kernel(uint32_t* p, int64_t nwords)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) p[i] = 0u;
}

__device__ __forceinline__ float block_max(float v, float* sh)
{
    uint32_t w = wave_max(__float_as_uint(v));      // non-negative floats order like their bits
    if (threadIdx.x % kWave == 0) sh[threadIdx.x / kWave] = __uint_as_float(w);
    __syncthreads();
    float m = sh[0];
#pragma unroll
    for (int i = 1; i < kPrepThreads / kWave; ++i) m = fmaxf(m, sh[i]);
    __syncthreads();
    return m;
}

// One block per output channel n (row of W[N,K]): Sec. 3, Eq. 1 applied to the row.
template <bool INT4>
__global__ __launch_bounds__(kPrepThreads) void quantize_weight_kernel(
    const float* __restrict__ w, uint8_t* __restrict__ wq, float* __restrict__ s_w, int64_t K)
{
    __shared__ float sh[kPrepThreads / kWave];
    const int64_t n = blockIdx.x;
    const float* row = w + n * K;
    float amax = 0.0f;
    for (int64_t k = threadIdx.x; k < K; k += kPrepThreads) amax = fmaxf(amax, fabsf(row[k]));
    amax = block_max(amax, sh);
    const int bits = INT4 ? 4 : 8;
    const float Qp = (float)((1 << (bits - 1)) - 1);
    const float sw = amax == 0.0f ? 1.0f : amax / Qp;
    if (threadIdx.x == 0) s_w[n] = sw;
    const QConst kc = make_qconst(sw, bits);
    if (INT4) {
        uint8_t* out = wq + n * (K / 2);
        for (int64_t j = threadIdx.x; j < K / 2; j += kPrepThreads) {
            int lo = code_of(quantize(row[2 * j], kc));
            int hi = code_of(quantize(row[2 * j + 1], kc));
            out[j] = (uint8_t)((lo & 15) | ((hi & 15) << 4));
        }
    } else {
        uint8_t* out = wq + n * K;
        for (int64_t k = threadIdx.x; k < K; k += kPrepThreads)
            out[k] = (uint8_t)(code_of(quantize(row[k], kc)) & 0xFF);
    }
}

// Re-arrange row-major int8 weight codes [N,K] into the GEMM's operand blocks: 16 rows x 64
// K-bytes per 1 KB block, block (nb, kb) at (nb * K/64 + kb) * 1024, the 16-byte chunk c of row
// r at 16 * (4r + (c ^ swz(r))), swz(r) = ((r >> 1) & 3) ^ ((r >> 3) & 1).  One thread per
// destination chunk; rows past N are zero.
__global__ __launch_bounds__(kPrepThreads) void pack_weight_i8_kernel(
    const uint8_t* __restrict__ wq, u32x4* __restrict__ out, int64_t N, int64_t K, int64_t nchunks)
{
    const int64_t i = (int64_t)blockIdx.x * kPrepThreads + threadIdx.x;
    if (i >= nchunks) return;
    const int64_t blk = i >> 6, KT = K >> 6;
    const int sl = (int)(i & 63), r = sl >> 2;
    const int ch = (sl & 3) ^ (((r >> 1) & 3) ^ ((r >> 3) & 1));
    const int64_t n = (blk / KT) * 16 + r, k0 = (blk % KT) * 64 + ch * 16;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (n < N) v = *reinterpret_cast<const u32x4*>(wq + n * K + k0);
    out[i] = v;
}

// Re-arrange row-major packed int4 weight codes [N,K/2] into 1 KB blocks of 32 rows x 64 k:
// block (nb, kb) at (nb * K/64 + kb) * 1024; the 16 codes k = 64 kb + 32 kk + 16 g + (0..15) of
// row r are the 8 bytes at 512 kk + 256 g + 8 r; in them byte b of the first dword holds code b
// (low nibble) and 4 + b (high nibble), byte b of the second dword codes 8 + b and 12 + b.
// One thread per 8 destination bytes; rows past N are zero.
__global__ __launch_bounds__(kPrepThreads) void pack_weight_i4_kernel(
    const uint8_t* __restrict__ wq, u32x2* __restrict__ out, int64_t N, int64_t K, int64_t nslots)
{
    const int64_t i = (int64_t)blockIdx.x * kPrepThreads + threadIdx.x;
    if (i >= nslots) return;
    const int64_t blk = i >> 7, KT = K >> 6;
    const int sl = (int)(i & 127), kk = sl >> 6, g = (sl >> 5) & 1, r = sl & 31;
    const int64_t n = (blk / KT) * 32 + r, k0 = (blk % KT) * 64 + 32 * kk + 16 * g;
    u32x2 o = {0u, 0u};
    if (n < N) {
        const u32x2 sv = *reinterpret_cast<const u32x2*>(wq + n * (K / 2) + k0 / 2);
        const uint64_t src = (uint64_t)sv[0] | ((uint64_t)sv[1] << 32);     // code j at bits 4j
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t c0 = (uint32_t)(src >> (4 * b)) & 15u, c4 = (uint32_t)(src >> (4 * (4 + b))) & 15u;
            const uint32_t c8 = (uint32_t)(src >> (4 * (8 + b))) & 15u, c12 = (uint32_t)(src >> (4 * (12 + b))) & 15u;
            o[0] |= (c0 | (c4 << 4)) << (8 * b);
            o[1] |= (c8 | (c12 << 4)) << (8 * b);
        }
    }
    out[i] = o;
}

// max |x| over a flat 16-bit tensor: magnitudes of finite values and infinities order like their
// 15 low bits, so the reduction is an integer max (exact and order-independent).
template <int DT>
__global__ __launch_bounds__(kPrepThreads) void absmax_kernel(
    const uint16_t* __restrict__ x, float* __restrict__ s, uint32_t* __restrict__ ws_head,
    uint32_t* __restrict__ partials, int64_t n, int bits)
{
    using S = Store16<DT>;
    uint32_t m = 0;
    const int64_t nvec = n / 8;
    const u32x4* xv = reinterpret_cast<const u32x4*>(x);
    for (int64_t i = (int64_t)blockIdx.x * kPrepThreads + threadIdx.x; i < nvec;
         i += (int64_t)gridDim.x * kPrepThreads) {
        u32x4 v = xv[i];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            uint32_t lo = v[w] & 0x7FFFu, hi = (v[w] >> 16) & 0x7FFFu;
            m = lo > m ? lo : m;
            m = hi > m ? hi : m;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(n - nvec * 8)) {
        uint32_t a = x[nvec * 8 + threadIdx.x] & 0x7FFFu;
        m = a > m ? a : m;
    }
    __shared__ uint32_t sh[kPrepThreads / kWave];
    __shared__ bool is_last;
    m = wave_max(m);
    if (threadIdx.x % kWave == 0) sh[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kPrepThreads / kWave; ++i) m = sh[i] > m ? sh[i] : m;
        const uint32_t ticket = publish_then_ticket(&partials[blockIdx.x], m, &ws_head[0]);
        is_last = (ticket == kTicketBase + gridDim.x - 1);
        if (ticket - kTicketBase >= gridDim.x) *s = __uint_as_float(0x7FC00000u);
    }
    __syncthreads();
    if (!is_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    constexpr int kPer = kMaxAbsmaxBlocks / kPrepThreads;
    uint32_t pv[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = j * kPrepThreads + threadIdx.x;
        pv[j] = __hip_atomic_load(&partials[i < (int)gridDim.x ? i : 0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    uint32_t t = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) t = pv[j] > t ? pv[j] : t;     // a duplicate of partial 0 cannot change a max
    t = wave_max(t);
    __syncthreads();
    if (threadIdx.x % kWave == 0) sh[threadIdx.x / kWave] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 0; i < kPrepThreads / kWave; ++i) t = sh[i] > t ? sh[i] : t;
        float amax = S::one((uint16_t)t);
        *s = amax / (float)((1 << (bits - 1)) - 1);
        __hip_atomic_store(&ws_head[0], kTicketBase, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}  // namespace sasq

using namespace sasq;

extern "C" const char* sasq_status_string(int status)
{
    switch (status) {
        case SASQ_OK: return "SASQ_OK";
        case SASQ_ERR_NULL: return "SASQ_ERR_NULL: a required pointer is NULL";
        case SASQ_ERR_SHAPE: return "SASQ_ERR_SHAPE: bad size";
        case SASQ_ERR_ALIGN: return "SASQ_ERR_ALIGN: pointer not 16-byte aligned";
        case SASQ_ERR_UNSUPPORTED: return "SASQ_ERR_UNSUPPORTED: unknown enum or bits outside [2,8]";
        case SASQ_ERR_WORKSPACE: return "SASQ_ERR_WORKSPACE: workspace missing or too small";
        case SASQ_ERR_LAUNCH: return "SASQ_ERR_LAUNCH: HIP launch error";
        default: return "unknown sasq_status";
    }
}

extern "C" int sasq_version(void) { return 200; }

namespace sasq { int g_tuning[SASQ_TUNE_COUNT] = {0}; }

extern "C" int sasq_set_tuning(int knob, int value)
{
    static const int kMax[SASQ_TUNE_COUNT] = {2, 3, 2, 3, 2};
    if (knob < 0 || knob >= SASQ_TUNE_COUNT || value < 0 || value > kMax[knob]) return SASQ_ERR_UNSUPPORTED;
    sasq::g_tuning[knob] = value;
    return SASQ_OK;
}

extern "C" int sasq_workspace_init(void* workspace, size_t workspace_bytes, void* stream)
{
    if (!workspace) return SASQ_ERR_NULL;
    if (workspace_bytes < kWsMinBytes) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;
    const int64_t words = (int64_t)((workspace_bytes < kWsHeaderBytes ? workspace_bytes : kWsHeaderBytes) / 4);
    fill_zero_kernel<<<1, 256, 0, as_stream(stream)>>>(static_cast<uint32_t*>(workspace), words);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" int sasq_quantize_weight(const float* w, void* wq, float* s_w, int64_t N, int64_t K,
                                    sasq_wfmt wf, void* stream)
{
    if (!w || !wq || !s_w) return SASQ_ERR_NULL;
    if (N <= 0 || K <= 0 || N > 0x7FFFFFFF || N > (INT64_C(1) << 40) / K) return SASQ_ERR_SHAPE;
    if (wf != SASQ_W_INT8 && wf != SASQ_W_INT4_PACKED) return SASQ_ERR_UNSUPPORTED;
    if (wf == SASQ_W_INT4_PACKED && (K & 1)) return SASQ_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(wq)) return SASQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    if (wf == SASQ_W_INT8)
        quantize_weight_kernel<false><<<(int)N, kPrepThreads, 0, st>>>(w, static_cast<uint8_t*>(wq), s_w, K);
    else
        quantize_weight_kernel<true><<<(int)N, kPrepThreads, 0, st>>>(w, static_cast<uint8_t*>(wq), s_w, K);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" size_t sasq_packed_weight_bytes(int64_t N, int64_t K, sasq_wfmt wf)
{
    if (N <= 0 || K <= 0 || (K % 64) != 0) return 0;
    if (wf == SASQ_W_INT8_BLOCKED) return (size_t)((N + 15) / 16 * 16) * (size_t)K;
    if (wf == SASQ_W_INT4_BLOCKED) return (size_t)((N + 31) / 32 * 32) * (size_t)(K / 2);
    return 0;
}

extern "C" int sasq_pack_weight(const void* wq, void* packed, int64_t N, int64_t K, sasq_wfmt wf_src, void* stream)
{
    if (!wq || !packed) return SASQ_ERR_NULL;
    if (N <= 0 || K <= 0 || N > 0x7FFFFFFF || N > (INT64_C(1) << 40) / K) return SASQ_ERR_SHAPE;
    if (wf_src != SASQ_W_INT8 && wf_src != SASQ_W_INT4_PACKED) return SASQ_ERR_UNSUPPORTED;
    if (K % 64) return SASQ_ERR_SHAPE;
    if (!aligned16(wq) || !aligned16(packed)) return SASQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    if (wf_src == SASQ_W_INT8) {
        const int64_t nchunks = (int64_t)(sasq_packed_weight_bytes(N, K, SASQ_W_INT8_BLOCKED) / 16);
        pack_weight_i8_kernel<<<(unsigned)((nchunks + kPrepThreads - 1) / kPrepThreads), kPrepThreads, 0, st>>>(
            static_cast<const uint8_t*>(wq), static_cast<u32x4*>(packed), N, K, nchunks);
    } else {
        const int64_t nslots = (int64_t)(sasq_packed_weight_bytes(N, K, SASQ_W_INT4_BLOCKED) / 8);
        pack_weight_i4_kernel<<<(unsigned)((nslots + kPrepThreads - 1) / kPrepThreads), kPrepThreads, 0, st>>>(
            static_cast<const uint8_t*>(wq), static_cast<u32x2*>(packed), N, K, nslots);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" size_t sasq_absmax_scale_workspace(int64_t rows, int64_t cols)
{
    (void)rows; (void)cols;
    return kWsHeaderBytes + sizeof(uint32_t) * kMaxAbsmaxBlocks;
}

extern "C" int sasq_absmax_scale(const void* x, float* s, int64_t rows, int64_t cols, int bits,
                                 sasq_dtype dt, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !s) return SASQ_ERR_NULL;
    if (rows <= 0 || cols <= 0 || rows > (INT64_C(1) << 40) / cols) return SASQ_ERR_SHAPE;
    if (bits < 2 || bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    if (!aligned16(x)) return SASQ_ERR_ALIGN;
    if (!workspace || workspace_bytes < sasq_absmax_scale_workspace(rows, cols)) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;
    const int64_t n = rows * cols;
    int64_t need = (n / 8 + kPrepThreads * 4 - 1) / (kPrepThreads * 4);
    int grid = (int)(need < 1 ? 1 : (need > kMaxAbsmaxBlocks ? kMaxAbsmaxBlocks : need));
    auto head = static_cast<uint32_t*>(workspace);
    auto parts = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + kWsHeaderBytes);
    hipStream_t st = as_stream(stream);
    if (dt == SASQ_F16)
        absmax_kernel<SASQ_F16><<<grid, kPrepThreads, 0, st>>>(static_cast<const uint16_t*>(x), s, head, parts, n, bits);
    else
        absmax_kernel<SASQ_BF16><<<grid, kPrepThreads, 0, st>>>(static_cast<const uint16_t*>(x), s, head, parts, n, bits);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}
