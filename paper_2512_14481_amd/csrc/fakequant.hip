// Fake-quant forward / backward kernels (HBM-bound streaming kernels) and their C entry points.
//
// Forward  (Sec. 4.2; Sec. 3, Eq. 1; Sec. 4.3, Eq. 5):  y = s * clamp(round(x/s), Qn, Qp)
// Backward (Sec. 4.2, Eq. 4 + chain rule):               dx = dy * m,  ds = sum dy * (q - m*x/s)
//
// Both treat the [rows, cols] tensor as a flat array: each lane moves 8 elements per 128-bit
// access, a block covers kUnroll such accesses per lane back to back so enough bytes are in
// flight to cover HBM latency, and a scalar tail handles the last (n mod 8) elements.
#include "sasq_device.h"
#include <cstdlib>
#include <cmath>
#include <mutex>

namespace sasq {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;                       // 128-bit accesses in flight per lane per stream
constexpr int kMaxReduceBlocks = 256;            // one block per CU: every block ends with one
                                                 // agent-scope store + ticket atomic on a single
                                                 // address, so more blocks only lengthen the tail
constexpr int kMaxFwdBlocks = 2048;

// Forward on one 8-element vector.
template <int DT, bool CODES>
__device__ __forceinline__ void fwd_vec(const u32x4& in, const QConst& k, u32x4& out, u32x2& cw)
{
    using S = Store16<DT>;
    float c[8];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        QElem a = quantize(S::lo(in[w]), k);
        QElem b = quantize(S::hi(in[w]), k);
        out[w] = S::pack(codef_of(a) * k.s, codef_of(b) * k.s);
        c[2 * w] = a.c;
        c[2 * w + 1] = b.c;
    }
    if (CODES) {
        cw[0] = pack_codes4(c[0], c[1], c[2], c[3]);
        cw[1] = pack_codes4(c[4], c[5], c[6], c[7]);
    }
}

// Forward over one tensor by block `block` of the `nblocks` that share it.
template <int DT, bool CODES>
// (y may alias x: neither is restrict-qualified.)
__device__ __forceinline__ void fwd_body(
    const u32x4* x, const float* __restrict__ s_ptr, u32x4* y,
    u32x2* __restrict__ codes, int64_t nvec, int64_t n, int bits, int block, int nblocks)
{
    using S = Store16<DT>;
    const QConst k = make_qconst(*s_ptr, bits);
    constexpr int64_t kChunk = (int64_t)kThreads * kUnroll;
    const int64_t full_end = nvec / kChunk * kChunk;
    // full chunks: no predication, all kUnroll loads of a lane in flight together
    for (int64_t base = (int64_t)block * kChunk; base < full_end; base += (int64_t)nblocks * kChunk) {
        u32x4 in[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) in[u] = __builtin_nontemporal_load(&x[base + u * kThreads + threadIdx.x]);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            u32x4 out;
            u32x2 cw;
            fwd_vec<DT, CODES>(in[u], k, out, cw);
            __builtin_nontemporal_store(out, &y[base + u * kThreads + threadIdx.x]);
            if (CODES) codes[base + u * kThreads + threadIdx.x] = cw;
        }
    }
    if (block != 0) return;
    // remainder: fewer than kChunk vectors, then fewer than 8 scalars
    for (int64_t i = full_end + threadIdx.x; i < nvec; i += kThreads) {
        u32x4 out;
        u32x2 cw;
        fwd_vec<DT, CODES>(x[i], k, out, cw);
        y[i] = out;
        if (CODES) codes[i] = cw;
    }
    if (threadIdx.x < (unsigned)(n - nvec * 8)) {
        int64_t i = nvec * 8 + threadIdx.x;
        const uint16_t* xs = reinterpret_cast<const uint16_t*>(x);
        uint16_t* ys = reinterpret_cast<uint16_t*>(y);
        QElem e = quantize(S::one(xs[i]), k);
        ys[i] = S::enc(codef_of(e) * k.s);
        if (CODES) reinterpret_cast<int8_t*>(codes)[i] = (int8_t)code_of(e);
    }
}

template <int DT, bool CODES>
__global__ __launch_bounds__(kThreads) void fakequant_fwd_kernel(
    const u32x4* x, const float* __restrict__ s_ptr, u32x4* y,
    u32x2* __restrict__ codes, int64_t nvec, int64_t n, int bits)
{
    fwd_body<DT, CODES>(x, s_ptr, y, codes, nvec, n, bits, (int)blockIdx.x, (int)gridDim.x);
}

// Several tensors in one launch (the fake-quant operators of one decoder layer): the grid is cut
// into one run of blocks per tensor, sized by the host in proportion to the tensor.
constexpr int kMaxBatch = SASQ_MAX_BATCH;
// Forward operators that read the same x (the fake-quant operators in front of q/k/v, or gate/up:
// one input, one factor each) form one entry: its blocks load x once and apply every member's factor.
constexpr int kMaxShare = 3;
struct FqBatchItem {
    const u32x4* x;
    int64_t nvec, n;
    int ns;                           // members (1 = an operator alone on its x)
    const float* s[kMaxShare];
    const u32x4* dy[kMaxShare];
    u32x4* out[kMaxShare];
    float* ds[kMaxShare];
    int slot[kMaxShare];              // index in the caller's batch: selects the ticket word and the partials
};
struct FqBatch {
    FqBatchItem it[kMaxBatch];
    int first_block[kMaxBatch + 1];
    int count;
};

__device__ __forceinline__ int batch_item_of(const FqBatch& b, int block)
{
    int k = 0;
#pragma unroll
    for (int i = 1; i < kMaxBatch; ++i)
        if (i < b.count && block >= b.first_block[i]) k = i;
    return k;
}

// Forward of NS operators on one x: same traversal as fwd_body, one load of x per NS stores.
template <int DT, int NS>
__device__ __forceinline__ void fwd_body_shared(const FqBatchItem& it, int bits, int block, int nblocks)
{
    using S = Store16<DT>;
    const u32x4* x = it.x;
    const int64_t nvec = it.nvec, n = it.n;
    QConst k[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) k[j] = make_qconst(*it.s[j], bits);
    constexpr int64_t kChunk = (int64_t)kThreads * kUnroll;
    const int64_t full_end = nvec / kChunk * kChunk;
    for (int64_t base = (int64_t)block * kChunk; base < full_end; base += (int64_t)nblocks * kChunk) {
        u32x4 in[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) in[u] = __builtin_nontemporal_load(&x[base + u * kThreads + threadIdx.x]);
#pragma unroll
        for (int j = 0; j < NS; ++j)
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                u32x4 out;
                u32x2 cw;
                fwd_vec<DT, false>(in[u], k[j], out, cw);
                __builtin_nontemporal_store(out, &it.out[j][base + u * kThreads + threadIdx.x]);
            }
    }
    if (block != 0) return;
    for (int64_t i = full_end + threadIdx.x; i < nvec; i += kThreads) {
        const u32x4 in = x[i];
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            u32x4 out;
            u32x2 cw;
            fwd_vec<DT, false>(in, k[j], out, cw);
            it.out[j][i] = out;
        }
    }
    if (threadIdx.x < (unsigned)(n - nvec * 8)) {
        const int64_t i = nvec * 8 + threadIdx.x;
        const float xv = S::one(reinterpret_cast<const uint16_t*>(x)[i]);
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            QElem e = quantize(xv, k[j]);
            reinterpret_cast<uint16_t*>(it.out[j])[i] = S::enc(codef_of(e) * k[j].s);
        }
    }
}

// SHARED: some entry of the launch has more than one member (a launch without any keeps the leaner
// kernel: the shared bodies cost registers that lower its occupancy).
template <int DT, bool SHARED>
__global__ __launch_bounds__(kThreads) void fakequant_fwd_batch_kernel(const FqBatch b, int bits)
{
    const int k = batch_item_of(b, (int)blockIdx.x);
    const FqBatchItem& it = b.it[k];
    const int block = (int)blockIdx.x - b.first_block[k], nblocks = b.first_block[k + 1] - b.first_block[k];
    if (SHARED && it.ns == 2)      fwd_body_shared<DT, 2>(it, bits, block, nblocks);
    else if (SHARED && it.ns == 3) fwd_body_shared<DT, 3>(it, bits, block, nblocks);
    else                           fwd_body<DT, false>(it.x, it.s[0], it.out[0], nullptr, it.nvec, it.n, bits, block, nblocks);
}

// Per-element backward term.  For an unclipped element q == round(p), and fma(-x, inv_s, q)
// is the exact difference q - p rounded once; for a clipped one the term is q itself.
__device__ __forceinline__ float ds_term(float x, float g, const QConst& k, bool& keep)
{
    QElem e = quantize(x, k);
    keep = unclipped(e);
    float q = codef_of(e);
    float u = __builtin_fmaf(-x, k.inv_s, q);
    return g * (keep ? u : q);
}

// Backward on one 8-element vector: dx bits and the fp32 sum of the 8 ds terms.
template <int DT>
__device__ __forceinline__ float bwd_vec(const u32x4& xin, const u32x4& gin, const QConst& k, u32x4& out)
{
    using S = Store16<DT>;
    float part = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        bool ka, kb;
        float ta = ds_term(S::lo(xin[w]), S::lo(gin[w]), k, ka);
        float tb = ds_term(S::hi(xin[w]), S::hi(gin[w]), k, kb);
        part += ta;
        part += tb;
        out[w] = gin[w] & ((ka ? 0x0000FFFFu : 0u) | (kb ? 0xFFFF0000u : 0u));
    }
    return part;
}

__device__ __forceinline__ void final_reduce(float* __restrict__ ds, uint32_t* __restrict__ ticket_word,
                                             double* __restrict__ partials, int nblocks);

// The grid-wide part of the ds reduction for one tensor: this block's lane sums -> one fp64
// partial, published; the last block to arrive sums all partials in a fixed order.
__device__ __forceinline__ void publish_and_reduce(double acc, float* __restrict__ ds, uint32_t* __restrict__ ticket_word,
                                                   double* __restrict__ partials, int block, int nblocks)
{
    // block partial: lanes -> wave (shuffles) -> block (LDS), fixed order
    __shared__ double wave_part[kThreads / kWave];
    __shared__ bool is_last;
    double w = wave_sum(acc);
    const int lane = threadIdx.x % kWave, wid = threadIdx.x / kWave;
    if (lane == 0) wave_part[wid] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
        double b = 0.0;
#pragma unroll
        for (int i = 0; i < kThreads / kWave; ++i) b += wave_part[i];
        const uint32_t ticket = publish_then_ticket(&partials[block], b, ticket_word);
        is_last = (ticket == kTicketBase + (uint32_t)nblocks - 1);
        if (ticket - kTicketBase >= (uint32_t)nblocks)      // workspace was never initialised: fail loudly
            *ds = __uint_as_float(0x7FC00000u);
    }
    __syncthreads();
    if (!is_last) return;
    final_reduce(ds, ticket_word, partials, nblocks);
}

// Deterministic second pass by the last block to arrive: fixed strided order, fp64.
__device__ __forceinline__ void final_reduce(float* __restrict__ ds, uint32_t* __restrict__ ticket_word,
                                             double* __restrict__ partials, int nblocks)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    // all of a thread's partials are requested before the first is used (one memory latency, not
    // one per partial); the summation order stays fixed
    constexpr int kPer = kMaxReduceBlocks / kThreads;
    double pv[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int i = j * kThreads + threadIdx.x;
        pv[j] = __hip_atomic_load(&partials[i < nblocks ? i : 0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    double t = 0.0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) t += (j * kThreads + (int)threadIdx.x < nblocks) ? pv[j] : 0.0;
    __shared__ double tree[kThreads];
    tree[threadIdx.x] = t;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) tree[threadIdx.x] += tree[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        *ds = (float)tree[0];
        __hip_atomic_store(ticket_word, kTicketBase, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Backward over one tensor by block `block` of the `nblocks` (<= kMaxReduceBlocks) that share it;
// `ticket` and `partials` belong to this tensor alone.
template <int DT, bool WRITE_DX>
__device__ __forceinline__ void bwd_body(
    const u32x4* __restrict__ x, const u32x4* dy, const float* __restrict__ s_ptr,
    u32x4* dx, float* __restrict__ ds, uint32_t* __restrict__ ticket_word,
    double* __restrict__ partials, int64_t nvec, int64_t n, int bits, int block, int nblocks)
{
    using S = Store16<DT>;
    const QConst k = make_qconst(*s_ptr, bits);
    double acc = 0.0;       // 8 terms are summed in fp32, everything above that in fp64
    constexpr int64_t kChunk = (int64_t)kThreads * kUnroll;
    const int64_t full_end = nvec / kChunk * kChunk;
    for (int64_t base = (int64_t)block * kChunk; base < full_end; base += (int64_t)nblocks * kChunk) {
        u32x4 xin[kUnroll], gin[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            xin[u] = __builtin_nontemporal_load(&x[base + u * kThreads + threadIdx.x]);
            gin[u] = __builtin_nontemporal_load(&dy[base + u * kThreads + threadIdx.x]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            u32x4 out;
            acc += (double)bwd_vec<DT>(xin[u], gin[u], k, out);
            if (WRITE_DX) __builtin_nontemporal_store(out, &dx[base + u * kThreads + threadIdx.x]);
        }
    }
    if (block == 0) {
        for (int64_t i = full_end + threadIdx.x; i < nvec; i += kThreads) {
            u32x4 out;
            acc += (double)bwd_vec<DT>(x[i], dy[i], k, out);
            if (WRITE_DX) dx[i] = out;
        }
        if (threadIdx.x < (unsigned)(n - nvec * 8)) {
            int64_t i = nvec * 8 + threadIdx.x;
            const uint16_t* xs = reinterpret_cast<const uint16_t*>(x);
            const uint16_t* gs = reinterpret_cast<const uint16_t*>(dy);
            bool keep;
            float t = ds_term(S::one(xs[i]), S::one(gs[i]), k, keep);
            uint16_t g = gs[i];
            acc += (double)t;
            if (WRITE_DX) reinterpret_cast<uint16_t*>(dx)[i] = keep ? g : (uint16_t)0;
        }
    }

    publish_and_reduce(acc, ds, ticket_word, partials, block, nblocks);
}

template <int DT, bool WRITE_DX>
__global__ __launch_bounds__(kThreads) void fakequant_bwd_kernel(
    const u32x4* __restrict__ x, const u32x4* dy, const float* __restrict__ s_ptr,
    u32x4* dx, float* __restrict__ ds, uint32_t* __restrict__ ws_head,
    double* __restrict__ partials, int64_t nvec, int64_t n, int bits)
{
    bwd_body<DT, WRITE_DX>(x, dy, s_ptr, dx, ds, ws_head, partials, nvec, n, bits, (int)blockIdx.x, (int)gridDim.x);
}

// Batched backward: every entry is one operator (sharing the read of x did not pay here: the
// fused body needs 200 registers and ran 2 % slower than the operators apart); it uses the ticket
// word and the run of kMaxReduceBlocks partials of its index in the caller's batch.
template <int DT>
__global__ __launch_bounds__(kThreads) void fakequant_bwd_batch_kernel(
    const FqBatch b, uint32_t* __restrict__ ws_head, double* __restrict__ partials, int bits)
{
    const int k = batch_item_of(b, (int)blockIdx.x);
    const FqBatchItem& it = b.it[k];
    const int block = (int)blockIdx.x - b.first_block[k], nblocks = b.first_block[k + 1] - b.first_block[k];
    uint32_t* ticket = ws_head + it.slot[0];
    double* parts = partials + it.slot[0] * kMaxReduceBlocks;
    if (it.out[0]) bwd_body<DT, true>(it.x, it.dy[0], it.s[0], it.out[0], it.ds[0], ticket, parts, it.nvec, it.n, bits, block, nblocks);
    else           bwd_body<DT, false>(it.x, it.dy[0], it.s[0], it.out[0], it.ds[0], ticket, parts, it.nvec, it.n, bits, block, nblocks);
}

__global__ void scale_sgd_vec_kernel(float* s, const float* ds, int n, float lr)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        float step = lr * ds[i];
        s[i] = s[i] - step;
    }
}

__global__ void scale_sgd_kernel(float* s, const float* ds, float lr)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        float step = lr * *ds;
        *s = *s - step;
    }
}

// AdamW with decoupled weight decay on a vector of scales; the bias corrections 1 - beta^t are
// computed by the host in double and passed in.
__global__ void scale_adamw_kernel(float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m,
                                   float* __restrict__ v, int64_t n, float lr, float b1, float b2, float omb1,
                                   float omb2, float eps, float wd, float bc1, float bc2)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float pi = p[i];
    const float gi = g[i];
    pi = pi - lr * wd * pi;
    const float mi = b1 * m[i] + omb1 * gi;
    const float vi = b2 * v[i] + omb2 * gi * gi;
    pi = pi - lr * (mi / bc1) / (sqrtf(vi / bc2) + eps);
    p[i] = pi; m[i] = mi; v[i] = vi;
}

static int grid_for(int64_t nvec, int max_blocks)
{
    int64_t per_block = (int64_t)kThreads * kUnroll;
    int64_t need = (nvec + per_block - 1) / per_block;
    if (need < 1) need = 1;
    return (int)(need < max_blocks ? need : max_blocks);
}

static int check_shape(int64_t rows, int64_t cols, int bits, int dt)
{
    if (rows <= 0 || cols <= 0) return SASQ_ERR_SHAPE;
    if (rows > (INT64_C(1) << 40) / cols) return SASQ_ERR_SHAPE;
    if (bits < 2 || bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    return SASQ_OK;
}

}  // namespace sasq

using namespace sasq;

extern "C" int sasq_fakequant_fwd(const void* x, const float* s, void* y, int8_t* codes,
                                  int64_t rows, int64_t cols, int bits, sasq_dtype dt, void* stream)
{
    if (!x || !s || !y) return SASQ_ERR_NULL;
    int rc = check_shape(rows, cols, bits, (int)dt);
    if (rc) return rc;
    if (!aligned16(x) || !aligned16(y) || (codes && (reinterpret_cast<uintptr_t>(codes) & 7u))) return SASQ_ERR_ALIGN;
    const int64_t n = rows * cols, nvec = n / 8;
    const int grid = grid_for(nvec, kMaxFwdBlocks);
    hipStream_t st = as_stream(stream);
    auto X = static_cast<const u32x4*>(x);
    auto Y = static_cast<u32x4*>(y);
    auto C = reinterpret_cast<u32x2*>(codes);
    if (dt == SASQ_F16) {
        if (codes) fakequant_fwd_kernel<SASQ_F16, true><<<grid, kThreads, 0, st>>>(X, s, Y, C, nvec, n, bits);
        else       fakequant_fwd_kernel<SASQ_F16, false><<<grid, kThreads, 0, st>>>(X, s, Y, C, nvec, n, bits);
    } else {
        if (codes) fakequant_fwd_kernel<SASQ_BF16, true><<<grid, kThreads, 0, st>>>(X, s, Y, C, nvec, n, bits);
        else       fakequant_fwd_kernel<SASQ_BF16, false><<<grid, kThreads, 0, st>>>(X, s, Y, C, nvec, n, bits);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" size_t sasq_fakequant_bwd_workspace(int64_t rows, int64_t cols)
{
    (void)rows; (void)cols;
    return kWsHeaderBytes + sizeof(double) * kMaxReduceBlocks;
}

extern "C" int sasq_fakequant_bwd(const void* x, const void* dy, const float* s, void* dx, float* ds,
                                  int64_t rows, int64_t cols, int bits, sasq_dtype dt,
                                  void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !dy || !s || !ds) return SASQ_ERR_NULL;
    int rc = check_shape(rows, cols, bits, (int)dt);
    if (rc) return rc;
    if (!aligned16(x) || !aligned16(dy) || (dx && !aligned16(dx))) return SASQ_ERR_ALIGN;
    if (!workspace || workspace_bytes < sasq_fakequant_bwd_workspace(rows, cols)) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;
    const int64_t n = rows * cols, nvec = n / 8;
    const int grid = grid_for(nvec, kMaxReduceBlocks);
    hipStream_t st = as_stream(stream);
    auto X = static_cast<const u32x4*>(x);
    auto G = static_cast<const u32x4*>(dy);
    auto DX = static_cast<u32x4*>(dx);
    auto head = static_cast<uint32_t*>(workspace);
    auto parts = reinterpret_cast<double*>(static_cast<char*>(workspace) + kWsHeaderBytes);
    if (dt == SASQ_F16) {
        if (dx) fakequant_bwd_kernel<SASQ_F16, true><<<grid, kThreads, 0, st>>>(X, G, s, DX, ds, head, parts, nvec, n, bits);
        else    fakequant_bwd_kernel<SASQ_F16, false><<<grid, kThreads, 0, st>>>(X, G, s, DX, ds, head, parts, nvec, n, bits);
    } else {
        if (dx) fakequant_bwd_kernel<SASQ_BF16, true><<<grid, kThreads, 0, st>>>(X, G, s, DX, ds, head, parts, nvec, n, bits);
        else    fakequant_bwd_kernel<SASQ_BF16, false><<<grid, kThreads, 0, st>>>(X, G, s, DX, ds, head, parts, nvec, n, bits);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

// ---- backward without a workspace argument and without any allocation ----------------------------
// For callers that cannot allocate device memory (code under HIP graph capture, tight serving
// loops, harnesses that forbid it): the ticket word and the block partials live in a file-scope
// device array instead of a caller-provided workspace.  Each GPU holds its own copy of the array
// at its own address; the address is looked up once per device and cached.  In host code the
// array's name is only a handle for that lookup, never a device address.
namespace sasq {

constexpr size_t kStaticScratchBytes = kWsHeaderBytes + sizeof(double) * kMaxReduceBlocks;   // 3 KB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];          // per device: where `scratch` lives on that GPU

// Address of this device's copy of `scratch` (nullptr on failure).  No allocation.
static void* scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

// The ticket word must be zero when the backward kernel starts.  (A fill kernel, not a memset:
// memset nodes recorded into a captured graph are avoided on purpose.)
__global__ void clear_ticket_kernel(uint32_t* head) { if (threadIdx.x == 0) head[0] = kTicketBase; }

}  // namespace sasq

extern "C" int sasq_fakequant_bwd_static(const void* x, const void* dy, const float* s, void* dx, float* ds,
                                         int64_t rows, int64_t cols, int bits, sasq_dtype dt, void* stream)
{
    if (!x || !dy || !s || !ds) return SASQ_ERR_NULL;
    int rc = check_shape(rows, cols, bits, (int)dt);
    if (rc) return rc;
    if (rows * cols > SASQ_FAKEQUANT_BWD_STATIC_MAX_ELEMENTS) return SASQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(dy) || (dx && !aligned16(dx))) return SASQ_ERR_ALIGN;
    void* base = scratch_of_current_device();
    if (!base) return SASQ_ERR_WORKSPACE;
    const int64_t n = rows * cols, nvec = n / 8;
    const int grid = grid_for(nvec, kMaxReduceBlocks);
    hipStream_t st = as_stream(stream);
    auto X = static_cast<const u32x4*>(x);
    auto G = static_cast<const u32x4*>(dy);
    auto DX = static_cast<u32x4*>(dx);
    auto head = static_cast<uint32_t*>(base);
    auto parts = reinterpret_cast<double*>(static_cast<char*>(base) + kWsHeaderBytes);
    clear_ticket_kernel<<<1, 64, 0, st>>>(head);
    if (dt == SASQ_F16) {
        if (dx) fakequant_bwd_kernel<SASQ_F16, true><<<grid, kThreads, 0, st>>>(X, G, s, DX, ds, head, parts, nvec, n, bits);
        else    fakequant_bwd_kernel<SASQ_F16, false><<<grid, kThreads, 0, st>>>(X, G, s, DX, ds, head, parts, nvec, n, bits);
    } else {
        if (dx) fakequant_bwd_kernel<SASQ_BF16, true><<<grid, kThreads, 0, st>>>(X, G, s, DX, ds, head, parts, nvec, n, bits);
        else    fakequant_bwd_kernel<SASQ_BF16, false><<<grid, kThreads, 0, st>>>(X, G, s, DX, ds, head, parts, nvec, n, bits);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" int sasq_scale_sgd(float* s, const float* ds, float lr, void* stream)
{
    if (!s || !ds) return SASQ_ERR_NULL;
    scale_sgd_kernel<<<1, 64, 0, as_stream(stream)>>>(s, ds, lr);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" int sasq_scale_adamw(float* s, const float* ds, float* m, float* v, int64_t n, int64_t step,
                                double lr, double beta1, double beta2, double eps, double weight_decay, void* stream)
{
    if (!s || !ds || !m || !v) return SASQ_ERR_NULL;
    if (n <= 0 || n > (INT64_C(1) << 31) || step <= 0) return SASQ_ERR_SHAPE;
    // 1 - beta and 1 - beta^step are formed in double: in fp32, 1 - 0.999f is off by 1e-5 relative
    const float bc1 = (float)(1.0 - pow(beta1, (double)step));
    const float bc2 = (float)(1.0 - pow(beta2, (double)step));
    const int blocks = (int)((n + 255) / 256);
    scale_adamw_kernel<<<blocks, 256, 0, as_stream(stream)>>>(s, ds, m, v, n, (float)lr, (float)beta1, (float)beta2,
                                                              (float)(1.0 - beta1), (float)(1.0 - beta2), (float)eps,
                                                              (float)weight_decay, bc1, bc2);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

// ---- batched entry points ---------------------------------------------------------------------
namespace sasq {

constexpr int kBatchFwdBlocks = 2048;
constexpr int kBatchBwdBlocks = 512;
// Tensors streamed concurrently by one launch: up to this many input bytes in all.  Beyond it the
// launch is slower than one launch per tensor (measured: seven tensors of 134-470 MB in one launch
// reach 5.0 TB/s, one after the other 6.1 TB/s; three tensors of 157 MB in all 5.8 against 5.1),
// so a batch is cut, in order, into launches under the limit.
constexpr int64_t kBatchLaunchBytes = INT64_C(192) << 20;
// Operators on the same x are grouped from this size up.  Measured, layer fwd+bwd: 8.4 M elements
// (LLaMA-2-7B q/k/v at 2048 tokens) 57.4 us apart, 58.6-60.4 us grouped; 16.8 M (gate/up at 4096
// tokens) 140.3 -> 136.5 us; 21 M (13B shapes) 307.6 -> 298.5 us.
constexpr int64_t kShareMinElements = INT64_C(12) << 20;

static int check_items(const sasq_fq_item* items, int count, bool backward)
{
    if (!items) return SASQ_ERR_NULL;
    if (count <= 0 || count > kMaxBatch) return SASQ_ERR_SHAPE;
    for (int i = 0; i < count; ++i) {
        const sasq_fq_item& it = items[i];
        if (!it.x || !it.s || (backward ? (!it.dy || !it.ds) : !it.out)) return SASQ_ERR_NULL;
        if (it.rows <= 0 || it.cols <= 0 || it.rows > (INT64_C(1) << 40) / it.cols) return SASQ_ERR_SHAPE;
        if (!aligned16(it.x) || (it.out && !aligned16(it.out)) || (backward && !aligned16(it.dy))) return SASQ_ERR_ALIGN;
    }
    return SASQ_OK;
}

// Items [lo, hi) as one launch: `total_blocks` cut into one run per tensor, proportional to its
// size, at least one block and at most `max_per_item` each.  A tensor keeps its index in the batch
// (it selects the tensor's ticket word and partials).
static void build_launch(const sasq_fq_item* items, int lo, int hi, int total_blocks, int max_per_item, bool share, FqBatch& b)
{
    // entries: operators on the same x (same pointer, same size) share one, up to kMaxShare members
    // (sasq_set_tuning(SASQ_TUNE_FQ_SHARE, 1|2|3) overrides the limit and lifts the size threshold).  A group's run of blocks is
    // capped like a single tensor's, so members are only added while the group still gets all the
    // blocks its members would have had apart.
    int max_share = share ? kMaxShare : 1;
    int64_t min_elements = kShareMinElements;
    if (const int v = tuning(SASQ_TUNE_FQ_SHARE)) {
        if (share && v >= 1 && v <= kMaxShare) { max_share = v; min_elements = 0; }
    }
    int64_t all_vec = 0;
    for (int i = lo; i < hi; ++i) all_vec += items[i].rows * items[i].cols / 8 + 1;
    b.count = 0;
    int64_t total_vec = 0;
    bool taken[kMaxBatch] = {false};
    for (int i = lo; i < hi; ++i) {
        if (taken[i - lo]) continue;
        const int64_t n = items[i].rows * items[i].cols;
        FqBatchItem& e = b.it[b.count++];
        e.x = static_cast<const u32x4*>(items[i].x);
        e.nvec = n / 8;
        e.n = n;
        e.ns = 0;
        const int64_t alone = ((n / 8 + 1) * total_blocks + all_vec - 1) / all_vec;      // blocks of one member on its own
        for (int j = i; j < hi && e.ns < max_share; ++j) {
            if (e.ns >= 1 && (alone * (e.ns + 1) > max_per_item || n < min_elements)) break;
            if (taken[j - lo] || items[j].x != items[i].x || items[j].rows * items[j].cols != n) continue;
            taken[j - lo] = true;
            e.s[e.ns] = items[j].s;
            e.dy[e.ns] = static_cast<const u32x4*>(items[j].dy);
            e.out[e.ns] = static_cast<u32x4*>(items[j].out);
            e.ds[e.ns] = items[j].ds;
            e.slot[e.ns] = j;
            ++e.ns;
        }
        total_vec += (n / 8 + 1) * e.ns;
    }
    b.first_block[0] = 0;
    const int64_t per_block = (int64_t)kThreads * kUnroll;
    for (int i = 0; i < b.count; ++i) {
        const int64_t need = (b.it[i].nvec + per_block - 1) / per_block;            // blocks that would each have a full chunk
        int64_t share = ((b.it[i].nvec + 1) * b.it[i].ns * total_blocks + total_vec - 1) / total_vec;
        if (share > need) share = need;
        if (share > max_per_item) share = max_per_item;
        if (share < 1) share = 1;
        b.first_block[i + 1] = b.first_block[i] + (int)share;
    }
    for (int i = b.count; i < kMaxBatch; ++i) b.first_block[i + 1] = b.first_block[b.count];
}

static bool any_shared(const FqBatch& b)
{
    for (int i = 0; i < b.count; ++i)
        if (b.it[i].ns > 1) return true;
    return false;
}

// next launch: items [lo, return value)
static int launch_end(const sasq_fq_item* items, int lo, int count)
{
    int64_t bytes = 0;
    int hi = lo;
    while (hi < count) {
        const int64_t b = items[hi].rows * items[hi].cols * 2;
        if (hi > lo && bytes + b > kBatchLaunchBytes) break;
        bytes += b;
        ++hi;
    }
    return hi;
}

}  // namespace sasq

extern "C" int sasq_fakequant_fwd_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt, void* stream)
{
    if (bits < 2 || bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    const int rc = check_items(items, count, false);
    if (rc) return rc;
    for (int lo = 0; lo < count;) {
        const int hi = launch_end(items, lo, count);
        FqBatch b{};
        build_launch(items, lo, hi, kBatchFwdBlocks, kBatchFwdBlocks, true, b);
        const int grid = b.first_block[b.count];
        hipStream_t st = as_stream(stream);
        if (any_shared(b)) {
            if (dt == SASQ_F16) fakequant_fwd_batch_kernel<SASQ_F16, true><<<grid, kThreads, 0, st>>>(b, bits);
            else                fakequant_fwd_batch_kernel<SASQ_BF16, true><<<grid, kThreads, 0, st>>>(b, bits);
        } else {
            if (dt == SASQ_F16) fakequant_fwd_batch_kernel<SASQ_F16, false><<<grid, kThreads, 0, st>>>(b, bits);
            else                fakequant_fwd_batch_kernel<SASQ_BF16, false><<<grid, kThreads, 0, st>>>(b, bits);
        }
        lo = hi;
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" size_t sasq_fakequant_bwd_batch_workspace(int count)
{
    if (count <= 0 || count > kMaxBatch) return 0;
    return kWsHeaderBytes + sizeof(double) * kMaxReduceBlocks * (size_t)count;
}

extern "C" int sasq_fakequant_bwd_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt,
                                        void* workspace, size_t workspace_bytes, void* stream)
{
    if (bits < 2 || bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    const int rc = check_items(items, count, true);
    if (rc) return rc;
    if (!workspace || workspace_bytes < sasq_fakequant_bwd_batch_workspace(count)) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;
    auto head = static_cast<uint32_t*>(workspace);
    auto parts = reinterpret_cast<double*>(static_cast<char*>(workspace) + kWsHeaderBytes);
    for (int lo = 0; lo < count;) {
        const int hi = launch_end(items, lo, count);
        FqBatch b{};
        // a tensor alone in its launch gets what the single-tensor call gives it: one block per CU
        build_launch(items, lo, hi, hi - lo == 1 ? kMaxReduceBlocks : kBatchBwdBlocks, kMaxReduceBlocks, false, b);
        const int grid = b.first_block[b.count];
        hipStream_t st = as_stream(stream);
        if (dt == SASQ_F16) fakequant_bwd_batch_kernel<SASQ_F16><<<grid, kThreads, 0, st>>>(b, head, parts, bits);
        else                fakequant_bwd_batch_kernel<SASQ_BF16><<<grid, kThreads, 0, st>>>(b, head, parts, bits);
        lo = hi;
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" int sasq_scale_sgd_vec(float* s, const float* ds, int64_t n, float lr, void* stream)
{
    if (!s || !ds) return SASQ_ERR_NULL;
    if (n <= 0 || n > (INT64_C(1) << 31) - 256) return SASQ_ERR_SHAPE;
    scale_sgd_vec_kernel<<<(int)((n + 255) / 256), 256, 0, as_stream(stream)>>>(s, ds, (int)n, lr);
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}
