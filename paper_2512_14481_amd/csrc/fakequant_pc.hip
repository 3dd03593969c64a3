// Per-channel fake quantization: one learned factor per activation column (the granularity Sec. 4
// adopts for activations and weights; Sec. 2, Fig. 2(b): per-channel = the elements of a column
// share a factor).  Same element arithmetic as the per-tensor operator
// (Sec. 3, Eq. 1; Sec. 4.2, Eq. 4); the scale gradient becomes a column reduction:
//     ds[k] = sum_m dy[m,k] * (q[m,k] - m[m,k] * x[m,k]/s[k]).
//
// Traversal: a lane owns 8 consecutive columns (one 128-bit access) for the whole kernel, so its
// eight scales and reciprocals live in registers; a wave covers 512 consecutive columns of one
// row (1 KB, fully coalesced); the 4 waves of a block take rows r, r+1, r+2, r+3 of the block's
// row chunk.  Grid = column chunks x row chunks.
#include "sasq_device.h"
#include <cstring>

namespace sasq {

constexpr int kPcThreads = 256;
constexpr int kPcWaves = kPcThreads / kWave;
constexpr int kPcColsPerBlock = kWave * 8;        // 512
constexpr int kPcRowUnroll = 4;                   // rows in flight per wave
constexpr int kPcMaxRowChunks = 128;              // more row chunks than this lengthen the reduction tail (measured)
constexpr int kPcTargetBlocks = 2048;             // 8 blocks per CU

struct PcConst {
    float inv_s[8];
    float s[8];
    float lo, hi;
};

__device__ __forceinline__ PcConst load_pc(const float* __restrict__ s, int64_t col0, int64_t cols, int bits)
{
    PcConst c;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v = s[col0 + e < cols ? col0 + e : cols - 1];
        c.s[e] = v;
        c.inv_s[e] = 1.0f / v;
    }
    c.lo = kMagic - (float)(1 << (bits - 1));
    c.hi = kMagic + (float)((1 << (bits - 1)) - 1);
    return c;
}

__device__ __forceinline__ QElem quantize_pc(float x, float inv_s, const PcConst& c)
{
    QElem e;
    e.f = __builtin_fmaf(x, inv_s, kMagic);
    e.c = __builtin_amdgcn_fmed3f(e.f, c.lo, c.hi);
    return e;
}

// The block (col_block, row_chunk) of one tensor's grid: the kernels below pass their block
// indices, or (batched) the position inside the tensor's run of blocks.
template <int DT, bool CODES>
__device__ __forceinline__ void fwd_pc_body(
    const uint16_t* __restrict__ x, const float* __restrict__ s, uint16_t* __restrict__ y,
    int8_t* __restrict__ codes, int64_t rows, int64_t cols, int64_t rows_per_chunk, int bits,
    int col_block, int row_chunk)
{
    using S = Store16<DT>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t col0 = (int64_t)col_block * kPcColsPerBlock + lane * 8;
    if (col0 >= cols) return;
    const int64_t r_begin = (int64_t)row_chunk * rows_per_chunk;
    const int64_t r_end = min(rows, r_begin + rows_per_chunk);
    // Groups of kPcRowUnroll rows per wave, double-buffered: the next group's loads are in flight
    // while the current one is computed, and the first group's loads are issued before the
    // column factors are fetched and inverted (few waves per CU: latency must be hidden in-wave).
    constexpr int64_t kStep = kPcWaves * kPcRowUnroll;
    auto full = [&](int64_t rr) { return rr + (kPcRowUnroll - 1) * kPcWaves < r_end; };
    auto load_group = [&](u32x4 (&buf)[kPcRowUnroll], int64_t rr) {
#pragma unroll
        for (int u = 0; u < kPcRowUnroll; ++u)
            buf[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + (rr + u * kPcWaves) * cols + col0));
    };
    int64_t r = r_begin + wave;
    u32x4 bufa[kPcRowUnroll], bufb[kPcRowUnroll];
    bool have = full(r);
    if (have) load_group(bufa, r);
    const PcConst c = load_pc(s, col0, cols, bits);
    auto one_row = [&](const u32x4 in, int64_t rr) {
        u32x4 out;
        float cc[8];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            QElem a = quantize_pc(S::lo(in[w]), c.inv_s[2 * w], c);
            QElem b = quantize_pc(S::hi(in[w]), c.inv_s[2 * w + 1], c);
            out[w] = S::pack(codef_of(a) * c.s[2 * w], codef_of(b) * c.s[2 * w + 1]);
            cc[2 * w] = a.c;
            cc[2 * w + 1] = b.c;
        }
        __builtin_nontemporal_store(out, reinterpret_cast<u32x4*>(y + rr * cols + col0));
        if (CODES) {
            u32x2 cw = {pack_codes4(cc[0], cc[1], cc[2], cc[3]), pack_codes4(cc[4], cc[5], cc[6], cc[7])};
            *reinterpret_cast<u32x2*>(codes + rr * cols + col0) = cw;
        }
    };
    // full groups without per-row predication (a clamp or an early exit inside the unrolled loop
    // makes the compiler serialize the loads), then the leftover rows
    while (have) {
        bool more = full(r + kStep);
        if (more) load_group(bufb, r + kStep);
#pragma unroll
        for (int u = 0; u < kPcRowUnroll; ++u) one_row(bufa[u], r + u * kPcWaves);
        r += kStep;
        have = more;
        if (!have) break;
        more = full(r + kStep);
        if (more) load_group(bufa, r + kStep);
#pragma unroll
        for (int u = 0; u < kPcRowUnroll; ++u) one_row(bufb[u], r + u * kPcWaves);
        r += kStep;
        have = more;
    }
    for (; r < r_end; r += kPcWaves)
        one_row(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + r * cols + col0)), r);
}

template <int DT, bool CODES>
__global__ __launch_bounds__(kPcThreads) void fakequant_fwd_pc_kernel(
    const uint16_t* __restrict__ x, const float* __restrict__ s, uint16_t* __restrict__ y,
    int8_t* __restrict__ codes, int64_t rows, int64_t cols, int64_t rows_per_chunk, int bits)
{
    fwd_pc_body<DT, CODES>(x, s, y, codes, rows, cols, rows_per_chunk, bits, (int)blockIdx.x, (int)blockIdx.y);
}

template <int DT, bool WRITE_DX>
__device__ __forceinline__ void bwd_pc_body(
    const uint16_t* __restrict__ x, const uint16_t* dy, const float* __restrict__ s,
    uint16_t* dx, float* __restrict__ ds, uint32_t* __restrict__ tickets, float* __restrict__ partials,
    int64_t rows, int64_t cols, int64_t rows_per_chunk, int bits,
    int col_block, int row_chunk, int nchunks, float (&red)[kPcWaves][kPcColsPerBlock], bool& is_last)
{
    using S = Store16<DT>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t cbase = (int64_t)col_block * kPcColsPerBlock;
    const int64_t col0 = cbase + lane * 8;
    const bool active = col0 < cols;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (active) {
        const int64_t r_begin = (int64_t)row_chunk * rows_per_chunk;
        const int64_t r_end = min(rows, r_begin + rows_per_chunk);
        // same double-buffered traversal as the forward kernel, two input streams
        constexpr int64_t kStep = kPcWaves * kPcRowUnroll;
        auto full = [&](int64_t rr) { return rr + (kPcRowUnroll - 1) * kPcWaves < r_end; };
        auto load_group = [&](u32x4 (&bx)[kPcRowUnroll], u32x4 (&bg)[kPcRowUnroll], int64_t rr) {
#pragma unroll
            for (int u = 0; u < kPcRowUnroll; ++u) {
                bx[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + (rr + u * kPcWaves) * cols + col0));
                bg[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dy + (rr + u * kPcWaves) * cols + col0));
            }
        };
        int64_t r = r_begin + wave;
        u32x4 xa_[kPcRowUnroll], ga_[kPcRowUnroll], xb_[kPcRowUnroll], gb_[kPcRowUnroll];
        bool have = full(r);
        if (have) load_group(xa_, ga_, r);
        const PcConst c = load_pc(s, col0, cols, bits);
        auto one_row = [&](const u32x4 xin, const u32x4 gin, int64_t rr) {
            u32x4 out;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float xa = S::lo(xin[w]), xb = S::hi(xin[w]);
                QElem a = quantize_pc(xa, c.inv_s[2 * w], c);
                QElem b = quantize_pc(xb, c.inv_s[2 * w + 1], c);
                const bool ka = unclipped(a), kb = unclipped(b);
                const float qa = codef_of(a), qb = codef_of(b);
                const float ua = __builtin_fmaf(-xa, c.inv_s[2 * w], qa), ub = __builtin_fmaf(-xb, c.inv_s[2 * w + 1], qb);
                acc[2 * w] += S::lo(gin[w]) * (ka ? ua : qa);
                acc[2 * w + 1] += S::hi(gin[w]) * (kb ? ub : qb);
                out[w] = gin[w] & ((ka ? 0x0000FFFFu : 0u) | (kb ? 0xFFFF0000u : 0u));
            }
            if (WRITE_DX) __builtin_nontemporal_store(out, reinterpret_cast<u32x4*>(dx + rr * cols + col0));
        };
        // full groups, then the leftover rows (same row order per wave either way)
        while (have) {
            bool more = full(r + kStep);
            if (more) load_group(xb_, gb_, r + kStep);
#pragma unroll
            for (int u = 0; u < kPcRowUnroll; ++u) one_row(xa_[u], ga_[u], r + u * kPcWaves);
            r += kStep;
            have = more;
            if (!have) break;
            more = full(r + kStep);
            if (more) load_group(xa_, ga_, r + kStep);
#pragma unroll
            for (int u = 0; u < kPcRowUnroll; ++u) one_row(xb_[u], gb_[u], r + u * kPcWaves);
            r += kStep;
            have = more;
        }
        for (; r < r_end; r += kPcWaves)
            one_row(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + r * cols + col0)),
                    __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dy + r * cols + col0)), r);
    }
    // block partial per column: waves in fixed order
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wave][lane * 8 + e] = acc[e];
    __syncthreads();
    // One 128-bit store per 4 columns, with the agent-scope cache policy the compiler gives its own
    // agent-scope atomic stores (sc1): 4-byte stores of the same data are four times as many
    // write-through transactions, and every block waits for their acknowledgement below.
    if (threadIdx.x < kPcColsPerBlock / 4) {
        const int c4 = threadIdx.x * 4;
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float a = 0.0f;
#pragma unroll
            for (int w = 0; w < kPcWaves; ++w) a += red[w][c4 + e];
            v[e] = a;
        }
        if (cbase + c4 < cols) {        // cols is a multiple of 8: a group of 4 is all in or all out
            float* dst = &partials[(int64_t)row_chunk * cols + cbase + c4];
            asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst), "v"(v) : "memory");
        }
    }
    // the stores above are agent-scope (sc1: written through to the level all XCDs share) and
    // acknowledged before the ticket is taken: see publish_then_ticket in sasq_device.h
    wait_stores_acknowledged();
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t ticket = __hip_atomic_fetch_add(&tickets[col_block], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (ticket == (uint32_t)nchunks - 1);
        if (ticket >= (uint32_t)nchunks) ds[cbase < cols ? cbase : 0] = __uint_as_float(0x7FC00000u);   // uninitialised workspace
    }
    __syncthreads();
    if (!is_last) return;
    // last block of this column chunk: row chunks summed in ascending order, in fp64.  The
    // acquire fence makes the other blocks' write-through partials visible to ordinary loads.  A
    // thread takes four adjacent columns (one 128-bit load per row chunk) of one half of the row
    // chunks and keeps 32 loads in flight (loading them a few at a time leaves the whole grid's
    // tail waiting on a chain of memory latencies); the halves meet in LDS, lower half first.
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    {
        constexpr int kBatch = 32;
        const int half = threadIdx.x >> 7;                               // 0: first half of the chunks, 1: second
        const int c4 = (threadIdx.x & 127) * 4;
        const bool ok = cbase + c4 < cols;                               // cols is a multiple of 8
        const uint32_t colv = ok ? (uint32_t)c4 : 0u;
        const int split = (nchunks + 1) >> 1;
        const int rc_begin = half ? split : 0, rc_end = half ? nchunks : split;
        double t[4] = {0.0, 0.0, 0.0, 0.0};
        for (int rc0 = rc_begin; rc0 < rc_end; rc0 += kBatch) {
            f32x4 pv[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int rc = rc0 + j < rc_end ? rc0 + j : nchunks - 1;
                const float* rowp = partials + (int64_t)rc * cols + cbase;  // uniform: scalar base, lane offset
                pv[j] = *reinterpret_cast<const f32x4*>(rowp + colv);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j)
                if (rc0 + j < rc_end) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[e] += (double)pv[j][e];
                }
        }
        double* meet = reinterpret_cast<double*>(&red[0][0]);            // 512 doubles of the 8 KB
        __syncthreads();                                                 // red's earlier contents are consumed
        if (half) {
#pragma unroll
            for (int e = 0; e < 4; ++e) meet[c4 + e] = t[e];
        }
        __syncthreads();
        if (!half && ok) {
            f32x4 out;
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = (float)(t[e] + meet[c4 + e]);
            *reinterpret_cast<f32x4*>(&ds[cbase + c4]) = out;
        }
    }
    if (threadIdx.x == 0) __hip_atomic_store(&tickets[col_block], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int DT, bool WRITE_DX>
__global__ __launch_bounds__(kPcThreads) void fakequant_bwd_pc_kernel(
    const uint16_t* __restrict__ x, const uint16_t* dy, const float* __restrict__ s,
    uint16_t* dx, float* __restrict__ ds, uint32_t* __restrict__ tickets, float* __restrict__ partials,
    int64_t rows, int64_t cols, int64_t rows_per_chunk, int bits)
{
    __shared__ float red[kPcWaves][kPcColsPerBlock];
    __shared__ bool is_last;
    bwd_pc_body<DT, WRITE_DX>(x, dy, s, dx, ds, tickets, partials, rows, cols, rows_per_chunk, bits,
                              (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.y, red, is_last);
}

// ---- several tensors in one launch -------------------------------------------------------------
// Each tensor owns a run of consecutive block ids, column block fastest (the order a 2-D grid
// dispatches in); one launch for the fake-quant operators of a layer pays one ramp and one drain.
struct PcItem {
    const uint16_t* x;
    const uint16_t* dy;
    const float* s;
    uint16_t* out;        // y (forward) or dx (backward, may be null)
    float* ds;
    uint32_t* tickets;
    float* partials;
    int64_t rows, cols, rpc;
    int col_blocks, chunks;
};
struct PcBatch {
    PcItem it[SASQ_MAX_BATCH];
    int first_block[SASQ_MAX_BATCH + 1];
    int count;
};

__device__ __forceinline__ int pc_item_of(const PcBatch& b, int bid)
{
    int k = 0;
#pragma unroll
    for (int i = 1; i < SASQ_MAX_BATCH; ++i)
        if (i < b.count && bid >= b.first_block[i]) k = i;
    return k;
}

template <int DT>
__global__ __launch_bounds__(kPcThreads) void fakequant_fwd_pc_batch_kernel(const PcBatch b, int bits)
{
    const int k = pc_item_of(b, (int)blockIdx.x);
    const PcItem& it = b.it[k];
    const int lb = (int)blockIdx.x - b.first_block[k];
    fwd_pc_body<DT, false>(it.x, it.s, it.out, nullptr, it.rows, it.cols, it.rpc, bits, lb % it.col_blocks, lb / it.col_blocks);
}

template <int DT>
__global__ __launch_bounds__(kPcThreads) void fakequant_bwd_pc_batch_kernel(const PcBatch b, int bits)
{
    __shared__ float red[kPcWaves][kPcColsPerBlock];
    __shared__ bool is_last;
    const int k = pc_item_of(b, (int)blockIdx.x);
    const PcItem& it = b.it[k];
    const int lb = (int)blockIdx.x - b.first_block[k];
    const int cb = lb % it.col_blocks, rc = lb / it.col_blocks;
    if (it.out) bwd_pc_body<DT, true>(it.x, it.dy, it.s, it.out, it.ds, it.tickets, it.partials, it.rows, it.cols, it.rpc, bits,
                                      cb, rc, it.chunks, red, is_last);
    else        bwd_pc_body<DT, false>(it.x, it.dy, it.s, nullptr, it.ds, it.tickets, it.partials, it.rows, it.cols, it.rpc, bits,
                                       cb, rc, it.chunks, red, is_last);
}

// cols not a multiple of 8: one thread per column walks the rows (rarely used, kept simple)
template <int DT>
__global__ void fakequant_pc_scalar_kernel(const uint16_t* __restrict__ x, const uint16_t* dy, const float* __restrict__ s,
                                           uint16_t* y, int8_t* codes, uint16_t* dx, float* ds,
                                           int64_t rows, int64_t cols, int bits, int backward)
{
    using S = Store16<DT>;
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= cols) return;
    const QConst c = make_qconst(s[k], bits);
    double acc = 0.0;
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t i = r * cols + k;
        const float xv = S::one(x[i]);
        const QElem e = quantize(xv, c);
        if (!backward) {
            y[i] = S::enc(codef_of(e) * c.s);
            if (codes) codes[i] = (int8_t)code_of(e);
        } else {
            const bool keep = unclipped(e);
            const float q = codef_of(e);
            const uint16_t g = dy[i];
            acc += (double)(S::one(g) * (keep ? __builtin_fmaf(-xv, c.inv_s, q) : q));
            if (dx) dx[i] = keep ? g : (uint16_t)0;
        }
    }
    if (backward) ds[k] = (float)acc;
}

static int pc_row_chunks(int64_t rows, int64_t col_blocks)
{
    // enough blocks to fill the chip, at least 16 rows per block, at most kPcMaxRowChunks
    int64_t want = (kPcTargetBlocks + col_blocks - 1) / col_blocks;
    int64_t by_rows = (rows + 15) / 16;
    int64_t rc = want < by_rows ? want : by_rows;
    if (rc < 1) rc = 1;
    if (rc > kPcMaxRowChunks) rc = kPcMaxRowChunks;
    return (int)rc;
}

// rows per chunk: a multiple of 16 (whole unpredicated groups in every chunk but the last)
static void pc_geometry(int64_t rows, int64_t cols, int64_t& col_blocks, int64_t& rpc, int& chunks)
{
    col_blocks = (cols + kPcColsPerBlock - 1) / kPcColsPerBlock;
    const int want = pc_row_chunks(rows, col_blocks);
    rpc = ((rows + want - 1) / want + 15) / 16 * 16;
    chunks = (int)((rows + rpc - 1) / rpc);
}

static int check_pc(int64_t rows, int64_t cols, int bits, int dt)
{
    if (rows <= 0 || cols <= 0) return SASQ_ERR_SHAPE;
    if (rows > (INT64_C(1) << 40) / cols) return SASQ_ERR_SHAPE;
    if ((cols + kPcColsPerBlock - 1) / kPcColsPerBlock > (int64_t)(kWsHeaderBytes / 4)) return SASQ_ERR_SHAPE;
    if (bits < 2 || bits > 8) return SASQ_ERR_UNSUPPORTED;
    if (dt != SASQ_F16 && dt != SASQ_BF16) return SASQ_ERR_UNSUPPORTED;
    return SASQ_OK;
}

}  // namespace sasq

using namespace sasq;

extern "C" int sasq_fakequant_fwd_pc(const void* x, const float* s, void* y, int8_t* codes,
                                     int64_t rows, int64_t cols, int bits, sasq_dtype dt, void* stream)
{
    if (!x || !s || !y) return SASQ_ERR_NULL;
    int rc = check_pc(rows, cols, bits, (int)dt);
    if (rc) return rc;
    if (!aligned16(x) || !aligned16(y) || (codes && (reinterpret_cast<uintptr_t>(codes) & 7u))) return SASQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    auto X = static_cast<const uint16_t*>(x);
    auto Y = static_cast<uint16_t*>(y);
    if (cols % 8 != 0) {
        const int blocks = (int)((cols + 255) / 256);
        if (dt == SASQ_F16) fakequant_pc_scalar_kernel<SASQ_F16><<<blocks, 256, 0, st>>>(X, nullptr, s, Y, codes, nullptr, nullptr, rows, cols, bits, 0);
        else                fakequant_pc_scalar_kernel<SASQ_BF16><<<blocks, 256, 0, st>>>(X, nullptr, s, Y, codes, nullptr, nullptr, rows, cols, bits, 0);
        return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
    }
    int64_t col_blocks, rpc;
    int chunks;
    pc_geometry(rows, cols, col_blocks, rpc, chunks);
    dim3 grid((unsigned)col_blocks, (unsigned)chunks);
    if (dt == SASQ_F16) {
        if (codes) fakequant_fwd_pc_kernel<SASQ_F16, true><<<grid, kPcThreads, 0, st>>>(X, s, Y, codes, rows, cols, rpc, bits);
        else       fakequant_fwd_pc_kernel<SASQ_F16, false><<<grid, kPcThreads, 0, st>>>(X, s, Y, codes, rows, cols, rpc, bits);
    } else {
        if (codes) fakequant_fwd_pc_kernel<SASQ_BF16, true><<<grid, kPcThreads, 0, st>>>(X, s, Y, codes, rows, cols, rpc, bits);
        else       fakequant_fwd_pc_kernel<SASQ_BF16, false><<<grid, kPcThreads, 0, st>>>(X, s, Y, codes, rows, cols, rpc, bits);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

extern "C" size_t sasq_fakequant_bwd_pc_workspace(int64_t rows, int64_t cols)
{
    (void)rows;
    if (cols <= 0) return kWsHeaderBytes;
    return kWsHeaderBytes + sizeof(float) * (size_t)kPcMaxRowChunks * (size_t)cols;
}

extern "C" int sasq_fakequant_bwd_pc(const void* x, const void* dy, const float* s, void* dx, float* ds,
                                     int64_t rows, int64_t cols, int bits, sasq_dtype dt,
                                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !dy || !s || !ds) return SASQ_ERR_NULL;
    int rc = check_pc(rows, cols, bits, (int)dt);
    if (rc) return rc;
    if (!aligned16(x) || !aligned16(dy) || (dx && !aligned16(dx))) return SASQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    auto X = static_cast<const uint16_t*>(x);
    auto G = static_cast<const uint16_t*>(dy);
    auto DX = static_cast<uint16_t*>(dx);
    if (cols % 8 != 0) {
        const int blocks = (int)((cols + 255) / 256);
        if (dt == SASQ_F16) fakequant_pc_scalar_kernel<SASQ_F16><<<blocks, 256, 0, st>>>(X, G, s, nullptr, nullptr, DX, ds, rows, cols, bits, 1);
        else                fakequant_pc_scalar_kernel<SASQ_BF16><<<blocks, 256, 0, st>>>(X, G, s, nullptr, nullptr, DX, ds, rows, cols, bits, 1);
        return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
    }
    if (!workspace || workspace_bytes < sasq_fakequant_bwd_pc_workspace(rows, cols)) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;
    int64_t col_blocks, rpc;
    int chunks;
    pc_geometry(rows, cols, col_blocks, rpc, chunks);
    dim3 grid((unsigned)col_blocks, (unsigned)chunks);
    auto tickets = static_cast<uint32_t*>(workspace);
    auto parts = reinterpret_cast<float*>(static_cast<char*>(workspace) + kWsHeaderBytes);
    if (dt == SASQ_F16) {
        if (dx) fakequant_bwd_pc_kernel<SASQ_F16, true><<<grid, kPcThreads, 0, st>>>(X, G, s, DX, ds, tickets, parts, rows, cols, rpc, bits);
        else    fakequant_bwd_pc_kernel<SASQ_F16, false><<<grid, kPcThreads, 0, st>>>(X, G, s, DX, ds, tickets, parts, rows, cols, rpc, bits);
    } else {
        if (dx) fakequant_bwd_pc_kernel<SASQ_BF16, true><<<grid, kPcThreads, 0, st>>>(X, G, s, DX, ds, tickets, parts, rows, cols, rpc, bits);
        else    fakequant_bwd_pc_kernel<SASQ_BF16, false><<<grid, kPcThreads, 0, st>>>(X, G, s, DX, ds, tickets, parts, rows, cols, rpc, bits);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

// ---- batched entry points ----------------------------------------------------------------------
namespace sasq {

constexpr size_t kPcBatchLaunchBytes = (size_t)192 << 20;   // bytes of x per launch: more concurrent streams run slower

static int check_pc_items(const sasq_fq_item* items, int count, int bits, sasq_dtype dt, bool backward)
{
    if (!items) return SASQ_ERR_NULL;
    if (count < 1 || count > SASQ_MAX_BATCH) return SASQ_ERR_SHAPE;
    for (int i = 0; i < count; ++i) {
        const sasq_fq_item& it = items[i];
        if (!it.x || !it.s || (backward ? (!it.dy || !it.ds) : !it.out)) return SASQ_ERR_NULL;
        int rc = check_pc(it.rows, it.cols, bits, (int)dt);
        if (rc) return rc;
        if (it.cols % 8) return SASQ_ERR_SHAPE;              // such tensors take the single-tensor call
        if (!aligned16(it.x) || (it.out && !aligned16(it.out)) || (backward && !aligned16(it.dy))) return SASQ_ERR_ALIGN;
    }
    return SASQ_OK;
}

// Workspace of a batch: the 1 KB header holds the tickets of all items back to back (one word per
// column block; sasq_workspace_init clears exactly that header), each item's partials follow.
struct PcBatchLayout {
    size_t ticket_word[SASQ_MAX_BATCH];
    size_t partials_off[SASQ_MAX_BATCH];
    size_t total;
    bool fits;
};

static PcBatchLayout pc_batch_layout(const sasq_fq_item* items, int count)
{
    PcBatchLayout L;
    size_t words = 0, off = kWsHeaderBytes;
    for (int i = 0; i < count; ++i) {
        L.ticket_word[i] = words;
        L.partials_off[i] = off;
        const int64_t cols = items[i].cols > 0 ? items[i].cols : 0;
        words += (size_t)((cols + kPcColsPerBlock - 1) / kPcColsPerBlock);
        off += sizeof(float) * (size_t)kPcMaxRowChunks * (size_t)cols;
    }
    L.total = off;
    L.fits = words <= kWsHeaderBytes / 4;
    return L;
}

// Launches items [i0, i1) as one grid.
template <bool BACKWARD>
static int launch_pc_batch(const sasq_fq_item* items, int i0, int i1, int bits, sasq_dtype dt, char* ws,
                           const PcBatchLayout* L, hipStream_t st)
{
    PcBatch b;
    memset(&b, 0, sizeof(b));
    int64_t blocks = 0;
    for (int i = i0; i < i1; ++i) {
        const sasq_fq_item& src = items[i];
        PcItem& it = b.it[i - i0];
        int64_t col_blocks;
        pc_geometry(src.rows, src.cols, col_blocks, it.rpc, it.chunks);
        it.col_blocks = (int)col_blocks;
        it.x = static_cast<const uint16_t*>(src.x);
        it.dy = static_cast<const uint16_t*>(src.dy);
        it.s = src.s;
        it.out = static_cast<uint16_t*>(src.out);
        it.ds = src.ds;
        it.rows = src.rows;
        it.cols = src.cols;
        if (BACKWARD) {
            it.tickets = reinterpret_cast<uint32_t*>(ws) + L->ticket_word[i];
            it.partials = reinterpret_cast<float*>(ws + L->partials_off[i]);
        }
        b.first_block[i - i0] = (int)blocks;
        blocks += col_blocks * it.chunks;
        if (blocks > 0x7FFFFFFF) return SASQ_ERR_SHAPE;
    }
    b.count = i1 - i0;
    b.first_block[b.count] = (int)blocks;
    if (BACKWARD) {
        if (dt == SASQ_F16) fakequant_bwd_pc_batch_kernel<SASQ_F16><<<(int)blocks, kPcThreads, 0, st>>>(b, bits);
        else                fakequant_bwd_pc_batch_kernel<SASQ_BF16><<<(int)blocks, kPcThreads, 0, st>>>(b, bits);
    } else {
        if (dt == SASQ_F16) fakequant_fwd_pc_batch_kernel<SASQ_F16><<<(int)blocks, kPcThreads, 0, st>>>(b, bits);
        else                fakequant_fwd_pc_batch_kernel<SASQ_BF16><<<(int)blocks, kPcThreads, 0, st>>>(b, bits);
    }
    return hipGetLastError() == hipSuccess ? SASQ_OK : SASQ_ERR_LAUNCH;
}

template <bool BACKWARD>
static int run_pc_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt, char* ws, const PcBatchLayout* L,
                        hipStream_t st)
{
    // consecutive items share a launch while their input stays under the per-launch cap
    int i0 = 0;
    while (i0 < count) {
        size_t bytes = 0;
        int i1 = i0;
        while (i1 < count) {
            const size_t add = (size_t)items[i1].rows * (size_t)items[i1].cols * 2;      // bytes of x, as the per-tensor batch counts
            if (i1 > i0 && bytes + add > kPcBatchLaunchBytes) break;
            bytes += add;
            ++i1;
        }
        int rc = launch_pc_batch<BACKWARD>(items, i0, i1, bits, dt, ws, L, st);
        if (rc) return rc;
        i0 = i1;
    }
    return SASQ_OK;
}

}  // namespace sasq

extern "C" int sasq_fakequant_fwd_pc_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt, void* stream)
{
    int rc = check_pc_items(items, count, bits, dt, false);
    if (rc) return rc;
    return run_pc_batch<false>(items, count, bits, dt, nullptr, nullptr, as_stream(stream));
}

extern "C" size_t sasq_fakequant_bwd_pc_batch_workspace(const sasq_fq_item* items, int count)
{
    if (!items || count < 1 || count > SASQ_MAX_BATCH) return 0;
    const PcBatchLayout L = pc_batch_layout(items, count);
    return L.fits ? L.total : 0;
}

extern "C" int sasq_fakequant_bwd_pc_batch(const sasq_fq_item* items, int count, int bits, sasq_dtype dt,
                                           void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_pc_items(items, count, bits, dt, true);
    if (rc) return rc;
    const PcBatchLayout L = pc_batch_layout(items, count);
    if (!L.fits) return SASQ_ERR_SHAPE;                      // more than 256 column blocks in all
    if (!workspace || workspace_bytes < L.total) return SASQ_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SASQ_ERR_ALIGN;
    return run_pc_batch<true>(items, count, bits, dt, static_cast<char*>(workspace), &L, as_stream(stream));
}
