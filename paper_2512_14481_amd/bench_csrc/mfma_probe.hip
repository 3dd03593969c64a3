// Benchmark tooling, not part of the SASQ library or its C ABI (built into libsasq_bench.so, loaded
// by bench.py --mfma-peak only).
// Diagnostic: what the matrix units of this part sustain with nothing else going on.  A
// register-only loop of MFMAs in the GEMM kernels' register pattern (4 x 4 accumulator tiles of
// 32x32, one wave per SIMD, 256 workgroups): no LDS, no memory traffic inside the loop.  The
// benchmark times it (bench.py --mfma-peak) to put the GEMMs' figures next to the part's own
// ceiling, which depends on the operand bit patterns (the part is power-limited under MFMA load).
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace sasq_bench {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t probe_hash(uint32_t v)
{
    v *= 2654435761u; v ^= v >> 15; v *= 2246822519u; v ^= v >> 13;
    return v;
}

// KIND 0: zero operands; 1: random bits; 2: GEMM-like codes (activation bytes in {-1, 0, 0, 1},
// weight bytes uniform in [-32, 31]; the weight-like operand is the MFMA's first source, as in the
// library's GEMMs: the other way round the same loop sustains about 10 % less)
template <int KIND>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void mfma_probe_i8_kernel(int* sink, int iters)
{
    i32x16 acc[4][4];
    for (int u = 0; u < 4; ++u) for (int w = 0; w < 4; ++w) for (int v = 0; v < 16; ++v) acc[u][w][v] = 0;
    i32x4 a[4], b[4];
    for (int u = 0; u < 4; ++u)
        for (int j = 0; j < 4; ++j) {
            const uint32_t h = probe_hash(threadIdx.x * 16 + u * 4 + j), g = h * 40503u + 17u;
            uint32_t av = 0, bv = 0;
            if (KIND == 1) { av = h; bv = g; }
            if (KIND == 2)
                for (int e = 0; e < 4; ++e) {
                    const uint32_t s2 = (h >> (2 * e)) & 3u;
                    av |= (s2 == 0 ? 0xFFu : (s2 == 3 ? 1u : 0u)) << (8 * e);
                    bv |= ((((g >> (6 * e)) & 63u) - 32u) & 0xFFu) << (8 * e);
                }
            a[u][j] = (int)av;
            b[u][j] = (int)bv;
        }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                if (KIND == 2) acc[u][w] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[w], a[u], acc[u][w], 0, 0, 0);
                else           acc[u][w] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[u], b[w], acc[u][w], 0, 0, 0);
            }
    }
    int s = 0;
    for (int u = 0; u < 4; ++u) for (int w = 0; w < 4; ++w) for (int v = 0; v < 16; ++v) s += acc[u][w][v];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same 128x128 block per wave as 8 x 8 tiles of v_mfma_i32_16x16x64_i8, GEMM-like codes; the weight-like operand is
// the MFMA's first source as in the library's GEMM.
template <bool ZERO>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void mfma_probe_i8_k64_kernel(int* sink, int iters)
{
    i32x4 acc[8][8];
    for (int u = 0; u < 8; ++u) for (int w = 0; w < 8; ++w) for (int v = 0; v < 4; ++v) acc[u][w][v] = 0;
    i32x4 a[8], b[8];
    for (int u = 0; u < 8; ++u)
        for (int j = 0; j < 4; ++j) {
            const uint32_t h = probe_hash(threadIdx.x * 32 + u * 4 + j), g = h * 40503u + 17u;
            uint32_t av = 0, bv = 0;
            for (int e = 0; e < 4; ++e) {
                const uint32_t s2 = (h >> (2 * e)) & 3u;
                av |= (s2 == 0 ? 0xFFu : (s2 == 3 ? 1u : 0u)) << (8 * e);
                bv |= ((((g >> (6 * e)) & 63u) - 32u) & 0xFFu) << (8 * e);
            }
            a[u][j] = ZERO ? 0 : (int)av;                      // ZERO: the issue rate without data-dependent power
            b[u][j] = ZERO ? 0 : (int)bv;
        }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int w = 0; w < 8; ++w) acc[u][w] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b[w], a[u], acc[u][w], 0, 0, 0);
    }
    int s = 0;
    for (int u = 0; u < 8; ++u) for (int w = 0; w < 8; ++w) for (int v = 0; v < 4; ++v) s += acc[u][w][v];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void mfma_probe_f16_kernel(int* sink, int iters)
{
    f32x16 acc[4][4];
    for (int u = 0; u < 4; ++u) for (int w = 0; w < 4; ++w) for (int v = 0; v < 16; ++v) acc[u][w][v] = 0.0f;
    f16x8 a[4], b[4];
    for (int u = 0; u < 4; ++u)
        for (int j = 0; j < 8; ++j) {
            const uint32_t h = probe_hash(threadIdx.x * 32 + u * 8 + j);
            a[u][j] = (_Float16)(((int)(h & 1023u) - 512) * (1.0f / 20000.0f));
            b[u][j] = (_Float16)(((int)((h >> 10) & 1023u) - 512) * (1.0f / 20000.0f));
        }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int w = 0; w < 4; ++w) acc[u][w] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[u], b[w], acc[u][w], 0, 0, 0);
    }
    float s = 0.0f;
    for (int u = 0; u < 4; ++u) for (int w = 0; w < 4; ++w) for (int v = 0; v < 16; ++v) s += acc[u][w][v];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = (int)s;
}

}  // namespace sasq_bench

using namespace sasq_bench;

// kind 0: v_mfma_i32_32x32x32_i8 on zero operands, 1: on random bits, 2: on GEMM-like codes (activation bytes in
// {-1, 0, 0, 1}, weight bytes in [-32, 31]); 3: v_mfma_f32_32x32x16_f16 on small random values; 4: v_mfma_i32_16x16x64_i8
// on the codes of kind 2, 5: the same on zero operands.  256 workgroups of 4 waves, `iters` x 16 MFMAs of 32x32 (64 of 16x16) per wave; sink: 65536 ints.
// Returns 0, or 1 for a bad argument, 2 for a launch error.
extern "C" int sasq_bench_mfma_probe(int kind, int iters, int* sink, void* stream)
{
    if (!sink) return 1;
    if (iters < 1 || iters > (1 << 22)) return 1;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    switch (kind) {
        case 0: mfma_probe_i8_kernel<0><<<256, 256, 0, st>>>(sink, iters); break;
        case 1: mfma_probe_i8_kernel<1><<<256, 256, 0, st>>>(sink, iters); break;
        case 2: mfma_probe_i8_kernel<2><<<256, 256, 0, st>>>(sink, iters); break;
        case 3: mfma_probe_f16_kernel<<<256, 256, 0, st>>>(sink, iters); break;
        case 4: mfma_probe_i8_k64_kernel<false><<<256, 256, 0, st>>>(sink, iters); break;
        case 5: mfma_probe_i8_k64_kernel<true><<<256, 256, 0, st>>>(sink, iters); break;
        default: return 1;
    }
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
