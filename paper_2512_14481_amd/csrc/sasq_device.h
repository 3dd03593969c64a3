// Device-side building blocks shared by the HIP kernels of the SASQ library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sasq.h"

namespace sasq {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// 1.5 * 2^23.  For |p| < 2^22, fma(x, inv_s, kMagic) is the exact product x*inv_s rounded ONCE
// (hardware round-to-nearest-even) to the integer grid, offset by kMagic; in [2^23, 2^24) the
// fp32 bit pattern is linear in the value, so the low bits carry the signed integer.
constexpr float kMagic = 12582912.0f;
constexpr int32_t kMagicBits = 0x4B400000;

// Quantizer constants for one call: Sec. 3, Eq. 1 with S = s and N = bits.
struct QConst {
    float inv_s;   // fl32(1/s), one IEEE division
    float s;
    float lo;      // kMagic + Qn
    float hi;      // kMagic + Qp
};

__device__ __forceinline__ QConst make_qconst(float s, int bits)
{
    QConst q;
    q.s = s;
    q.inv_s = 1.0f / s;                       // correctly rounded (no fast-math)
    q.lo = kMagic - (float)(1 << (bits - 1));
    q.hi = kMagic + (float)((1 << (bits - 1)) - 1);
    return q;
}

// One quantized element in the "magic" domain.
//   f  = round(x*inv_s) + kMagic  (single rounding; saturating garbage far out of range)
//   c  = clamp(f) = q + kMagic
struct QElem {
    float f;
    float c;
};

__device__ __forceinline__ QElem quantize(float x, const QConst& k)
{
    QElem e;
    e.f = __builtin_fmaf(x, k.inv_s, kMagic);
    e.c = __builtin_amdgcn_fmed3f(e.f, k.lo, k.hi);
    return e;
}

__device__ __forceinline__ int code_of(const QElem& e) { return __float_as_int(e.c) - kMagicBits; }
__device__ __forceinline__ float codef_of(const QElem& e) { return e.c - kMagic; }   // exact
__device__ __forceinline__ bool unclipped(const QElem& e) { return e.f == e.c; }

// ---- 16-bit storage types -------------------------------------------------------------------
template <int DT> struct Store16;

// An fp32 value whose rounding to fp32 is part of the numerical contract, made opaque to the
// compiler before it is narrowed to 16 bits.  Without this, clang folds "multiply, then convert
// to half" into v_fma_mixlo_f16, which rounds the exact product once; the contract (and the plain
// two-step code) rounds to fp32 first, and the two differ when the fp32 product lands on a
// half-precision tie.
// (The paired conversion in pack() compiles to v_cvt_pk_f16_f32, which has no fused form.)
__device__ __forceinline__ float rounded_f32(float f)
{
    asm("" : "+v"(f));
    return f;
}

template <> struct Store16<SASQ_F16> {
    static __device__ __forceinline__ float lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFFu)); }
    static __device__ __forceinline__ float hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
    static __device__ __forceinline__ float one(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
    static __device__ __forceinline__ uint16_t enc(float f) { return __builtin_bit_cast(uint16_t, (_Float16)rounded_f32(f)); }
    static __device__ __forceinline__ uint32_t pack(float a, float b)
    {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        h2 v = {(_Float16)a, (_Float16)b};
        return __builtin_bit_cast(uint32_t, v);
    }
};

template <> struct Store16<SASQ_BF16> {
    static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
    static __device__ __forceinline__ float one(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
    static __device__ __forceinline__ uint16_t enc(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
    static __device__ __forceinline__ uint32_t pack(float a, float b)
    {
        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
        b2 v = {(__bf16)a, (__bf16)b};
        return __builtin_bit_cast(uint32_t, v);
    }
};

// Pack the low bytes of four "magic domain" floats (their int8 codes) into one dword.
__device__ __forceinline__ uint32_t pack_codes4(float c0, float c1, float c2, float c3)
{
    uint32_t a = __builtin_amdgcn_perm(__float_as_uint(c1), __float_as_uint(c0), 0x0c0c0400u);  // [c0.b0, c1.b0, 0, 0]
    uint32_t b = __builtin_amdgcn_perm(__float_as_uint(c3), __float_as_uint(c2), 0x04000c0cu);  // [0, 0, c2.b0, c3.b0]
    return a | b;
}

// ---- reductions -----------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ uint32_t wave_max(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}

// ---- publishing a block's partial result to the block that finishes a grid-wide reduction ----
// Protocol: every block stores its partial with an agent-scope atomic store, waits until that
// store is acknowledged, then takes a ticket with an agent-scope atomic add; the block that draws
// the last ticket issues an agent-scope acquire fence and reads all partials with agent-scope
// atomic loads.
// Why this is ordered on gfx950 (8 XCDs, one L2 each, coherent with each other only at the memory
// side): an agent-scope atomic store is a store with the sc1 bit, which is written through this
// XCD's L2 to the level all XCDs share, and the wave's vmcnt entry for it is released only when
// that write has been performed there; so after s_waitcnt vmcnt(0) the partial is visible to every
// XCD before the ticket is even requested.  This is the compiler's own agent-scope release sequence
// (write back L2, then s_waitcnt vmcnt(0)) without the L2 write-back: the write-back exists to push
// out earlier plain stores that may sit dirty in L2, and here nothing but the sc1 store itself has
// to be published (a full release fence costs a write-back of the XCD's L2 per block: measured
// 117 us against 35 us for a 16.8 M element backward).  On the reading side the fence invalidates
// this XCD's non-coherent L2 lines and the sc1 loads are served from the shared level.
__device__ __forceinline__ void wait_stores_acknowledged() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <typename T>
__device__ __forceinline__ uint32_t publish_then_ticket(T* slot, T value, uint32_t* ticket_word)
{
    __hip_atomic_store(slot, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    wait_stores_acknowledged();
    return __hip_atomic_fetch_add(ticket_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Workspace header used by the grid-wide reductions: arrival tickets (word 0 for the scalar
// reductions, words 0..255 one per column chunk for the per-channel backward).
constexpr size_t kWsHeaderBytes = 1024;
constexpr size_t kWsMinBytes = 256;
constexpr uint32_t kTicketBase = 0;

// Kernel-variant overrides set through sasq_set_tuning (a test and tuning aid; 0 = choose by shape).
extern int g_tuning[SASQ_TUNE_COUNT];
inline int tuning(int knob) { return g_tuning[knob]; }

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace sasq
