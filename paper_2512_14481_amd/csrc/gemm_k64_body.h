// The tile body shared by the GEMM kernels on the 16-row MFMA shapes (v_mfma_i32_16x16x64_i8 for the static linear,
// v_mfma_f32_16x16x32_{f16,bf16} for the backward of the frozen linear): K pipeline, fragment reads, epilogue.
// Included by static_linear_k64.hip and linear_bwd.hip; the description of the machine shape is at the top of the former.
#pragma once

#include "sasq_device.h"
#include "gemm_tile.h"
#include <type_traits>

namespace sasq {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int DT> struct Mfma16x16;
template <> struct Mfma16x16<SASQ_F16> {
    static __device__ __forceinline__ f32x4 mma(const i32x4& a, const i32x4& b, const f32x4& c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mfma16x16<SASQ_BF16> {
    static __device__ __forceinline__ f32x4 mma(const i32x4& a, const i32x4& b, const f32x4& c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};

// Weight paths (values shared with static_linear.hip): int8 row-major, int8 pre-arranged in 1 KB blocks, int4
// pre-arranged (it stays packed through L2 -> LDS and is unpacked between the fragment read and the MFMA: a nibble
// moved to the high half of a byte is the int8 value 16 w, so two mask/shift operations per dword turn 8 nibbles into
// 8 bytes; the accumulators are then exactly 16 acc and are shifted back in the epilogue).
enum { KW_I8 = 0, KW_I8B = 2, KW_I4B = 3 };

constexpr int kFacBytes = 1024;      // per wave: the epilogue's per-column factors (BN/2 floats, loaded twice over)
template <int BM, int BN> constexpr int lds_bytes_k64() { return Tile<BM, BN>::kLds + 4 * kFacBytes; }

// One direct 128-bit-per-lane load from global memory into LDS: lane i deposits its 16 bytes at
// LDS address lds_addr + 16 i.  The memory address is a scalar base plus a 32-bit per-lane offset,
// so that the instruction needs no vector address arithmetic.  The compiler does not see the LDS
// write: the callers order it against their LDS reads with s_waitcnt vmcnt and barriers.
__device__ __forceinline__ void lds_load16(uint32_t lds_addr, const void* base, uint32_t lane_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}
// The same with the LDS address given as a sum of two scalars (a slot's fixed address + the stage's offset): the
// addition writes M0 itself, one scalar instruction less in front of every load of the K loop.
__device__ __forceinline__ void lds_load16(uint32_t lds_a, uint32_t lds_b, const void* base, uint32_t lane_off)
{
    asm volatile("s_add_i32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
                 :: "s"(lds_a), "s"(lds_b), "v"(lane_off), "s"(base) : "memory", "scc");
}

// Measurement hook: a translation unit that wants cycle and wall-clock stamps at five points of every tile (body start,
// pipeline filled, K loop done, stages drained, epilogue done) defines SASQ_TILE_TS(k) before including this file (the
// benchmark's instrumented build of static_linear_k64.hip does); everywhere else it expands to nothing.
#ifndef SASQ_TILE_TS
#define SASQ_TILE_TS(k)
#endif

// GROUPED (Sec. 3, Eq. 3): one activation factor per group of `group_tiles` K tiles; s_ptr then
// points at the factors.  The int32 accumulators cover one group at a time (a group's first K tile
// multiplies into a zero accumulator operand) and are folded into fp32 sums at its end,
// f = fma(fl32(acc), s_g, f) in ascending group order; the epilogue applies s_w and the bias to f,
// and acc_out receives f (as float bits).  Tiles of 128 rows only (f doubles the accumulator registers);
// with 128x128 tiles two waves share a SIMD and one wave's fold runs under the other's MFMAs.
// GROUPED = 2: groups of 32 channels, two per K tile.  One MFMA contracts the whole 64-byte stage, so every K tile
// is multiplied twice, once with the activation fragments of channels 32..63 zeroed and once with those of 0..31
// zeroed (lanes 32..63 resp. 0..31 of a fragment), each pass into zero accumulators and folded with its own factor:
// twice the matrix work and a fold per 32 channels, an order of magnitude faster than the scalar kernel all the same.
// OP 1: the same machine on v_mfma_f32_16x16x32_{f16,bf16} (DT picks the type): both operands hold 16-bit floats, 32
// per 64-byte stage row; the "activation" operand xq is then read ROW-MAJOR (rows of K bytes, the 16-byte chunks of a
// row gathered per lane as for row-major weights), the weight operand from 1 KB blocks; K is the contraction length in
// BYTES; the accumulators are fp32, written out rounded to 16 bits without any factor (s_ptr, s_w, bias unused), and
// acc_out receives the fp32 sums.  This is the backward GEMM of the frozen linear (linear_bwd.hip).
template <int DT, int WMODE, int BM, int BN, bool ROWS, int GROUPED = 0, int OP = 0>
__device__ __forceinline__
void gemm_k64_body(const int8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
                   const float* __restrict__ s_ptr, const float* __restrict__ s_w,
                   const float* __restrict__ bias, uint16_t* __restrict__ y,
                   int32_t* __restrict__ acc_out, int M, int N, int K,
                   int tm, int tn, char* lds, int group_tiles = 0)
{
    static_assert(!GROUPED || (BM == 128 && !ROWS), "grouped factors: 128-row tiles");
    static_assert(OP == 0 || (WMODE == KW_I8B && !ROWS && !GROUPED), "float contraction: pre-arranged weight blocks, no factors");
    constexpr bool FLT = OP != 0;
    using AccT = std::conditional_t<FLT, f32x4, i32x4>;
    using S = Store16<DT>;
    using T = Tile<BM, BN>;
    constexpr int MF = BM / 32, NF = BN / 32;          // 16x16 tiles per wave along m, n
    constexpr int XS = T::XS, WS = T::WS;              // 1 KB slabs per wave per stage
    constexpr bool I4 = WMODE == KW_I4B;
    constexpr int WSL = I4 ? WS / 2 : WS;              // weight loads per wave per K tile (packed int4: half the bytes)
    constexpr int kLoads = XS + WSL;                   // direct loads per wave per K tile
    constexpr int kAccShift = I4 ? 4 : 0;
    auto stage_ptr = [&](int st, int operand) -> char* { return &lds[st * T::kStageBytes + operand * T::kXBytes]; };

    const int m0 = tm * BM, n0 = tn * BN;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // uniform: LDS addresses of the loads stay scalar
    const int wm = wave & 1, wn = wave >> 1;
    const int KT = K / kBK;

    // ---- direct L2 -> LDS loads: load j of wave w fills rows (4j + w)*16 .. +16 of a stage ----
    // Address of a load = scalar base of the operand panel at the K tile (advanced once per K tile)
    // + a per-lane 32-bit offset fixed for the whole tile: the load itself then costs the wave two
    // scalar instructions and the load (anything more does not fit behind a 16-cycle MFMA).
    const int lrow = lane >> 2;
    const int lchunk = (lane & 3) ^ (((lane >> 3) & 3) ^ ((lane >> 5) & 1));
    const int last_rb = (M - 1) >> 4;
    const int8_t* xpanel = FLT ? xq + (int64_t)m0 * K : xq + (int64_t)(m0 >> 4) * KT * 1024;
    constexpr int kXTileStep = FLT ? kBK : 1024;
    const int8_t* wpanel = reinterpret_cast<const int8_t*>(wq) + (WMODE == KW_I8B ? (int64_t)(n0 >> 4) * KT * 1024
                                                                  : I4 ? (int64_t)(n0 >> 5) * KT * 1024 : (int64_t)n0 * K);
    uint32_t xoff[XS], woff[WSL];
#pragma unroll
    for (int j = 0; j < XS; ++j)
        xoff[j] = FLT ? (uint32_t)(min((4 * j + wave) * 16 + lrow, M - 1 - m0) * K + lchunk * 16)
                      : (uint32_t)(min(4 * j + wave, last_rb - (m0 >> 4)) * KT * 1024 + lane * 16);
#pragma unroll
    for (int j = 0; j < WSL; ++j) {
        if (I4) woff[j] = (uint32_t)(min(4 * j + wave, ((N - 1) >> 5) - (n0 >> 5)) * KT * 1024 + lane * 16);   // blocks of 32 rows
        else if (WMODE == KW_I8B) woff[j] = (uint32_t)(min(4 * j + wave, ((N - 1) >> 4) - (n0 >> 4)) * KT * 1024 + lane * 16);
        else                 woff[j] = (uint32_t)(min((4 * j + wave) * 16 + lrow, N - 1 - n0) * K + lchunk * 16);
    }
    constexpr int kWTileStep = (WMODE == KW_I8B || I4) ? 1024 : kBK;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_ptr_t)&lds[0] + (uint32_t)wave * 1024u;
    auto dma_at = [&](const int8_t* xtile, const int8_t* wtile, int j, int st) {   // loads 0..XS-1: activations, XS..: weights
        const uint32_t st_off = (uint32_t)st * T::kStageBytes;
        if (j < XS) lds_load16(lds_base + j * 4096, st_off, xtile, xoff[j]);
        else        lds_load16(lds_base + T::kXBytes + (j - XS) * 4096, st_off, wtile, woff[j - XS < WSL ? j - XS : 0]);
    };
    auto dma = [&](int Tk, int j, int st) {          // K tile Tk into stage st = Tk & 3
        dma_at(xpanel + (int64_t)Tk * kXTileStep, wpanel + (int64_t)Tk * kWTileStep, j, st);
    };
    // The steady loop keeps the operands' addresses at its current group of four K tiles here: a load of
    // tile i + 4 then adds a constant to them.
    const int8_t* xrun = xpanel;
    const int8_t* wrun = wpanel;

    // ---- LDS -> MFMA fragments: lane l reads chunk l/16 of row l%16 of a 16-row tile ----
    const int frow = lane & 15, fq = lane >> 4;
    const int foff = frow * kBK + ((fq ^ swz64(frow)) << 4);
    const int xbase = wm * (BM / 2) * kBK, wbase = wn * (BN / 2) * kBK;
    // Packed int4: a 1 KB block holds 32 rows x 64 k; the 16 codes k = 16 G .. + 15 of row r are the 8 bytes at
    // 256 G + 8 r (G = 2 kk + g in the layout's own terms), so lane l fetches 8 bytes at 256 (l/16) + 8 (16 h + l%16),
    // h = the 16-row half of the block its tile is.
    using WFrag = std::conditional_t<I4, u32x2, i32x4>;
    i32x4 fx[2][MF];
    WFrag fw[2][NF];
    auto read_frag = [&](int set, int st, int idx) {   // the MF activation fragments first, then the NF weight ones
        if (idx < MF) {
            fx[set][idx] = *reinterpret_cast<const i32x4*>(stage_ptr(st, 0) + xbase + idx * 16 * kBK + foff);
        } else if constexpr (I4) {
            const int g = idx - MF;
            fw[set][g] = *reinterpret_cast<const u32x2*>(stage_ptr(st, 1) + (wn * (BN / 64) + (g >> 1)) * 1024 + 256 * fq + 8 * (16 * (g & 1) + frow));
        } else {
            fw[set][idx - MF] = *reinterpret_cast<const i32x4*>(stage_ptr(st, 1) + wbase + (idx - MF) * 16 * kBK + foff);
        }
    };
    auto wfrag_piece = [&](const WFrag& f, int j) -> int {   // output dword j of the unpacked operand
        if constexpr (I4) {
            const uint32_t p = f[j >> 1];
            return (int)(((j & 1) ? p : (p << 4)) & 0xF0F0F0F0u);
        } else {
            return f[j];
        }
    };
    i32x4 wv_ahead = {0, 0, 0, 0}, wv_next = {0, 0, 0, 0};   // packed int4: the weight operand of the row to come
    auto wfrag = [&](const WFrag& f) -> i32x4 {         // the MFMA's weight operand: as read, or unpacked here
        if constexpr (I4) {
            const uint32_t p0 = f[0], p1 = f[1];
            return i32x4{(int)((p0 << 4) & 0xF0F0F0F0u), (int)(p0 & 0xF0F0F0F0u), (int)((p1 << 4) & 0xF0F0F0F0u), (int)(p1 & 0xF0F0F0F0u)};
        } else {
            return f;
        }
    };

    AccT acc[NF][MF];
    f32x4 fsum[GROUPED ? NF : 1][GROUPED ? MF : 1];           // fp32 sums over groups
#pragma unroll
    for (int g = 0; g < (GROUPED ? NF : 1); ++g)
#pragma unroll
        for (int b = 0; b < (GROUPED ? MF : 1); ++b) fsum[g][b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // ---- K pipeline ----
    // Iteration i multiplies K tile i from fragment set i&1 while it reads the fragments of tile
    // i+1 into the other set and issues the loads of tile i+4 into the stage tile i has just left.
    // At its top: this wave's fragment reads of tile i are complete and its own loads of tile i+1
    // have landed (loads return in issue order, so that is one s_waitcnt vmcnt with the loads of
    // the later tiles still allowed in flight); after the barrier the same holds for every wave,
    // so tile i+1 may be read and stage i&3 refilled.
    // Side work is dealt out behind the MFMAs (one wave per SIMD: nothing else hides a clump of
    // issue): the fragment reads first, every `kFragStep` MFMAs, then the loads.
    // The last four or five iterations (TAIL) request a tile only if there is one left and wait for
    // what is still due.
    constexpr int NM = MF * NF, NFR = MF + NF;
    constexpr int kFragStep = NM / 2 / NFR >= 1 ? NM / 2 / NFR : 1;
    constexpr int kLoadStep = (NM - kFragStep * NFR) / kLoads;
    static_assert(kLoadStep >= 1, "side work does not fit behind the MFMAs");
    auto fold = [&](int group_idx) {                           // f = fma(fl32(acc), s_g, f) for every accumulator
        const float sg = s_ptr[GROUPED ? group_idx : 0];
#pragma unroll
        for (int g = 0; g < NF; ++g)
#pragma unroll
            for (int b = 0; b < MF; ++b)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    fsum[GROUPED ? g : 0][GROUPED ? b : 0][e] =
                        __builtin_fmaf((float)((int)acc[g][b][e] >> kAccShift), sg, fsum[GROUPED ? g : 0][GROUPED ? b : 0][e]);
    };
    auto iteration = [&](int i, auto cur_tag, auto stage_tag, auto first_tag, auto tail_tag) {
        constexpr int CUR = decltype(cur_tag)::value;
        constexpr int STG = decltype(stage_tag)::value;        // i & 3 where the copy of the body knows it, else -1
        constexpr bool FIRST = decltype(first_tag)::value;
        constexpr bool TAIL = decltype(tail_tag)::value;
        if (!TAIL) {
            __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(2 * kLoads));
        } else {
            const int later = min(i + 3, KT - 1) - (i + 1);    // tiles after i+1 already requested
            if (later >= 2)      __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(2 * kLoads));
            else if (later == 1) __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(kLoads));
            else                 __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(0));
        }
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        const int stn = STG >= 0 ? (STG + 1) & 3 : (i + 1) & 3;
        const bool more = !TAIL || i + 1 < KT;                 // a next tile to read fragments of
        i32x4 xhalf[GROUPED == 2 ? MF : 1];                    // GROUPED 2: the fragments with one half of the channels zeroed
        if constexpr (GROUPED == 2) {
#pragma unroll
            for (int b = 0; b < MF; ++b) xhalf[b] = fq < 2 ? fx[CUR][b] : i32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            // Packed int4: the operand of this row was unpacked while the previous row multiplied (wv_ahead), and the next
            // row's -- at the end of the tile, row 0 of the next tile -- is unpacked one output dword behind each of this
            // row's first four MFMAs: done at the top of a row, the six VALU operations and their latency stand in front of
            // the row's first MFMA (195 of 1405 cycles per K tile on the 13B layer).
            const i32x4 wv = I4 ? wv_ahead : wfrag(fw[CUR][g]);
            const bool ahead_in_tile = g + 1 < NF;
            const WFrag& fnext = ahead_in_tile ? fw[CUR][g + 1 < NF ? g + 1 : 0] : fw[1 - CUR][0];
#pragma unroll
            for (int b = 0; b < MF; ++b) {
                // K tile 0 multiplies into a zero accumulator operand instead of clearing the accumulators
                if constexpr (FLT) {
                    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
                    acc[g][b] = Mfma16x16<DT>::mma(wv, fx[CUR][b], FIRST ? zero : acc[g][b]);
                } else {
                    const i32x4 zero = {0, 0, 0, 0};
                    acc[g][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wv, GROUPED == 2 ? xhalf[GROUPED == 2 ? b : 0] : fx[CUR][b],
                                                                      FIRST ? zero : acc[g][b], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                const int t = g * MF + b;
                if (t < kFragStep * NFR) {
                    if (t % kFragStep == 0 && more) read_frag(1 - CUR, stn, t / kFragStep);
                } else if (!TAIL || i + 4 < KT) {
                    const int u = t - kFragStep * NFR;
                    if (u % kLoadStep == 0 && u / kLoadStep < kLoads) {
                        if constexpr (STG >= 0) dma_at(xrun + (STG + 4) * kXTileStep, wrun + (STG + 4) * kWTileStep, u / kLoadStep, STG);
                        else                    dma(i + 4, u / kLoadStep, i & 3);
                    }
                }
                if constexpr (I4) {
                    if (b < 4 && (ahead_in_tile || more)) wv_next[b] = wfrag_piece(fnext, b);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (I4) wv_ahead = wv_next;
        }
        if constexpr (GROUPED == 2) {
            // channels 0..31 of this K tile are in acc: fold them, then the same tile with channels 32..63
            fold(2 * i);
#pragma unroll
            for (int b = 0; b < MF; ++b) xhalf[b] = fq < 2 ? i32x4{0, 0, 0, 0} : fx[CUR][b];
#pragma unroll
            for (int g = 0; g < NF; ++g) {
                const i32x4 wv = wfrag(fw[CUR][g]);
#pragma unroll
                for (int b = 0; b < MF; ++b)
                    acc[g][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wv, xhalf[GROUPED == 2 ? b : 0], i32x4{0, 0, 0, 0}, 0, 0, 0);
            }
            fold(2 * i + 1);
        }
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    using S3 = std::integral_constant<int, 3>;
    using SR = std::integral_constant<int, -1>;               // stage known only at run time
    using Yes = std::true_type;
    using No = std::false_type;
    // one K tile; with grouped factors also the group bookkeeping (all of it uniform)
    int in_group = 0, group_idx = 0;
    auto step = [&](int i, auto cur_tag, auto stage_tag, auto first_tag, auto tail_tag) {
        if constexpr (!GROUPED) {
            iteration(i, cur_tag, stage_tag, first_tag, tail_tag);
        } else if constexpr (GROUPED == 2) {
            iteration(i, cur_tag, stage_tag, Yes{}, tail_tag);     // both folds of the tile happen inside
        } else {
            if (in_group == 0) iteration(i, cur_tag, stage_tag, Yes{}, tail_tag);
            else               iteration(i, cur_tag, stage_tag, No{}, tail_tag);
            if (++in_group == group_tiles) {
                fold(group_idx);
                in_group = 0;
                ++group_idx;
            }
        }
    };
    SASQ_TILE_TS(0);
    // fill: the first four tiles requested, tile 0 landed for everyone, its fragments read
    const int nfill = min(KT, 4);
    for (int t = 0; t < nfill; ++t)
#pragma unroll
        for (int j = 0; j < kLoads; ++j) dma(t, j, t);
    if (nfill == 4)      __builtin_amdgcn_s_waitcnt(waitcnt_vm(3 * kLoads));
    else if (nfill == 3) __builtin_amdgcn_s_waitcnt(waitcnt_vm(2 * kLoads));
    else if (nfill == 2) __builtin_amdgcn_s_waitcnt(waitcnt_vm(kLoads));
    else                 __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int k = 0; k < NFR; ++k) read_frag(0, 0, k);
    if constexpr (I4) wv_ahead = wfrag(fw[0][0]);
    SASQ_TILE_TS(1);
    // A multiple of four steady iterations (they always have a tile i+4 to request), then the tail.
    // The steady loop is written out four iterations at a time: every copy of the body then knows
    // its fragment set and its LDS stages at compile time, and the addresses of its fragment reads
    // and loads are constants instead of a chain of scalar arithmetic in front of the first read.
    // (Whole-tile groups keep two iterations with run-time stages: their body exists once per accumulator
    // mode already, and four copies of each push the register allocator into scratch memory.)
    constexpr bool kBy4 = GROUPED != 1;
    const int steady = !kBy4 ? (KT >= 6 ? ((KT - 4) & ~1) : 0) : KT >= 8 ? ((KT - 4) & ~3) : 0;
    if constexpr (!kBy4) {
        if (steady > 0) {
            step(0, C0{}, SR{}, Yes{}, No{});
            step(1, C1{}, SR{}, No{}, No{});
#pragma unroll 1
            for (int it = 2; it < steady; it += 2) {
                step(it, C0{}, SR{}, No{}, No{});
                step(it + 1, C1{}, SR{}, No{}, No{});
            }
        }
    } else if (steady > 0) {
        step(0, C0{}, S0{}, Yes{}, No{});
        step(1, C1{}, S1{}, No{}, No{});
        step(2, C0{}, S2{}, No{}, No{});
        step(3, C1{}, S3{}, No{}, No{});
#pragma unroll 1
        for (int it = 4; it < steady; it += 4) {
            xrun += 4 * kXTileStep;
            wrun += 4 * kWTileStep;
            step(it, C0{}, S0{}, No{}, No{});
            step(it + 1, C1{}, S1{}, No{}, No{});
            step(it + 2, C0{}, S2{}, No{}, No{});
            step(it + 3, C1{}, S3{}, No{}, No{});
        }
    } else if (!GROUPED) {
#pragma unroll
        for (int g = 0; g < NF; ++g)
#pragma unroll
            for (int b = 0; b < MF; ++b) acc[g][b] = AccT{0, 0, 0, 0};
    }
    // The per-column factors of the epilogue are requested here, a few K tiles before they are
    // needed (fetched inside the epilogue they cost eight memory latencies in a row): one direct
    // load per wave parks the BN/2 factors of its block in LDS, behind the stages.  (An extra load
    // in the in-order queue only makes the counted waits of the tail wait for more, never less.)
    const int wn0 = n0 + wn * (BN / 2), wm0 = m0 + wm * (BM / 2);
    const bool cols_inside = !FLT && wn0 + BN / 2 <= N && (reinterpret_cast<uintptr_t>(s_w) & 15u) == 0 &&
                             (bias == nullptr || (reinterpret_cast<uintptr_t>(bias) & 15u) == 0);
    char* fac = &lds[T::kLds + wave * kFacBytes];
    if (cols_inside)
        lds_load16(lds_base - (uint32_t)wave * 1024u + T::kLds + (uint32_t)wave * kFacBytes, s_w + wn0,
                   (uint32_t)(lane & (BN / 8 - 1)) * 16u);   // lanes past BN/8 fetch the same factors again: no lane reads past the block
    if constexpr (kBy4) {
#pragma unroll 1
        for (int i = steady; i < KT; i += 2) {                  // KT - steady is 1 .. 7, steady is even
            step(i, C0{}, SR{}, No{}, Yes{});
            if (i + 1 < KT) step(i + 1, C1{}, SR{}, No{}, Yes{});
        }
    } else {
        step(steady, C0{}, SR{}, No{}, Yes{});                  // KT - steady is 1 .. 5
        if (steady + 1 < KT) {
            step(steady + 1, C1{}, SR{}, No{}, Yes{});
            if (steady + 2 < KT) {
                step(steady + 2, C0{}, SR{}, No{}, Yes{});
                if (steady + 3 < KT) {
                    step(steady + 3, C1{}, SR{}, No{}, Yes{});
                    if (steady + 4 < KT) step(steady + 4, C0{}, SR{}, No{}, Yes{});
                }
            }
        }
    }
    SASQ_TILE_TS(2);
    // the last fragment reads (none pending) and loads (none in flight) are complete; LDS is reused
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0 & waitcnt_vm(0));
    SASQ_TILE_TS(3);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ---- epilogue: Y = fl32(fl32(acc) * fl32(s * s_w[n])) (+ bias), staged through LDS in [m][n]
    // order as 16-bit values, written with 128-bit stores, BN contiguous bytes per row ----
    const float s = (ROWS || GROUPED || FLT) ? 1.0f : *s_ptr;
    const bool has_bias = !FLT && bias != nullptr;
    char* epi = &lds[wave * T::kEpiBytes];
    float srow[MF];                                            // ROWS: the factor of each row this lane holds
#pragma unroll
    for (int b = 0; b < MF; ++b) srow[b] = ROWS ? s_ptr[min(wm0 + b * 16 + frow, M - 1)] : 1.0f;
    // Common case (block inside the matrix): the block goes out in chunks of 16 rows through a small
    // staging buffer, software-pipelined: while chunk b is dequantized, the LDS reads of chunk b-1 are
    // in flight; then chunk b-1 is stored, chunk b written to the buffer and read back.  LDS serves a
    // wave's requests in order, so one buffer is enough.  (Staging the whole block first and storing
    // it afterwards left the wave waiting for LDS and for the store queue in turn: 11 k cycles per
    // 256x256 tile against 5 k.)
    const bool vec_ok = (N & 7) == 0;
    constexpr int kChunksPerRow = BN / 16;                      // 16-byte chunks in a wave-block row
    constexpr int kRowsPerPass = 64 / kChunksPerRow;
    const int crow = lane / kChunksPerRow, cchunk = lane % kChunksPerRow;
    auto write_tile_chunked = [&](auto bias_tag) {
        constexpr bool BIAS = decltype(bias_tag)::value;
        constexpr int kPasses = 16 / kRowsPerPass;             // read-back passes per 16-row chunk
        float cs[NF][4], bs[NF][4];
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            const int nl = g * 16 + 4 * fq;
            f32x4 sv = {1.0f, 1.0f, 1.0f, 1.0f}, bv = {0.0f, 0.0f, 0.0f, 0.0f};
            if (FLT) {
            } else if (cols_inside) {
                sv = *reinterpret_cast<const f32x4*>(fac + nl * 4);
                if (BIAS) bv = *reinterpret_cast<const f32x4*>(bias + wn0 + nl);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) { sv[e] = s_w[wn0 + nl + e]; if (BIAS) bv[e] = bias[wn0 + nl + e]; }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) { cs[g][e] = (ROWS || GROUPED) ? sv[e] : s * sv[e]; bs[g][e] = bv[e]; }
        }
        char* wr = epi + frow * T::kEpiStride + 4 * fq * 2;
        const char* rd = epi + crow * T::kEpiStride + cchunk * 16;
        char* dst = reinterpret_cast<char*>(y + (int64_t)(wm0 + crow) * N + wn0 + cchunk * 8);
        const int64_t row_step = (int64_t)kRowsPerPass * N * 2, chunk_step = (int64_t)16 * N * 2;
        u32x4 back[kPasses];
#pragma unroll
        for (int b = 0; b <= MF; ++b) {
            u32x2 pk[NF];
            if (b < MF) {
#pragma unroll
                for (int g = 0; g < NF; ++g) {
                    float yv[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float cc = ROWS ? srow[b < MF ? b : 0] * cs[g][e] : cs[g][e];
                        float v;
                        if constexpr (FLT)          v = acc[g][b < MF ? b : 0][e];
                        else if constexpr (GROUPED) v = fsum[GROUPED ? g : 0][GROUPED ? (b < MF ? b : 0) : 0][e] * cc;   // Y = fl32(f * s_w[n])
                        else                        v = (float)((int)acc[g][b < MF ? b : 0][e] >> kAccShift) * cc;
                        if (BIAS) v = v + bs[g][e];
                        yv[e] = v;
                    }
                    pk[g] = u32x2{S::pack(yv[0], yv[1]), S::pack(yv[2], yv[3])};
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (b > 0) {
#pragma unroll
                for (int p = 0; p < kPasses; ++p) *reinterpret_cast<u32x4*>(dst + (b - 1) * chunk_step + p * row_step) = back[p];
            }
            if (b < MF) {
#pragma unroll
                for (int g = 0; g < NF; ++g) *reinterpret_cast<u32x2*>(wr + g * 32) = pk[g];
#pragma unroll
                for (int p = 0; p < kPasses; ++p) back[p] = *reinterpret_cast<const u32x4*>(rd + p * kRowsPerPass * T::kEpiStride);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (vec_ok && wm0 + BM / 2 <= M && wn0 + BN / 2 <= N) {
        if (has_bias) write_tile_chunked(std::true_type{});
        else          write_tile_chunked(std::false_type{});
    } else {
    auto write_tile = [&](auto bias_tag) {
        constexpr bool BIAS = decltype(bias_tag)::value;
        f32x4 svs[NF];                                         // all parked factors requested together: one LDS latency
#pragma unroll
        for (int g = 0; g < NF; ++g) svs[g] = *reinterpret_cast<const f32x4*>(fac + (g * 16 + 4 * fq) * 4);
#pragma unroll
        for (int g = 0; g < NF; ++g) {
            const int nl = g * 16 + 4 * fq;                    // column within the wave's block
            float cs[4], bs[4];
            if (FLT) {
#pragma unroll
                for (int e = 0; e < 4; ++e) { cs[e] = 1.0f; bs[e] = 0.0f; }
            } else if (cols_inside) {
                const f32x4 sv = svs[g];
                f32x4 bv = {0.0f, 0.0f, 0.0f, 0.0f};
                if (BIAS) bv = *reinterpret_cast<const f32x4*>(bias + wn0 + nl);
#pragma unroll
                for (int e = 0; e < 4; ++e) { cs[e] = (ROWS || GROUPED) ? sv[e] : s * sv[e]; bs[e] = bv[e]; }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ne = min(wn0 + nl + e, N - 1);
                    cs[e] = (ROWS || GROUPED) ? s_w[ne] : s * s_w[ne];
                    bs[e] = BIAS ? bias[ne] : 0.0f;
                }
            }
#pragma unroll
            for (int b = 0; b < MF; ++b) {
                const int ml = b * 16 + frow;
                float yv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float cc = ROWS ? srow[b] * cs[e] : cs[e];
                    float v;
                    if constexpr (FLT)          v = acc[g][b][e];
                    else if constexpr (GROUPED) v = fsum[GROUPED ? g : 0][GROUPED ? b : 0][e] * cc;      // Y = fl32(f * s_w[n])
                    else                        v = (float)((int)acc[g][b][e] >> kAccShift) * cc;
                    if (BIAS) v = v + bs[e];
                    yv[e] = v;
                }
                u32x2 pk = {S::pack(yv[0], yv[1]), S::pack(yv[2], yv[3])};
                *reinterpret_cast<u32x2*>(epi + ml * T::kEpiStride + nl * 2) = pk;
            }
        }
    };
    if (has_bias) write_tile(std::true_type{});
    else          write_tile(std::false_type{});
    // each wave reads back only what it wrote itself: no workgroup barrier needed
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
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
    }   // block at an edge of the matrix
    // inspection output (int32 accumulators): straight from the registers, apart from the common path
    if (acc_out) {
#pragma unroll
        for (int g = 0; g < NF; ++g)
#pragma unroll
            for (int b = 0; b < MF; ++b) {
                const int m = wm0 + b * 16 + frow, n = wn0 + g * 16 + 4 * fq;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (m < M && n + e < N)
                        acc_out[(int64_t)m * N + n + e] = GROUPED ? __float_as_int(fsum[GROUPED ? g : 0][GROUPED ? b : 0][e])
                                                                  : FLT ? __float_as_int((float)acc[g][b][e]) : ((int)acc[g][b][e] >> kAccShift);
            }
    }
    SASQ_TILE_TS(4);
}

}  // namespace sasq
