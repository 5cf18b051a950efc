// The window kernel of the SGNS trainer for gfx950 (MI355X) and its device helpers.  Included by
// the translation units that instantiate it (one per row shape, see w2v_train_inst.inc).
//
// Window kernel in one paragraph (paper Sections 3.1, 3.2, 4.2, re-mapped to CDNA4):
// one wavefront owns one sentence, or one stretch of a long sentence, at a time (device work queue,
// lock-free between wavefronts).  The 64 lanes split every embedding row; the N+1 output rows of a window
// (target + shared negatives) sit in VGPRs while the window lasts, the context rows sit in an
// LDS ring from the moment the window span reaches them until it has passed them.  All
// (context, output) dot products of a window are formed as per-lane partial sums and reduced
// together by one transposing butterfly (v_permlane32_swap / v_permlane16_swap / DPP), after
// which lane v holds pairing v and the sigmoid is evaluated lane-parallel.  The window's
// update is the sum over all pairings evaluated at the values the rows had when the window
// began.  Sampling decisions (subsampling, width, negatives) are computed lane-parallel for
// 64 positions at a time from a counter-based generator.
#pragma once
#include "w2v_internal.h"
#include "w2v_rng.h"

#include <type_traits>
#include <utility>

namespace w2v {
namespace {

constexpr int kLanes = 64;
constexpr int KC = 6;              // output rows held in registers at once
constexpr int CC = 10;             // most context rows whose pairings are reduced together (CC*KC <= 64)
constexpr int FCAP = 256;          // kept-token FIFO entries per wavefront (power of two) of most shapes
// Windows sampled at a time and FIFO entries by shape (e: floats of a row per lane, wcap: widest window of the
// instantiation, summed: the summed-update variant).  Two kinds of shape sample 32 windows at a time into a FIFO of 128,
// because the 2.7 to 3.3 KB of LDS this saves lets a CU hold more wavefronts: rows of five floats per lane (d = 260..320;
// ring of 16.6 KB at W <= 5: 8 instead of 7 wavefronts per CU), and rows of two floats per lane with windows up to 10
// (d = 65..128; ring of 11.8 KB: 11 instead of 9).  The
// price is a sampling stage that runs half empty.  The FIFO holds the kept positions from W before the chunk's first
// window to the last one scanned: at most chunk + 2W + 64 entries.
// Context rows whose pairings are reduced together.  The summed width-10 kernel of rows of two floats per lane takes 5
// at a time (a second or third reduction for windows wider than 2, but 40 registers fewer): it then fits 3 wavefronts
// per SIMD without a spill on the window path, and 11 per CU instead of 8 hide its waits better (walk workload 172 ->
// 164 ms per epoch).
constexpr int block_slots(int e, int wcap, bool summed) { return (summed && wcap == 10 && e == 2) ? 5 : CC; }
constexpr int wcap_of(uint32_t window) { return window <= 5 ? 5 : window <= 10 ? 10 : 16; }
constexpr int chunk_windows(int e, int wcap, bool summed) { (void)summed; return ((e == 5 && wcap <= 10) || (e == 2 && wcap == 10)) ? 32 : 64; }
constexpr int fifo_entries(int e, int wcap, bool summed) { return chunk_windows(e, wcap, summed) == 32 ? 128 : FCAP; }
constexpr uint32_t kIdBits = 27;
constexpr uint32_t kIdMask = (1u << kIdBits) - 1u;

__device__ __forceinline__ uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ uint64_t uni64(uint64_t v)
{
    return ((uint64_t)uni((uint32_t)(v >> 32)) << 32) | uni((uint32_t)v);
}
__device__ __forceinline__ float lane_value(float v, uint32_t lane)
{
    return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), lane));
}
__device__ __forceinline__ uint32_t lane_value(uint32_t v, uint32_t lane) { return __builtin_amdgcn_readlane(v, lane); }

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
constexpr int kDppRowRor8 = 0x128, kDppHalfMirror = 0x141, kDppQuadXor2 = 0x4E, kDppQuadXor1 = 0xB1;

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// Broadcast of per-lane results to every lane without going through scalar registers.
// rows_to_all: G[r] gets lanes 16r .. 16r+15 of g in each of its four rows of 16 lanes (r < ROWS).
// mul_row_lane<S>(G, o) = o * G[lane S of the caller's row], fma_row_lane adds that product to acc: the
// multiplier comes through the row-broadcast DPP operand, so it costs no instruction of its own.
// The compiler does not see that these instructions read G across lanes, so rows_to_all ends with the two
// wait states a DPP read of a freshly written register needs.  All 64 lanes must be active.
template <int ROWS>
__device__ __forceinline__ void rows_to_all(float g, float (&G)[4])
{
    static_assert(ROWS >= 1 && ROWS <= 4, "a wavefront has four rows");
    const uint32_t u = __float_as_uint(g);
    const auto h = __builtin_amdgcn_permlane32_swap(u, u, false, false);      // [r0 r1 r0 r1], [r2 r3 r2 r3]
    const auto lo = __builtin_amdgcn_permlane16_swap(h[0], h[0], false, false);
    G[0] = __uint_as_float(lo[0]);
    G[1] = __uint_as_float(lo[1]);
    G[2] = G[3] = 0.0f;
    if constexpr (ROWS > 2) {
        const auto hi = __builtin_amdgcn_permlane16_swap(h[1], h[1], false, false);
        G[2] = __uint_as_float(hi[0]);
        G[3] = __uint_as_float(hi[1]);
    }
    asm volatile("s_nop 1" : "+v"(G[0]), "+v"(G[1]), "+v"(G[2]), "+v"(G[3]));
}
template <int S>
__device__ __forceinline__ float mul_row_lane(float G, float o)
{
    float r;
    asm("v_mul_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(G), "v"(o), "n"(S));
    return r;
}
template <int S>
__device__ __forceinline__ void fma_row_lane(float &acc, float G, float o)
{
    asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(G), "v"(o), "n"(S));
}

// Transposing reduction: sums each of M per-lane values over the 64 lanes; lane v (v < M) returns
// the total of value v.  Stage B (32, 16, .., 1) pairs register i with register i+B: lanes with bit B
// set continue with the upper one, so every stage halves the registers and the lanes a value is
// spread over.  A register without a partner (i+B >= M) is carried on unchanged and its two halves
// are folded once at the end, which costs one operation per stage instead of one per register.
template <int IN, int BIT, int CTRL>
__device__ __forceinline__ void row_stage(const float *in, float *out, int lane)
{
    constexpr int OUT = IN > BIT ? BIT : IN;
    const bool up = (lane & BIT) != 0;
#pragma unroll
    for (int i = 0; i < OUT; ++i) {
        if (i + BIT < IN) {
            const float a = in[i], b = in[i + BIT];
            if constexpr (BIT == 8 || BIT == 4) {
                // Lanes whose BIT is clear continue with a (own + partner's), the others with b: two adds that take
                // the partner's value through the DPP operand and write disjoint banks of four lanes (bank_mask),
                // instead of two selects and an add.  The s_nop covers the two wait states a DPP read needs after
                // the write of its register (the compiler does not look into the statement).
                float o;
                if constexpr (BIT == 8)
                    asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
                                 "v_add_f32_dpp %0, %2, %2 row_ror:8 row_mask:0xf bank_mask:0xc" : "=&v"(o) : "v"(a), "v"(b));
                else
                    asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
                                 "v_add_f32_dpp %0, %2, %2 row_half_mirror row_mask:0xf bank_mask:0xa" : "=&v"(o) : "v"(a), "v"(b));
                out[i] = o;
                continue;
            }
            const float mine = up ? b : a;
            const float theirs = up ? a : b;
            out[i] = mine + dpp_move<CTRL>(theirs);
        } else {
            out[i] = in[i];
        }
    }
}

template <int M>
__device__ __forceinline__ float transpose_reduce(const float *v, int lane)
{
    static_assert(M >= 8 && M <= 64, "between 8 and 64 values");
    constexpr int N32 = M < 32 ? M : 32;
    constexpr int N16 = N32 < 16 ? N32 : 16;
    constexpr int N8 = N16 < 8 ? N16 : 8;
    float s32[N32], s16[N16], s8[N8], s4[4], s2[2], s1[1];
#pragma unroll
    for (int i = 0; i < N32; ++i) {   // halves: lanes >= 32 continue with value i+32
        if (i + 32 < M) {
            auto p = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[i]), __float_as_uint(v[i + 32]), false, false);
            s32[i] = __uint_as_float(p[0]) + __uint_as_float(p[1]);
        } else {
            s32[i] = v[i];
        }
    }
#pragma unroll
    for (int i = 0; i < N16; ++i) {   // rows: odd rows continue with value i+16
        if (i + 16 < N32) {
            auto p = __builtin_amdgcn_permlane16_swap(__float_as_uint(s32[i]), __float_as_uint(s32[i + 16]), false, false);
            s16[i] = __uint_as_float(p[0]) + __uint_as_float(p[1]);
        } else {
            s16[i] = s32[i];
        }
    }
    row_stage<N16, 8, kDppRowRor8>(s16, s8, lane);
    row_stage<N8, 4, kDppHalfMirror>(s8, s4, lane);
    row_stage<4, 2, kDppQuadXor2>(s4, s2, lane);
    row_stage<2, 1, kDppQuadXor1>(s2, s1, lane);
    float x = s1[0];
    // late folds, innermost first.  Lane l ends on the register chain of value (l mod B) at stage B
    // (lower stages are always paired for M >= 8); that register had no partner iff (l mod B) + B >= M.
    if constexpr (M < 16) {
        const float t = x + dpp_move<kDppRowRor8>(x);
        x = ((lane & 7) + 8 >= M) ? t : x;
    }
    if constexpr (M < 32) {
        auto p = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
        const float t = __uint_as_float(p[0]) + __uint_as_float(p[1]);
        constexpr int B = M < 16 ? 8 : 16;          // bits of the chain index known at this stage
        x = ((lane & (B - 1)) + 16 >= M) ? t : x;
    }
    {
        auto p = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
        const float t = __uint_as_float(p[0]) + __uint_as_float(p[1]);
        constexpr int B = M < 16 ? 8 : (M < 32 ? 16 : 32);
        x = ((lane & (B - 1)) + 32 >= M) ? t : x;
    }
    return x;
}

// plain 64-lane sum, every lane gets the total (used once per wavefront for the loss)
__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, kLanes);
    return x;
}

template <int VW> __device__ __forceinline__ void load_vec(const float *p, float *dst)
{
    if constexpr (VW == 1) { dst[0] = *p; }
    else if constexpr (VW == 2) { const float2 t = *reinterpret_cast<const float2 *>(p); dst[0] = t.x; dst[1] = t.y; }
    else { const float4 t = *reinterpret_cast<const float4 *>(p); dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w; }
}
template <int VW> __device__ __forceinline__ void store_vec(float *p, const float *src)
{
    if constexpr (VW == 1) { *p = src[0]; }
    else if constexpr (VW == 2) { *reinterpret_cast<float2 *>(p) = make_float2(src[0], src[1]); }
    else { *reinterpret_cast<float4 *>(p) = make_float4(src[0], src[1], src[2], src[3]); }
}

// the same store at system scope (written through to the memory side that all XCDs share): relaxed atomic stores of
// 4 or 8 bytes are what the compiler turns into global_store ... sc0 sc1
template <int VW> __device__ __forceinline__ void store_vec_system(float *p, const float *src)
{
    if constexpr (VW == 1) {
        __hip_atomic_store(reinterpret_cast<uint32_t *>(p), __float_as_uint(src[0]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    } else {
#pragma unroll
        for (int h = 0; h < VW / 2; ++h) {
            const uint64_t v = ((uint64_t)__float_as_uint(src[2 * h + 1]) << 32) | __float_as_uint(src[2 * h]);
            __hip_atomic_store(reinterpret_cast<uint64_t *>(p) + h, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

// Rows whose length does not fill the lanes' shares (dim < 64 * floats per lane) are reached through a buffer
// resource per row, dim floats long: a lane whose share lies past the last column loads 0 and its stores are
// dropped by the hardware's range check, so no lane needs a test of its own, and the lane's constant byte offset
// is the only vector operand.  Whole rows use plain global accesses (measured faster for them).
typedef unsigned int vec2u __attribute__((ext_vector_type(2)));
typedef unsigned int vec4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_resource(const float *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0, (int)bytes, 0x00020000);
}
// AUX is the cache-policy operand of the buffer instructions: 0 = ordinary (served by the L2 of the wavefront's own
// XCD), kSystemScope = sc0 sc1: the access is made at the memory side that all XCDs share (loads do not hit in
// L2, stores are written through), which is what keeps rows coherent between wavefronts on different XCDs.
constexpr int kSystemScope = 0x11;
template <int VW, int AUX = 0>
__device__ __forceinline__ void row_load_vec(__amdgpu_buffer_rsrc_t rs, int lane_bytes, uint32_t row_bytes_off, float *dst)
{
    if constexpr (VW == 1) {
        dst[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, lane_bytes, (int)row_bytes_off, AUX));
    } else if constexpr (VW == 2) {
        const vec2u t = __builtin_amdgcn_raw_buffer_load_b64(rs, lane_bytes, (int)row_bytes_off, AUX);
        dst[0] = __uint_as_float(t.x); dst[1] = __uint_as_float(t.y);
    } else {
        const vec4u t = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_bytes, (int)row_bytes_off, AUX);
        dst[0] = __uint_as_float(t.x); dst[1] = __uint_as_float(t.y); dst[2] = __uint_as_float(t.z); dst[3] = __uint_as_float(t.w);
    }
}
template <int VW, int AUX = 0>
__device__ __forceinline__ void row_store_vec(__amdgpu_buffer_rsrc_t rs, int lane_bytes, uint32_t row_bytes_off, const float *src)
{
    if constexpr (VW == 1) {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(src[0]), rs, lane_bytes, (int)row_bytes_off, AUX);
    } else if constexpr (VW == 2) {
        vec2u t; t.x = __float_as_uint(src[0]); t.y = __float_as_uint(src[1]);
        __builtin_amdgcn_raw_buffer_store_b64(t, rs, lane_bytes, (int)row_bytes_off, AUX);
    } else {
        vec4u t; t.x = __float_as_uint(src[0]); t.y = __float_as_uint(src[1]); t.z = __float_as_uint(src[2]); t.w = __float_as_uint(src[3]);
        __builtin_amdgcn_raw_buffer_store_b128(t, rs, lane_bytes, (int)row_bytes_off, AUX);
    }
}

// bfloat16 storage: a row of dim elements of 2 bytes.  A chunk of VW elements is one 2-, 4- or 8-byte access; a
// stored value is the upper half of the float's bit pattern.  A load leaves the chunk's words as they are in the
// first registers of the chunk (a row that has been requested but not yet arrived must not be touched: widening it at
// once would put a wait for the data right behind every load and no prefetch would hide anything); widen_chunk
// turns them into floats where the row is first needed.
template <int VW>
__device__ __forceinline__ void row_load_bf16(__amdgpu_buffer_rsrc_t rs, int lane_bytes, float *dst)
{
    if constexpr (VW == 1) {
        dst[0] = __uint_as_float((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(rs, lane_bytes, 0, 0));
    } else if constexpr (VW == 2) {
        dst[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, lane_bytes, 0, 0));
    } else {
        const vec2u t = __builtin_amdgcn_raw_buffer_load_b64(rs, lane_bytes, 0, 0);
        dst[0] = __uint_as_float(t.x); dst[1] = __uint_as_float(t.y);
    }
}
// dst[0 .. VW) = the floats of the chunk whose words lie in src[0 .. (VW+1)/2); dst may be src
template <int VW>
__device__ __forceinline__ void widen_chunk(float *dst, const float *src)
{
    if constexpr (VW == 1) {
        dst[0] = __uint_as_float(__float_as_uint(src[0]) << 16);
    } else if constexpr (VW == 2) {
        const uint32_t w = __float_as_uint(src[0]);
        dst[1] = __uint_as_float(w & 0xFFFF0000u); dst[0] = __uint_as_float(w << 16);
    } else {
        const uint32_t w0 = __float_as_uint(src[0]), w1 = __float_as_uint(src[1]);
        dst[3] = __uint_as_float(w1 & 0xFFFF0000u); dst[2] = __uint_as_float(w1 << 16);
        dst[1] = __uint_as_float(w0 & 0xFFFF0000u); dst[0] = __uint_as_float(w0 << 16);
    }
}
// Stochastic rounding of a working value to bfloat16: 16 random bits are added to the float's bit pattern and the
// low half is dropped (infinities stay, a NaN stays a NaN).  The bits of element e of a row written with the 64-bit
// draw S are the upper half of  a = lo24(S) * c_e + hi32(S)  (one v_mad_u32_u24), with c_e an odd 24-bit constant of
// the element that the caller keeps in a register.  v_cvt_sr_bf16_f32 does the rest in one instruction: it adds the
// upper half of its second operand to the float and writes the upper half of the sum into one half of its
// destination, so two calls fill one 32-bit word of the row.
template <bool HIGH>
__device__ __forceinline__ void round_to_bf16(uint32_t &word, float x, uint32_t s_lo, uint32_t s_hi, uint32_t c)
{
    const uint32_t a = __umul24(s_lo, c) + s_hi;
    if constexpr (HIGH) asm("v_cvt_sr_bf16_f32 %0, %1, %2 op_sel:[0,0,1]" : "+v"(word) : "v"(x), "v"(a));
    else asm("v_cvt_sr_bf16_f32 %0, %1, %2" : "+v"(word) : "v"(x), "v"(a));
}
// h: the row's chunk as packed words (element x of the chunk in half x & 1 of word x >> 1)
template <int VW>
__device__ __forceinline__ void row_store_bf16(__amdgpu_buffer_rsrc_t rs, int lane_bytes, const uint32_t *h)
{
    if constexpr (VW == 1) {
        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)h[0], rs, lane_bytes, 0, 0);
    } else if constexpr (VW == 2) {
        __builtin_amdgcn_raw_buffer_store_b32(h[0], rs, lane_bytes, 0, 0);
    } else {
        vec2u t; t.x = h[0]; t.y = h[1];
        __builtin_amdgcn_raw_buffer_store_b64(t, rs, lane_bytes, 0, 0);
    }
}

// learning rate of the sentence that starts at global token offset `start` of this epoch
__device__ __forceinline__ float sentence_lr(const KernelArgs &A, uint64_t start)
{
    const double done = (double)(A.lr_done_base + start);
    double frac = 1.0 - done / (double)A.lr_all;
    if (frac < A.lr_min_frac) frac = A.lr_min_frac;
    return (float)(A.lr0 * frac);
}

// ---------------------------------------------------------------------------------------------
// the window kernel
// ---------------------------------------------------------------------------------------------
// Per-window scalars the sampling stage leaves in LDS for the window loop (one uint4 per window):
//   x = width b | (reload bits << 8) | (atomic << 16) | (plain << 17) | (special << 18),  w = dupmask
//       reload bit k': output row k' (k' < KC) of this window is also an output row of the previous
//       window, so a copy fetched before that window's write-back is stale;
//       dupmask bit c: context slot c holds the same word as a later slot and is represented by it;
//       atomic: a word fills more than 15 slots, weights are not used and ring rows are added to;
//       plain: every negative distinct and different from the target;
//       special: some context slot of the window is absent or repeats a word (slot weights differ from 1)
//       idle (bit 19): a lead-in token of the unit; it has no window of its own and needs no output rows
//       hand-over (bit 20): the next window uses the same negatives; their rows stay in registers for it
//   y = target word, z = word of the kept position that enters the ring at this window (or none)
constexpr uint32_t kNoWord = 0xFFFFFFFFu;

// VW, R, TAIL: a lane's share of a row (R chunks of VW floats, then TAIL single floats); WCAP: widest window of
// the instantiation; FULL: the rows fill the shares exactly (dim = 64 * floats per lane), so rows are reached
// with plain global accesses and no bounds check.
// KMODE: how the N + 1 output rows of a window relate to the KC rows handled at a time:
//   0: fewer than KC rows, 1: exactly KC rows (every row-exists test folds away), 2: up to 2 KC rows (two passes,
//   each fetching the rows of the next while it computes), 3: more (further rows fetched when their pass begins)

// wavefronts per SIMD the register allocator is asked to make room for (512 VGPRs per lane in all)
// (e: floats of a row per lane, wcap: widest window of the instantiation; measured: rows of one float per lane
// gain 17 % from 4 per SIMD (128 VGPRs, 16 spilled), 5 spills 56; rows of two floats gain nothing from 4
// because LDS then limits the CU; 3 for rows of 4 floats per lane spills)
constexpr bool rounding_draws_in_lds(int kmode) { return kmode <= 1; }
constexpr int occupancy_goal(int e, int wcap, bool summed = false)
{
    (void)summed;
    return (e == 1 && wcap <= 5) ? 4 : (e <= 2 && wcap <= 10) ? 3 : ((e * wcap <= 25) ? 2 : 1);
}

// SUMMED: lock-free updates are added to what memory holds when a row goes back, instead of overwriting it with a copy
// that was fetched up to 2W+1 windows earlier (see "summed updates" below); the rows are then stored at system scope.
// BF16: the tables hold bfloat16 (2 bytes per element, row stride A.ld elements); rows are widened to fp32 when they are
// fetched into registers / the ring and rounded stochastically when they go back (an extension; the paper stores fp32).
template <int VW, int R, int TAIL, int WCAP, bool FULL, int KMODE, bool SUMMED, bool BF16>
__global__ void __launch_bounds__(kLanes) __attribute__((amdgpu_waves_per_eu(occupancy_goal(VW * R + TAIL, WCAP, SUMMED))))
train_kernel(KernelArgs A)
{
    static_assert(!(BF16 && (FULL || SUMMED)), "bfloat16 rows go through buffer resources and are overwritten");
    constexpr int E = VW * R + TAIL;     // floats of a row per lane
    constexpr int NCH = R + TAIL;        // chunks of a row per lane: R of VW floats, then TAIL single floats
    constexpr int ROWF = kLanes * E;     // floats of a ring row in LDS
    constexpr int CCK = block_slots(E, WCAP, SUMMED);   // most context rows reduced together
    constexpr int CHUNK = chunk_windows(E, WCAP, SUMMED);   // windows sampled at a time (one per lane)
    constexpr int FQ = fifo_entries(E, WCAP, SUMMED);       // kept-token FIFO entries
    constexpr int NCTX = 2 * WCAP;       // context positions a window can have
    constexpr bool MULTI = KMODE >= 2;   // output rows beyond the first KC are handled in further passes
    constexpr bool TWO = KMODE == 2;     // ... in exactly one further pass (KC < N + 1 <= 2 KC)
    constexpr bool KFULL = KMODE >= 1;   // the first KC output rows all exist
    constexpr bool KEXACT = KMODE == 1;  // ... and there are no others
    constexpr bool NREG = KMODE <= 1;    // at most KC - 1 negatives: the sampling stage keeps them in registers
    // bfloat16 storage: the rounding draws of 64 windows are computed lane-parallel in the sampling stage and kept in
    // LDS, except where that kilobyte would cost the CU a wavefront (the shapes with two passes over the output
    // rows): there the scalar unit computes the two draws of a window when the window begins
    constexpr bool DRAWS_IN_LDS = BF16 && rounding_draws_in_lds(KMODE);

    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int lane = threadIdx.x;
    const uint32_t W = A.window, N = A.negatives;
    const uint32_t nslots = 2 * W + 2;
    float *ring = reinterpret_cast<float *>(lds_raw);
    // ring row `nslots` is never assigned to a word: it holds zeros and stands in for context slots that do not exist
    int32_t *kw = reinterpret_cast<int32_t *>(ring + (size_t)(nslots + 1) * ROWF);  // kept word ids (FIFO)
    uint32_t *kp = reinterpret_cast<uint32_t *>(kw + FQ);                  // their offsets in the sentence
    uint4 *cb_meta = reinterpret_cast<uint4 *>(kp + FQ);                   // per-window scalars of the chunk
    uint32_t *cb_cm = reinterpret_cast<uint32_t *>(cb_meta + CHUNK);        // [64][4] context multiplicities, 4 bits per slot
    uint32_t *cb_pack = cb_cm + 4 * CHUNK;                                  // [64][N] negative id | multiplicity<<27
    // bfloat16 storage: [64] the 64-bit draws that key the roundings of a window: of its centre (output rows) and of
    // the position that leaves the span after it (that position's context row)
    uint4 *cb_rnd = reinterpret_cast<uint4 *>(cb_pack + (size_t)CHUNK * A.negatives);

    // A lane's share of a row: chunk r < R is VW consecutive floats at (r*64 + lane)*VW, chunk R + t is the
    // single float at 64*VW*R + t*64 + lane.  `chunks` calls f(chunk index, its width, its place in a register row).
    auto chunks = [&](auto &&f) {
        static_for<NCH>([&](auto r_tag) {
            constexpr int r = decltype(r_tag)::value;
            f(r_tag, std::integral_constant<int, (r < R ? VW : 1)>{},
              std::integral_constant<int, (r < R ? r * VW : R * VW + (r - R))>{});
        });
    };
    // element offsets of this lane inside a row (they may lie beyond dim: such elements are zero in registers and
    // in the ring, and the bounds check of the row accesses keeps them out of memory)
    int eoff[NCH];
#pragma unroll
    for (int r = 0; r < NCH; ++r)
        eoff[r] = r < R ? (r * kLanes + lane) * VW : kLanes * VW * R + (r - R) * kLanes + lane;
    const int lane_c0 = lane / KC, lane_k0 = lane % KC;   // pairing handled by this lane after the reduction

    const uint32_t row_bytes = A.dim * 4u;
    // row `word` of a table -> registers (zeros beyond dim) / registers -> the row (nothing beyond dim)
    // (summed mode: stores are made at system scope, i.e. written through to the memory side that all XCDs share;
    // measured on walks over a 1M-node graph, system-scope loads on top of that change nothing)
    // per-element constants of the stochastic rounding (bfloat16 storage only)
    uint32_t round_c[BF16 ? E : 1] = {};
    if constexpr (BF16) {
        chunks([&](auto r_, auto w_, auto o_) {
            constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
#pragma unroll
            for (int x = 0; x < CW; ++x) round_c[RO + x] = ((uint32_t)(mix64(0x726F756E64ull + (uint64_t)(eoff[r] + x)) >> 32) >> 8) | 1u;
        });
    }
    auto load_row = [&](const float *table, uint32_t word, float *dst) {
        if constexpr (BF16) {
            const uint16_t *row16 = reinterpret_cast<const uint16_t *>(table) + (size_t)word * A.ld;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(row16), 0, (int)(A.dim * 2u), 0x00020000);
            chunks([&](auto r_, auto w_, auto o_) {
                constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
                row_load_bf16<CW>(rs, eoff[r] * 2, dst + RO);
            });
            return;
        }
        const float *row = table + (size_t)word * A.ld;
        if constexpr (FULL) {
            chunks([&](auto r_, auto w_, auto o_) {
                constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
                load_vec<CW>(row + eoff[r], dst + RO);
            });
        } else {
            const __amdgpu_buffer_rsrc_t rs = row_resource(row, row_bytes);
            chunks([&](auto r_, auto w_, auto o_) {
                constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
                row_load_vec<CW>(rs, eoff[r] * 4, 0u, dst + RO);
            });
        }
    };
    // sbits: the 64-bit draw that keys the rounding of this write (bfloat16 storage only)
    auto store_row = [&](float *table, uint32_t word, const float *src, uint64_t sbits) {
        if constexpr (BF16) {
            uint16_t *row16 = reinterpret_cast<uint16_t *>(table) + (size_t)word * A.ld;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(row16, 0, (int)(A.dim * 2u), 0x00020000);
            const uint32_t s_lo = (uint32_t)sbits, s_hi = (uint32_t)(sbits >> 32);
            chunks([&](auto r_, auto w_, auto o_) {
                constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
                uint32_t h[(CW + 1) / 2] = {};
                static_for<CW>([&](auto x_) {
                    constexpr int x = decltype(x_)::value;
                    round_to_bf16<(x & 1) != 0>(h[x >> 1], src[RO + x], s_lo, s_hi, round_c[RO + x]);
                });
                row_store_bf16<CW>(rs, eoff[r] * 2, h);
            });
            return;
        }
        float *row = table + (size_t)word * A.ld;
        if constexpr (FULL) {
            chunks([&](auto r_, auto w_, auto o_) {
                constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
                if constexpr (SUMMED) store_vec_system<CW>(row + eoff[r], src + RO);
                else store_vec<CW>(row + eoff[r], src + RO);
            });
        } else {
            const __amdgpu_buffer_rsrc_t rs = row_resource(row, row_bytes);
            chunks([&](auto r_, auto w_, auto o_) {
                constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
                row_store_vec<CW, SUMMED ? kSystemScope : 0>(rs, eoff[r] * 4, 0u, src + RO);
            });
        }
    };
    // Summed updates.  A wavefront works on copies: a context row stays in its ring for up to 2W+1 windows, an
    // output row in its registers from the fetch one window ahead to the end of its window.  Writing the copy back
    // discards whatever other wavefronts added to the row meanwhile.  In the summed mode a row goes back as
    // (what memory holds now) + (copy - value the copy started from): the update is added, and the time in which
    // another wavefront's update can be lost shrinks from the copy's lifetime to one memory round trip.  The
    // starting value of a ring slot is kept in a snapshot row of the wavefront's own in global memory (written
    // when the slot is filled, read when it is evicted); an output row's starting value is still in registers.
    constexpr bool sum_ring = SUMMED;
    float *snap_base = SUMMED ? A.snap + (size_t)blockIdx.x * A.snap_stride : nullptr;
    auto snap_store = [&](uint32_t slot, const float *src) {
        float *row = snap_base + (size_t)slot * ROWF;
        chunks([&](auto r_, auto w_, auto o_) {
            constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
            store_vec<CW>(row + eoff[r], src + RO);
        });
    };
    auto snap_load = [&](uint32_t slot, float *dst) {
        const float *row = snap_base + (size_t)slot * ROWF;
        chunks([&](auto r_, auto w_, auto o_) {
            constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
            load_vec<CW>(row + eoff[r], dst + RO);
        });
    };
    auto load_ctx = [&](uint32_t word, float *dst) { load_row(A.syn0, word, dst); };
    auto load_out = [&](uint32_t word, float *dst) { load_row(A.syn1neg, word, dst); };
    auto store_out = [&](uint32_t word, const float *src, uint64_t sbits) { store_row(A.syn1neg, word, src, sbits); };
    // bfloat16 storage: a fetched row (words as loaded) becomes floats, in place or on its way into another row
    auto widen_into = [&](float *dst, const float *src) {
        if constexpr (BF16) {
            chunks([&](auto r_, auto w_, auto o_) {
                constexpr int CW = decltype(w_)::value, RO = decltype(o_)::value;
                widen_chunk<CW>(dst + RO, src + RO);
            });
        }
    };
    auto widen_row = [&](float *row) { widen_into(row, row); };
    auto ring_to_regs = [&](const float *lrow, float *dst) {      // LDS ring row -> registers
        chunks([&](auto r_, auto w_, auto o_) {
            constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
            load_vec<CW>(lrow + eoff[r], dst + RO);
        });
    };
    auto regs_to_ring = [&](float *lrow, const float *src) {      // registers -> LDS ring row
        chunks([&](auto r_, auto w_, auto o_) {
            constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
            store_vec<CW>(lrow + eoff[r], src + RO);
        });
    };
    {
        float zero[E];
#pragma unroll
        for (int x = 0; x < E; ++x) zero[x] = 0.0f;
        regs_to_ring(ring + (size_t)nslots * ROWF, zero);
    }

    double loss_acc = 0.0;
    unsigned long long pairs_acc = 0, dropped_acc = 0, kept_acc = 0;
    // the launch's work plan (written by the planning kernel that precedes the launch on the stream)
    const uint32_t plan_unit_shift = uni(A.accum->unit_shift), plan_fine_shift = uni(A.accum->fine_shift);
    const uint64_t plan_coarse = uni64(A.accum->coarse_sent), plan_units = uni64(A.accum->n_units);

    for (;;) {
        // ---- next unit of work from the queue ---------------------------------------------------
        // A unit is one of 2^shift equal stretches of a sentence's tokens.  Its windows are those of the
        // kept tokens inside the stretch; the W kept tokens before it and after it are read as context only,
        // so the windows are exactly those the whole sentence has (units of one sentence that run at the same
        // time race like any two sentences do; one wavefront taking all units in order reproduces strict order).
        unsigned long long q_raw = 0;
        if (lane == 0) q_raw = atomicAdd(&A.accum->next_sentence, 1ull);
        const uint64_t q = uni64(q_raw);
        // (sentences from plan_coarse on are cut into 2^fine_shift stretches instead: the queue ends in small units)
        const uint64_t n_coarse = plan_coarse << plan_unit_shift;
        if (q >= plan_units) break;
        const bool fine = q >= n_coarse;
        const uint32_t shift = fine ? plan_fine_shift : plan_unit_shift;
        const uint64_t qs = fine ? q - n_coarse : q;                 // index among the units of its own kind
        const uint64_t s = (fine ? plan_coarse : 0ull) + (qs >> shift);
        const uint64_t t0 = uni64(A.sent_off[s]);
        const uint64_t t1 = uni64(A.sent_off[s + 1]);
        const uint32_t len = (t1 > t0) ? (uint32_t)(t1 - t0) : 0u;
        const float alpha = sentence_lr(A, A.first_pos + t0);
        const uint32_t unit_len = (uint32_t)(((uint64_t)len + (1u << shift) - 1u) >> shift);
        const uint64_t u0_64 = (qs & ((1ull << shift) - 1ull)) * unit_len;
        const uint32_t u0 = u0_64 < len ? (uint32_t)u0_64 : len;                  // the unit's tokens: [u0, u1)
        const uint32_t u1 = (len - u0 > unit_len) ? u0 + unit_len : len;
        if (u0 >= u1) continue;

        // is the token at offset `off` of the sentence kept?  (w: its word; bad: id outside the vocabulary)
        auto keep_token = [&](uint32_t off, int32_t &w, bool &bad) -> bool {
            w = A.tokens[t0 + off];
            bool k = w >= 0 && (uint32_t)w < A.vocab;
            bad = !k;
            if (k && A.subsample) {
                const uint32_t th = A.thr[w];
                if (th != 0xFFFFFFFFu) k = keep_decision(position_base(A.key, A.first_pos + t0 + off), th);
            }
            return k;
        };
        // the scan starts at the W-th kept token before the unit (or at the sentence start): n_lead of them
        uint32_t n_lead = 0, raw_first = u0;
        for (uint32_t hi = u0; n_lead < W && hi > 0;) {
            const uint32_t lo = hi >= (uint32_t)kLanes ? hi - kLanes : 0u;
            const uint32_t off = lo + lane;
            int32_t w;
            bool bad;
            const bool k = off < hi && keep_token(off, w, bad);
            uint64_t km = __ballot(k);
            const uint32_t cnt = (uint32_t)__popcll(km);
            raw_first = lo;
            if (n_lead + cnt >= W) {
                for (uint32_t drop = W - n_lead; drop > 1; --drop) km &= ~(1ull << (63 - __builtin_clzll(km)));
                raw_first = lo + (63u - (uint32_t)__builtin_clzll(km));     // the (W - n_lead)-th kept token from the top
                n_lead = W;
            } else {
                n_lead += cnt;
            }
            hi = lo;
        }

        int32_t meta_word = -1;       // lane p&63: word of resident kept position p (-1: none)
        uint32_t meta_slot = 0;       // lane p&63: its ring slot
        uint32_t free_slots = (nslots >= 32) ? 0xFFFFFFFFu : ((1u << nslots) - 1u);
        uint32_t free_hi = (nslots > 32) ? ((1u << (nslots - 32)) - 1u) : 0u;   // slots 32..33 (W = 16)
        uint32_t n_prod = 0;          // kept tokens found so far (counted from the scan's start)
        uint32_t n_own = 0;           // ... of them before the unit's end: windows exist for [n_lead, n_own)
        uint32_t raw_next = raw_first;   // next token offset to look at
        uint32_t n_ins = 0;           // kept positions [0, n_ins) have entered the ring
        uint32_t i0 = 0;              // first window of the current chunk

        auto take_slot = [&]() -> uint32_t {
            uint32_t sl;
            if (free_slots) { sl = __builtin_ctz(free_slots); free_slots &= free_slots - 1u; }
            else { sl = 32u + __builtin_ctz(free_hi); free_hi &= free_hi - 1u; }
            return sl;
        };
        auto give_slot = [&](uint32_t sl) {
            if (sl < 32u) free_slots |= 1u << sl; else free_hi |= 1u << (sl - 32u);
        };
        // kept position p (word `word`) enters the ring; true when its row must be fetched into `slot`
        auto ring_enter = [&](uint32_t p, int32_t word, uint32_t &slot) -> bool {
            const uint64_t same = __ballot(meta_word == word);
            bool fetch;
            if (same) { slot = lane_value(meta_slot, (uint32_t)__builtin_ctzll(same)); fetch = false; }
            else { slot = take_slot(); fetch = true; }
            if (lane == (int)(p & 63u)) { meta_word = word; meta_slot = slot; }
            return fetch;
        };
        // position p leaves the ring: true if its row must go back to syn0 (no other position shares it)
        auto leave_decide = [&](uint32_t p, uint32_t &slot, uint32_t &word) -> bool {
            const uint32_t l = p & 63u;
            slot = lane_value(meta_slot, l);
            word = lane_value((uint32_t)meta_word, l);
            if (lane == (int)l) meta_word = -1;
            return __ballot(meta_word >= 0 && meta_slot == slot) == 0;
        };
        // the row of `slot` goes back: as it is, or (summed) as fresh + (row - snapshot)
        // bfloat16 storage: the 64-bit draw of kept position p, which keys the rounding of its context row; inside the
        // window loop the sampling stage has computed it (lane-parallel), here it is formed by the scalar unit
        auto leave_draw = [&](uint32_t p) -> uint64_t {
            if constexpr (!BF16) return 0ull;
            else return draw_u64(position_base(A.key, A.first_pos + t0 + uni(kp[p & (FQ - 1)])), 64u);
        };
        auto leave_finish = [&](uint32_t slot, uint32_t word, bool summed, const float *fresh, const float *snapv, uint64_t sbits) {
            float t[E];
            ring_to_regs(ring + (size_t)slot * ROWF, t);
            if (summed) {
#pragma unroll
                for (int x = 0; x < E; ++x) t[x] = fresh[x] + (t[x] - snapv[x]);
            }
            store_row(A.syn0, word, t, sbits);
            give_slot(slot);
        };
        // draw: the 64-bit draw of position p (bfloat16 storage)
        auto ring_leave = [&](uint32_t p, uint64_t draw) {
            uint32_t slot, word;
            if (leave_decide(p, slot, word)) {
                float fresh[E] = {}, snapv[E] = {};
                const bool summed = sum_ring;
                if (summed) { load_row(A.syn0, word, fresh); snap_load(slot, snapv); }
                leave_finish(slot, word, summed, fresh, snapv, BF16 ? row_key(draw, 32u) : 0ull);
            }
        };

        for (;;) {
            // ---- look at more tokens until this chunk's windows know all their context ----------
            while (n_prod < i0 + CHUNK + W + 1 && raw_next < len) {
                const uint32_t off = raw_next + lane;
                bool k = false, bad = false;
                int32_t w = -1;
                if (off < len) k = keep_token(off, w, bad);
                if (bad && off >= u0 && off < u1) ++dropped_acc;
                const uint64_t km = __ballot(k);
                if (k) {
                    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(km >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)km, 0u));
                    kw[(n_prod + rank) & (FQ - 1)] = w;
                    kp[(n_prod + rank) & (FQ - 1)] = off;
                }
                n_own += (uint32_t)__popcll(__ballot(k && off < u1));
                n_prod += (uint32_t)__popcll(km);
                raw_next += kLanes;
            }
            __syncthreads();
            if (i0 >= n_own) break;
            const uint32_t nwin = (n_own - i0 < (uint32_t)CHUNK) ? n_own - i0 : (uint32_t)CHUNK;

            // ---- width and negatives of the chunk's windows, one window per lane ----------------
            // Negative k of a window carries a multiplicity: 0 if it equals the target or an earlier negative,
            // otherwise the number of times its id was drawn.  With at most KC-1 negatives (NREG) ids and
            // multiplicities stay in registers and every comparison is unrolled; otherwise they are worked on
            // in LDS.  Negatives that do not exist (k >= N) get ids no word has, so they match nothing.
            int32_t my_w = -1;
            uint32_t my_b = 0, my_enter = kNoWord, my_plain = 0, my_stretch = 0;
            uint32_t nid[NREG ? KC - 1 : 1] = {}, nmult[NREG ? KC - 1 : 1] = {};
            const bool have = (uint32_t)lane < nwin;
            if (have) {
                const uint32_t idx = (i0 + lane) & (FQ - 1);
                my_w = kw[idx];
                const uint32_t my_off = kp[idx];
                const uint64_t base = position_base(A.key, A.first_pos + t0 + my_off);
                my_b = (i0 + lane < n_lead) ? 0u : window_width(base, W, A.window_mode);   // lead-in tokens: context only
                if constexpr (DRAWS_IN_LDS) {
                    const uint64_t d_own = draw_u64(base, 64u);
                    uint64_t d_leave = 0ull;
                    const uint32_t me = i0 + lane;
                    if (me >= W) d_leave = draw_u64(position_base(A.key, A.first_pos + t0 + kp[(me - W) & (FQ - 1)]), 64u);
                    cb_rnd[lane] = make_uint4((uint32_t)d_own, (uint32_t)(d_own >> 32), (uint32_t)d_leave, (uint32_t)(d_leave >> 32));
                }
                // negatives: drawn at my own position, or at the first position of my stretch of 2^neg_shift tokens
                my_stretch = my_off >> A.neg_shift;
                const bool dump = A.dump.keep != nullptr && i0 + lane >= n_lead;   // test surface: my own decisions
                if (dump) { A.dump.keep[t0 + my_off] = 1; A.dump.width[t0 + my_off] = (uint8_t)my_b; }
                const uint64_t nbase = A.neg_shift ? position_base(A.key, A.first_pos + t0 + (my_stretch << A.neg_shift)) : base;
                const uint32_t pe = i0 + lane + W + 1;
                if (pe < n_prod) my_enter = (uint32_t)kw[pe & (FQ - 1)];
                uint32_t *pk = cb_pack + (size_t)lane * N;
                my_plain = 1u;
                if constexpr (NREG) {
#pragma unroll
                    for (int k = 0; k < KC - 1; ++k) {
                        nid[k] = kIdMask + 1u + (uint32_t)k;
                        if (KEXACT || (uint32_t)k < N) nid[k] = (uint32_t)A.table[negative_slot(nbase, (uint32_t)k, A.table_size)];
                        if (dump && (KEXACT || (uint32_t)k < N)) A.dump.neg[(t0 + my_off) * N + k] = (int32_t)nid[k];
                    }
#pragma unroll
                    for (int k = 0; k < KC - 1; ++k) {
                        bool first = nid[k] != (uint32_t)my_w;
                        uint32_t m = 1u;
#pragma unroll
                        for (int k1 = 0; k1 < k; ++k1) first = first && nid[k1] != nid[k];
#pragma unroll
                        for (int k2 = k + 1; k2 < KC - 1; ++k2) m += (nid[k2] == nid[k]) ? 1u : 0u;
                        nmult[k] = first ? m : 0u;
                        if (KEXACT || (uint32_t)k < N) {
                            pk[k] = nid[k] | (nmult[k] << kIdBits);
                            if (nmult[k] != 1u) my_plain = 0u;
                        }
                    }
                } else {
                    for (uint32_t k = 0; k < N; ++k) pk[k] = (uint32_t)A.table[negative_slot(nbase, k, A.table_size)];
                    if (dump) for (uint32_t k = 0; k < N; ++k) A.dump.neg[(t0 + my_off) * N + k] = (int32_t)pk[k];
                    for (uint32_t k = 0; k < N; ++k) {
                        const uint32_t id = pk[k] & kIdMask;
                        uint32_t m = (id == (uint32_t)my_w) ? 0u : 1u;
                        for (uint32_t k1 = 0; k1 < k && m; ++k1) if ((pk[k1] & kIdMask) == id) m = 0u;
                        if (m) for (uint32_t k2 = k + 1; k2 < N; ++k2) if ((pk[k2] & kIdMask) == id) ++m;
                        pk[k] = id | (m << kIdBits);
                        if (m != 1u) my_plain = 0u;
                    }
                }
            }
            __syncthreads();
            uint32_t reload = 0, dupmask = 0, overflow = 0, special = 0;
            if (have) {
                // which of my first KC output rows does the previous window also write?
                if (lane > 0) {
                    const uint32_t pw = (uint32_t)kw[(i0 + lane - 1) & (FQ - 1)];
                    const uint32_t *prev = cb_pack + (size_t)(lane - 1) * N;
                    if constexpr (NREG) {
                        uint32_t pid[KC];           // rows the previous window writes (others: an id no word has)
                        pid[0] = pw;
#pragma unroll
                        for (int k = 0; k < KC - 1; ++k) {
                            uint32_t pv = 0u;
                            if (KEXACT || (uint32_t)k < N) pv = prev[k];
                            pid[k + 1] = (pv >> kIdBits) ? (pv & kIdMask) : 0xFFFFFFFFu;
                        }
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk) {
                            const uint32_t id = kk ? nid[kk - 1] : (uint32_t)my_w;
                            bool hit = false;
#pragma unroll
                            for (int k = 0; k < KC; ++k) hit = hit || pid[k] == id;
                            if (kk && nmult[kk - 1] == 0u) hit = false;
                            if (hit) reload |= 1u << kk;
                        }
                    } else {
                        const uint32_t *mine = cb_pack + (size_t)lane * N;
                        for (uint32_t kk = 0; kk < (uint32_t)KC && kk <= N; ++kk) {
                            uint32_t id;
                            if (kk == 0) id = (uint32_t)my_w;
                            else { const uint32_t p = mine[kk - 1]; if ((p >> kIdBits) == 0) continue; id = p & kIdMask; }
                            bool hit = id == pw;
                            for (uint32_t k = 0; k < N && !hit; ++k) hit = (prev[k] >> kIdBits) != 0 && (prev[k] & kIdMask) == id;
                            if (hit) reload |= 1u << kk;
                        }
                    }
                }
                // Context slots of my window (slot c <-> distance (c>>1)+1, right side if c is odd) get a 4-bit
                // weight: 0 for a slot whose position does not exist, 0 for a slot whose word comes again in a
                // later slot (dupmask), and for the last slot of a word the number of slots that hold it.  Slots
                // of one word share one ring row and one set of dot products, so the last one stands for all.
                // The words of all slots are fetched once; a slot outside the width or the sentence gets a
                // value of its own that no word has, so the unrolled comparisons need no further tests.
                const uint32_t me = i0 + lane;
                int32_t sw[NCTX];
                uint32_t exist = 0;
#pragma unroll
                for (int c = 0; c < NCTX; ++c) {
                    const uint32_t a = (uint32_t)(c >> 1) + 1u;
                    const uint32_t p = (c & 1) ? me + a : me - a;
                    const bool ok = a <= my_b && ((c & 1) ? p < n_prod : me >= a);
                    sw[c] = -2 - c;
                    if (ok) { sw[c] = kw[p & (FQ - 1)]; exist |= 1u << c; }
                }
                uint32_t cm[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int c = 0; c < NCTX; ++c) {
                    bool later = false;
                    uint32_t m = 1u;
#pragma unroll
                    for (int c2 = c + 1; c2 < NCTX; ++c2) later = later || sw[c2] == sw[c];
#pragma unroll
                    for (int c2 = 0; c2 < c; ++c2) m += (sw[c2] == sw[c]) ? 1u : 0u;
                    if ((exist >> c) & 1u) {
                        if (later) dupmask |= 1u << c;
                        else {
                            if (m > 15u) overflow = 1u;
                            cm[c >> 3] |= (m & 15u) << (4 * (c & 7));
                        }
                    }
                }
                // special: some slot inside the width is absent, or two slots hold one word
                const uint32_t inside = (my_b >= 16u) ? 0xFFFFFFFFu : ((1u << (2u * my_b)) - 1u);
                special = (exist != inside || dupmask != 0u) ? 1u : 0u;
                if (overflow) dupmask = 0u;      // pathological repetition: every slot stays on, rows are added to atomically
                reinterpret_cast<uint4 *>(cb_cm)[lane] = make_uint4(cm[0], cm[1], cm[2], cm[3]);
            }
            // Negatives shared by a stretch of tokens stay in registers from one window to the next: window j
            // "hands over" to window j+1 when both are ordinary windows of one stretch (straight-line path, every
            // negative distinct and different from either target, some context to train on).  The handing window
            // skips the stores of its negative rows, the receiving one skips their fetch.
            uint32_t hand_over = 0;
            if constexpr (!MULTI && !SUMMED && !BF16) {
                const uint32_t ok = (have && A.neg_shift && my_b != 0u && my_plain && !overflow && n_prod > 1u) ? 1u : 0u;
                const uint32_t mine = (my_stretch << 1) | ok;
                const uint32_t next = (uint32_t)__shfl_down((int)mine, 1, kLanes);
                const uint32_t prev = (uint32_t)__shfl_up((int)mine, 1, kLanes);
                hand_over = (ok && (uint32_t)lane + 1u < nwin && next == mine) ? 1u : 0u;
                const bool receive = ok && lane > 0 && prev == mine;
                if (receive) reload &= 1u;       // only my target row can have been rewritten in memory by the previous window
            }
            if (have)
                cb_meta[lane] = make_uint4(my_b | (reload << 8) | (overflow << 16) | (my_plain << 17) | (special << 18) |
                                               ((my_b == 0u ? 1u : 0u) << 19) | (hand_over << 20),
                                           (uint32_t)my_w, my_enter, dupmask);
            __syncthreads();

            // ---- first chunk of a sentence: positions 0..W enter the ring before the first window ----
            if (i0 == 0) {
                const uint32_t want = (W + 1 < n_prod) ? W + 1 : n_prod;
                while (n_ins < want) {
                    const int32_t word = (int32_t)uni((uint32_t)kw[n_ins & (FQ - 1)]);
                    uint32_t slot;
                    if (ring_enter(n_ins, word, slot)) {
                        float t[E];
                        load_ctx((uint32_t)word, t);
                        widen_row(t);
                        regs_to_ring(ring + (size_t)slot * ROWF, t);
                        if (sum_ring) snap_store(slot, t);
                    }
                    ++n_ins;
                }
            }

            // ---- the chunk's windows, strictly in order -----------------------------------------
            // scalars and output rows of the first window; later windows get theirs one window ahead
            uint4 mraw = cb_meta[0];
            uint32_t packv = 0;
            if (lane_k0 >= 1 && (KFULL || (uint32_t)lane_k0 <= N)) packv = cb_pack[lane_k0 - 1];
            if (lane_k0 == 0) packv = mraw.y | (1u << kIdBits);
            float O[KC][E];
            const bool first_idle = (uni(mraw.x) >> 19) & 1u;
#pragma unroll
            for (int kk = 0; kk < KC; ++kk) {
                const uint32_t pk = lane_value(packv, (uint32_t)kk);
#pragma unroll
                for (int x = 0; x < E; ++x) O[kk][x] = 0.0f;
                if (!first_idle && (KFULL || (uint32_t)kk <= N)) load_out(pk & kIdMask, O[kk]);
            }
            // The rows of the chunk's first window are waited for here, once per 64 windows.  Without this wait the
            // registers of O carry loads in flight into the window loop on one of its two entry paths, the compiler's
            // wait-count bookkeeping merges the paths conservatively, and every window gets a full vmcnt(0) in front of
            // its first multiply-add: right behind the prefetch of the next window's rows, which then hides nothing.
            __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0), the other counters left alone
            if constexpr (BF16 && !TWO) {
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) widen_row(O[kk]);
            }

            for (uint32_t j = 0; j < nwin; ++j) {
                const uint32_t i = i0 + j;
                const uint32_t b = uni(mraw.x) & 0xFFu;
                const bool shared_rows = (uni(mraw.x) >> 16) & 1u;
                const bool plain = (uni(mraw.x) >> 17) & 1u;
                const bool special = (uni(mraw.x) >> 18) & 1u;
                const uint32_t dupmask = uni(mraw.w);
                const uint32_t enter_word = uni(mraw.z);
                const bool has_next = j + 1 < nwin;

                // The pairing a lane handles after the reduction.  In the shapes under register pressure (windows wider
                // than 5, two passes over the output rows, five floats per lane) it is taken through an empty asm
                // statement once per window: the compiler then forms what follows from it (labels, weights, addresses
                // and shifts of the slot weights, one set per block of every width) where it is used, two or three
                // instructions each, instead of computing all of it once at kernel entry, where it filled some twenty
                // registers that were spilled; a reload from scratch waits behind every row prefetch in flight
                // (vector memory operations complete in order), which cost those shapes 2 to 5 % of their time.  The
                // other shapes spill nothing on the window path and are 1 to 2 % faster with the values hoisted.
                uint32_t lane_c = (uint32_t)lane_c0, lane_k = (uint32_t)lane_k0;
                if constexpr (WCAP > 5 || MULTI || E > 4) asm volatile("" : "+v"(lane_c), "+v"(lane_k));
                uint64_t win_draw = 0ull, leave_draw_j = 0ull;      // bfloat16 storage: this window's rounding draws
                if constexpr (DRAWS_IN_LDS) {
                    const uint4 r = cb_rnd[j];
                    win_draw = uni64(((uint64_t)r.y << 32) | r.x);
                    leave_draw_j = uni64(((uint64_t)r.w << 32) | r.z);
                } else if constexpr (BF16) {
                    win_draw = leave_draw(i);
                    if (i >= W) leave_draw_j = leave_draw(i - W);
                }
                // bfloat16 storage, two passes: the window's first batch of rows was fetched into O as words (between the
                // passes of the window before, or at the chunk start) and becomes floats here
                if constexpr (BF16 && TWO) {
#pragma unroll
                    for (int kk = 0; kk < KC; ++kk) widen_row(O[kk]);
                }
                // (a) ask LDS for the next window's scalars now, use them after the ring work below
                uint4 mraw_next = make_uint4(0u, 0u, kNoWord, 0u);
                uint32_t pack_next = 0;
                if (has_next) {
                    mraw_next = cb_meta[j + 1];
                    if (lane_k >= 1 && (KFULL || (uint32_t)lane_k <= N)) pack_next = cb_pack[(size_t)(j + 1) * N + (lane_k - 1)];
                }

                // (b) the kept position i+W+1 enters the span: its row is fetched now and written into
                //     the ring after this window's arithmetic
                uint32_t pend_slot = 0;
                bool pend = false;
                float pend_row[E] = {};
                if (enter_word != kNoWord) {
                    pend = ring_enter(n_ins, (int32_t)enter_word, pend_slot);
                    if (pend) load_ctx(enter_word, pend_row);
                    ++n_ins;
                }
                //     summed mode: the position that leaves the span after this window is known now; what memory holds
                //     of its row and the slot's snapshot are requested here and used in step (h)
                bool lv = false, lv_summed = false;
                uint32_t lv_slot = 0, lv_word = 0;
                float lv_fresh[SUMMED ? E : 1] = {}, lv_snap[SUMMED ? E : 1] = {};
                if constexpr (SUMMED) {
                    if (sum_ring && i >= W) {
                        lv = leave_decide(i - W, lv_slot, lv_word);
                        if (lv) {
                            lv_summed = true;
                            if (lv_summed) { load_row(A.syn0, lv_word, lv_fresh); snap_load(lv_slot, lv_snap); }
                        }
                    }
                }

                // (c) contexts of this window: slot c <-> distance a=(c>>1)+1, right side if c odd;
                //     amask bit c set when that position exists and lies within the width
                const uint32_t nl = (b < i) ? b : i;
                const uint32_t nr = (b < n_prod - 1 - i) ? b : n_prod - 1 - i;
                const uint32_t amask_all = uni((0x55555555u & (uint32_t)((1ull << (2 * nl)) - 1ull)) | (0xAAAAAAAAu & (uint32_t)((1ull << (2 * nr)) - 1ull)));
                const uint32_t nact = nl + nr;
                const uint32_t amask = amask_all & ~dupmask;          // slots that take part

                // (d) the next window's output rows start their trip from memory
                uint32_t packv_next = pack_next;
                float On[KC][E];
                //     (negative rows that this window hands over in registers are not fetched).
                //     Windows with two passes over their output rows fetch them between the passes instead.
                const bool hand_over = !MULTI && ((uni(mraw.x) >> 20) & 1u);
                auto fetch_next_window = [&](auto &dst) {
                    if (has_next && !((uni(mraw_next.x) >> 19) & 1u)) {
                        if (lane_k == 0) packv_next = mraw_next.y | (1u << kIdBits);
                        if (hand_over) {                        // one branch, two straight-line variants
                            load_out(lane_value(packv_next, 0u) & kIdMask, dst[0]);
                        } else {
#pragma unroll
                            for (int kk = 0; kk < KC; ++kk) {
                                const uint32_t pk = lane_value(packv_next, (uint32_t)kk);
#pragma unroll
                                for (int x = 0; x < E; ++x) dst[kk][x] = 0.0f;
                                if (KFULL || (uint32_t)kk <= N) load_out(pk & kIdMask, dst[kk]);
                            }
                        }
                    }
                };
                if constexpr (!TWO) fetch_next_window(On);
                else if (nact == 0) fetch_next_window(O);

                // Called when the window's last pass is about to store its output rows.  Everything fetched so far (the
                // entering context row, the next window's rows; summed mode: the fresh row and the snapshot of the
                // position that leaves) has had the window's arithmetic to arrive and is waited for HERE, before this
                // window's stores are issued: vector memory operations complete in order and the compiler's waits are
                // all-or-nothing where paths merge, so a wait placed after the stores also waits for their
                // acknowledgements.  After this point the loop waits for nothing that has a store in front of it.
                auto arrivals_before_stores = [&](bool window_done) {
                    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0), the other counters left alone
                    if (pend) {
                        widen_row(pend_row);
                        regs_to_ring(ring + (size_t)pend_slot * ROWF, pend_row);
                        if (sum_ring) snap_store(pend_slot, pend_row);
                        pend = false;
                    }
                    if constexpr (SUMMED) {      // (the leaving row has received all of the window's deltas only then)
                        if (window_done && sum_ring && lv) { leave_finish(lv_slot, lv_word, lv_summed, lv_fresh, lv_snap, 0ull); lv = false; }
                    }
                };

                // (e) the window's arithmetic over context slots 0..NCW-1.
                //     GENERAL = false: straight-line code for the common window: all NCW slots exist, no two
                //     of them share a ring row, every negative is distinct and differs from the target.
                //     GENERAL = true: slot c takes part only if bit c of amask is set (windows cut by a
                //     sentence end), multiplicities are honoured, shared ring rows are added to.
                auto do_window = [&](auto ncw_tag, auto general_tag) {
                    constexpr int NCW = decltype(ncw_tag)::value;
                    constexpr bool MASKED = decltype(general_tag)::value;
                    constexpr bool GENERAL = MASKED;
                    // the NCW slots are handled in NQW blocks of nearly equal size (BASE or BASE+1 slots)
                    constexpr int NQW = (NCW + CCK - 1) / CCK;
                    constexpr int BASE = NCW / NQW, REM = NCW % NQW;
                    // Straight-line windows whose output rows are handled in one pass take the context rows out of
                    // the ring block by block (fewer rows live at a time): no two slots that take part share a row,
                    // so a block never sees an earlier block's update.  Otherwise (several passes, or rows that
                    // are added to by several slots) every dot product needs the rows as they were when the
                    // window began, and all of them are fetched first.
                    constexpr bool LOAD_PER_BLOCK = !MULTI && !MASKED && NQW > 1;
                    float I[NCW][E];
                    uint32_t cslot[NCW];
                    auto fetch_slot = [&](auto c_tag) {
                        constexpr int c = decltype(c_tag)::value;
                        cslot[c] = 0;
#pragma unroll
                        for (int x = 0; x < E; ++x) I[c][x] = 0.0f;
                        if (!MASKED || ((amask >> c) & 1u)) {
                            const uint32_t a = (uint32_t)(c >> 1) + 1u;
                            const uint32_t p = (c & 1) ? i + a : i - a;
                            cslot[c] = lane_value(meta_slot, p & 63u);
                            if (!MASKED && !((amask_all >> c) & 1u)) cslot[c] = nslots;    // absent: the zero row
                            ring_to_regs(ring + (size_t)cslot[c] * ROWF, I[c]);
                        }
                    };
                    if constexpr (!LOAD_PER_BLOCK) static_for<NCW>(fetch_slot);
                    // One pass: the KC output rows held in OB (ids in pv, rows kb .. kb+KC-1 of the window) against
                    // all context slots.
                    // bfloat16 storage: the centre's draw keys the rounding of this window's output rows
                    auto out_bits = [&](uint32_t tag) -> uint64_t { return BF16 ? row_key(win_draw, tag) : 0ull; };
                    auto run_pass = [&](uint32_t kb, auto &OB, uint32_t pv, bool early_wait, bool last) {
                        const uint32_t gk = kb + lane_k;
                        const float mult_lane = (KEXACT || gk <= N) ? (GENERAL ? (float)(pv >> kIdBits) : 1.0f) : 0.0f;
                        const float label = (gk == 0) ? 1.0f : 0.0f;
                        const float gscale = GENERAL ? alpha * mult_lane : alpha;
                        float dO[KC][E];
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk)
#pragma unroll
                            for (int x = 0; x < E; ++x) dO[kk][x] = 0.0f;
                        // summed mode: what memory holds of the output rows now is fetched into registers of its own
                        // when the last block of context slots begins, so that the block's arithmetic covers the trip,
                        // and takes the deltas in step (f)
                        bool fresh_loaded = false;
                        float FR[SUMMED ? KC : 1][SUMMED ? E : 1];
                        auto load_fresh = [&]() {
                            if constexpr (SUMMED) {
#pragma unroll
                                for (int kk = 0; kk < KC; ++kk) {
                                    const uint32_t pk = lane_value(pv, (uint32_t)kk);
#pragma unroll
                                    for (int x = 0; x < E; ++x) FR[kk][x] = 0.0f;
                                    if ((KEXACT || kb + kk <= N) && (!GENERAL || (pk >> kIdBits))) load_out(pk & kIdMask, FR[kk]);
                                }
                            }
                            fresh_loaded = true;
                        };

                        static_for<NQW>([&](auto q_tag) {
                            // NC context rows (slots C0 .. C0+NC-1) against the KC output rows
                            constexpr int q = decltype(q_tag)::value;
                            constexpr int NC = (q < REM) ? BASE + 1 : BASE;
                            constexpr int C0 = q * BASE + (q < REM ? q : REM);
                            if (MASKED && !(amask >> C0)) return;       // no slot from here on takes part
                            if constexpr (SUMMED && q == NQW - 1) load_fresh();
                            if constexpr (LOAD_PER_BLOCK)
                                static_for<NC>([&](auto cc_tag) { fetch_slot(std::integral_constant<int, C0 + decltype(cc_tag)::value>{}); });
                            float acc[CCK * KC];
#pragma unroll
                            for (int cc = 0; cc < CCK; ++cc) {
                                const int c = C0 + cc;
#pragma unroll
                                for (int kk = 0; kk < KC; ++kk) {
                                    float p = 0.0f;
                                    if (cc < NC && (!MASKED || ((amask >> c) & 1u))) {
#pragma unroll
                                        for (int x = 0; x < E; ++x) p = __builtin_fmaf(I[c][x], OB[kk][x], p);
                                    }
                                    acc[cc * KC + kk] = p;
                                }
                            }
                            const float xraw = (q < REM) ? transpose_reduce<(REM ? BASE + 1 : BASE) * KC>(acc, lane)
                                                         : transpose_reduce<BASE * KC>(acc, lane);
                            bool act = lane < NC * KC && (GENERAL ? mult_lane > 0.0f : (KEXACT || gk <= N));
                            float cmult = 1.0f;                      // how many context positions this slot stands for
                            {
                                const uint32_t gc = (uint32_t)(C0 + lane_c);
                                if (MASKED) act = act && gc < 32u && ((amask >> gc) & 1u);
                                if ((MASKED ? dupmask != 0u : special) && gc < 32u) {
                                    cmult = (float)((cb_cm[4 * j + (gc >> 3)] >> (4u * (gc & 7u))) & 15u);
                                    if (!MASKED) act = act && cmult > 0.0f;
                                }
                            }
                            // sigmoid and log-loss from u = 1 + exp(-x): sigma = 1/u, -log sigma(x) = log u,
                            // -log sigma(-x) = x + log u   (x clamped where exp would overflow)
                            // (hardware exp2 / log2 / rcp: about 1 ulp each, far inside the parity budget)
                            const float xv = __builtin_amdgcn_fmed3f(xraw, -80.0f, 80.0f);
                            const float u = 1.0f + __builtin_amdgcn_exp2f(xv * -1.44269504088896341f);
                            const float g = act ? gscale * cmult * (label - __builtin_amdgcn_rcpf(u)) : 0.0f;
                            if (act) {
                                const float l1 = __builtin_fmaf(__builtin_amdgcn_logf(u), 0.693147180559945309f, (gk == 0) ? 0.0f : xv);
                                loss_acc += (double)(GENERAL ? mult_lane * cmult * l1 : cmult * l1);
                            }
                            // every lane needs every g: straight-line windows take it through the row-broadcast
                            // operand of the multiply-adds, the general path through scalar registers
                            float G[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                            if constexpr (!MASKED) rows_to_all<(NC * KC + 15) / 16>(g, G);
                            // the deltas of both sides from the block's gradients: DO_I / DO_O say which side(s) this
                            // sweep over the block forms (one sweep for both, except the summed mode's last block)
                            auto sweep = [&](auto do_i_tag, auto do_o_tag) {
                            constexpr bool DO_I = decltype(do_i_tag)::value, DO_O = decltype(do_o_tag)::value;
                            static_for<CCK>([&](auto cc_tag) {
                                constexpr int cc = decltype(cc_tag)::value;
                                constexpr int c = C0 + cc;
                                if constexpr (cc < NC) if (!MASKED || ((amask >> c) & 1u)) {
                                    float dI[E];
#pragma unroll
                                    for (int x = 0; x < E; ++x) dI[x] = 0.0f;
                                    static_for<KC>([&](auto kk_tag) {
                                        constexpr int kk = decltype(kk_tag)::value;
                                        constexpr int v = cc * KC + kk;         // lane that holds this pairing's g
                                        if constexpr (!MASKED) {
#pragma unroll
                                            for (int x = 0; x < E; ++x) {
                                                if constexpr (DO_I) {
                                                    if (kk == 0) dI[x] = mul_row_lane<v % 16>(G[v / 16], OB[kk][x]);
                                                    else fma_row_lane<v % 16>(dI[x], G[v / 16], OB[kk][x]);
                                                }
                                                if constexpr (DO_O) {
                                                    if (q == 0 && cc == 0) dO[kk][x] = mul_row_lane<v % 16>(G[v / 16], I[c][x]);
                                                    else fma_row_lane<v % 16>(dO[kk][x], G[v / 16], I[c][x]);
                                                }
                                            }
                                        } else {
                                            const float gs = lane_value(g, (uint32_t)v);
#pragma unroll
                                            for (int x = 0; x < E; ++x) {
                                                if constexpr (DO_I) dI[x] = __builtin_fmaf(gs, OB[kk][x], dI[x]);
                                                if constexpr (DO_O) dO[kk][x] = __builtin_fmaf(gs, I[c][x], dO[kk][x]);
                                            }
                                        }
                                    });
                                    if constexpr (!DO_I) return;
                                    float *dst = ring + (size_t)cslot[c] * ROWF;
                                    if (GENERAL && shared_rows) {
                                        // positions that share a ring row add up (LDS float add)
                                        chunks([&](auto r_, auto w_, auto o_) {
                                            constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
#pragma unroll
                                            for (int x = 0; x < CW; ++x)
                                                __hip_atomic_fetch_add(dst + eoff[r] + x, dI[RO + x], __ATOMIC_RELAXED,
                                                                       __HIP_MEMORY_SCOPE_WAVEFRONT);
                                        });
                                    } else if (MULTI && kb) {
                                        // later output chunks: the row already carries the earlier chunks' deltas
                                        chunks([&](auto r_, auto w_, auto o_) {
                                            constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
                                            float t[CW];
                                            load_vec<CW>(dst + eoff[r], t);
#pragma unroll
                                            for (int x = 0; x < CW; ++x) t[x] += dI[RO + x];
                                            store_vec<CW>(dst + eoff[r], t);
                                        });
                                    } else {
                                        // the row still equals the copy in registers: plain write of copy + delta
                                        chunks([&](auto r_, auto w_, auto o_) {
                                            constexpr int r = decltype(r_)::value, CW = decltype(w_)::value, RO = decltype(o_)::value;
                                            float t[CW];
#pragma unroll
                                            for (int x = 0; x < CW; ++x) t[x] = I[c][RO + x] + dI[RO + x];
                                            store_vec<CW>(dst + eoff[r], t);
                                        });
                                    }
                                }
                            });
                            };
                            using std::true_type;
                            using std::false_type;
                            sweep(true_type{}, true_type{});
                        });

                        // (f) output rows go back (lock-free) once per window
                        if (early_wait) arrivals_before_stores(last);
                        if (hand_over) {
                            // the negatives' rows stay in registers for the next window (every row exists and
                            // counts once in a window that hands over)
                            float t[E];
#pragma unroll
                            for (int x = 0; x < E; ++x) t[x] = OB[0][x] + dO[0][x];
                            store_out(lane_value(pv, 0u) & kIdMask, t, out_bits(0u));
#pragma unroll
                            for (int kk = 1; kk < KC; ++kk)
#pragma unroll
                                for (int x = 0; x < E; ++x) OB[kk][x] += dO[kk][x];
                        } else {
                            if constexpr (SUMMED) { if (!fresh_loaded) load_fresh(); }
#pragma unroll
                            for (int kk = 0; kk < KC; ++kk) {
                                const uint32_t pk = lane_value(pv, (uint32_t)kk);
                                if ((KEXACT || kb + kk <= N) && (!GENERAL || (pk >> kIdBits))) {
                                    float t[E];
#pragma unroll
                                    for (int x = 0; x < E; ++x) {
                                        if constexpr (SUMMED) t[x] = FR[kk][x] + dO[kk][x];
                                        else t[x] = OB[kk][x] + dO[kk][x];
                                    }
                                    store_out(pk & kIdMask, t, out_bits(kb + (uint32_t)kk));
                                }
                            }
                        }
                    };
                    if constexpr (!MULTI) {
                        run_pass(0u, O, packv, true, true);
                    } else if constexpr (TWO) {
                        // two passes: the second batch of rows travels into On while the first batch is worked on,
                        // and the next window's first batch travels into O while the second is worked on
                        const uint32_t gk2 = (uint32_t)KC + lane_k;
                        const uint32_t pv2 = (gk2 <= N) ? cb_pack[(size_t)j * N + (gk2 - 1)] : 0u;
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk) {
                            const uint32_t pk = lane_value(pv2, (uint32_t)kk);
#pragma unroll
                            for (int x = 0; x < E; ++x) On[kk][x] = 0.0f;
                            if ((uint32_t)KC + kk <= N) load_out(pk & kIdMask, On[kk]);
                        }
                        // (the early wait sits before the first pass's stores: the second batch is needed right after
                        // it anyway; before the second pass's stores it would wait for the next window's first batch,
                        // which has only had the second pass to arrive: measured 2 % slower than letting the next
                        // window wait for it)
                        run_pass(0u, O, packv, true, false);
                        fetch_next_window(O);
                        if constexpr (BF16) {
#pragma unroll
                            for (int kk = 0; kk < KC; ++kk) widen_row(On[kk]);
                        }
                        run_pass((uint32_t)KC, On, pv2, false, true);
                    } else {
                        for (uint32_t kb = 0; kb <= N; kb += KC) {
                            uint32_t pv = packv;
                            if (kb) {                               // further output rows: fetched here
                                const uint32_t gk = kb + lane_k;
                                pv = (gk <= N) ? cb_pack[(size_t)j * N + (gk - 1)] : 0u;
#pragma unroll
                                for (int kk = 0; kk < KC; ++kk) {
                                    const uint32_t pk = lane_value(pv, (uint32_t)kk);
#pragma unroll
                                    for (int x = 0; x < E; ++x) O[kk][x] = 0.0f;
                                    if (kb + kk <= N) load_out(pk & kIdMask, O[kk]);
                                }
                            }
                            run_pass(kb, O, pv, kb + (uint32_t)KC > N, kb + (uint32_t)KC > N);
                        }
                    }
                };
                if (nact) {
                    pairs_acc += nact;
                    using std::integral_constant;
                    using T = integral_constant<bool, true>;
                    using F = integral_constant<bool, false>;
#define W2V_WIN(NCV) do_window(integral_constant<int, (NCV)>{}, F{})
                    bool done = false;
                    if (plain && !shared_rows) {
                        // straight-line code per width; absent and repeated slots carry weight 0
                        done = true;
                        switch (b) {
                        case 1: W2V_WIN(2); break;
                        case 2: W2V_WIN(4); break;
                        case 3: W2V_WIN(6); break;
                        case 4: W2V_WIN(8); break;
                        case 5: W2V_WIN(10); break;
                        default: done = false; break;
                        }
                        if constexpr (WCAP >= 10) {
                            if (!done) {
                                done = true;
                                switch (b) {
                                case 6: W2V_WIN(12); break;
                                case 7: W2V_WIN(14); break;
                                case 8: W2V_WIN(16); break;
                                case 9: W2V_WIN(18); break;
                                case 10: W2V_WIN(20); break;
                                default: done = false; break;
                                }
                            }
                        }
                    }
#undef W2V_WIN
                    if (!done) do_window(integral_constant<int, NCTX>{}, T{});   // anything else
                } else {
                    // a position without context (a lead-in token, a sentence of one kept word): nothing to compute,
                    // but the same wait, so that every path through the window has made it before the paths join
                    arrivals_before_stores(true);
                }

                // (g) rows of the next window that this window has just rewritten are fetched again
                //     (a load issued after a store of the same wavefront sees the stored data)
                if (has_next) {
                    const uint32_t reload = nact ? ((uni(mraw_next.x) >> 8) & 0x3Fu) : 0u;
                    if (reload) {
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk)
                            if ((reload >> kk) & 1u) {
                                const uint32_t pk = lane_value(packv_next, (uint32_t)kk);
                                load_out(pk & kIdMask, TWO ? O[kk] : On[kk]);
                            }
                        // (rare; waited for at once, so that where this path joins the other no register of the next
                        // window's rows has a load in flight: the compiler would wait for the stores above as well)
                        __builtin_amdgcn_s_waitcnt(0x0F70);
                    }
                }

                // (h) the fetched context row enters the ring, the oldest position leaves it
                //     (every lane only touches its own elements of a ring row: no barrier needed)
                if (pend) {
                    widen_row(pend_row);
                    regs_to_ring(ring + (size_t)pend_slot * ROWF, pend_row);
                    if (sum_ring) snap_store(pend_slot, pend_row);
                }
                if constexpr (SUMMED) {
                    if (sum_ring) { if (lv) leave_finish(lv_slot, lv_word, lv_summed, lv_fresh, lv_snap, 0ull); }
                    else if (i >= W) ring_leave(i - W, 0ull);
                } else {
                    if (i >= W) ring_leave(i - W, leave_draw_j);
                }

                // (i) next window's scalars and rows become current
                if (has_next) {
                    mraw = mraw_next;
                    packv = packv_next;
                    if constexpr (!TWO) {
                        if (hand_over) {
#pragma unroll
                            for (int x = 0; x < E; ++x) O[0][x] = On[0][x];
                        } else {
#pragma unroll
                            for (int kk = 0; kk < KC; ++kk) {
                                if constexpr (BF16) {
                                    widen_into(O[kk], On[kk]);        // the rows arrive as words and become floats here
                                } else {
#pragma unroll
                                    for (int x = 0; x < E; ++x) O[kk][x] = On[kk][x];
                                }
                            }
                        }
                    }
                }
            }
            i0 += nwin;
        }
        kept_acc += n_own - n_lead;

        // ---- sentence done: the rows still in the ring go back -------------------------------------
        {
            const uint32_t first = (n_own > W) ? n_own - W : 0u;     // positions < first left already
            if (sum_ring) {
                // four rows at a time: their loads travel together
                uint32_t p = first;
                while (p < n_ins) {
                    uint32_t sl[4], wd[4];
                    bool on[4], sm[4];
                    float fr[4][E], sn[4][E];
                    static_for<4>([&](auto b_) {
                        constexpr int b = decltype(b_)::value;
                        on[b] = false;
                        if (p < n_ins) { on[b] = leave_decide(p, sl[b], wd[b]); ++p; }
                    });
                    static_for<4>([&](auto b_) {
                        constexpr int b = decltype(b_)::value;
                        sm[b] = on[b];
                        if (sm[b]) { load_row(A.syn0, wd[b], fr[b]); snap_load(sl[b], sn[b]); }
                    });
                    static_for<4>([&](auto b_) {
                        constexpr int b = decltype(b_)::value;
                        if (on[b]) leave_finish(sl[b], wd[b], sm[b], fr[b], sn[b], 0ull);
                    });
                }
            } else {
                for (uint32_t p = first; p < n_ins; ++p) ring_leave(p, leave_draw(p));
            }
        }
        __syncthreads();
    }

    const double lsum = wave_sum(loss_acc);
    const unsigned long long dsum = (unsigned long long)wave_sum((double)dropped_acc);
    if (lane == 0) {
        atomicAdd(&A.accum->loss_sum, lsum);
        atomicAdd(&A.accum->pairs, pairs_acc);
        atomicAdd(&A.accum->kept, kept_acc);
        if (dsum) atomicAdd(&A.accum->dropped, dsum);
    }
}

}  // namespace
}  // namespace w2v
