// Counter-based random numbers of the SGNS trainer (host and device).
//
// Every random decision is a pure function of (seed, epoch, global token position, draw index),
// so it is the same whichever wavefront handles the sentence and however many run at once.
// The mixer is the output function of the SplitMix64 generator (Steele, Lea, Flood 2014).
//   key   = mix64(seed + G*(epoch+1))
//   base  = mix64(key ^ mix64(position))
//   draw  = mix64(base + G*(index+1));   the high 32 bits are used
//   index 0: subsampling decision, 1: window width, 2+k: negative k,
//   64: the 64 bits S that key the stochastic roundings of the rows written for this position (bfloat16 storage).
//   The key of one row is row_key(S, t): both halves of S times odd constants of the tag t (0 the window's target
//   row, 1+k its negative k, 32 the token's own context row when it leaves the span); multiplying by an odd number
//   permutes the 32-bit words, so the halves of a key stay uniform and independent of each other.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define W2V_HD __host__ __device__ __forceinline__
#else
#define W2V_HD inline
#endif

namespace w2v {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

W2V_HD constexpr uint64_t mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

W2V_HD uint64_t epoch_key(uint64_t seed, uint32_t epoch) { return mix64(seed + kGolden * ((uint64_t)epoch + 1u)); }
W2V_HD uint64_t position_base(uint64_t key, uint64_t pos) { return mix64(key ^ mix64(pos)); }
W2V_HD uint32_t draw_u32(uint64_t base, uint32_t index) { return (uint32_t)(mix64(base + kGolden * ((uint64_t)index + 1u)) >> 32); }
W2V_HD uint64_t draw_u64(uint64_t base, uint32_t index) { return mix64(base + kGolden * ((uint64_t)index + 1u)); }
W2V_HD constexpr uint64_t row_key(uint64_t draw, uint32_t tag)
{
    const uint64_t m = mix64(0x6B6579ull + tag);
    const uint32_t lo = (uint32_t)draw * ((uint32_t)m | 1u);
    const uint32_t hi = (uint32_t)(draw >> 32) * ((uint32_t)(m >> 32) | 1u);
    return ((uint64_t)hi << 32) | lo;
}
W2V_HD uint32_t mul_hi_u32(uint32_t a, uint32_t n) { return (uint32_t)(((uint64_t)a * (uint64_t)n) >> 32); }

// subsampling: threshold 0xFFFFFFFF keeps always, otherwise keep iff draw < threshold
W2V_HD bool keep_decision(uint64_t base, uint32_t threshold)
{
    return threshold == 0xFFFFFFFFu || draw_u32(base, 0) < threshold;
}

// window width: uniform on 1..W (mode 0), ceil(W/2) (mode 1), or W itself (mode 2: the caller has already
// replaced W by the fixed width)
W2V_HD uint32_t window_width(uint64_t base, uint32_t W, uint32_t mode)
{
    return mode == 2u ? W : (mode == 1u ? (W + 1u) / 2u : 1u + mul_hi_u32(draw_u32(base, 1), W));
}

// slot of the sampling table that negative k of this position reads
W2V_HD uint32_t negative_slot(uint64_t base, uint32_t k, uint32_t table_size)
{
    return mul_hi_u32(draw_u32(base, 2u + k), table_size);
}

}  // namespace w2v
