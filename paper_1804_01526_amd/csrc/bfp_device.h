// Device-side arithmetic of the FP32 -> BFP conversion (Sec. 4.1, Sec. 5.3).
// The public header states the number format and the stochastic-rounding hash.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hbfp {

// Counter hash of the element's logical index; the xorshift triple is the generator
// Sec. 5.3 names, the two multiply rounds make consecutive counters independent.
__device__ __forceinline__ uint32_t sr_hash(uint32_t lo, uint32_t hi, uint32_t s0, uint32_t s1) {
    uint32_t x = lo ^ s0;
    x ^= x << 13;
    x ^= x >> 17;
    x ^= x << 5;
    x += hi ^ s1;
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

// Shared exponent byte from the largest magnitude bit pattern of a block.  Adding
// the rounding increment to the bit pattern carries into the exponent field
// exactly when the rounded maximum would need one more magnitude bit.
template <int ROUND>
__device__ __forceinline__ uint32_t block_exponent(uint32_t amax_bits, int m) {
    const int sh0 = 25 - m;
    const uint32_t rb = ROUND ? ((1u << sh0) - 1u) : (1u << (sh0 - 1));
    uint32_t e = (amax_bits + rb) >> 23;  // amax_bits < 2^31, no wrap
    e = e < 1u ? 1u : e;
    return e > 255u ? 255u : e;
}

// Round to nearest even through the FP32 adder: x * 2^-(unit exponent) is exact, and
// adding 1.5 * 2^23 rounds it to an integer held in the low mantissa bits (two's
// complement for negative x).  |q| <= 2^15 here, far inside the trick's 2^22 range.
__device__ __forceinline__ int quant_rne(float x, int neg_unit_exp) {
    const float y = __builtin_amdgcn_ldexpf(x, neg_unit_exp);
    const float t = y + 12582912.0f;
    return __float_as_int(t) - 0x4B400000;
}

// Stochastic rounding: q = floor(|x| / unit + h / 2^32), sign applied afterwards, where an element whose significand
// would have to move right by more than 32 bits becomes 0.  |x| / unit is exact in FP32 (a power-of-two scaling), its
// integer part is the mantissa before rounding and its fraction, scaled by 2^32, is an exact integer below 2^32
// whenever the shift is at most 32 bits; the carry of fraction + h is the rounding decision.  With
// sh = 25 - m + Eb - (exponent field of x, at least 1) this is the definition
//     q = (sig + (h >> (32 - sh))) >> sh   (sh <= 31),   carry of sig + h   (sh = 32),   0   (sh > 32)
// bit for bit: the bits of h that the definition drops before adding are a fraction below one unit of sig and cannot
// change the floor.  neg_unit_exp = 125 + m - Eb; small_bits: bit patterns below it need more than 32 bits of shift.
__device__ __forceinline__ uint32_t sr_small_bits(uint32_t Eb, int m) {
    const int t = (int)Eb - 7 - m;                 // elements whose exponent field (at least 1) is below t vanish
    return t <= 1 ? 0u : (uint32_t)t << 23;
}
// the rounded magnitude, at most 2^(m-1) - 1
__device__ __forceinline__ uint32_t quant_sr_magnitude(float x, int neg_unit_exp, uint32_t small_bits, uint32_t h) {
    const uint32_t bits = __float_as_uint(x);
    const float ax = (bits & 0x7fffffffu) < small_bits ? 0.0f : __builtin_fabsf(x);
    const float y = __builtin_amdgcn_ldexpf(ax, neg_unit_exp);
    const uint32_t whole = (uint32_t)y;                                                // truncation: y >= 0
    const uint32_t frac = (uint32_t)__builtin_amdgcn_ldexpf(__builtin_amdgcn_fractf(y), 32);
    return whole + ((frac + h) < h ? 1u : 0u);
}
__device__ __forceinline__ int quant_sr(float x, int neg_unit_exp, uint32_t small_bits, uint32_t h) {
    const uint32_t q = quant_sr_magnitude(x, neg_unit_exp, small_bits, h);
    const uint32_t sgn = (uint32_t)((int32_t)__float_as_uint(x) >> 31);
    return (int)((q ^ sgn) - sgn);
}
// Two magnitudes (each below 2^15) with the signs of two floats, as two 16-bit two's-complement halves of one word:
// the sign words come from the floats' upper halves with one byte permute and one packed shift, and the conditional
// negation (m ^ s) - s runs on both halves at once.
typedef short v2s16 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t signed_pair16(uint32_t mag0, uint32_t mag1, float x0, float x1) {
    const uint32_t mags = __builtin_amdgcn_perm(mag1, mag0, 0x05040100u);                                       // mag0.lo16, mag1.lo16
    const uint32_t tops = __builtin_amdgcn_perm(__float_as_uint(x1), __float_as_uint(x0), 0x07060302u);        // x0.hi16, x1.hi16
    const v2s16 s = __builtin_bit_cast(v2s16, tops) >> (short)15;
    const v2s16 r = __builtin_bit_cast(v2s16, mags ^ __builtin_bit_cast(uint32_t, s)) - s;
    return __builtin_bit_cast(uint32_t, r);
}

// The hash in two parts.  Its first three steps (the xorshift triple) are linear over GF(2), so the part of the
// counter that is common to a run of elements can be pushed through them once: for counters c0 + e with c0 a
// multiple of 8 and e < 8, c0 + e = c0 ^ e and triple(c0 ^ e ^ s0) = triple(c0 ^ s0) ^ triple(e).
__host__ __device__ constexpr uint32_t sr_triple(uint32_t x) {
    x ^= x << 13;
    x ^= x >> 17;
    x ^= x << 5;
    return x;
}
// after_triple: the counter's low word ^ s0 after the three xorshift steps; high_term = (high word of the counter) ^ s1
__device__ __forceinline__ uint32_t sr_hash_tail(uint32_t after_triple, uint32_t high_term) {
    uint32_t x = after_triple + high_term;
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

template <int ROUND>
__device__ __forceinline__ int quantise(float x, uint32_t Eb, int m, uint32_t idx_lo, uint32_t idx_hi,
                                        uint32_t s0, uint32_t s1) {
    if (ROUND == 0) return quant_rne(x, 125 + m - (int)Eb);
    return quant_sr(x, 125 + m - (int)Eb, sr_small_bits(Eb, m), sr_hash(idx_lo, idx_hi, s0, s1));
}

}  // namespace hbfp
