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

// Stochastic rounding in integer arithmetic on the bit pattern.  shbase = 25 - m + Eb, so the shift
// sh = shbase - (element's exponent) is at least 25 - m >= 9.  The definition
//     q = (sig + (h >> (32 - sh))) >> sh   (sh <= 31),   carry of sig + h   (sh = 32),   0   (sh > 32)
// equals bits 32 and up of (sig << (32 - sh)) + h for every sh <= 32: the bits of h dropped before the
// sum of the definition are a fraction below one unit of sig and cannot change the floor.  So one
// add-with-carry serves all cases; a zero (padding) value always gives 0.
__device__ __forceinline__ int quant_sr(uint32_t bits, int shbase, uint32_t h) {
    const uint32_t a = bits & 0x7fffffffu;
    const uint32_t be = a >> 23;
    uint32_t sig = be ? ((a & 0x7fffffu) | 0x800000u) : a;
    const int sh = shbase - (int)(be ? be : 1u);
    sig = sh > 32 ? 0u : sig;
    const uint32_t lo = sig << ((32 - sh) & 31);
    const uint32_t hi = (sig >> 8) >> ((sh - 8) & 31);
    const uint32_t q = hi + ((lo + h) < h ? 1u : 0u);
    const uint32_t sgn = (uint32_t)((int32_t)bits >> 31);
    return (int)((q ^ sgn) - sgn);
}

template <int ROUND>
__device__ __forceinline__ int quantise(float x, uint32_t Eb, int m, uint32_t idx_lo, uint32_t idx_hi,
                                        uint32_t s0, uint32_t s1) {
    if (ROUND == 0) return quant_rne(x, 125 + m - (int)Eb);
    return quant_sr(__float_as_uint(x), 25 - m + (int)Eb, sr_hash(idx_lo, idx_hi, s0, s1));
}

}  // namespace hbfp
