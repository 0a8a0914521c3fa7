// Layout of an operand packed for the bf16 product kernel, and the per-lane conversion of stored mantissas into it;
// shared by the pack kernel and the product kernel (gemm_bf.hip) and by the conversion kernel that packs what it has
// just converted (encode_pack.hip).  Each translation unit gets its own copy.
//
// A BFP value with a mantissa of at most 9 bits (sign included) is a bf16 number: its magnitude has at most 8
// significant bits and mant * 2^(E - 125 - m) keeps the 8-bit exponent range of the stored exponent byte.  So an
// operand of the 6..9-bit class is packed as the bf16 values of its elements (Eq. (1) applied once, exactly), the
// matrix instruction multiplies 8-bit significands and adds exponents as the block arithmetic of Eq. (2) prescribes,
// and nothing has to be scaled per block.
//
// Packed operand: [panel of 256 rows][k-step of 32][row tile of 32][half h of the k-step][lane][8 bf16].
// Lane l of a half stands for operand row (l % 32) and the 8 k at 16 h + 8 (l / 32): the operand registers of one
// v_mfma_f32_32x32x16_bf16, 16 bytes per lane, 1 KB per half, read from LDS with one 16-byte read per lane.
// Exponent blocks of 8, 16 or 24 elements, which are STORED padded to 32, are packed without their padding (octet j of
// the packed k axis lies in block j / ob at offset 8 (j % ob), ob octets per block); the packed k axis is padded with
// zeros to a multiple of 128.
#pragma once
#include "gemm_common.h"

namespace hbfp {
namespace {

typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kBfTileBytes = 2048;                // 32 rows x 32 k
constexpr int kBfStageBytes = 8 * kBfTileBytes;   // a panel of 256 rows, one k-step

// mantissa widths packed as bf16 planes: below, one 4-bit limb on the block-scaled instruction is twice as fast;
// above, the significand does not fit
inline bool bf_class(int m) { return m >= 6 && m <= 9; }
// octets per exponent block when the packed k axis leaves out the padding of the stored blocks, else 0
inline int bf_dense_octets(int64_t kbp, int64_t kblock, int m) {
    return (kbp == 32 && kblock < 32 && kblock % 8 == 0 && m <= 8) ? (int)(kblock / 8) : 0;
}
// octets of a densely packed row: those of all blocks, less the ones of the last block that lie wholly behind the end
// of the contraction
inline int64_t bf_dense_row_octets(int ob, int64_t nblk, int64_t kdim) {
    const int64_t all = nblk * ob, used = (kdim + 7) / 8;
    return kdim > 0 && used < all ? used : all;
}
// length of the packed k axis (a multiple of 128)
inline int64_t bf_klen(int64_t kpad, int64_t kbp, int64_t kblock, int64_t nblk, int64_t kdim, int m) {
    const int ob = bf_dense_octets(kbp, kblock, m);
    return ob ? (bf_dense_row_octets(ob, nblk, kdim) * 8 + 127) / 128 * 128 : kpad;
}
inline size_t bf_packed_bytes(int64_t rows, int64_t kpad) { return 256 + (size_t)((rows + 255) / 256) * 256 * (size_t)kpad * 2; }

__device__ __forceinline__ uint32_t bf_dense_block_of(uint32_t j, int ob) {
    return ob == 3 ? __umulhi(j, 0xAAAAAAABu) >> 1 : ob == 2 ? j >> 1 : j;
}

// byte offset of the 16 bytes of (row tile rt of the operand, k-step ks of 32, half h, wave half lh, row r32 of the tile)
__device__ __forceinline__ int64_t bf_piece_offset(int64_t rt, int64_t ks, int64_t ksteps, int h, int lh, int r32) {
    return (((rt >> 3) * ksteps + ks) * 8 + (rt & 7)) * kBfTileBytes + h * 1024 + lh * 512 + r32 * 16;
}

// An exponent byte above 253 (values from 2^127 on) could take an element beyond the largest bf16 number; the operand is
// then marked and the int8 kernels compute the product.  Small exponents need nothing: the matrix instruction takes
// subnormal bf16 operands and accumulates subnormal FP32 sums exactly.
__device__ __forceinline__ bool bf_exponent_ok(int E) { return E <= 253; }

// two mantissas times 2^shift as bf16 numbers in one word (the conversions are exact: at most 8 significant bits)
__device__ __forceinline__ uint32_t bf_pair(int lo, int hi, int shift) {
    const float a = __builtin_ldexpf((float)lo, shift), b = __builtin_ldexpf((float)hi, shift);
    return __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x07060302u);
}
// an octet of int8 mantissas (8 bytes) with exponent byte E and mantissa width m
__device__ __forceinline__ v4u bf_octet_i8(const v2i &raw, int E, int m) {
    const int shift = E - 125 - m;
    v4u out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int w = raw[i >> 1] >> (16 * (i & 1));
        out[i] = bf_pair((int)(int8_t)w, (int)(int8_t)(w >> 8), shift);
    }
    return out;
}
// an octet of int16 mantissas (16 bytes)
__device__ __forceinline__ v4u bf_octet_i16(const v4i &raw, int E, int m) {
    const int shift = E - 125 - m;
    v4u out;
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = bf_pair((int)(int16_t)raw[i], raw[i] >> 16, shift);
    return out;
}

// ------------------------------------------------------------------------------------------------
// Mantissas of 10 to 12 bits do not fit a bf16 significand, but they fit an FP16 one (11 bits), and FP16's narrow
// exponent range is enough once every operand row is taken relative to its own largest block exponent Eref: an element
// becomes mant * 2^(E - Eref + 4), at most 2^15 in magnitude, exact in FP16 (subnormals included) as long as its block
// lies no more than 28 binades below the row's largest, and the row's factor 2^(Eref - 4 - 125 - m) is applied to the
// FP32 sums when they are stored.  Same planes as above with FP16 elements, preceded by one scale word per row:
// [256-byte header][rows padded to 256: int32 Eref - 129 - m][planes].  A non-zero block further down marks the operand.
constexpr int kF16Lift = 4;
constexpr int kF16MinShift = -24;                 // weight of the last bit of an FP16 subnormal
inline size_t f16_scale_bytes(int64_t rows) { return (size_t)((rows + 255) / 256) * 256 * 4; }
inline size_t f16_packed_bytes(int64_t rows, int64_t kpad) { return 256 + f16_scale_bytes(rows) + (size_t)((rows + 255) / 256) * 256 * (size_t)kpad * 2; }
// an octet of int16 mantissas times 2^shift as FP16 numbers (exact for shift >= kF16MinShift)
__device__ __forceinline__ v4u f16_octet_i16(const v4i &raw, int shift) {
    v4u out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a = __builtin_ldexpf((float)(int)(int16_t)raw[i], shift), b = __builtin_ldexpf((float)(raw[i] >> 16), shift);
        out[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
    }
    return out;
}

}  // namespace
}  // namespace hbfp
