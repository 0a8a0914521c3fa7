// Layout of an operand packed for the block-scaled matrix instruction, and the per-lane conversion of int8 mantissas
// into it; shared by the pack kernel (gemm_mx.hip) and by the conversion kernel that packs what it has just converted
// (encode_pack.hip).  Each translation unit gets its own copy.
//
// Packed operand: [panel of 256 rows][k-step of 64][row tile of 32][limb planes, most significant first | scale words].
// Lane l of a row tile stands for operand row (l % 32) and the 32 k of half (l / 32) of the k-step: the 32 codes
// of a limb are 192 bits, code e in bits 6 e .. 6 e + 5, stored at [l * 24] of the limb plane; the scale word of the
// lane holds the exponent byte of limb j in byte j.
#pragma once
#include "gemm_common.h"

namespace hbfp {
namespace {

struct __attribute__((aligned(4))) Bytes12 {   // 12 bytes stored at a 4-byte aligned address
    uint32_t a, b, c;
};

// limbs of 4 magnitude bits that a mantissa of m bits (sign included) needs
inline int limbs_of(int m) { return m <= 5 ? 1 : m <= 9 ? 2 : 3; }

constexpr int kLimbBytes = 1536;                 // one limb of 32 rows x 64 k: 24 bytes per lane
constexpr int kScaleBytes = 256;                 // [64 lanes] one word: exponent byte of limb j in byte j
constexpr int kRowTiles = 8;                     // 32-row tiles per 256-row panel
__host__ __device__ constexpr int chunk_bytes(int L) { return L * kLimbBytes + kScaleBytes; }
__host__ __device__ constexpr int panel_stage_bytes(int L) { return kRowTiles * chunk_bytes(L); }   // a multiple of 2048

// Scale bytes of the limbs of one group of 32 codes with stored exponent byte E; `bad` if one is out of range.
template <int L>
__device__ __forceinline__ uint32_t mx_scale_word(int E, int m, bool &bad) {
    E = E > 254 ? 254 : E;
    uint32_t word = 0;
    bad = false;
#pragma unroll
    for (int j = 0; j < L; ++j) {
        int byte = E + 5 + 4 * (L - 1 - j) - m;
        if (byte < 0 || byte > 254) {
            bad = true;
            byte = byte < 0 ? 0 : 254;
        }
        word |= (uint32_t)byte << (8 * j);
    }
    return word;
}

// ------------------------------------------------------------------------------------------------
// Dense layout for exponent blocks of 8, 16 or 24 elements.  Such blocks are STORED padded to 32, and packing them as
// stored would make a quarter (24), half (16) or three quarters (8) of the matrix instructions multiply zeros.  The
// instruction scales groups of 32 codes, but an E2M3 code carries two exponent bits of its own: the integer n * 2^d
// (n in 0..15, d in 0..2) is still a code.  So the k axis is packed without the padding, a group of 32 consecutive
// elements takes the SMALLEST exponent among its (two to four) blocks as its scale, and the elements of a block whose
// exponent is d binades above it are stored as n * 2^d: the same numbers, exactly (and one more binade comes for
// free where the mantissas leave a spare bit in their limbs, see pack_half_group_dense).  A group whose non-zero
// blocks are further apart cannot be written that way; it marks the operand's header like an exponent out of range,
// and the int8 kernels queued behind the product compute it from the stored operand.  For values drawn from one
// normal distribution, block maxima 4 binades apart do not occur in practice (3 apart: about once in 3 million
// groups of config 4's operands); heavy-tailed gradients do take the fallback.  Both operands of a product
// pack k the same way (the rule depends on the block length alone).
//
// Unit of the mapping is the octet (8 consecutive elements; block lengths are multiples of 8): octet j of the dense
// axis lies in block j / ob at offset 8 * (j % ob), i.e. at stored position 32 * (j / ob) + 8 * (j % ob).
__device__ __forceinline__ uint32_t dense_block_of(uint32_t j, int ob) {
    return ob == 3 ? __umulhi(j, 0xAAAAAAABu) >> 1 : ob == 2 ? j >> 1 : j;
}
// the code of twice the value of each byte's code: normal codes (>= 8) gain one in their exponent field (+ 8),
// subnormal codes (< 8) double as integers (7 -> 14 is the normal code of 14 / 8)
// 0xff in every byte whose bit 0 is set in `ones` (a value of 0 or 1 per byte) in two instructions; written as
// (ones << 8) - ones the compiler turns it back into a 32-bit multiplication by 255 with its constant in a register
__device__ __forceinline__ uint32_t byte_mask(uint32_t ones) { return (0x80808080u - ones) ^ 0x80808080u; }
__device__ __forceinline__ uint32_t e2m3_double_bytes(uint32_t c) {
    const uint32_t normal = ((c + 0x78787878u) >> 7) & 0x01010101u;   // 1 in the bytes that hold a code >= 8
    return c + (normal << 3) + (c & ~byte_mask(normal));
}

// One lane's share of a densely packed group: 16 consecutive elements of the unpadded k axis as two octets, raw[o]
// their 8 int8 mantissas and E[o] the exponent byte of the block octet o lies in, or 255 when the octet holds no
// non-zero mantissa (it then takes any exponent).  Lanes q and q ^ 1 of a quad hold the two halves of a group of 32:
// q even the first 16.  Writes this lane's 12 bytes of every limb plane of the row tile at `chunk` (lane `lo` of the
// matrix instruction: operand row + 32 * half of the k-step) and, from the even lane, the group's scale word.
// Returns true when the group cannot be expressed (blocks more than 3 binades apart, 2 for 5-bit mantissas, or a scale
// byte out of range).
//
// An octet d binades above the group's exponent holds its magnitudes times 2^d.  When the mantissas leave a spare bit
// in their limbs (m <= 4 L: 8-bit mantissas in two limbs, 4-bit ones in one) the first binade costs nothing: twice the
// magnitude still splits into L limbs of 4 bits.  What remains goes into the exponent bits of the codes
// (e2m3_double_bytes), which only a few groups need then.
template <int L>
__device__ __forceinline__ bool pack_half_group_dense(const v2i (&raw)[2], const int (&E)[2], int m, uint8_t *chunk, int lo, int q) {
    int emin = E[0] < E[1] ? E[0] : E[1];
    const int other = __builtin_amdgcn_update_dpp(0, emin, 0xB1, 0xF, 0xF, false);   // quad_perm [1, 0, 3, 2]
    emin = other < emin ? other : emin;
    const bool empty = emin == 255;                       // the whole group is zero
    bool far = false;
    uint32_t g[L][4];
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        const int d = E[o] == 255 ? 0 : E[o] - emin;
        const int sh = (m <= 4 * L && d > 0) ? 1 : 0;                     // binades taken by doubling the magnitudes
        const int dbl = d - sh;                                           // and by doubling the codes: at most two
        far = far || dbl > 2;
        uint32_t w[L][2], sign[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint32_t x = (uint32_t)raw[o][i];
            const uint32_t sg = (x >> 7) & 0x01010101u;                   // 1 in the bytes of negative mantissas
            const uint32_t a = ((x ^ byte_mask(sg)) + sg) << sh;        // magnitudes, byte by byte
            sign[i] = sg << 5;
#pragma unroll
            for (int j = 0; j < L; ++j) w[j][i] = (a >> (4 * (L - 1 - j))) & 0x0f0f0f0fu;   // limb j of four mantissas, one per byte
        }
        if (dbl > 0) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < L; ++j) w[j][i] = e2m3_double_bytes(w[j][i]);
        }
        if (dbl > 1) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < L; ++j) w[j][i] = e2m3_double_bytes(w[j][i]);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < L; ++j) {
                const uint32_t c = w[j][i] | sign[i];
                const uint32_t t = (c & 0x003f003fu) | ((c >> 2) & 0x0fc00fc0u);              // two 12-bit pairs
                g[j][2 * o + i] = (t & 0xfffu) | ((t >> 4) & 0xfff000u);                      // four 6-bit codes in 24 bits
            }
    }
    bool bad = false;
    const uint32_t word = empty ? 0u : mx_scale_word<L>(emin, m, bad);
#pragma unroll
    for (int j = 0; j < L; ++j) {
        const Bytes12 three = {g[j][0] | (g[j][1] << 24), (g[j][1] >> 8) | (g[j][2] << 16), (g[j][2] >> 16) | (g[j][3] << 8)};
        *reinterpret_cast<Bytes12 *>(chunk + j * kLimbBytes + lo * 24 + (q & 1) * 12) = three;
    }
    if ((q & 1) == 0) *reinterpret_cast<uint32_t *>(chunk + L * kLimbBytes + lo * 4) = word;
    return far || (!empty && bad);
}

}  // namespace
}  // namespace hbfp
