// BFP matrix product on the block-scaled matrix instruction of gfx950 (Eq. (2) of Sec. 4 with the
// per-block FP accumulation of Sec. 4 / Sec. 4.2 "Tiling"):
//     C[i][j] = sum_b 2^(eA[i][b] + eB[j][b]) * sum_{k in b} mA[i][k] * mB[j][k]
//
// v_mfma_scale_f32_32x32x64_f8f6f4 is a BFP dot-product unit in hardware: every lane hands it 32
// narrow values along k together with one shared 8-bit exponent, it multiplies the narrow values,
// applies 2^(sA + sB - 254) per pair of 32-element groups and accumulates in FP32.  The per-block
// scaling that costs the int8 kernels two vector instructions per output and block is free here.
// Its narrow values are floats, the widest significand at the fast rate being 4 bits (FP6 E2M3, twice
// the int8 rate), so a mantissa is cut into limbs of 4 magnitude bits:
//     |v| = sum_i n_i * 16^i,  n_i in 0..15,  limb i stored as the E2M3 code (sign << 5) | n_i = +-n_i / 8
// (codes 0..7 are the subnormals n/8, codes 8..15 the first binade (1 + (n-8)/8), so the code of an
// integer n in 0..15 is n itself: an E2M3 plane is a plane of sign-magnitude 4-bit fixed-point numbers).
// Limb products are exact (8 bits), a group of 32 sums exactly inside the instruction, and each limb pair
// gets its own exponent byte  E + 5 + 4 i - m  (E the stored block exponent, m the mantissa width), so
// LA x LB matrix instructions per k-step of 64 accumulate the full product straight into the FP32
// accumulator: 8-bit mantissas take 2 x 2, 12-bit mantissas 3 x 3, mantissas of at most 5 bits 1 x 1.
//
// pack kernel:  stored operand (int8 / int16 mantissas [rows][kpad], exponent bytes) -> limb planes in
//               the register order of the matrix instruction, 256 operand rows x 64 k at a time, so the
//               product kernel moves whole stages with contiguous asynchronous copies and every fragment
//               read is three conflict-free 8-byte LDS reads per lane (lanes 24 bytes apart cover all 64 banks).
// gemm_mx_kernel: 256 x 256 tile of C per workgroup, 8 waves of 64 x 128, three-stage LDS ring, one
//               barrier per k-step, fragment reads one column tile ahead of the matrix instructions that use them
//               and issued between the matrix instructions of the column tile before.
// An exponent byte outside 0..254 (blocks below 2^-120 or above 2^126) cannot be expressed; the pack
// kernel then marks the header of the packed operand, the product kernel does nothing when either header
// is marked and the int8 kernels, launched behind it with the opposite condition, compute the product instead.
// A packed operand (header + limb planes) stays valid until the operand is encoded again, so weights are
// packed once per update and serve every product until the next.
#include <atomic>
#include <chrono>

#include "bfp_device.h"
#include "mx_out.h"
#include "mx_pack.h"

namespace hbfp {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
constexpr int kMxThreads = 512;

// ------------------------------------------------------------------------------------------------
// Packed operand: [panel of 256 rows][k-step of 64][row tile of 32][limb planes, most significant first | scale words].
// Lane l of a row tile stands for operand row (l % 32) and the 32 k of half (l / 32) of the k-step: the 32 codes
// of a limb are 192 bits, code e in bits 6 e .. 6 e + 5, stored at [l * 24] of the limb plane.
struct PackParams {
    const void *mant;
    const uint8_t *exps;
    uint8_t *out;
    int *header;                 // first 256 bytes of the packed operand: word 1 = this pack's mark, word 0 = the mark of
                                 // the last pack that found an exponent byte out of range
    int64_t R, kpad, exp_ld;
    int32_t ksteps, nks4, chunks32_per_block, m;
    int32_t mark;
    int32_t ob, noct;            // dense layout: octets (8 elements) per exponent block and in the whole row; ob = 0: padded layout
};

// int8 mantissas: a lane converts 16 consecutive mantissas (one 16-byte load; the 4 lanes of a row read its 64 bytes
// of the k-step, so a wave instruction reads 16 whole 64-byte pieces) into the 12 bytes they occupy in each limb plane.
template <int L>
__device__ __forceinline__ void mx_pack_block_i8(const PackParams &p, uint32_t block) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (block == 0 && threadIdx.x == 0) p.header[1] = p.mark;
    const int64_t rt = block / p.nks4;
    const int ks = (int)(block % p.nks4) * 4 + wave;
    if (ks >= p.ksteps) return;
    const int q = lane & 3;                                   // quarter of the k-step: 16 mantissas
    const int kb = 2 * ks + (q >> 1);                         // 32-element chunk of the stored row
    uint8_t *chunk = p.out + (((rt >> 3) * p.ksteps + ks) * kRowTiles + (rt & 7)) * (int64_t)chunk_bytes(L);
    v4i raw[2];
    int E[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int64_t row = rt * 32 + h * 16 + (lane >> 2);
        const int64_t rs = row < p.R ? row : 0;               // rows past the end read row 0 and store zeros
        raw[h] = *reinterpret_cast<const v4i *>(reinterpret_cast<const int8_t *>(p.mant) + rs * p.kpad + (int64_t)ks * 64 + q * 16);
        E[h] = p.exps[rs * p.exp_ld + kb / p.chunks32_per_block];
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = h * 16 + (lane >> 2);
        const bool live = rt * 32 + r < p.R;
        // four mantissas per register at a time: |v| byte-wise (v = -128 does not occur), limbs and signs as bytes,
        // then the four 6-bit codes of a register squeezed into 24 bits and four such groups laid end to end
        uint32_t g[L][4], any = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t x = live ? (uint32_t)raw[h][i] : 0u;
            const uint32_t sg = (x >> 7) & 0x01010101u;                   // 1 in the bytes of negative mantissas
            const uint32_t a = (x ^ byte_mask(sg)) + sg;                  // byte-wise two's complement negation
            any |= a;
#pragma unroll
            for (int j = 0; j < L; ++j) {
                const uint32_t w = ((a >> (4 * (L - 1 - j))) & 0x0f0f0f0fu) | (sg << 5);       // codes, one per byte
                const uint32_t t = (w & 0x003f003fu) | ((w >> 2) & 0x0fc00fc0u);              // two 12-bit pairs
                g[j][i] = (t & 0xfffu) | ((t >> 4) & 0xfff000u);
            }
        }
        bool bad;
        const uint32_t word = live ? mx_scale_word<L>(E[h], p.m, bad) : (bad = false, 0u);
        if (bad && any) p.header[0] = p.mark;                 // all-zero groups (padding) take any exponent
        const int lo = r + 32 * (q >> 1);                     // the lane of the matrix instruction that owns these codes
#pragma unroll
        for (int j = 0; j < L; ++j) {
            const Bytes12 three = {g[j][0] | (g[j][1] << 24), (g[j][1] >> 8) | (g[j][2] << 16), (g[j][2] >> 16) | (g[j][3] << 8)};
            *reinterpret_cast<Bytes12 *>(chunk + j * kLimbBytes + lo * 24 + (q & 1) * 12) = three;
        }
        if ((q & 1) == 0) *reinterpret_cast<uint32_t *>(chunk + L * kLimbBytes + lo * 4) = word;
    }
}

template <int L>
__device__ __forceinline__ void mx_pack_block_i8_dense(const PackParams &p, uint32_t block) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (block == 0 && threadIdx.x == 0) p.header[1] = p.mark;
    const int64_t rt = block / p.nks4;
    const int ks = (int)(block % p.nks4) * 4 + wave;
    if (ks >= p.ksteps) return;
    const int q = lane & 3;                                   // quarter of the k-step: 16 elements = 2 octets
    uint8_t *chunk = p.out + (((rt >> 3) * p.ksteps + ks) * kRowTiles + (rt & 7)) * (int64_t)chunk_bytes(L);
    v2i raw[2][2];
    int E[2][2];
    // all loads first (mantissas and exponent bytes side by side), then the conversion
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int64_t row = rt * 32 + h * 16 + (lane >> 2);
        const bool live = row < p.R;
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            const uint32_t j = (uint32_t)ks * 8u + (uint32_t)q * 2u + (uint32_t)o;
            const bool there = live && j < (uint32_t)p.noct;
            const uint32_t b = there ? dense_block_of(j, p.ob) : 0u;
            const int64_t rs = there ? row : 0;               // octets that do not exist read the first one and become zero
            raw[h][o] = *reinterpret_cast<const v2i *>(reinterpret_cast<const int8_t *>(p.mant) + rs * p.kpad + (int64_t)b * 32 +
                                                       (there ? 8 * (int)(j - b * (uint32_t)p.ob) : 0));
            E[h][o] = p.exps[rs * p.exp_ld + b];
            if (!there) raw[h][o] = v2i{0, 0};
        }
    }
    bool bad = false;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int o = 0; o < 2; ++o) E[h][o] = (raw[h][o][0] | raw[h][o][1]) ? (E[h][o] > 254 ? 254 : E[h][o]) : 255;
        const int r = h * 16 + (lane >> 2);
        bad |= pack_half_group_dense<L>(raw[h], E[h], p.m, chunk, r + 32 * (q >> 1), q);
    }
    if (bad) p.header[0] = p.mark;
}

template <int L, typename MT>
__device__ __forceinline__ void mx_pack_block(const PackParams &p, uint32_t block) {
    if constexpr (sizeof(MT) == 1) {
        if (p.ob) mx_pack_block_i8_dense<L>(p, block);
        else mx_pack_block_i8<L>(p, block);
        return;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (block == 0 && threadIdx.x == 0) p.header[1] = p.mark;
    const int64_t rt = block / p.nks4;
    const int ks = (int)(block % p.nks4) * 4 + wave;
    if (ks >= p.ksteps) return;
    const int64_t row = rt * 32 + (lane & 31);
    const int kb = 2 * ks + (lane >> 5);                      // 32-element chunk of the stored row
    uint32_t limb[L][6];
#pragma unroll
    for (int j = 0; j < L; ++j)
#pragma unroll
        for (int d = 0; d < 6; ++d) limb[j][d] = 0;
    uint32_t word = 0;
    if (row < p.R) {
        constexpr int NV = 32 * (int)sizeof(MT) / 16;
        v4i raw[NV];
        const MT *src = reinterpret_cast<const MT *>(p.mant) + row * p.kpad + (int64_t)kb * 32;
#pragma unroll
        for (int i = 0; i < NV; ++i) raw[i] = reinterpret_cast<const v4i *>(src)[i];
        uint32_t any = 0;
        {
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                const int v = (int)(int16_t)((uint32_t)raw[e >> 3][(e >> 1) & 3] >> (16 * (e & 1)));
                const uint32_t s = v < 0 ? 32u : 0u;
                const uint32_t a = (uint32_t)(v < 0 ? -v : v);
                any |= a;
#pragma unroll
                for (int j = 0; j < L; ++j) {
                    const uint32_t code = s | ((a >> (4 * (L - 1 - j))) & 15u);
                    const int bit = 6 * e;
                    limb[j][bit >> 5] |= code << (bit & 31);
                    if ((bit & 31) > 26) limb[j][(bit >> 5) + 1] |= code >> (32 - (bit & 31));
                }
            }
        }
        bool bad;
        word = mx_scale_word<L>(p.exps[row * p.exp_ld + kb / p.chunks32_per_block], p.m, bad);
        if (bad && any) p.header[0] = p.mark;                 // all-zero groups (padding) take any exponent
    }
    uint8_t *chunk = p.out + (((rt >> 3) * p.ksteps + ks) * kRowTiles + (rt & 7)) * (int64_t)chunk_bytes(L);
#pragma unroll
    for (int j = 0; j < L; ++j) {
#pragma unroll
        for (int d = 0; d < 3; ++d) {
            const v2i two = {(int)limb[j][2 * d], (int)limb[j][2 * d + 1]};
            *reinterpret_cast<v2i *>(chunk + j * kLimbBytes + lane * 24 + d * 8) = two;
        }
    }
    *reinterpret_cast<uint32_t *>(chunk + L * kLimbBytes + lane * 4) = word;
}

// both operands of a product in one launch: the first blocks_a workgroups pack A, the rest B
struct PackPair {
    PackParams op[2];
    uint32_t blocks_a;
};
template <int LA, int LB, typename MT>
__global__ __launch_bounds__(256) void mx_pack_kernel(const PackPair q) {
    if (blockIdx.x < q.blocks_a) mx_pack_block<LA, MT>(q.op[0], blockIdx.x);
    else mx_pack_block<LB, MT>(q.op[1], blockIdx.x - q.blocks_a);
}

// under graph capture a pack is replayed with the same mark: the out-of-range word is reset first
__global__ void mx_clear_flag_kernel(int *header_a, int *header_b) {
    if (threadIdx.x == 0) {
        if (header_a) header_a[0] = 0;
        if (header_b) header_b[0] = 0;
    }
}

// ------------------------------------------------------------------------------------------------
struct MxParams {
    const uint8_t *pa, *pb;      // limb planes of the packed operands
    const int *ha, *hb;          // their headers: words 0 and 1 equal = outside the range of the scale bytes
    float *C;
    int64_t M, N, ldc;
    int32_t ksteps, tiles_m, tiles_n, beta;
};

// Up to kMxGroup independent products in one launch (the data-gradient and weight-gradient products of a layer, the
// products of several layers or micro-batches): workgroups first[i] .. first[i + 1] - 1 belong to product i.  A
// CU that finishes a tile of one product goes on with a tile of the next, so the stores of the first drain under the
// matrix instructions of the second; launched one by one, every product ends with all CUs storing at once.
constexpr int kMxGroup = 4;

// Workgroups behind the tiles (kMxWordWgs per product that has a job): they prepare the scale words of the 8-wave int8
// kernel that stands by behind this launch, and only if that kernel is going to run (an operand is marked); otherwise
// they are gone at once.  This keeps the stand-by path at one launch without tying it to the slower kernel that
// reads exponent bytes itself.
constexpr int kMxWordWgs = 64;
struct MxGroup {
    MxParams p[kMxGroup];
    int32_t first[kMxGroup + 1];
    int32_t n;
    int32_t word_jobs;           // bit i: product i has a scale-word job
    MxOut out;                   // of product 0 of a launch with a single product
    WordParams words[kMxGroup];
};

// The product kernel is a set of macros over its local arrays (function templates taking the fragment arrays by
// reference left them in scratch memory).
// Fragment registers: af[buffer][row tile][3 * limb + piece], bf[buffer][3 * limb + piece]: the codes of a lane are read
// 8 bytes at a time, limb l at l * kLimbBytes; as / bs are the scale words.
#define HBFP_MX_READ_A1(buf, i, base_)                                                                                      \
    {                                                                                                                      \
        _Pragma("unroll") for (int l = 0; l < LA; ++l)                                                                     \
            _Pragma("unroll") for (int d = 0; d < 3; ++d)                                                                  \
                af[buf][i][3 * l + d] =                                                                                    \
                    *reinterpret_cast<const v2i *>((base_) + abase[ONE_A ? 0 : (i)][l] + (ONE_A ? (i) * CHA : 0) + d * 8); \
        as[buf][i] = *reinterpret_cast<const int *>((base_) + a4 + (i) * CHA);                                             \
    }
#define HBFP_MX_READ_A(buf, base_)                                                                                          \
    {                                                                                                                      \
        HBFP_MX_READ_A1(buf, 0, base_);                                                                                    \
        HBFP_MX_READ_A1(buf, 1, base_);                                                                                    \
    }
#define HBFP_MX_READ_B(buf, j, base_)                                                                                       \
    {                                                                                                                      \
        _Pragma("unroll") for (int l = 0; l < LB; ++l)                                                                     \
            _Pragma("unroll") for (int d = 0; d < 3; ++d)                                                                  \
                bf[buf][3 * l + d] = *reinterpret_cast<const v2i *>((base_) + bbase[l] + (j) * CHB + d * 8);               \
        bs[buf] = *reinterpret_cast<const int *>((base_) + b4 + (j) * CHB);                                                \
    }
// Two-limb fragments in pieces, so that the reads of the next column tile can be issued between the matrix
// instructions of the current one (a wave that finds the LDS queue full then still has matrix instructions in flight)
#define HBFP_MX_READ_B_PIECE(buf, j, base_, FIRST, LAST, SCALE)                                                             \
    {                                                                                                                      \
        _Pragma("unroll") for (int x = (FIRST); x <= (LAST); ++x)                                                          \
            bf[buf][x] = *reinterpret_cast<const v2i *>((base_) + bbase[x / 3] + (j) * CHB + (x % 3) * 8);                 \
        if (SCALE) bs[buf] = *reinterpret_cast<const int *>((base_) + b4 + (j) * CHB);                                     \
    }
// the builtin takes 8 registers per operand and drops the last two for this format
#define HBFP_MX_MFMA(abuf, bbuf, JA, JB, i, j)                                                                              \
    {                                                                                                                      \
        const v8i av_ = {af[abuf][i][3 * (JA)][0],     af[abuf][i][3 * (JA)][1],     af[abuf][i][3 * (JA) + 1][0],         \
                         af[abuf][i][3 * (JA) + 1][1], af[abuf][i][3 * (JA) + 2][0], af[abuf][i][3 * (JA) + 2][1], 0, 0};  \
        const v8i bv_ = {bf[bbuf][3 * (JB)][0],     bf[bbuf][3 * (JB)][1],     bf[bbuf][3 * (JB) + 1][0],                  \
                         bf[bbuf][3 * (JB) + 1][1], bf[bbuf][3 * (JB) + 2][0], bf[bbuf][3 * (JB) + 2][1], 0, 0};           \
        /* TR: operands exchanged, the 32 x 32 result arrives transposed (same products, same sums) */                    \
        if (TR) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bv_, av_, acc[i][j], 2, 2, JB, bs[bbuf], JA, as[abuf][i]); \
        else acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av_, bv_, acc[i][j], 2, 2, JA, as[abuf][i], JB, bs[bbuf]); \
    }
// limb pair (JA, JB) of column tile j for both row tiles, which alternate so that a matrix instruction never waits
// for the one just before it; then this pair's share of the stage copies, if the k-step hands over a buffer
#define HBFP_MX_PAIR(abuf, bbuf, JA, JB, j, COPY)                                                                           \
    {                                                                                                                      \
        HBFP_MX_MFMA(abuf, bbuf, JA, JB, 0, j);                                                                            \
        HBFP_MX_MFMA(abuf, bbuf, JA, JB, 1, j);                                                                            \
        if (COPY) {                                                                                                        \
            constexpr int slot = (JA) * LB + (JB), per = (NCOPY + LA * LB - 1) / (LA * LB);                                \
            _Pragma("unroll") for (int c_ = slot * per; c_ < (slot + 1) * per && c_ < NCOPY; ++c_) {                       \
                async_copy16(cptr[c_], voff, copy_ring * STAGE + coff[c_]);                                                \
                cptr[c_] += cstep[c_];                                                                                     \
            }                                                                                                              \
        }                                                                                                                  \
    }
// PART 0: every limb pair of column tile j;  1: only the first pair;  2: all but the first
#define HBFP_MX_COLUMN(abuf, bbuf, j, COPY, PART)                                                                           \
    {                                                                                                                      \
        constexpr int A1 = LA > 1 ? 1 : 0, A2 = LA > 2 ? 2 : 0, B1 = LB > 1 ? 1 : 0, B2 = LB > 2 ? 2 : 0;                  \
        if (PART != 2) HBFP_MX_PAIR(abuf, bbuf, 0, 0, j, COPY);                                                            \
        if (PART != 1) {                                                                                                   \
            if (LB > 1) HBFP_MX_PAIR(abuf, bbuf, 0, B1, j, COPY);                                                          \
            if (LB > 2) HBFP_MX_PAIR(abuf, bbuf, 0, B2, j, COPY);                                                          \
            if (LA > 1) {                                                                                                  \
                HBFP_MX_PAIR(abuf, bbuf, A1, 0, j, COPY);                                                                  \
                if (LB > 1) HBFP_MX_PAIR(abuf, bbuf, A1, B1, j, COPY);                                                     \
                if (LB > 2) HBFP_MX_PAIR(abuf, bbuf, A1, B2, j, COPY);                                                     \
            }                                                                                                              \
            if (LA > 2) {                                                                                                  \
                HBFP_MX_PAIR(abuf, bbuf, A2, 0, j, COPY);                                                                  \
                if (LB > 1) HBFP_MX_PAIR(abuf, bbuf, A2, B1, j, COPY);                                                     \
                if (LB > 2) HBFP_MX_PAIR(abuf, bbuf, A2, B2, j, COPY);                                                     \
            }                                                                                                              \
        }                                                                                                                  \
    }

// the same products for one row tile only, each followed by one stage copy if the k-step hands over a buffer
#define HBFP_MX_ONE(abuf, bbuf, JA, JB, i, j, COPY)                                                                         \
    {                                                                                                                      \
        HBFP_MX_MFMA(abuf, bbuf, JA, JB, i, j);                                                                            \
        constexpr int c_ = (i) * LA * LB + (JA) * LB + (JB);                                                               \
        if ((COPY) && c_ < NCOPY) {                                                                                        \
            async_copy16(cptr[c_], voff, copy_ring * STAGE + coff[c_]);                                                    \
            cptr[c_] += cstep[c_];                                                                                         \
        }                                                                                                                  \
    }
#define HBFP_MX_COLUMN_ROW(abuf, bbuf, i, j, COPY, PART)                                                                        \
    {                                                                                                                      \
        constexpr int A1 = LA > 1 ? 1 : 0, A2 = LA > 2 ? 2 : 0, B1 = LB > 1 ? 1 : 0, B2 = LB > 2 ? 2 : 0;                  \
        if (PART != 2) HBFP_MX_ONE(abuf, bbuf, 0, 0, i, j, COPY);                                                          \
        if (PART != 1) {                                                                                                   \
            if (LB > 1) HBFP_MX_ONE(abuf, bbuf, 0, B1, i, j, COPY);                                                        \
            if (LB > 2) HBFP_MX_ONE(abuf, bbuf, 0, B2, i, j, COPY);                                                        \
            if (LA > 1) {                                                                                                  \
                HBFP_MX_ONE(abuf, bbuf, A1, 0, i, j, COPY);                                                                \
                if (LB > 1) HBFP_MX_ONE(abuf, bbuf, A1, B1, i, j, COPY);                                                   \
                if (LB > 2) HBFP_MX_ONE(abuf, bbuf, A1, B2, i, j, COPY);                                                   \
            }                                                                                                              \
            if (LA > 2) {                                                                                                  \
                HBFP_MX_ONE(abuf, bbuf, A2, 0, i, j, COPY);                                                                \
                if (LB > 1) HBFP_MX_ONE(abuf, bbuf, A2, B1, i, j, COPY);                                                   \
                if (LB > 2) HBFP_MX_ONE(abuf, bbuf, A2, B2, i, j, COPY);                                                   \
            }                                                                                                              \
        }                                                                                                                  \
    }

// TR: the variant whose output is an encoded operand (g.out)
template <int LA, int LB, bool TR>
__global__ __launch_bounds__(kMxThreads, 2) void gemm_mx_kernel(const MxGroup g) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int CHA = chunk_bytes(LA), CHB = chunk_bytes(LB);
    constexpr int SA = panel_stage_bytes(LA), SB = panel_stage_bytes(LB), STAGE = SA + SB;
    constexpr int RING = 3 * STAGE <= 160 * 1024 ? 3 : 2;
    constexpr int PIECES = STAGE / 1024;                       // 1 KB = one copy instruction of a wave
    constexpr int NCOPY = (PIECES + 7) / 8;                    // per wave and stage
    constexpr bool ONE_A = LA > 2 || LB > 2;                   // three limbs: no room for a second set of row-tile registers

    // which product this workgroup belongs to: selected with constant indices, so that the parameters stay in
    // scalar registers (the copy instructions take their base addresses from there)
    if ((int)blockIdx.x >= g.first[kMxGroup]) {
        // behind the tiles: scale words for the int8 stand-by of product i, 256 threads per operand
        const int extra = (int)blockIdx.x - g.first[kMxGroup], i = extra / kMxWordWgs;
        WordParams w = g.words[0];
#pragma unroll
        for (int j = 1; j < kMxGroup; ++j)
            if (j == i) w = g.words[j];
        if (!((g.word_jobs >> i) & 1) || stands_down(w.run_a, w.run_b)) return;
        const uint32_t blocks = (uint32_t)w.row_blocks * (uint32_t)(w.slots / 4);
        // few workgroups (each costs launch time when there is nothing to do), so several blocks at a time: their loads
        // are independent
        for (uint32_t b = (uint32_t)(extra - i * kMxWordWgs); b < blocks; b += 4 * kMxWordWgs) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (b + u * kMxWordWgs < blocks) scale_words_block(w, b + u * kMxWordWgs, (int)(threadIdx.x >> 8), (int)(threadIdx.x & 255));
        }
        return;
    }
    MxParams p = g.p[0];
    int first_wg = 0;
#pragma unroll
    for (int i = 1; i < kMxGroup; ++i)
        if (i < g.n && (int)blockIdx.x >= g.first[i]) {
            p = g.p[i];
            first_wg = g.first[i];
        }
    if (p.ha[0] == p.ha[1] || p.hb[0] == p.hb[1]) return;      // uniform: the int8 kernels take over
    int tm, tn;
    if (!tile_of_workgroup((int)blockIdx.x - first_wg, p.tiles_m, p.tiles_n, tm, tn)) return;   // whole workgroup, before any barrier

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave & 3, wn = wave >> 2;

    // ---- copies: a stage is PIECES pieces of 1 KB, A's first; wave w moves pieces w, w + 8, ... (the last ones
    // clamped, so every wave issues NCOPY copies per stage and one wait count fits all).  The source of piece c
    // advances by one stage of its operand per k-step.
    const uint32_t voff = lane * 16;
    const uint8_t *cptr[NCOPY];
    uint32_t coff[NCOPY], cstep[NCOPY];
#pragma unroll
    for (int i = 0; i < NCOPY; ++i) {
        int c = wave + 8 * i;
        c = c < PIECES ? c : PIECES - 1;
        const int byte = c * 1024;
        coff[i] = byte;
        cptr[i] = byte < SA ? p.pa + (int64_t)tm * p.ksteps * SA + byte : p.pb + (int64_t)tn * p.ksteps * SB + (byte - SA);
        cstep[i] = byte < SA ? SA : SB;
    }
#define HBFP_MX_COPY_STAGE(ring_)                                                                  \
    {                                                                                              \
        _Pragma("unroll") for (int i = 0; i < NCOPY; ++i) {                                        \
            async_copy16(cptr[i], voff, (uint32_t)((ring_) * STAGE) + coff[i]);                    \
            cptr[i] += cstep[i];                                                                   \
        }                                                                                          \
    }

    // ---- fragment addresses inside a stage
    // (one opaque base register per limb plane read in the same phase: reads that share a base get merged into
    // two-address reads across fragments, whose results then have to be copied into the operand registers)
    const int a4 = lane * 4 + 2 * wm * CHA + LA * kLimbBytes, b4 = lane * 4 + SA + 4 * wn * CHB + LB * kLimbBytes;
    int abase[2][LA], bbase[LB];
#pragma unroll
    for (int l = 0; l < LA; ++l) {
        abase[0][l] = lane * 24 + 2 * wm * CHA + l * kLimbBytes;
        abase[1][l] = abase[0][l] + CHA;
        asm volatile("" : "+v"(abase[0][l]), "+v"(abase[1][l]));
    }
#pragma unroll
    for (int l = 0; l < LB; ++l) {
        bbase[l] = lane * 24 + SA + 4 * wn * CHB + l * kLimbBytes;
        asm volatile("" : "+v"(bbase[l]));
    }

    v16f acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // Software pipeline.  The fragments of column tile j + 1 are read while the matrix instructions of column tile j
    // run; during the last column tile of a k-step the wave reads the row tiles and the first column tile of the next
    // k-step.  That needs the next stage, so the hand-over sits there: wait for this wave's copies of stage ks + 1,
    // barrier (now every wave's copies of it have landed and every wave has finished reading stage ks), and the
    // buffer of stage ks takes the copy of stage ks + RING, issued between the matrix instructions of the last
    // column tile.  A copy has RING - 1 k-steps to land.
    v2i af[2][2][3 * LA], bf[2][3 * LB];
    int as[2][2], bs[2];
    HBFP_MX_COPY_STAGE(0);
    HBFP_MX_COPY_STAGE(1);                                     // there are at least two k-steps
    if (RING == 3 && p.ksteps > 2) {
        HBFP_MX_COPY_STAGE(2);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NCOPY) : "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCOPY) : "memory");
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    HBFP_MX_READ_A(0, lds);
    HBFP_MX_READ_B(0, 0, lds);
    int ring = 0;
    // Neither the optimiser (memory clobber) nor the instruction scheduler moves LDS reads or matrix instructions
    // across a fence: the order below is the schedule.  A k-step is straight-line code (the start-up and drain cases
    // are separate expansions chosen by MODE), because matrix instructions are otherwise sunk past a branch.
#define HBFP_MX_FENCE                   \
    asm volatile("" ::: "memory");      \
    __builtin_amdgcn_sched_barrier(0)
    // MODE 0: hand-over with a copy of stage ks + RING;  1: hand-over, nothing left to copy, one more stage in flight;
    //      2: hand-over, nothing left to copy, the next stage is the last;  3: last k-step
    /* column tile j from B buffer bbuf, fragment of column tile jn into B buffer bn in four pieces */
#define HBFP_MX_COLUMN22(abuf, bbuf, j, bn, jn, base_, COPY)                                                               \
    {                                                                                                                      \
        HBFP_MX_PAIR(abuf, bbuf, 0, 0, j, COPY);                                                                           \
        HBFP_MX_READ_B_PIECE(bn, jn, base_, 0, 1, false);                                                                  \
        HBFP_MX_FENCE;                                                                                                     \
        HBFP_MX_PAIR(abuf, bbuf, 0, 1, j, COPY);                                                                           \
        HBFP_MX_READ_B_PIECE(bn, jn, base_, 2, 2, true);                                                                   \
        HBFP_MX_FENCE;                                                                                                     \
        HBFP_MX_PAIR(abuf, bbuf, 1, 0, j, COPY);                                                                           \
        HBFP_MX_READ_B_PIECE(bn, jn, base_, 3, 4, false);                                                                  \
        HBFP_MX_FENCE;                                                                                                     \
        HBFP_MX_PAIR(abuf, bbuf, 1, 1, j, COPY);                                                                           \
        HBFP_MX_READ_B_PIECE(bn, jn, base_, 5, 5, false);                                                                  \
        HBFP_MX_FENCE;                                                                                                     \
    }
#define HBFP_MX_HANDOVER(MODE)                                                                                             \
    {                                                                                                                      \
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                                                 \
        if (RING == 3 && MODE != 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCOPY) : "memory");                           \
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                                              \
        __builtin_amdgcn_s_barrier();                                                                                      \
        asm volatile("" ::: "memory");                                                                                     \
    }
#define HBFP_MX_KSTEP(abuf, MODE)                                                                                          \
    {                                                                                                                      \
        const uint8_t *base = lds + ring * STAGE;                                                                          \
        const int copy_ring = ring;                                                                                        \
        const int next = ring + 1 == RING ? 0 : ring + 1;                                                                  \
        const uint8_t *nbase = lds + next * STAGE;                                                                         \
        if (LA == 2 && LB == 2) {                                                                                          \
            /* two limbs each: four pairs of matrix instructions per column tile, a quarter of the next column   */       \
            /* tile's fragment requested after each pair                                                         */       \
            HBFP_MX_COLUMN22(abuf, 0, 0, 1, 1, base, false);                                                               \
            HBFP_MX_COLUMN22(abuf, 1, 1, 0, 2, base, false);                                                               \
            HBFP_MX_COLUMN22(abuf, 0, 2, 1, 3, base, false);                                                               \
            if (MODE != 3) HBFP_MX_HANDOVER(MODE);                                                                         \
            HBFP_MX_PAIR(abuf, 1, 0, 0, 3, MODE == 0);                                                                     \
            if (MODE != 3) HBFP_MX_READ_B(0, 0, nbase);                                                                    \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_PAIR(abuf, 1, 0, 1, 3, MODE == 0);                                                                     \
            if (MODE != 3) HBFP_MX_READ_A1(1 - (abuf), 0, nbase);                                                          \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_PAIR(abuf, 1, 1, 0, 3, MODE == 0);                                                                     \
            if (MODE != 3) HBFP_MX_READ_A1(1 - (abuf), 1, nbase);                                                          \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_PAIR(abuf, 1, 1, 1, 3, MODE == 0);                                                                     \
            HBFP_MX_FENCE;                                                                                                 \
        } else if (!ONE_A) {                                                                                               \
            /* the first matrix instructions wait for the reads of the previous hand-over; the next column    */          \
            /* tile is requested behind them so that this wait does not cover it                              */          \
            HBFP_MX_COLUMN(abuf, 0, 0, false, 1);                                                                          \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_READ_B(1, 1, base);                                                                                    \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN(abuf, 0, 0, false, 2);                                                                          \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_READ_B(0, 2, base);                                                                                    \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN(abuf, 1, 1, false, 0);                                                                            \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_READ_B(1, 3, base);                                                                                    \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN(abuf, 0, 2, false, 0);                                                                            \
            HBFP_MX_FENCE;                                                                                                 \
            if (MODE != 3) {                                                                                               \
                HBFP_MX_HANDOVER(MODE);                                                                                    \
                HBFP_MX_READ_A(1 - (abuf), nbase);                                                                         \
                HBFP_MX_READ_B(0, 0, nbase);                                                                               \
            }                                                                                                              \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN(abuf, 1, 3, MODE == 0, 0);                                                                        \
            HBFP_MX_FENCE;                                                                                                 \
        } else {                                                                                                           \
            /* one set of row-tile registers: row tile 0 of the next k-step is read as soon as the last column    */      \
            /* tile has used it, row tile 1 after that; all products of a row tile run back to back               */      \
            HBFP_MX_COLUMN_ROW(0, 0, 0, 0, false, 1);                                                                      \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_READ_B(1, 1, base);                                                                                    \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN_ROW(0, 0, 0, 0, false, 2);                                                                      \
            HBFP_MX_COLUMN_ROW(0, 0, 1, 0, false, 0);                                                                       \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_READ_B(0, 2, base);                                                                                    \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN_ROW(0, 1, 0, 1, false, 0);                                                                         \
            HBFP_MX_COLUMN_ROW(0, 1, 1, 1, false, 0);                                                                         \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_READ_B(1, 3, base);                                                                                    \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN_ROW(0, 0, 0, 2, false, 0);                                                                         \
            HBFP_MX_COLUMN_ROW(0, 0, 1, 2, false, 0);                                                                         \
            HBFP_MX_FENCE;                                                                                                 \
            if (MODE != 3) {                                                                                               \
                HBFP_MX_HANDOVER(MODE);                                                                                    \
                HBFP_MX_READ_B(0, 0, nbase);                                                                               \
            }                                                                                                              \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN_ROW(0, 1, 0, 3, MODE == 0, 0);                                                                     \
            HBFP_MX_FENCE;                                                                                                 \
            if (MODE != 3) HBFP_MX_READ_A1(0, 0, nbase);                                                                   \
            HBFP_MX_FENCE;                                                                                                 \
            HBFP_MX_COLUMN_ROW(0, 1, 1, 3, MODE == 0, 0);                                                                     \
            HBFP_MX_FENCE;                                                                                                 \
            if (MODE != 3) HBFP_MX_READ_A1(0, 1, nbase);                                                                   \
            HBFP_MX_FENCE;                                                                                                 \
        }                                                                                                                  \
        ring = next;                                                                                                       \
    }
    // the number of k-steps is even (the stored contraction length is a multiple of 128)
    int ks = 0;
    if (RING == 3) {
        for (; ks + 6 <= p.ksteps; ks += 2) {
            HBFP_MX_KSTEP(0, 0);
            HBFP_MX_KSTEP(1, 0);
        }
        if (p.ksteps - ks == 4) {
            HBFP_MX_KSTEP(0, 0);
            HBFP_MX_KSTEP(1, 1);
        }
    } else {
        for (; ks + 4 <= p.ksteps; ks += 2) {
            HBFP_MX_KSTEP(0, 0);
            HBFP_MX_KSTEP(1, 0);
        }
    }
    HBFP_MX_KSTEP(0, 2);
    HBFP_MX_KSTEP(1, 3);
#undef HBFP_MX_KSTEP
#undef HBFP_MX_HANDOVER
#undef HBFP_MX_COLUMN22
#undef HBFP_MX_FENCE
#undef HBFP_MX_COPY_STAGE

    const int l32 = lane & 31, lh = lane >> 5;
    const int64_t row0 = (int64_t)tm * 256 + wm * 64, col0 = (int64_t)tn * 256 + wn * 128;
    if (TR) {
        if (g.out.rounding) mx_store_encoded<1>(g.out, acc, row0, col0, p.M, p.N, lane);
        else mx_store_encoded<0>(g.out, acc, row0, col0, p.M, p.N, lane);
        return;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = col0 + j * 32 + l32;
            if (col >= p.N) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = row0 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (row < p.M) {
                    float *dst = p.C + row * p.ldc + col;
                    // C is written once and not read again here: streaming stores leave the operand panels in the caches
                    if (p.beta) *dst = *dst + acc[i][j][v];
                    else __builtin_nontemporal_store(acc[i][j][v], dst);
                }
            }
        }
}

constexpr int mx_lds_bytes(int LA, int LB) {
    const int stage = panel_stage_bytes(LA) + panel_stage_bytes(LB);
    return (3 * stage <= 160 * 1024 ? 3 : 2) * stage;
}

#undef HBFP_MX_COLUMN
#undef HBFP_MX_COLUMN_ROW
#undef HBFP_MX_ONE
#undef HBFP_MX_READ_A1
#undef HBFP_MX_PAIR
#undef HBFP_MX_MFMA
#undef HBFP_MX_READ_A
#undef HBFP_MX_READ_B
#undef HBFP_MX_READ_B_PIECE


inline size_t packed_bytes(int64_t rows, int64_t kpad, int L) {
    return (size_t)ceil_div(rows, 256) * (size_t)(kpad / 64) * (size_t)panel_stage_bytes(L);
}

// A pack marks the operand with a value of its own (word 1 of the header) and copies it to word 0 when an exponent
// is out of range, so nothing has to be cleared between packs: whatever an earlier pack (or nobody) left in word 0
// differs from this pack's mark.  (Should stale memory match by accident, the int8 kernels compute the product:
// slower, still correct.)  A captured pack is replayed with the same mark, so there word 0 is cleared by a small
// kernel first.
int32_t next_mark() {
    static std::atomic<uint32_t> counter{(uint32_t)std::chrono::steady_clock::now().time_since_epoch().count() * 2654435761u};
    uint32_t e;
    do e = counter.fetch_add(1, std::memory_order_relaxed); while (e == 0);
    return (int32_t)e;
}

// octets per exponent block when the operands of `a` are packed densely (8-bit class, blocks of 8, 16 or 24), else 0
int dense_octets(const GemmArgs &a) {
    return (a.kbp == 32 && a.kblock < 32 && a.kblock % 8 == 0 && a.mA <= 8 && a.mB <= 8) ? (int)(a.kblock / 8) : 0;
}
// octets of a densely packed row: those of all exponent blocks, less the ones of the last block that lie wholly behind
// the end of the contraction (a last block of 16 elements in blocks of 24 has two, not three)
static int64_t dense_row_octets(const GemmArgs &a) {
    const int64_t all = a.nblk * dense_octets(a), used = ceil_div(a.kdim, 8);
    return a.kdim > 0 && used < all ? used : all;
}
// k-steps of 64 that the product kernel walks: the stored length, or the unpadded one for the dense layout
int64_t mx_ksteps(const GemmArgs &a) { return (dense_octets(a) ? round_up(dense_row_octets(a) * 8, 128) : a.kpad) / 64; }

PackParams pack_params(const GemmArgs &a, const void *mant, const uint8_t *exps, int64_t R, int64_t exp_ld, int m, void *packed) {
    const int64_t kpad = a.kpad, kbp = a.kbp;
    PackParams q;
    q.mant = mant;
    q.exps = exps;
    q.header = (int *)packed;
    q.out = (uint8_t *)packed + 256;
    q.mark = next_mark();
    q.R = R;
    q.kpad = kpad;
    q.exp_ld = exp_ld;
    q.ksteps = (int32_t)mx_ksteps(a);
    q.nks4 = (q.ksteps + 3) / 4;
    q.chunks32_per_block = (int32_t)(kbp / 32);
    q.m = m;
    q.ob = dense_octets(a);
    q.noct = (int32_t)dense_row_octets(a);
    return q;
}

template <int LA, int LB, typename MT>
int launch_pack_t(const PackPair &q, unsigned blocks, hipStream_t s) {
    hipLaunchKernelGGL((mx_pack_kernel<LA, LB, MT>), dim3(blocks), dim3(256), 0, s, q);
    return launch_status();
}

// The conversion of an FP32 product into the same encoded output, queued behind the int8 kernels that stand by for the
// block-scaled kernel: runs only when they ran.  One half wave per row and exponent block (padding entries included).
template <int ROUND>
__device__ __forceinline__ void encode_block_of_c(const float *C, int64_t ldc, int64_t M, int64_t N, const MxOut &o, int64_t unit,
                                                  int l32) {
    const int64_t row = unit / o.exp_ld, blk = unit - row * o.exp_ld;
    float x[2];
    uint32_t am = 0;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int64_t col = blk * o.kblock + e * 32 + l32;
        x[e] = (e * 32 < o.kblock && col < N) ? C[row * ldc + col] : 0.0f;
        if (o.relu) x[e] = x[e] < 0.0f ? 0.0f : x[e];
        am = max(am, __float_as_uint(x[e]) & 0x7fffffffu);
    }
    am = max_of_half_wave(am);
    const uint32_t eb = block_exponent<ROUND>(am, o.m);
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int64_t col = blk * o.kblock + e * 32 + l32;
        const uint64_t idx = (uint64_t)row * (uint64_t)N + (uint64_t)col;
        const int q = quantise<ROUND>(x[e], eb, o.m, (uint32_t)idx, (uint32_t)(idx >> 32), o.s0, o.s1);
        if (e * 32 < o.kblock && col < o.kpad) {
            if (o.wide) reinterpret_cast<int16_t *>(o.mant)[row * o.kpad + col] = (int16_t)q;
            else reinterpret_cast<int8_t *>(o.mant)[row * o.kpad + col] = (int8_t)q;
        }
    }
    if (l32 == 0) o.exps[row * o.exp_ld + blk] = blk < o.nblk ? (uint8_t)eb : (uint8_t)1;
}

__global__ __launch_bounds__(256) void mx_encode_standby_kernel(const float *C, int64_t ldc, int64_t M, int64_t N, const MxOut o,
                                                                const int *run_a, const int *run_b) {
    if (stands_down(run_a, run_b)) return;
    // a small grid that strides over the blocks: in the usual case, where it has nothing to do, it is gone in microseconds
    for (int64_t unit = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5); unit < M * o.exp_ld; unit += (int64_t)gridDim.x * 8) {   // per half wave
        if (o.rounding) encode_block_of_c<1>(C, ldc, M, N, o, unit, threadIdx.x & 31);
        else encode_block_of_c<0>(C, ldc, M, N, o, unit, threadIdx.x & 31);
    }
}

__global__ __launch_bounds__(256) void relu_kernel(float *x, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) x[i] = x[i] < 0.0f ? 0.0f : x[i];
}

template <int LA, int LB, bool TR>
int launch_mx_tr(const MxGroup &g, hipStream_t s) {
    constexpr int bytes = mx_lds_bytes(LA, LB);
    static std::atomic<bool> configured{false};
    if (allow_dynamic_lds(configured, reinterpret_cast<const void *>(&gemm_mx_kernel<LA, LB, TR>), bytes) != HBFP_OK) return HBFP_ERR_LAUNCH;
    const unsigned grid = (unsigned)g.first[g.n] + (g.word_jobs ? (unsigned)(g.n * kMxWordWgs) : 0u);
    hipLaunchKernelGGL((gemm_mx_kernel<LA, LB, TR>), dim3(grid), dim3(kMxThreads), bytes, s, g);
    return launch_status();
}

template <int LA, int LB>
int launch_mx_t(const MxGroup &g, hipStream_t s) {
    return g.out.mant ? launch_mx_tr<LA, LB, true>(g, s) : launch_mx_tr<LA, LB, false>(g, s);
}

}  // namespace

// The block-scaled path pays for itself when its 256 x 256 tiles fill the chip and it spends less energy than the int8
// kernels (both are limited by the power the chip may draw, not by issue slots).  Measured on 4096^3 and 8192^3
// products: four limb products per k-step (6..9-bit mantissas) beat the int8 kernel where that one scales after every
// matrix instruction (blocks of at most 32, stored padded to 32: 8 to 20 % faster), not for longer blocks; one or two
// limb products (an operand of at most 5 bits: 2 x faster) and the 12-bit formats (6 or 9 limb products against four
// int8 products plus five vector instructions per output and block: 1.4 x faster) win for every block length.
bool mx_same_limbs(const GemmArgs &a, const GemmArgs &b) {
    return limbs_of(a.mA) == limbs_of(b.mA) && limbs_of(a.mB) == limbs_of(b.mB);
}

bool gemm_mx_possible(const GemmArgs &a) {
    return !a.P && ceil_div(a.M, 256) * ceil_div(a.N, 256) <= 0x7ffffff0 && a.kpad / 64 <= 0x7fffffff && a.nblk * 4 <= 0x7fffffff;
}

bool gemm_mx_ok(const GemmArgs &a) {
    if (!gemm_mx_possible(a)) return false;
    const int64_t tiles = ceil_div(a.M, 256) * ceil_div(a.N, 256);
    // 128 tiles on 256 CUs (4096 x 2048) lose to the int8 kernels at every contraction length measured (30 to 45 %);
    // 144 tiles (3072^2) win from a contraction of 2048 to 3072 on
    if (tiles < 144) return false;
    if ((double)a.M * (double)a.N < 0.75 * 65536.0 * (double)tiles) return false;   // ragged edges would waste the tiles
    // short contractions do not repay the packing and the start-up of the three-stage ring: blocks of 32 at 4096^2 are
    // 5 to 9 % ahead from 2048 on and 6 % behind at 1024; with two or more rounds of tiles (8192 x 4096, 8192^2) the
    // break-even is 1024 (2 to 5 % ahead there, 10 to 20 % behind at 512)
    if (a.kpad < (tiles >= 512 ? 1024 : 2048)) return false;
    const int products = limbs_of(a.mA) * limbs_of(a.mB);
    // blocks of exactly 32: 3 to 8 % ahead at 4096^3, 20 % at 8192^3; shorter blocks, stored padded to 32, cost the int8
    // kernel a scaling pass per padded block as well: 15 to 20 % ahead at 4096^3
    if (products == 4) return a.kbp == 32;
    return true;
}

// Products that share one launch.  Measured with 8-bit mantissas in blocks of 32 against the int8 kernels run one
// after the other: four products of 64 tiles each (2048 x 2048) 5 to 14 % ahead for contractions of 1024 to 4096;
// 128 tiles or fewer in the whole group (four of 2048 x 1024 x 8192, four of 1024 x 1024 x 4096) 5 to 7 % behind.
// Tiles of very different contraction lengths do not share well (the gate products of an LSTM step, contractions of
// 640, 2048 and 8192: 60 % behind, the few long tiles run on alone at the end), so the lengths must be within a
// factor of two of each other and none below the 1024 that a product of its own needs.
bool gemm_mx_group_ok(int n, const GemmArgs *args) {
    int64_t tiles = 0, kmin = args[0].kpad, kmax = args[0].kpad;
    double area = 0.0;
    for (int i = 0; i < n; ++i) {
        const GemmArgs &a = args[i];
        if (!gemm_mx_possible(a) || !mx_same_limbs(a, args[0])) return false;
        if (limbs_of(a.mA) * limbs_of(a.mB) == 4 && a.kbp != 32) return false;
        tiles += ceil_div(a.M, 256) * ceil_div(a.N, 256);
        area += (double)a.M * (double)a.N;
        kmin = a.kpad < kmin ? a.kpad : kmin;
        kmax = a.kpad > kmax ? a.kpad : kmax;
    }
    return tiles >= 256 && area >= 0.75 * 65536.0 * (double)tiles && kmin >= 1024 && kmax <= 2 * kmin;
}

// What a kernel that writes a packed operand itself needs first: this pack's mark and, under graph capture (where a
// replay repeats the mark), a cleared out-of-range word.
int mx_pack_begin(void *packed, hipStream_t s, int32_t *mark) {
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &capture) != hipSuccess || capture != hipStreamCaptureStatusNone) {
        hipLaunchKernelGGL(mx_clear_flag_kernel, dim3(1), dim3(64), 0, s, (int *)packed, (int *)nullptr);
        if (launch_status() != HBFP_OK) return HBFP_ERR_LAUNCH;
    }
    *mark = next_mark();
    return HBFP_OK;
}

size_t mx_packed_bytes(int64_t rows, int64_t kpad, int mant_bits) { return 256 + packed_bytes(rows, kpad, limbs_of(mant_bits)); }

int launch_mx_pack(const GemmArgs &a, void *packed_a, void *packed_b, hipStream_t s) {
    if (!packed_a && !packed_b) return HBFP_OK;
    PackPair q;
    int64_t ba = 0, bb = 0;
    int LA = limbs_of(a.mA), LB = limbs_of(a.mB);
    if (packed_a) {
        q.op[0] = pack_params(a, a.mantA, a.expA, a.M, a.expA_ld, a.mA, packed_a);
        ba = ceil_div(a.M, 256) * 8 * q.op[0].nks4;
    }
    if (packed_b) {
        q.op[1] = pack_params(a, a.mantB, a.expB, a.N, a.expB_ld, a.mB, packed_b);
        bb = ceil_div(a.N, 256) * 8 * q.op[1].nks4;
    }
    if (!packed_a) LA = LB;                                     // the absent operand has no workgroups; any instantiation does
    if (!packed_b) LB = LA;
    if (ba + bb > 0x7fffffff) return HBFP_ERR_ARG;
    q.blocks_a = (uint32_t)ba;
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &capture) != hipSuccess || capture != hipStreamCaptureStatusNone)
        hipLaunchKernelGGL(mx_clear_flag_kernel, dim3(1), dim3(64), 0, s, (int *)packed_a, (int *)packed_b);
    const unsigned blocks = (unsigned)(ba + bb);
    const bool wide = (packed_a ? a.mA : a.mB) > 8;             // both operands of a product are of the same mantissa class
    switch (LA * 4 + LB + (wide ? 16 : 0)) {
        case 1 * 4 + 1: return launch_pack_t<1, 1, int8_t>(q, blocks, s);
        case 1 * 4 + 2: return launch_pack_t<1, 2, int8_t>(q, blocks, s);
        case 2 * 4 + 1: return launch_pack_t<2, 1, int8_t>(q, blocks, s);
        case 2 * 4 + 2: return launch_pack_t<2, 2, int8_t>(q, blocks, s);
        case 16 + 2 * 4 + 2: return launch_pack_t<2, 2, int16_t>(q, blocks, s);
        case 16 + 2 * 4 + 3: return launch_pack_t<2, 3, int16_t>(q, blocks, s);
        case 16 + 3 * 4 + 2: return launch_pack_t<3, 2, int16_t>(q, blocks, s);
        case 16 + 3 * 4 + 3: return launch_pack_t<3, 3, int16_t>(q, blocks, s);
        default: return HBFP_ERR_FORMAT;
    }
}

// n <= kMxGroup products with the same limb counts in one launch
static int launch_mx_group(int n, GemmArgs *args, const void *const *packed_a, const void *const *packed_b, const MxOut *out,
                           void *const *standby_ws, hipStream_t s) {
    if (n < 1 || n > kMxGroup || (out && n != 1)) return HBFP_ERR_ARG;
    const int LA = limbs_of(args[0].mA), LB = limbs_of(args[0].mB);
    MxGroup g = {};
    g.n = n;
    if (out) g.out = *out;
    int64_t first = 0;
    for (int i = 0; i < n; ++i) {
        const GemmArgs &a = args[i];
        if (limbs_of(a.mA) != LA || limbs_of(a.mB) != LB) return HBFP_ERR_FORMAT;
        MxParams &p = g.p[i];
        p.ha = (const int *)packed_a[i];
        p.hb = (const int *)packed_b[i];
        p.pa = (const uint8_t *)packed_a[i] + 256;
        p.pb = (const uint8_t *)packed_b[i] + 256;
        p.C = a.C;
        p.M = a.M;
        p.N = a.N;
        p.ldc = a.ldc;
        p.ksteps = (int32_t)mx_ksteps(a);
        p.tiles_m = (int32_t)ceil_div(a.M, 256);
        p.tiles_n = (int32_t)ceil_div(a.N, 256);
        p.beta = a.beta != 0.0f;
        g.first[i] = (int32_t)first;
        first += ceil_div((int64_t)p.tiles_m * p.tiles_n, 8) * 8;      // a multiple of 8: the XCD of a tile does not depend on the group
        if (first > 0x7ffffff0) return HBFP_ERR_ARG;
    }
    for (int i = n; i <= kMxGroup; ++i) g.first[i] = (int32_t)first;
    for (int i = 0; i < n && standby_ws; ++i) {
        StandbyWords w;
        if (!standby_ws[i] || !gemm_i8_standby_words(args[i], standby_ws[i], &w)) continue;
        g.words[i] = scale_word_params(w.eA, w.ldA, w.M, w.eB, w.ldB, w.N, w.slots, w.a_or, w.wA, w.wB, (const int *)packed_a[i],
                                       (const int *)packed_b[i]);
        if (scale_word_blocks(g.words[i]) > 0x7fffffff) continue;
        g.word_jobs |= 1 << i;
        args[i].words_ready = 1;
    }
    switch (LA * 4 + LB) {
        case 1 * 4 + 1: return launch_mx_t<1, 1>(g, s);
        case 1 * 4 + 2: return launch_mx_t<1, 2>(g, s);
        case 2 * 4 + 1: return launch_mx_t<2, 1>(g, s);
        case 2 * 4 + 2: return launch_mx_t<2, 2>(g, s);
        case 2 * 4 + 3: return launch_mx_t<2, 3>(g, s);
        case 3 * 4 + 2: return launch_mx_t<3, 2>(g, s);
        case 3 * 4 + 3: return launch_mx_t<3, 3>(g, s);
        default: return HBFP_ERR_FORMAT;
    }
}

int launch_mx_products(int n, GemmArgs *args, const void *const *packed_a, const void *const *packed_b, void *const *standby_ws,
                       hipStream_t s) {
    return launch_mx_group(n, args, packed_a, packed_b, nullptr, standby_ws, s);
}

int launch_mx_product(GemmArgs &a, const void *packed_a, const void *packed_b, void *standby_ws, hipStream_t s) {
    return launch_mx_group(1, &a, &packed_a, &packed_b, nullptr, &standby_ws, s);
}

// The block-scaled kernel can write its accumulators as an encoded operand when the output's exponent blocks are
// runs of 32 or 64 columns of a row of C.
bool mx_encoded_output_ok(const hbfp_tensor &out) {
    return out.contract_axis == 1 && out.rblock == 1 && out.kshare == 1 && (out.kblock == 32 || out.kblock == 64) &&
           out.kblock_pad == out.kblock && out.rows * out.exp_ld < ((int64_t)1 << 33);
}

int launch_mx_product_encoded(const GemmArgs &a, const void *packed_a, const void *packed_b, const hbfp_tensor &out, int relu,
                              hipStream_t s) {
    if (!mx_encoded_output_ok(out)) return HBFP_ERR_FORMAT;
    const MxOut o = mx_out_of(out, relu);
    GemmArgs copy = a;
    return launch_mx_group(1, &copy, &packed_a, &packed_b, &o, nullptr, s);
}

// behind the int8 kernels that stood by for launch_mx_product_encoded and wrote the FP32 product to C
int launch_mx_encode_standby(const float *C, int64_t ldc, const hbfp_tensor &out, int relu, const int *run_a, const int *run_b,
                             hipStream_t s) {
    if (!mx_encoded_output_ok(out)) return HBFP_ERR_FORMAT;
    const int64_t units = out.rows * out.exp_ld;
    const int64_t wgs = ceil_div(units, 8);
    hipLaunchKernelGGL(mx_encode_standby_kernel, dim3((unsigned)(wgs < 2048 ? wgs : 2048)), dim3(256), 0, s, C, ldc, out.rows, out.src_cols,
                       mx_out_of(out, relu), run_a, run_b);
    return launch_status();
}

int launch_relu(float *x, int64_t n, hipStream_t s) {
    if (ceil_div(n, 256) > 0x7fffffff) return HBFP_ERR_ARG;
    hipLaunchKernelGGL(relu_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, x, n);
    return launch_status();
}

}  // namespace hbfp
