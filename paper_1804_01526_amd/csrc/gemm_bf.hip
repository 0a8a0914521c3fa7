// BFP matrix product for mantissas of 6 to 9 bits on the bf16 matrix instruction of gfx950 (Eq. (2) of Sec. 4):
//     C[i][j] = sum_b 2^(eA[i][b] + eB[j][b]) * sum_{k in b} mA[i][k] * mB[j][k]
//
// A mantissa of at most 9 bits times its block's power of two is a bf16 number (8 significant bits, the exponent
// range of the stored exponent byte), so the decode of Eq. (1) is exact in bf16 and v_mfma_f32_32x32x16_bf16 is the
// arithmetic of Eq. (2) in hardware: it multiplies the 8-bit significands as integers, adds the exponents, and
// accumulates in FP32 (Sec. 4: accumulation across blocks is in floating point).  One matrix instruction per 16 k
// does what the block-scaled instruction needs four 4-bit limb products for, at the same instruction rate and at
// a lower power per product, which is what bounds both kernels on this chip; and blocks whose exponents lie far apart
// (heavy-tailed gradients) need no other path.
//
// pack kernel:    stored operand (int8 / int16 mantissas [rows][kpad], exponent bytes) -> bf16 planes in the register
//                 order of the matrix instruction (bf_pack.h), blocks of 8, 16 and 24 without their padding.
// gemm_bf_kernel: 256 x 256 tile of C per workgroup, 8 waves of 64 x 128, four-stage LDS ring of k-steps of 32 filled
//                 by asynchronous copies of whole stages, one barrier per k-step, operand registers of the next half
//                 k-step read while the matrix instructions of this one run.
// Only a non-zero block with an exponent byte above 253 (values from 2^127 on) cannot be packed safely; the pack then
// marks the header of the packed operand as the block-scaled path does, and the product kernel computes such a product
// from the stored operands with plain integer and FP32 arithmetic (bf_marked_tile).  Small values need no such care:
// the instruction takes subnormal bf16 operands and keeps subnormal FP32 sums.
#include <atomic>
#include <type_traits>

#include "bf_pack.h"
#include "hbfp_internal.h"
#include "mx_out.h"

namespace hbfp {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef int v4i_t __attribute__((ext_vector_type(4)));

constexpr int kBfThreads = 512;
constexpr int kBfStage = 2 * kBfStageBytes;      // A's panel and B's panel of one k-step: 32 KB
constexpr int kBfRing = 4;
constexpr int kBfCopies = kBfStage / 1024 / 8;   // copy instructions (1 KB each) per wave and stage
constexpr int kBfGroup = HBFP_BATCH_MAX;

// ------------------------------------------------------------------------------------------------
struct BfPackParams {
    const void *mant;
    const uint8_t *exps;
    uint8_t *out;
    int *header;                 // word 1 = this pack's mark, word 0 = the mark of the last pack that found an exponent out of range
    int64_t R, kpad, exp_ld;
    int32_t ksteps;              // k-steps of 32 of the packed operand (a multiple of 4)
    int32_t chunks32_per_block, m, mark;
    int32_t ob, noct;            // dense layout: octets per exponent block and in the whole row; ob = 0: as stored
    int32_t *scale;              // FP16 planes: one word per row (rows padded to 256), Eref - 129 - m; else null
    int32_t nblk;
};
struct BfPackPair {
    BfPackParams op[2];
    uint32_t blocks_a;
};

// A workgroup of 4 waves packs one row tile of 32 rows over 4 x 64 k; a lane converts 16 consecutive k of one row (two
// octets) of rows r and r + 16.
template <typename MT, bool F16>
__device__ __forceinline__ void bf_pack_block(const BfPackParams &p, uint32_t block) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (block == 0 && threadIdx.x == 0) p.header[1] = p.mark;
    const int nk4 = (p.ksteps / 2 + 3) / 4;
    const int64_t rt = block / nk4;
    const int ks64 = (int)(block % nk4) * 4 + wave;
    if (2 * ks64 >= p.ksteps) return;
    const int q = lane & 3, r4 = lane >> 2;
    const int ks = 2 * ks64 + (q >> 1), h = q & 1;
    bool bad = false;
    // all loads first (mantissas and exponent bytes of both rows and both octets), then the conversions and the stores:
    // the compiler cannot move a load above a store through another pointer
    typedef typename std::conditional<sizeof(MT) == 1, v2i, v4i_t>::type raw_t;
    raw_t raw[2][2];
    int E[2][2], Eref[2] = {0, 0};
    bool there[2][2];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const int64_t row = rt * 32 + hh * 16 + r4;
        const bool live = row < p.R;
        if (F16) Eref[hh] = p.scale[rt * 32 + hh * 16 + r4] + 129 + p.m;      // written by f16_row_scale_kernel before this launch
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            const uint32_t j = (uint32_t)ks64 * 8u + (uint32_t)q * 2u + (uint32_t)o;          // octet of the packed k axis
            bool t = live;
            int64_t pos;                                                                       // its first element in the stored row
            uint32_t b;                                                                        // its exponent block
            if (p.ob) {
                t = t && j < (uint32_t)p.noct;
                b = t ? bf_dense_block_of(j, p.ob) : 0u;
                pos = t ? (int64_t)b * 32 + 8 * (int)(j - b * (uint32_t)p.ob) : 0;
            } else {
                pos = (int64_t)j * 8;
                b = (j >> 2) / (uint32_t)p.chunks32_per_block;
            }
            const int64_t rs = t ? row : 0;                                                    // what does not exist reads row 0 and stores zeros
            there[hh][o] = t;
            E[hh][o] = p.exps[rs * p.exp_ld + b];
            raw[hh][o] = *reinterpret_cast<const raw_t *>(reinterpret_cast<const MT *>(p.mant) + rs * p.kpad + pos);
        }
    }
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const int r32 = hh * 16 + r4;
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            v4u out = {0u, 0u, 0u, 0u};
            bool any;
            if constexpr (sizeof(MT) == 1) {
                any = (raw[hh][o][0] | raw[hh][o][1]) != 0;
                if (there[hh][o]) out = bf_octet_i8(raw[hh][o], E[hh][o], p.m);
            } else {
                any = (raw[hh][o][0] | raw[hh][o][1] | raw[hh][o][2] | raw[hh][o][3]) != 0;
                if (F16) {
                    const int shift = E[hh][o] - Eref[hh] + kF16Lift;
                    if (there[hh][o]) out = f16_octet_i16(raw[hh][o], shift);
                    bad = bad || (there[hh][o] && any && shift < kF16MinShift);
                } else if (there[hh][o]) {
                    out = bf_octet_i16(raw[hh][o], E[hh][o], p.m);
                }
            }
            if (!F16) bad = bad || (there[hh][o] && any && !bf_exponent_ok(E[hh][o]));
            __builtin_nontemporal_store(out, reinterpret_cast<v4u *>(p.out + bf_piece_offset(rt, ks, p.ksteps, h, o, r32)));
        }
    }
    if (bad) p.header[0] = p.mark;
}

template <typename MT, bool F16>
__global__ __launch_bounds__(256) void bf_pack_kernel(const BfPackPair q) {
    if (blockIdx.x < q.blocks_a) bf_pack_block<MT, F16>(q.op[0], blockIdx.x);
    else bf_pack_block<MT, F16>(q.op[1], blockIdx.x - q.blocks_a);
}

// FP16 planes: the scale word of every row, from the largest exponent byte of its blocks; one thread per row of either
// operand (rows behind the last: 0).  Runs before the pack kernel, which reads the words.
__global__ __launch_bounds__(256) void f16_row_scale_kernel(const BfPackPair q, uint32_t rows_a, uint32_t rows_b) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= rows_a + rows_b) return;
    const BfPackParams &p = i < rows_a ? q.op[0] : q.op[1];
    const int64_t row = i < rows_a ? i : i - rows_a;
    int word = 0;
    if (row < p.R) {
        int emax = 1;
        for (int b = 0; b < p.nblk; ++b) emax = max(emax, (int)p.exps[row * p.exp_ld + b]);
        word = emax - 129 - p.m;
    }
    p.scale[row] = word;
}

// ------------------------------------------------------------------------------------------------
struct BfParams {
    const uint8_t *pa, *pb;      // bf16 planes of the packed operands
    const int *ha, *hb;          // their headers: words 0 and 1 equal = marked
    float *C;
    int64_t M, N, ldc;
    int32_t ksteps, tiles_m, tiles_n, beta;
    // the stored operands, read only when a packed operand is marked
    const void *mantA, *mantB;
    const uint8_t *expA, *expB;
    int64_t kpad, expA_ld, expB_ld;
    int32_t chunks32_per_block, shift, wide;   // shift: -(2 * 125 + mA + mB)
    const int32_t *sa, *sb;                    // FP16 planes: the scale words of the rows of A and of B
};

// A tile of a product with a marked operand (an exponent byte above 253: values next to the largest finite FP32 number),
// from the stored operands with the arithmetic of Eq. (2) as written: an integer sum per stored chunk of 32, scaled by
// 2^(eA + eB) and accumulated in FP32.  Thread t owns column t % 256 of the tile and every second row.  Slow, and
// expected never to run on training data; it spares every product the launch of a stand-by kernel.
template <typename MT>
__device__ void bf_marked_tile(const BfParams &p, int tm, int tn) {
    const int64_t col = (int64_t)tn * 256 + (threadIdx.x & 255);
    if (col >= p.N) return;
    const MT *b = reinterpret_cast<const MT *>(p.mantB) + col * p.kpad;
    for (int i = 0; i < 128; ++i) {
        const int64_t row = (int64_t)tm * 256 + (threadIdx.x >> 8) + 2 * i;
        if (row >= p.M) break;
        const MT *a = reinterpret_cast<const MT *>(p.mantA) + row * p.kpad;
        float sum = 0.0f;
        for (int64_t c = 0; c < p.kpad / 32; ++c) {
            int P = 0;
            for (int k = 0; k < 32; ++k) P += (int)a[c * 32 + k] * (int)b[c * 32 + k];
            const int64_t blk = c / p.chunks32_per_block;
            sum += __builtin_ldexpf((float)P, (int)p.expA[row * p.expA_ld + blk] + (int)p.expB[col * p.expB_ld + blk] + p.shift);
        }
        float *dst = p.C + row * p.ldc + col;
        *dst = p.beta ? *dst + sum : sum;
    }
}
// Up to kBfGroup independent products in one launch: workgroups first[i] .. first[i + 1] - 1 belong to product i, so the
// stores of one product's tiles drain under the matrix instructions of the next.
struct BfGroup {
    BfParams p[kBfGroup];
    int32_t first[kBfGroup + 1];
    int32_t n;
    MxOut out;                   // of product 0 of a launch with a single product (TR)
};

// TR: the variant whose output is an encoded operand (g.out): the operands of the matrix instruction exchanged, so
// that every 32 x 32 result arrives transposed (same products, same sums) as mx_store_encoded wants them
// F16: FP16 planes (10..12-bit mantissas relative to their rows' largest exponents): the FP16 matrix instruction, and the
// rows' and columns' factors applied at the store
template <bool TR, bool F16>
__global__ __launch_bounds__(kBfThreads, 2) void gemm_bf_kernel(const BfGroup g) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // which product this workgroup belongs to: selected with constant indices, so that the parameters stay in scalar
    // registers (the copy instructions take their base addresses from there)
    BfParams p = g.p[0];
    int first_wg = 0;
#pragma unroll
    for (int i = 1; i < kBfGroup; ++i)
        if (i < g.n && (int)blockIdx.x >= g.first[i]) {
            p = g.p[i];
            first_wg = g.first[i];
        }
    int tm, tn;
    if (!tile_of_workgroup((int)blockIdx.x - first_wg, p.tiles_m, p.tiles_n, tm, tn)) return;   // whole workgroup, before any barrier
    if (p.ha[0] == p.ha[1] || p.hb[0] == p.hb[1]) {            // uniform
        if (p.wide) bf_marked_tile<int16_t>(p, tm, tn);
        else bf_marked_tile<int8_t>(p, tm, tn);
        return;
    }

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave & 3, wn = wave >> 2;

    // ---- copies: a stage is 32 pieces of 1 KB, A's 16 first; wave w moves pieces w, w + 8, w + 16, w + 24.  The source
    // of a piece advances by one stage of its operand per k-step.
    const uint32_t voff = lane * 16;
    const uint8_t *cptr[kBfCopies];
    uint32_t coff[kBfCopies];
#pragma unroll
    for (int i = 0; i < kBfCopies; ++i) {
        const int byte = (wave + 8 * i) * 1024;
        coff[i] = byte;
        cptr[i] = byte < kBfStageBytes ? p.pa + (int64_t)tm * p.ksteps * kBfStageBytes + byte
                                       : p.pb + (int64_t)tn * p.ksteps * kBfStageBytes + (byte - kBfStageBytes);
    }
#define HBFP_BF_COPY_STAGE(ring_)                                                                  \
    {                                                                                              \
        _Pragma("unroll") for (int i = 0; i < kBfCopies; ++i) {                                    \
            async_copy16(cptr[i], voff, (uint32_t)((ring_) * kBfStage) + coff[i]);                 \
            cptr[i] += kBfStageBytes;                                                              \
        }                                                                                          \
    }
    // ---- operand registers: row tiles 2 wm, 2 wm + 1 of A's panel, column tiles 4 wn .. 4 wn + 3 of B's
    int abase = lane * 16 + 2 * wm * kBfTileBytes, bbase = lane * 16 + kBfStageBytes + 4 * wn * kBfTileBytes;
    asm volatile("" : "+v"(abase), "+v"(bbase));

    v16f acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    v4i_t af[2][2], bf[2][4];
#define HBFP_BF_READ(buf, base_, h)                                                                                                             \
    {                                                                                                                                           \
        _Pragma("unroll") for (int i = 0; i < 2; ++i) af[buf][i] = *reinterpret_cast<const v4i_t *>((base_) + abase + i * kBfTileBytes + (h) * 1024); \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) bf[buf][j] = *reinterpret_cast<const v4i_t *>((base_) + bbase + j * kBfTileBytes + (h) * 1024); \
    }
#define HBFP_BF_MFMA(buf, i, j)                                                                                                    \
    if (F16)                                                                                                                       \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, af[buf][i]), __builtin_bit_cast(v8h, bf[buf][j]), \
                                                           acc[i][j], 0, 0, 0);                                                    \
    else                                                                                                                           \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, TR ? bf[buf][j] : af[buf][i]),                \
                                                            __builtin_bit_cast(v8bf, TR ? af[buf][i] : bf[buf][j]), acc[i][j], 0, 0, 0)
#define HBFP_BF_ROW(buf, i)        \
    {                              \
        HBFP_BF_MFMA(buf, i, 0);   \
        HBFP_BF_MFMA(buf, i, 1);   \
        HBFP_BF_MFMA(buf, i, 2);   \
        HBFP_BF_MFMA(buf, i, 3);   \
    }
    // Neither the optimiser (memory clobber) nor the instruction scheduler moves LDS reads or matrix instructions
    // across a fence: the order below is the schedule.
#define HBFP_BF_FENCE                   \
    asm volatile("" ::: "memory");      \
    __builtin_amdgcn_sched_barrier(0)
    // Matrix instructions touch no memory, so a fence alone does not keep them on their side of the hand-over: an empty
    // statement that reads and writes one register of every accumulator does (the next instruction on that
    // accumulator depends on it).
#define HBFP_BF_PIN                                                                                        \
    _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)                                                       \
        _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_) asm volatile("" : "+v"(acc[i_][j_][0]))
    // One k-step.  The registers of its second half are requested first and arrive under the matrix instructions of
    // the first half.  The hand-over sits between the two rows of the first half, so that matrix instructions are in
    // flight when a wave reaches the barrier and ready to issue when it leaves: wait for the second-half registers and
    // for this wave's copies of stage ks + 1, barrier (now every wave's copies of it have landed and every wave has
    // read all of stage ks).  After the first half the wave requests the first-half registers of stage ks + 1 and
    // hands the buffer of stage ks to the copy of stage ks + 4; both land under the second half.  (Measured: the
    // barrier after the whole first half, or inside the second, costs 1 to 5 % of the product.)
    // MODE 0: stages ks + 1 .. ks + 3 in flight and a copy to issue; 1: the same, nothing left to copy; 2: two stages
    // in flight; 3: one; 4: last k-step
#define HBFP_BF_KSTEP(MODE)                                                                                \
    {                                                                                                      \
        const uint8_t *base = lds + ring * kBfStage;                                                       \
        const int copy_ring = ring;                                                                        \
        const int next = ring + 1 == kBfRing ? 0 : ring + 1;                                               \
        const uint8_t *nbase = lds + next * kBfStage;                                                      \
        HBFP_BF_READ(1, base, 1);                                                                          \
        HBFP_BF_FENCE;                                                                                     \
        HBFP_BF_ROW(0, 0);                                                                                 \
        HBFP_BF_PIN;                                                                                       \
        if (MODE != 4) {                                                                                   \
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                             \
            if (MODE <= 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kBfCopies) : "memory");            \
            else if (MODE == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kBfCopies) : "memory");           \
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                          \
            __builtin_amdgcn_s_barrier();                                                                  \
            asm volatile("" ::: "memory");                                                                 \
        }                                                                                                  \
        HBFP_BF_PIN;                                                                                       \
        HBFP_BF_ROW(0, 1);                                                                                 \
        HBFP_BF_PIN;                                                                                       \
        HBFP_BF_FENCE;                                                                                     \
        if (MODE != 4) {                                                                                   \
            HBFP_BF_READ(0, nbase, 0);                                                                     \
            if (MODE == 0) HBFP_BF_COPY_STAGE(copy_ring);                                                  \
        }                                                                                                  \
        HBFP_BF_FENCE;                                                                                     \
        HBFP_BF_ROW(1, 0);                                                                                 \
        HBFP_BF_ROW(1, 1);                                                                                 \
        HBFP_BF_PIN;                                                                                       \
        ring = next;                                                                                       \
    }
    // the number of k-steps is a multiple of 4 (the packed k axis is a multiple of 128)
    HBFP_BF_COPY_STAGE(0);
    HBFP_BF_COPY_STAGE(1);
    HBFP_BF_COPY_STAGE(2);
    HBFP_BF_COPY_STAGE(3);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * kBfCopies) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    HBFP_BF_READ(0, lds, 0);
    int ring = 0;
    for (int ks = 0; ks + kBfRing < p.ksteps; ++ks) HBFP_BF_KSTEP(0);
    HBFP_BF_KSTEP(1);
    HBFP_BF_KSTEP(2);
    HBFP_BF_KSTEP(3);
    HBFP_BF_KSTEP(4);
#undef HBFP_BF_KSTEP
#undef HBFP_BF_FENCE
#undef HBFP_BF_PIN
#undef HBFP_BF_ROW
#undef HBFP_BF_MFMA
#undef HBFP_BF_READ
#undef HBFP_BF_COPY_STAGE

    const int l32 = lane & 31, lh = lane >> 5;
    const int64_t row0 = (int64_t)tm * 256 + wm * 64, col0 = (int64_t)tn * 256 + wn * 128;
    if (TR && !F16) {
        if (g.out.rounding) mx_store_encoded<1>(g.out, acc, row0, col0, p.M, p.N, lane);
        else mx_store_encoded<0>(g.out, acc, row0, col0, p.M, p.N, lane);
        return;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int sa[16];
        if (F16) {
#pragma unroll
            for (int v = 0; v < 16; ++v) sa[v] = p.sa[row0 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3)];      // padded to whole panels
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = col0 + j * 32 + l32;
            if (col >= p.N) continue;
            const int sb = F16 ? p.sb[col] : 0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = row0 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (row < p.M) {
                    float *dst = p.C + row * p.ldc + col;
                    const float x = F16 ? __builtin_ldexpf(acc[i][j][v], sa[v] + sb) : acc[i][j][v];
                    // C is written once and not read again here: streaming stores leave the operand panels in the caches
                    if (p.beta) *dst = *dst + x;
                    else __builtin_nontemporal_store(x, dst);
                }
            }
        }
    }
}

int64_t klen_of(const GemmArgs &a, int m) { return bf_klen(a.kpad, a.kbp, a.kblock, a.nblk, a.kdim, m); }

BfPackParams bf_pack_params(const GemmArgs &a, const void *mant, const uint8_t *exps, int64_t R, int64_t exp_ld, int m, void *packed,
                            int32_t mark, bool f16) {
    BfPackParams q;
    q.mant = mant;
    q.exps = exps;
    q.header = (int *)packed;
    q.scale = f16 ? (int32_t *)((uint8_t *)packed + 256) : nullptr;
    q.out = (uint8_t *)packed + 256 + (f16 ? f16_scale_bytes(R) : 0);
    q.nblk = (int32_t)a.nblk;
    q.mark = mark;
    q.R = R;
    q.kpad = a.kpad;
    q.exp_ld = exp_ld;
    q.ksteps = (int32_t)(klen_of(a, m) / 32);
    q.chunks32_per_block = (int32_t)(a.kbp / 32);
    q.m = m;
    q.ob = bf_dense_octets(a.kbp, a.kblock, m);
    q.noct = (int32_t)bf_dense_row_octets(q.ob, a.nblk, a.kdim);
    return q;
}

}  // namespace

bool bf_operand(int mant_bits) { return bf_class(mant_bits); }

size_t packed_operand_bytes(int64_t rows, int64_t kpad, int mant_bits) {
    return bf_class(mant_bits) ? bf_packed_bytes(rows, kpad) : mant_bits >= 10 ? f16_packed_bytes(rows, kpad) : mx_packed_bytes(rows, kpad, mant_bits);
}

static bool shape_ok(const GemmArgs &a) {
    return !a.P && ceil_div(a.M, 256) * ceil_div(a.N, 256) <= 0x7ffffff0 && a.kpad / 32 <= 0x7fffffff && a.nblk * 4 <= 0x7fffffff;
}
bool gemm_bf_possible(const GemmArgs &a) { return shape_ok(a) && bf_class(a.mA) && bf_class(a.mB); }
// 9..12-bit mantissas (int16 storage) as FP16 numbers relative to their rows' largest exponents
bool gemm_f16_planes_possible(const GemmArgs &a) {
    return shape_ok(a) && a.mA >= 9 && a.mA <= 12 && a.mB >= 9 && a.mB <= 12 && a.M <= 0x7fffff00 && a.N <= 0x7fffff00 && a.nblk <= 0x7fffffff;
}
size_t f16_planes_bytes(int64_t rows, int64_t kpad) { return f16_packed_bytes(rows, kpad); }

// packs operand A (rows a.M) and / or operand B (rows a.N) of `a` in one launch; a null buffer skips that operand
static int launch_pack(const GemmArgs &a, void *packed_a, void *packed_b, bool f16, hipStream_t s) {
    if (!packed_a && !packed_b) return HBFP_OK;
    BfPackPair q = {};
    int64_t ba = 0, bb = 0;
    if (packed_a) {
        int32_t mark;
        const int rc = mx_pack_begin(packed_a, s, &mark);
        if (rc != HBFP_OK) return rc;
        q.op[0] = bf_pack_params(a, a.mantA, a.expA, a.M, a.expA_ld, a.mA, packed_a, mark, f16);
    }
    if (packed_b) {
        int32_t mark;
        const int rc = mx_pack_begin(packed_b, s, &mark);
        if (rc != HBFP_OK) return rc;
        q.op[1] = bf_pack_params(a, a.mantB, a.expB, a.N, a.expB_ld, a.mB, packed_b, mark, f16);
    }
    if (f16) {      // the scale words of whole panels first: the pack kernel reads them
        const uint32_t ra = packed_a ? (uint32_t)(ceil_div(a.M, 256) * 256) : 0u, rb = packed_b ? (uint32_t)(ceil_div(a.N, 256) * 256) : 0u;
        hipLaunchKernelGGL(f16_row_scale_kernel, dim3((ra + rb + 255) / 256), dim3(256), 0, s, q, ra, rb);
        if (launch_status() != HBFP_OK) return HBFP_ERR_LAUNCH;
    }
    // whole panels are written: the row tiles behind the last row hold zeros
    if (packed_a) ba = ceil_div(a.M, 256) * 8 * ceil_div(q.op[0].ksteps / 2, 4);
    if (packed_b) bb = ceil_div(a.N, 256) * 8 * ceil_div(q.op[1].ksteps / 2, 4);
    if (ba + bb > 0x7fffffff) return HBFP_ERR_ARG;
    q.blocks_a = (uint32_t)ba;
    const bool wide = (packed_a ? a.mA : a.mB) > 8;             // both operands of a product are of the same storage class
    if (f16) hipLaunchKernelGGL((bf_pack_kernel<int16_t, true>), dim3((unsigned)(ba + bb)), dim3(256), 0, s, q);
    else if (wide) hipLaunchKernelGGL((bf_pack_kernel<int16_t, false>), dim3((unsigned)(ba + bb)), dim3(256), 0, s, q);
    else hipLaunchKernelGGL((bf_pack_kernel<int8_t, false>), dim3((unsigned)(ba + bb)), dim3(256), 0, s, q);
    return launch_status();
}
int launch_bf_pack(const GemmArgs &a, void *packed_a, void *packed_b, hipStream_t s) { return launch_pack(a, packed_a, packed_b, false, s); }
int launch_f16_planes_pack(const GemmArgs &a, void *packed_a, void *packed_b, hipStream_t s) {
    return launch_pack(a, packed_a, packed_b, true, s);
}

// n <= HBFP_BATCH_MAX products of operands packed as bf16 planes, in one launch; out: product 0 of a single-product
// launch is delivered as this encoded operand (a marked operand: the FP32 product goes to args[0].C instead)
static int launch_bf_group(int n, const GemmArgs *args, const void *const *packed_a, const void *const *packed_b, const MxOut *out,
                           bool f16, hipStream_t s) {
    if (n < 1 || n > kBfGroup || (out && (n != 1 || f16))) return HBFP_ERR_ARG;
    BfGroup g = {};
    g.n = n;
    if (out) g.out = *out;
    int64_t first = 0;
    for (int i = 0; i < n; ++i) {
        const GemmArgs &a = args[i];
        if (!(f16 ? gemm_f16_planes_possible(a) : gemm_bf_possible(a)) || klen_of(a, a.mA) != klen_of(a, a.mB)) return HBFP_ERR_FORMAT;
        BfParams &p = g.p[i];
        p.ha = (const int *)packed_a[i];
        p.hb = (const int *)packed_b[i];
        p.pa = (const uint8_t *)packed_a[i] + 256 + (f16 ? f16_scale_bytes(a.M) : 0);
        p.pb = (const uint8_t *)packed_b[i] + 256 + (f16 ? f16_scale_bytes(a.N) : 0);
        p.sa = f16 ? (const int32_t *)((const uint8_t *)packed_a[i] + 256) : nullptr;
        p.sb = f16 ? (const int32_t *)((const uint8_t *)packed_b[i] + 256) : nullptr;
        p.C = a.C;
        p.M = a.M;
        p.N = a.N;
        p.ldc = a.ldc;
        p.ksteps = (int32_t)(klen_of(a, a.mA) / 32);
        p.tiles_m = (int32_t)ceil_div(a.M, 256);
        p.tiles_n = (int32_t)ceil_div(a.N, 256);
        p.beta = a.beta != 0.0f;
        p.mantA = a.mantA;
        p.mantB = a.mantB;
        p.expA = a.expA;
        p.expB = a.expB;
        p.kpad = a.kpad;
        p.expA_ld = a.expA_ld;
        p.expB_ld = a.expB_ld;
        p.chunks32_per_block = (int32_t)(a.kbp / 32);
        p.shift = -(250 + a.mA + a.mB);
        p.wide = a.mA > 8;
        if (p.ksteps < kBfRing || p.ksteps % 4) return HBFP_ERR_ARG;    // the stored length is a multiple of 128
        g.first[i] = (int32_t)first;
        first += ceil_div((int64_t)p.tiles_m * p.tiles_n, 8) * 8;      // a multiple of 8: the XCD of a tile does not depend on the group
        if (first > 0x7ffffff0) return HBFP_ERR_ARG;
    }
    for (int i = n; i <= kBfGroup; ++i) g.first[i] = (int32_t)first;
    static std::atomic<bool> configured[3];
    const int which = f16 ? 2 : out ? 1 : 0;
    const void *kernel = f16   ? reinterpret_cast<const void *>(&gemm_bf_kernel<false, true>)
                         : out ? reinterpret_cast<const void *>(&gemm_bf_kernel<true, false>)
                               : reinterpret_cast<const void *>(&gemm_bf_kernel<false, false>);
    if (allow_dynamic_lds(configured[which], kernel, kBfRing * kBfStage) != HBFP_OK) return HBFP_ERR_LAUNCH;
    if (f16) hipLaunchKernelGGL((gemm_bf_kernel<false, true>), dim3((unsigned)first), dim3(kBfThreads), kBfRing * kBfStage, s, g);
    else if (out) hipLaunchKernelGGL((gemm_bf_kernel<true, false>), dim3((unsigned)first), dim3(kBfThreads), kBfRing * kBfStage, s, g);
    else hipLaunchKernelGGL((gemm_bf_kernel<false, false>), dim3((unsigned)first), dim3(kBfThreads), kBfRing * kBfStage, s, g);
    return launch_status();
}

int launch_bf_products(int n, const GemmArgs *args, const void *const *packed_a, const void *const *packed_b, hipStream_t s) {
    return launch_bf_group(n, args, packed_a, packed_b, nullptr, false, s);
}
// the same on FP16 planes (launch_f16_planes_pack)
int launch_f16_planes_products(int n, const GemmArgs *args, const void *const *packed_a, const void *const *packed_b, hipStream_t s) {
    return launch_bf_group(n, args, packed_a, packed_b, nullptr, true, s);
}

// The product as an encoded operand (output blocks of 32 or 64 along the columns of the product: mx_encoded_output_ok).
// a.C / a.ldc: FP32 scratch of M x N that receives the product when an operand is marked; the caller then queues
// launch_mx_encode_standby behind this launch, which converts it in that case only.
int launch_bf_product_encoded(const GemmArgs &a, const void *packed_a, const void *packed_b, const hbfp_tensor &out, int relu,
                              hipStream_t s) {
    if (!mx_encoded_output_ok(out)) return HBFP_ERR_FORMAT;
    const MxOut o = mx_out_of(out, relu);
    return launch_bf_group(1, &a, &packed_a, &packed_b, &o, false, s);
}

}  // namespace hbfp
