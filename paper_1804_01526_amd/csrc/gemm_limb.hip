// BFP matrix product for mantissas of 9..12 bits (Eq. (2), Sec. 4; the paper evaluates
// 12-bit mantissas in Sec. 6 "BFP design space").  The matrix cores multiply int8, so a
// mantissa v is split into two limbs, v = 64*h + l with h = v >> 6 in [-32, 31] and
// l = v & 63 in [0, 63], and a block sum becomes
//     P = 4096 * sum(hA*hB) + 64 * (sum(hA*lB) + sum(lA*hB)) + sum(lA*lB)
// with four int8 matrix instructions per k-step and three int32 accumulators (the two
// cross terms share one).  |P| <= kblock * 2047^2 < 2^31 is enforced by the host.
// P is recombined exactly in int32, converted to FP32 (round to nearest even above 2^24),
// scaled by the row and the column exponent and accumulated in FP32.
//
// Two kernels over 64 x 128 tiles of C, a stage being 64 bytes of k of both limb planes of both
// operands: gemm_limb_w8_kernel for blocks of 64 (8 waves, asynchronous copies; described where it
// starts) and gemm_limb_kernel for every other block length and for the dump of the integer block
// sums (4 waves, a wave owns 32 x 64 as 1 x 2 tiles of v_mfma_i32_32x32x32_i8, operands staged
// through registers).
#include "gemm_common.h"

namespace hbfp {
namespace {

constexpr int kThreads = 256;
constexpr int BM = 64, BN = 128, BK = 64;
constexpr int kPlaneA = BM * BK, kPlaneB = BN * BK;           // bytes of one limb plane of one stage
constexpr int kOffAH = 0, kOffAL = kPlaneA, kOffBH = 2 * kPlaneA, kOffBL = 2 * kPlaneA + kPlaneB;
constexpr int kOffWA = 2 * kPlaneA + 2 * kPlaneB;             // [2 slots][64 rows] float row scales
constexpr int kOffWB = kOffWA + 2 * BM * 4;                   // [2 slots][128 rows] float column scales
constexpr int kStageBytes = kOffWB + 2 * BN * 4;
constexpr int kLdsBytes = 2 * kStageBytes;

// int16 mantissas [rows][kpad] -> two int8 planes [rows][kpad]: hi = v >> 6, lo = v & 63
__global__ __launch_bounds__(kThreads) void limb_split_kernel(const int16_t *src, int8_t *hi, int8_t *lo, int64_t n8,
                                                              const int *run_a, const int *run_b) {
    if (stands_down(run_a, run_b)) return;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n8; i += (int64_t)gridDim.x * kThreads) {
        const v4i d = *reinterpret_cast<const v4i *>(src + i * 8);
        uint32_t h[2] = {0, 0}, l[2] = {0, 0};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int v = (int)(int16_t)((uint32_t)d[e >> 1] >> (16 * (e & 1)));
            h[e >> 2] |= (uint32_t)((v >> 6) & 0xff) << (8 * (e & 3));
            l[e >> 2] |= (uint32_t)(v & 63) << (8 * (e & 3));
        }
        *reinterpret_cast<uint2 *>(hi + i * 8) = make_uint2(h[0], h[1]);
        *reinterpret_cast<uint2 *>(lo + i * 8) = make_uint2(l[0], l[1]);
    }
}

struct LimbParams {
    const uint8_t *AH, *AL, *BH, *BL;   // int8 limb planes [rows][kpad]
    const uint8_t *eA, *eB;
    float *C;
    int32_t *P;
    int64_t M, N, kpad, eA_ld, eB_ld, ldc, nblk;
    int32_t nstage;                     // kpad / 64
    int32_t spb;                        // k-steps of 32 per exponent block
    int32_t tiles_n;
    int32_t beta;
    float final_scale;
    const int *run_a, *run_b;           // non-null: do nothing unless a packed operand is marked out of range
};

struct LimbRegs {
    v4i a[2], b[4];
    uint32_t e;
};

// SPB: k-steps per exponent block: 1, 2, or 0 = a multiple of 4 (blocks span whole stages)
template <int SPB, bool DUMP>
__global__ __launch_bounds__(kThreads, 2) void gemm_limb_kernel(const LimbParams p) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[kLdsBytes];
    if (stands_down(p.run_a, p.run_b)) return;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int tm = blockIdx.x / p.tiles_n, tn = blockIdx.x % p.tiles_n;
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;

    // staging roles: A planes are 512 pieces of 16 bytes (2 per thread), B planes 1024 (4 per thread)
    const uint8_t *gA[2], *gB[4];
    int ldsA[2], ldsB[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int idx = t + 256 * i, plane = idx >> 8, r = (idx & 255) >> 2, c = idx & 3;
        int64_t rr = row0 + r;
        rr = rr < p.M ? rr : p.M - 1;
        gA[i] = (plane ? p.AL : p.AH) + rr * p.kpad + c * 16;
        ldsA[i] = (plane ? kOffAL : kOffAH) + r * BK + ((c ^ ((r >> 1) & 3)) * 16);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = t + 256 * i, plane = idx >> 9, r = (idx & 511) >> 2, c = idx & 3;
        int64_t rr = col0 + r;
        rr = rr < p.N ? rr : p.N - 1;
        gB[i] = (plane ? p.BL : p.BH) + rr * p.kpad + c * 16;
        ldsB[i] = (plane ? kOffBL : kOffBH) + r * BK + ((c ^ ((r >> 1) & 3)) * 16);
    }
    // exponent rows: threads 0..63 take A rows, 64..191 B rows
    const bool e_a = t < 64, e_b = t >= 64 && t < 192;
    const int erow = e_a ? t : t - 64;
    const uint8_t *gE = nullptr;
    if (e_a) {
        int64_t r = row0 + erow;
        r = r < p.M ? r : p.M - 1;
        gE = p.eA + r * p.eA_ld;
    } else if (e_b) {
        int64_t r = col0 + erow;
        r = r < p.N ? r : p.N - 1;
        gE = p.eB + r * p.eB_ld;
    }
    const int stages_per_block = SPB == 0 ? p.spb / 2 : 1;

    auto load = [&](LimbRegs &r, int st) {
        const int64_t koff = (int64_t)st * BK;
#pragma unroll
        for (int i = 0; i < 2; ++i) r.a[i] = *reinterpret_cast<const v4i *>(gA[i] + koff);
#pragma unroll
        for (int i = 0; i < 4; ++i) r.b[i] = *reinterpret_cast<const v4i *>(gB[i] + koff);
        r.e = 0;
        if (gE) {
            if (SPB == 1) r.e = *reinterpret_cast<const uint16_t *>(gE + st * 2);
            else if (SPB == 2) r.e = gE[st];
            else r.e = gE[st / stages_per_block];
        }
    };
    auto store = [&](const LimbRegs &r, uint8_t *base) {
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<v4i *>(base + ldsA[i]) = r.a[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<v4i *>(base + ldsB[i]) = r.b[i];
        if (e_a || e_b) {
            uint32_t *w = reinterpret_cast<uint32_t *>(base + (e_a ? kOffWA : kOffWB));
            const int rows = e_a ? BM : BN;
            constexpr int NE = SPB == 1 ? 2 : 1;
#pragma unroll
            for (int s = 0; s < NE; ++s) {
                uint32_t e = (r.e >> (8 * s)) & 0xffu;
                e = e > 254u ? 254u : e;
                w[s * rows + erow] = e << 23;   // the float 2^(E - 127)
            }
        }
    };

    int offA = (wm * 32 + l32) * BK, swzA = ((wm * 32 + l32) >> 1) & 3;
    int offB[2], swzB[2];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const int r = wn * 64 + ni * 32 + l32;
        offB[ni] = r * BK;
        swzB[ni] = (r >> 1) & 3;
    }

    float acc[2][16];
    v16i hh[2], mid[2], ll[2];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            acc[ni][v] = 0.0f;
            hh[ni][v] = 0;
            mid[ni][v] = 0;
            ll[ni][v] = 0;
        }

    v16i zero;
#pragma unroll
    for (int v = 0; v < 16; ++v) zero[v] = 0;

    LimbRegs regs;
    if (p.nstage > 0) {
        load(regs, 0);
        store(regs, lds);
    }
    __syncthreads();

    for (int st = 0; st < p.nstage; ++st) {
        const bool more = st + 1 < p.nstage;
        if (more) load(regs, st + 1);
        const uint8_t *base = lds + (st & 1) * kStageBytes;

#pragma unroll 1
        for (int s = 0; s < 2; ++s) {
            bool first, last;
            int slot;
            if (SPB == 1) { first = true; last = true; slot = s; }
            else if (SPB == 2) { first = s == 0; last = s == 1; slot = 0; }
            else {
                first = s == 0 && (st % stages_per_block) == 0;
                last = s == 1 && ((st + 1) % stages_per_block) == 0;
                slot = 0;
            }
            const int chunkA = ((2 * s + lh) ^ swzA) * 16;
            const v4i aH = *reinterpret_cast<const v4i *>(base + kOffAH + offA + chunkA);
            const v4i aL = *reinterpret_cast<const v4i *>(base + kOffAL + offA + chunkA);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const int chunkB = ((2 * s + lh) ^ swzB[ni]) * 16;
                const v4i bH = *reinterpret_cast<const v4i *>(base + kOffBH + offB[ni] + chunkB);
                const v4i bL = *reinterpret_cast<const v4i *>(base + kOffBL + offB[ni] + chunkB);
                if (first) {   // a new exponent block starts from zero: no accumulator clearing
                    hh[ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aH, bH, zero, 0, 0, 0);
                    mid[ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aH, bL, zero, 0, 0, 0);
                    ll[ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aL, bL, zero, 0, 0, 0);
                } else {
                    hh[ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aH, bH, hh[ni], 0, 0, 0);
                    mid[ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aH, bL, mid[ni], 0, 0, 0);
                    ll[ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aL, bL, ll[ni], 0, 0, 0);
                }
                mid[ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aL, bH, mid[ni], 0, 0, 0);
            }
            if (last) {
                float sa[16];
                if (!DUMP) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const v4i w4 = *reinterpret_cast<const v4i *>(base + kOffWA + (slot * BM + wm * 32 + 8 * g + 4 * lh) * 4);
                        sa[4 * g + 0] = __int_as_float(w4[0]);
                        sa[4 * g + 1] = __int_as_float(w4[1]);
                        sa[4 * g + 2] = __int_as_float(w4[2]);
                        sa[4 * g + 3] = __int_as_float(w4[3]);
                    }
                }
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    const float sb = DUMP ? 0.0f
                                          : *reinterpret_cast<const float *>(base + kOffWB + (slot * BN + wn * 64 + ni * 32 + l32) * 4);
                    const int64_t blk = SPB == 0 ? st / stages_per_block : ((int64_t)st * 2 + s) / SPB;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int P = (hh[ni][v] << 12) + (mid[ni][v] << 6) + ll[ni][v];
                        if (!DUMP) {
                            acc[ni][v] = fmaf((float)P * sa[v], sb, acc[ni][v]);
                        } else {
                            const int64_t i = row0 + wm * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                            const int64_t j = col0 + wn * 64 + ni * 32 + l32;
                            if (blk < p.nblk && i < p.M && j < p.N) p.P[(i * p.N + j) * p.nblk + blk] = P;
                        }
                    }
                }
            }
        }
        if (more) store(regs, lds + ((st + 1) & 1) * kStageBytes);
        __syncthreads();
    }

    if (DUMP) return;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t i = row0 + wm * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
            const int64_t j = col0 + wn * 64 + ni * 32 + l32;
            if (i < p.M && j < p.N) {
                const float val = acc[ni][v] * p.final_scale;
                if (p.beta) p.C[i * p.ldc + j] += val;
                else __builtin_nontemporal_store(val, p.C + i * p.ldc + j);   // written once, not read again here
            }
        }
}

// ------------------------------------------------------------------------------------------------
// Blocks of 64 (the 12-bit configuration): same organisation as the 8-bit kernel for short blocks -
// 8 waves per workgroup at 4 waves per SIMD, asynchronous global -> LDS copies through a ring of LDS
// buffers, one barrier per stage, row scales spread over the output layout by one bf16 matrix
// instruction per block.  A workgroup owns 64 x 128 of C, a wave 32 x 32; a stage is one exponent block
// (64 bytes of k of the four limb planes, 24 KB, plus one scale word per operand row), three stages
// live in LDS.  Per wave and block: 8 matrix instructions, then 5 vector instructions per output.
constexpr int kLwThreads = 512;
constexpr int kLwAH = 0, kLwAL = 4096, kLwBH = 8192, kLwBL = 16384;   // [rows][64 bytes], 16-byte chunks XORed with (row >> 2) & 3
constexpr int kLwWA = 24576, kLwWB = 24832;                            // 64 row words, 128 column words
constexpr int kLwStage = 25344;
constexpr int kLwRing = 3;
constexpr int kLwLdsBytes = kLwRing * kLwStage;                        // 74.25 KB: two workgroups per CU

struct LimbW8Params {
    LimbParams g;
    const uint32_t *wA, *wB;     // scale words [block][rows rounded up to 128]: 2^(E - 127) as bf16 / as FP32
    int64_t mpad, npad;
    int32_t tiles_m;
};

__global__ __launch_bounds__(kLwThreads, 4) void gemm_limb_w8_kernel(const LimbW8Params q) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const LimbParams &p = q.g;
    if (stands_down(p.run_a, p.run_b)) return;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, lh = lane >> 5;

    int tm, tn;
    if (!tile_of_workgroup(blockIdx.x, q.tiles_m, p.tiles_n, tm, tn)) return;   // whole workgroup, before any barrier
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
    const int nst = p.nstage;

    // ---- copy roles, four per wave and stage: 16 rows of one A plane (wave >> 2 picks the plane), the
    // same 16 rows of both B planes, and 64 scale words (waves 0, 3, 6: A rows; 1, 4, 7 and 2, 5: the two
    // halves of the B rows; duplicates write the same words)
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    uint32_t voffA, voffB;
    {
        const int rows_a = (int)((p.M - row0) < BM ? (p.M - row0) : BM), rows_b = (int)((p.N - col0) < BN ? (p.N - col0) : BN);
        const int ra_ = 16 * (wave & 3) + (lane >> 2), rb_ = 16 * wave + (lane >> 2);
        const int ra = ra_ < rows_a ? ra_ : rows_a - 1;   // rows past the edge re-read the last row; never stored
        const int rb = rb_ < rows_b ? rb_ : rows_b - 1;
        voffA = (uint32_t)ra * (uint32_t)p.kpad + (((lane & 3) ^ ((ra_ >> 2) & 3)) * 16);
        voffB = (uint32_t)rb * (uint32_t)p.kpad + (((lane & 3) ^ ((rb_ >> 2) & 3)) * 16);
    }
    const uint32_t voffW = lane * 4;
    const uint8_t *planeA = (wave_u >> 2 ? p.AL : p.AH) + row0 * p.kpad;
    const uint8_t *planeBH = p.BH + col0 * p.kpad, *planeBL = p.BL + col0 * p.kpad;
    const int wsel = wave_u % 3;
    const uint32_t *wordsrc = wsel == 0 ? q.wA + row0 : q.wB + col0 + 64 * (wsel - 1);
    const int64_t wordpitch = wsel == 0 ? q.mpad : q.npad;
    const uint32_t ldsA = (wave_u >> 2 ? kLwAL : kLwAH) + (wave_u & 3) * 1024;
    const uint32_t ldsB = wave_u * 1024;
    const uint32_t ldsW = wsel == 0 ? kLwWA : kLwWB + 256 * (wsel - 1);

#define HBFP_COPY_STAGE(st, ring)                                                                       \
    {                                                                                                   \
        const uint32_t lb = (ring) * kLwStage;                                                          \
        async_copy16(planeA + (int64_t)(st) * BK, voffA, lb + ldsA);                                    \
        async_copy16(planeBH + (int64_t)(st) * BK, voffB, lb + kLwBH + ldsB);                           \
        async_copy16(planeBL + (int64_t)(st) * BK, voffB, lb + kLwBL + ldsB);                           \
        async_copy4(wordsrc + (int64_t)(st) * wordpitch, voffW, lb + ldsW);                             \
    }
#define HBFP_WAIT_COPIES(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")

    // ---- fragment addresses in ring buffer 0; k-step 1 flips the 32-byte half of the row
    const int r_a = wm * 32 + l32, r_b = wn * 32 + l32;
    const int fragA = r_a * 64 + ((lh ^ ((r_a >> 2) & 3)) * 16);
    const int fragB = kLwBH + r_b * 64 + ((lh ^ ((r_b >> 2) & 3)) * 16);
    const int offW = kLwWA + r_a * 4, offS = kLwWB + r_b * 4;
    const v2i one_hot = {lh ? 0 : 0x3F80, 0};

    float acc[16];
    v16i hh, mid, ll;
    v16i zero;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        acc[v] = 0.0f;
        zero[v] = 0;
    }
    v4i aH, aL, bH, bL;
    uint32_t rowc = 0;
    float sb = 0.0f;
#define HBFP_READ_FRAGS(ring, s)                                                                        \
    {                                                                                                   \
        const uint8_t *base_ = lds + (ring) * kLwStage;                                                 \
        aH = *reinterpret_cast<const v4i *>(base_ + (fragA ^ ((s) * 32)));                              \
        aL = *reinterpret_cast<const v4i *>(base_ + (fragA ^ ((s) * 32)) + kLwAL);                      \
        bH = *reinterpret_cast<const v4i *>(base_ + (fragB ^ ((s) * 32)));                              \
        bL = *reinterpret_cast<const v4i *>(base_ + (fragB ^ ((s) * 32)) + (kLwBL - kLwBH));            \
    }
#define HBFP_READ_WORDS(ring)                                                                           \
    {                                                                                                   \
        const uint8_t *base_ = lds + (ring) * kLwStage;                                                 \
        rowc = *reinterpret_cast<const uint32_t *>(base_ + offW);                                       \
        sb = *reinterpret_cast<const float *>(base_ + offS);                                            \
    }
    // One stage = one exponent block.  The hand-over sits right after the block's last matrix
    // instructions: every LDS read of the stage is consumed by then, so after the barrier its buffer
    // takes stage st + 3, and stage st + 1 has landed for everyone (copies complete in issue order: all
    // but the newest group of four).  The recombination and scaling of the block then cover the latency
    // of the next stage's first fragments.
#define HBFP_STAGE(ring)                                                                                \
    {                                                                                                   \
        hh = __builtin_amdgcn_mfma_i32_32x32x32_i8(aH, bH, zero, 0, 0, 0);                              \
        mid = __builtin_amdgcn_mfma_i32_32x32x32_i8(aH, bL, zero, 0, 0, 0);                             \
        ll = __builtin_amdgcn_mfma_i32_32x32x32_i8(aL, bL, zero, 0, 0, 0);                              \
        mid = __builtin_amdgcn_mfma_i32_32x32x32_i8(aL, bH, mid, 0, 0, 0);                              \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        HBFP_READ_FRAGS(ring, 1);                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        hh = __builtin_amdgcn_mfma_i32_32x32x32_i8(aH, bH, hh, 0, 0, 0);                                \
        mid = __builtin_amdgcn_mfma_i32_32x32x32_i8(aH, bL, mid, 0, 0, 0);                              \
        ll = __builtin_amdgcn_mfma_i32_32x32x32_i8(aL, bL, ll, 0, 0, 0);                                \
        mid = __builtin_amdgcn_mfma_i32_32x32x32_i8(aL, bH, mid, 0, 0, 0);                              \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        const int rem = nst - 1 - st;                                                                   \
        if (rem > 0) {                                                                                  \
            if (rem >= 2) HBFP_WAIT_COPIES(4); else HBFP_WAIT_COPIES(0);                                \
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                          \
            __builtin_amdgcn_s_barrier();                                                               \
            asm volatile("" ::: "memory");                                                              \
            if (rem >= 3) HBFP_COPY_STAGE(st + 3, ring);                                                \
            HBFP_READ_FRAGS(((ring) + 1) % 3, 0);                                                       \
        }                                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        const v16i sa = row_constants(rowc, one_hot);                                                   \
        asm volatile("" ::"v"(sa));   /* issued here: the recombination below covers its latency */     \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        int P[16];                                                                                      \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) P[v] = (((hh[v] << 6) + mid[v]) << 6) + ll[v];   \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(P[v]));                   \
        float x[16];                                                                                    \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) x[v] = (float)P[v];                              \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) x[v] *= __int_as_float(sa[v]);                   \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[v] = fmaf(x[v], sb, acc[v]);                 \
        _Pragma("unroll") for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(acc[v]));                 \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        if (rem > 0) HBFP_READ_WORDS(((ring) + 1) % 3);                                                 \
    }

    if (nst > 0) {
        HBFP_COPY_STAGE(0, 0);
        if (nst > 1) HBFP_COPY_STAGE(1, 1);
        if (nst > 2) HBFP_COPY_STAGE(2, 2);
        if (nst > 2) HBFP_WAIT_COPIES(8); else if (nst == 2) HBFP_WAIT_COPIES(4); else HBFP_WAIT_COPIES(0);
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (nst > 0) {
        HBFP_READ_FRAGS(0, 0);
        HBFP_READ_WORDS(0);
    }
    for (int st = 0; st < nst;) {
        HBFP_STAGE(0);
        if (++st >= nst) break;
        HBFP_STAGE(1);
        if (++st >= nst) break;
        HBFP_STAGE(2);
        ++st;
    }
#undef HBFP_STAGE
#undef HBFP_READ_WORDS
#undef HBFP_READ_FRAGS
#undef HBFP_COPY_STAGE
#undef HBFP_WAIT_COPIES

#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int64_t i = row0 + wm * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
        const int64_t j = col0 + wn * 32 + l32;
        if (i < p.M && j < p.N) {
            const float val = acc[v] * p.final_scale;
            if (p.beta) p.C[i * p.ldc + j] += val;
            else __builtin_nontemporal_store(val, p.C + i * p.ldc + j);   // written once, not read again here
        }
    }
}

template <int SPB, bool DUMP>
int launch_t(const LimbParams &p, dim3 grid, hipStream_t s) {
    hipLaunchKernelGGL((gemm_limb_kernel<SPB, DUMP>), grid, dim3(kThreads), 0, s, p);
    return launch_status();
}

size_t plane_bytes(int64_t rows, int64_t kpad) { return ((size_t)rows * (size_t)kpad + 255) & ~(size_t)255; }

}  // namespace

// workspace: [A hi][A lo][B hi][B lo] int8 planes, [A row words][B column words] (blocks of 64 only)
size_t gemm_limb_workspace(const hbfp_tensor *A, const hbfp_tensor *B) {
    size_t n = 2 * plane_bytes(A->rows, A->kpad) + 2 * plane_bytes(B->rows, B->kpad);
    if (A->kblock_pad == 64) n += word_bytes(A->rows, A->exp_ld) + word_bytes(B->rows, B->exp_ld);
    return n;
}

int launch_gemm_limb(const GemmArgs &a, void *workspace, hipStream_t s) {
    uint8_t *w = (uint8_t *)workspace;
    const size_t pa = plane_bytes(a.M, a.kpad), pb = plane_bytes(a.N, a.kpad);
    LimbParams p;
    p.AH = w;
    p.AL = w + pa;
    p.BH = w + 2 * pa;
    p.BL = w + 2 * pa + pb;
    {
        const int64_t na = a.M * a.kpad / 8, nb = a.N * a.kpad / 8;   // kpad is a multiple of 128
        int64_t ga = ceil_div(na, kThreads), gb = ceil_div(nb, kThreads);
        ga = ga > 65536 ? 65536 : ga;
        gb = gb > 65536 ? 65536 : gb;
        hipLaunchKernelGGL(limb_split_kernel, dim3((unsigned)ga), dim3(kThreads), 0, s, (const int16_t *)a.mantA,
                           (int8_t *)p.AH, (int8_t *)p.AL, na, a.run_a, a.run_b);
        hipLaunchKernelGGL(limb_split_kernel, dim3((unsigned)gb), dim3(kThreads), 0, s, (const int16_t *)a.mantB,
                           (int8_t *)p.BH, (int8_t *)p.BL, nb, a.run_a, a.run_b);
        if (launch_status() != HBFP_OK) return HBFP_ERR_LAUNCH;
    }
    p.eA = a.expA;
    p.eB = a.expB;
    p.C = a.C;
    p.P = a.P;
    p.M = a.M;
    p.N = a.N;
    p.kpad = a.kpad;
    p.eA_ld = a.expA_ld;
    p.eB_ld = a.expB_ld;
    p.ldc = a.ldc;
    p.nblk = a.nblk;
    if (a.kpad / BK > 0x7fffffff) return HBFP_ERR_ARG;
    p.nstage = (int32_t)(a.kpad / BK);
    p.spb = (int32_t)(a.kbp / 32);
    const int64_t tm = ceil_div(a.M, BM), tn = ceil_div(a.N, BN);
    if (tm * tn > 0x7fffffff) return HBFP_ERR_ARG;
    p.tiles_n = (int32_t)tn;
    p.beta = a.beta != 0.0f;
    p.final_scale = ldexpf(1.0f, 4 - a.mA - a.mB);
    p.run_a = a.run_a;
    p.run_b = a.run_b;
    const dim3 grid((unsigned)(tm * tn));
    if (!a.P && !a.run_a && p.spb == 2 && (uint64_t)127 * (uint64_t)a.kpad + 64 < ((uint64_t)1 << 32) && ceil_div(tm * tn, 8) * 8 <= 0x7fffffff) {
        static std::atomic<bool> configured{false};
        if (allow_dynamic_lds(configured, reinterpret_cast<const void *>(&gemm_limb_w8_kernel), kLwLdsBytes) != HBFP_OK) return HBFP_ERR_LAUNCH;
        LimbW8Params q;
        q.g = p;
        q.mpad = ceil_div(a.M, 128) * 128;
        q.npad = ceil_div(a.N, 128) * 128;
        q.tiles_m = (int32_t)tm;
        uint8_t *ww = w + 2 * pa + 2 * pb;
        q.wA = (const uint32_t *)ww;
        q.wB = (const uint32_t *)(ww + word_bytes(a.M, a.expA_ld));
        const int rc = launch_scale_words(a.expA, a.expA_ld, a.M, a.expB, a.expB_ld, a.N, (int)a.expA_ld, 0u,
                                          const_cast<uint32_t *>(q.wA), const_cast<uint32_t *>(q.wB), a.run_a, a.run_b, s);
        if (rc != HBFP_OK) return rc;
        hipLaunchKernelGGL(gemm_limb_w8_kernel, dim3((unsigned)(ceil_div(tm * tn, 8) * 8)), dim3(kLwThreads), kLwLdsBytes, s, q);
        return launch_status();
    }
    if (a.P) return p.spb == 1 ? launch_t<1, true>(p, grid, s) : p.spb == 2 ? launch_t<2, true>(p, grid, s) : launch_t<0, true>(p, grid, s);
    return p.spb == 1 ? launch_t<1, false>(p, grid, s) : p.spb == 2 ? launch_t<2, false>(p, grid, s) : launch_t<0, false>(p, grid, s);
}

}  // namespace hbfp
