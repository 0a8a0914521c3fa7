// BFP matrix product with one exponent per operand row (the basic scheme of Sec. 4: "one exponent per row
// of A and per column of B", Eq. (2) with a single block):
//     C[i][j] = 2^(eA[i] + eB[j]) * sum_k mA[i][k] * mB[j][k]
// Here nothing happens between the matrix instructions of a tile: the whole contraction is one chain of
// v_mfma_i32_32x32x32_i8 into int32 accumulators and the two exponents are applied once, when C is stored.
// The kernel is therefore built for the matrix core alone: a 256 x 256 tile of C per workgroup, four waves
// of 128 x 128 at one wave per SIMD (256 int32 accumulators per lane), so that a pair of matrix instructions
// needs one 16-byte LDS read per lane (64 B/clk per CU at the full matrix rate; a 64 x 128 wave tile would need
// 94 of the 128 the LDS can deliver).  Operands are read as they are stored (int8 [rows][kpad]): 64 bytes of k
// of 256 + 256 rows per stage (32 KB), copied global -> LDS asynchronously into a ring of four buffers, rows of
// 64 bytes with the 16-byte chunk index XORed with (row >> 2) & 3 as in the other int8 kernels (copies of 16 rows
// and fragment reads of 32 rows then both cover all banks).  Fragments are read one k-step (32) ahead, between
// the matrix instructions, and the hand-over of a ring buffer (one barrier per stage) sits in the middle of a stage.
#include "gemm_common.h"

namespace hbfp {
namespace {

constexpr int kWideThreads = 256;
constexpr int kWideRows = 256;                          // tile of C is 256 x 256
constexpr int kWideK = 64;                              // bytes of k per stage
constexpr int kWideOperand = kWideRows * kWideK;        // 16 KB
constexpr int kWideStage = 2 * kWideOperand;            // 32 KB
constexpr int kWideRing = 4;
constexpr int kWideLds = kWideRing * kWideStage;        // 128 KB
constexpr int kWideCopies = kWideStage / 1024 / 4;      // 8 copies of 1 KB (16 rows x 64 B) per wave and stage

struct WideParams {
    const uint8_t *A, *B;        // int8 mantissas [rows][kpad]
    const uint8_t *eA, *eB;      // exponent bytes [rows][exp_ld], block 0
    float *C;
    int64_t M, N, kpad, eA_ld, eB_ld, ldc;
    int32_t nstage;              // kpad / 64 (even)
    int32_t tiles_m, tiles_n, beta;
    int32_t exp_offset;          // C = acc * 2^(Ea + Eb + exp_offset)
    const int *run_a, *run_b;
};

__global__ __launch_bounds__(kWideThreads, 1) void gemm_i8_wide_kernel(const WideParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    if (stands_down(p.run_a, p.run_b)) return;
    int tm, tn;
    if (!tile_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn)) return;   // whole workgroup, before any barrier

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int64_t row0 = (int64_t)tm * kWideRows, col0 = (int64_t)tn * kWideRows;

    // ---- copies: piece c of a stage is 16 rows x 64 bytes; pieces 0..15 are A, 16..31 B; wave w moves pieces w, w + 4, ...
    // A lane copies 16 bytes: row 16 c + lane / 4, LDS chunk lane % 4, which holds source chunk (lane % 4) ^ ((row >> 2) & 3).
    // Rows past the edge re-read the last row (their results are never stored).
    const uint8_t *cbase[kWideCopies];
    uint32_t cvoff[kWideCopies], coff[kWideCopies];
#pragma unroll
    for (int i = 0; i < kWideCopies; ++i) {
        const int c = wave + 4 * i;
        const bool is_a = c < 16;
        const int r = 16 * (c & 15) + (lane >> 2);
        const int64_t lim = is_a ? p.M - row0 : p.N - col0;
        const int rr = r < lim ? r : (int)lim - 1;
        const int chunk = (lane & 3) ^ ((r >> 2) & 3);
        cbase[i] = is_a ? p.A + row0 * p.kpad : p.B + col0 * p.kpad;
        cvoff[i] = (uint32_t)rr * (uint32_t)p.kpad + chunk * 16;
        coff[i] = c * 1024;
    }
#define HBFP_WIDE_COPY(i, ring_)                                                                    \
    {                                                                                              \
        async_copy16(cbase[i], cvoff[i], (uint32_t)((ring_) * kWideStage) + coff[i]);              \
        cbase[i] += kWideK;                                                                        \
    }
#define HBFP_WIDE_COPY_STAGE(ring_)                                                                 \
    {                                                                                              \
        _Pragma("unroll") for (int i = 0; i < kWideCopies; ++i) HBFP_WIDE_COPY(i, ring_);          \
    }

    // ---- fragment addresses inside a stage: row tile i of A is rows 128 wm + 32 i + l32, k-step s the chunks 2 s + lh
    int fa[2], fb[2];                                   // per k-step: byte offset of (row tile 0, this lane); tiles are 2 KB apart
    {
        const int ra = 128 * wm + l32, rb = 128 * wn + l32;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            fa[s] = ra * kWideK + (((2 * s + lh) ^ ((ra >> 2) & 3)) * 16);
            fb[s] = kWideOperand + rb * kWideK + (((2 * s + lh) ^ ((rb >> 2) & 3)) * 16);
        }
    }

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    v4i a[2][4], b[2][4];                               // [buffer][tile]
#define HBFP_WIDE_FENCE                 \
    asm volatile("" ::: "memory");      \
    __builtin_amdgcn_sched_barrier(0)
#define HBFP_WIDE_READ(buf, base_, s, i)                                                                       \
    {                                                                                                         \
        a[buf][i] = *reinterpret_cast<const v4i *>((base_) + fa[s] + (i) * 2048);                             \
        b[buf][i] = *reinterpret_cast<const v4i *>((base_) + fb[s] + (i) * 2048);                             \
    }
    // one k-step of 32: 16 matrix instructions on buffer `buf`; after each group of four, one row tile and one column
    // tile of the next k-step are requested into the other buffer (EXTRA: the hand-over's copies ride along)
#define HBFP_WIDE_ROW(buf, i)                                                                                  \
    {                                                                                                         \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                         \
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[buf][i], b[buf][j], acc[i][j], 0, 0, 0);      \
    }
#define HBFP_WIDE_KSTEP(buf, NEXT, nbase_, ns, COPY, ring_)                                                     \
    {                                                                                                         \
        HBFP_WIDE_ROW(buf, 0);                                                                                \
        if (NEXT) HBFP_WIDE_READ(1 - (buf), nbase_, ns, 0);                                                   \
        if (COPY) { HBFP_WIDE_COPY(0, ring_); HBFP_WIDE_COPY(1, ring_); }                                     \
        HBFP_WIDE_FENCE;                                                                                      \
        HBFP_WIDE_ROW(buf, 1);                                                                                \
        if (NEXT) HBFP_WIDE_READ(1 - (buf), nbase_, ns, 1);                                                   \
        if (COPY) { HBFP_WIDE_COPY(2, ring_); HBFP_WIDE_COPY(3, ring_); }                                     \
        HBFP_WIDE_FENCE;                                                                                      \
        HBFP_WIDE_ROW(buf, 2);                                                                                \
        if (NEXT) HBFP_WIDE_READ(1 - (buf), nbase_, ns, 2);                                                   \
        if (COPY) { HBFP_WIDE_COPY(4, ring_); HBFP_WIDE_COPY(5, ring_); }                                     \
        HBFP_WIDE_FENCE;                                                                                      \
        HBFP_WIDE_ROW(buf, 3);                                                                                \
        if (NEXT) HBFP_WIDE_READ(1 - (buf), nbase_, ns, 3);                                                   \
        if (COPY) { HBFP_WIDE_COPY(6, ring_); HBFP_WIDE_COPY(7, ring_); }                                     \
        HBFP_WIDE_FENCE;                                                                                      \
    }
    // A stage: k-step 0 (its fragments were requested during the stage before), then the hand-over: this wave's copies
    // of the next stage have landed when only those of the stage after it are in flight; after the barrier everybody's
    // have, and everybody has read the last fragment of the stage before this one, whose buffer takes the copies of
    // stage st + 3 (issued between the matrix instructions of k-step 1).
    // MODE 0: hand-over with copies;  1: hand-over, nothing left to copy, one more stage in flight;  2: hand-over,
    // the next stage is the last;  3: last stage
#define HBFP_WIDE_STAGE(MODE)                                                                                  \
    {                                                                                                         \
        const uint8_t *base = lds + ring * kWideStage;                                                        \
        const int next = (ring + 1) & 3, free_ring = (ring + 3) & 3;                                          \
        HBFP_WIDE_KSTEP(0, true, base, 1, false, 0);                                                          \
        if (MODE != 3) {                                                                                      \
            if (MODE != 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kWideCopies) : "memory");                 \
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                             \
            __builtin_amdgcn_s_barrier();                                                                     \
            asm volatile("" ::: "memory");                                                                    \
        }                                                                                                     \
        HBFP_WIDE_KSTEP(1, MODE != 3, lds + next * kWideStage, 0, MODE == 0, free_ring);                      \
        ring = next;                                                                                          \
    }

    // prologue: stages 0..2 on their way (the contraction has at least two stages), fragments of k-step 0
    HBFP_WIDE_COPY_STAGE(0);
    HBFP_WIDE_COPY_STAGE(1);
    if (p.nstage > 2) {
        HBFP_WIDE_COPY_STAGE(2);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kWideCopies) : "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kWideCopies) : "memory");
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < 4; ++i) HBFP_WIDE_READ(0, lds, 0, i);
    int ring = 0;
    int st = 0;
    for (; st + 4 <= p.nstage; ++st) HBFP_WIDE_STAGE(0);     // stage st + 3 exists
    if (p.nstage - st == 3) {
        HBFP_WIDE_STAGE(1);
        ++st;
    }
    HBFP_WIDE_STAGE(2);
    HBFP_WIDE_STAGE(3);
#undef HBFP_WIDE_STAGE
#undef HBFP_WIDE_KSTEP
#undef HBFP_WIDE_ROW
#undef HBFP_WIDE_READ
#undef HBFP_WIDE_FENCE
#undef HBFP_WIDE_COPY_STAGE
#undef HBFP_WIDE_COPY

    // ---- C = acc * 2^(Ea + Eb + offset): int32 -> FP32 rounds to nearest even above 2^24, the scaling is exact
    int eb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t col = col0 + 128 * wn + 32 * j + l32;
        int e = col < p.N ? p.eB[col * p.eB_ld] : 1;
        eb[j] = (e > 254 ? 254 : e) + p.exp_offset;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t row = row0 + 128 * wm + 32 * i + 8 * (v >> 2) + 4 * lh + (v & 3);
            if (row >= p.M) continue;
            int ea = p.eA[row * p.eA_ld];
            ea = ea > 254 ? 254 : ea;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t col = col0 + 128 * wn + 32 * j + l32;
                if (col >= p.N) continue;
                const float val = ldexpf((float)acc[i][j][v], ea + eb[j]);
                float *dst = p.C + row * p.ldc + col;
                if (p.beta) *dst = *dst + val;
                else __builtin_nontemporal_store(val, dst);               // written once, not read again here
            }
        }
}

}  // namespace

// One exponent per operand row, 8-bit mantissas, rows of the stored operands addressable with 32-bit offsets
bool gemm_wide_possible(const GemmArgs &a) {
    return !a.P && a.nblk == 1 && a.mA <= 8 && a.mB <= 8 && (uint64_t)255 * (uint64_t)a.kpad + 64 < ((uint64_t)1 << 32) &&
           ceil_div(a.M, kWideRows) * ceil_div(a.N, kWideRows) <= 0x7ffffff0 && a.kpad / kWideK <= 0x7fffffff;
}

// ... and enough full tiles of 256 x 256 to fill the chip
bool gemm_wide_ok(const GemmArgs &a) {
    if (!gemm_wide_possible(a)) return false;
    const int64_t tiles = ceil_div(a.M, kWideRows) * ceil_div(a.N, kWideRows);
    return tiles >= 128 && (double)a.M * (double)a.N >= 0.75 * 65536.0 * (double)tiles;
}

int launch_gemm_wide(const GemmArgs &a, hipStream_t s) {
    static std::atomic<bool> configured{false};
    if (allow_dynamic_lds(configured, reinterpret_cast<const void *>(&gemm_i8_wide_kernel), kWideLds) != HBFP_OK) return HBFP_ERR_LAUNCH;
    WideParams p;
    p.A = (const uint8_t *)a.mantA;
    p.B = (const uint8_t *)a.mantB;
    p.eA = a.expA;
    p.eB = a.expB;
    p.C = a.C;
    p.M = a.M;
    p.N = a.N;
    p.kpad = a.kpad;
    p.eA_ld = a.expA_ld;
    p.eB_ld = a.expB_ld;
    p.ldc = a.ldc;
    p.nstage = (int32_t)(a.kpad / kWideK);
    p.tiles_m = (int32_t)ceil_div(a.M, kWideRows);
    p.tiles_n = (int32_t)ceil_div(a.N, kWideRows);
    p.beta = a.beta != 0.0f;
    p.exp_offset = -250 - a.mA - a.mB;
    p.run_a = a.run_a;
    p.run_b = a.run_b;
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    hipLaunchKernelGGL(gemm_i8_wide_kernel, dim3((unsigned)(ceil_div(tiles, 8) * 8)), dim3(kWideThreads), kWideLds, s, p);
    return launch_status();
}

}  // namespace hbfp
