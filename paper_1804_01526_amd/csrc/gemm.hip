// BFP matrix product for gfx950, Eq. (2) of Sec. 4 with per-block FP accumulation
// (Sec. 4 "tiled" products, Sec. 4.2 Tiling):
//     C[i][j] = sum_b 2^(eA[i][b] + eB[j][b]) * sum_{k in b} mA[i][k] * mB[j][k]
//
// Both operands are stored with k contiguous (public header), so this is an "NT"
// product.  A workgroup of 4 waves owns a 128 x 128 tile of C; a wave owns 64 x 64 as
// 2 x 2 tiles of v_mfma_i32_32x32x32_i8.  A stage is 128 bytes of k for all 256
// operand rows of the tile, staged through LDS (double buffered).
//
// The per-block scaling is the expensive part on this chip (one FP32 operation per 2*B
// integer operations is cheap next to 8-bit multipliers in the paper's accelerator,
// Sec. 4.2; here the matrix core retires 2048 integer operations per clock and SIMD while the
// vector ALU retires 16 lanes).  It is kept to two vector instructions per output and block:
//   1. the matrix core starts from a constant C input whose int32 bit pattern is the
//      float 1.5 * 2^(Ea - 127): adding the integer block sum P (|P| < 2^22) to those
//      bits gives the float (1.5 * 2^23 + P) * 2^(Ea - 150), so the int->float
//      conversion and the row exponent cost nothing;
//   2. one subtraction removes the constant (exact), one FMA multiplies by the column
//      scale 2^(Eb - 127) and accumulates.
// The remaining constant 2^(27 - mA - mB) is applied once when C is stored.
#include "hbfp_internal.h"

namespace hbfp {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BM = 128, BN = 128, BK = 128;            // tile of C, bytes of k per stage
constexpr int kMantBytes = BM * BK;                     // one operand tile of one stage
constexpr int kWordBytes = 4 * 128 * 4;                 // up to 4 exponent blocks per stage x 128 rows
constexpr int kStageBytes = 2 * kMantBytes + 2 * kWordBytes;
constexpr int kLdsBytes = 2 * kStageBytes;

struct GemmParams {
    const uint8_t *A, *B;        // int8 mantissas [rows][kpad]
    const uint8_t *eA, *eB;      // exponent bytes [rows][exp_ld]
    float *C;                    // [M][ldc]
    float *partial;              // split-K: [splits][M][N]
    int32_t *P;                  // partial dump [M][N][nblk]
    int64_t M, N, kpad, eA_ld, eB_ld, ldc, nblk;
    int32_t nstage;              // kpad / 128
    int32_t spb;                 // 32-byte k-steps per exponent block (kblock_pad / 32)
    int32_t stages_per_split;
    int32_t splits;
    int32_t tiles_m, tiles_n;
    int32_t beta;
    float final_scale;
};

struct StageRegs {
    v4i a[4], b[4];
    uint32_t e;
};

// global -> registers: 4 x 16 bytes of each operand and this thread's exponent bytes of stage st
template <int SPB>
__device__ __forceinline__ void load_stage(StageRegs &r, const uint8_t *const (&gA)[4], const uint8_t *const (&gB)[4],
                                           const uint8_t *gE, int st, int stages_per_block) {
    const int64_t koff = (int64_t)st * BK;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        r.a[i] = *reinterpret_cast<const v4i *>(gA[i] + koff);
        r.b[i] = *reinterpret_cast<const v4i *>(gB[i] + koff);
    }
    if (SPB == 1) r.e = *reinterpret_cast<const uint32_t *>(gE + st * 4);
    else if (SPB == 2) r.e = *reinterpret_cast<const uint16_t *>(gE + st * 2);
    else r.e = gE[st / stages_per_block];
}

// registers -> LDS; the exponent bytes become the 32-bit words the matrix core and the FMA use
template <int SPB, bool DUMP>
__device__ __forceinline__ void store_stage(const StageRegs &r, uint8_t *base, const int (&ldsoff)[4], bool exp_is_a,
                                            int erow) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<v4i *>(base + ldsoff[i]) = r.a[i];
        *reinterpret_cast<v4i *>(base + kMantBytes + ldsoff[i]) = r.b[i];
    }
    uint32_t *w = reinterpret_cast<uint32_t *>(base + 2 * kMantBytes + (exp_is_a ? 0 : kWordBytes));
    constexpr int NE = SPB == 1 ? 4 : SPB == 2 ? 2 : 1;
#pragma unroll
    for (int s = 0; s < NE; ++s) {
        uint32_t e = (r.e >> (8 * s)) & 0xffu;
        e = e > 254u ? 254u : e;
        uint32_t word = e << 23;                                // B side: the float 2^(E - 127)
        if (exp_is_a) word = DUMP ? 0u : (word | 0x400000u);    // A side: the float 1.5 * 2^(E - 127)
        w[s * 128 + erow] = word;
    }
}

// Workgroup -> tile.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  XCD x gets
// a contiguous eighth of the tiles, walked in bands of 8 tile rows column by column, so that the 64
// tiles an XCD works on at any time are an 8 x 8 patch: 8 row panels and 8 column panels of the current
// k range stay in that XCD's L2 and each is used 8 times.  Returns false for the padding workgroups.
__device__ __forceinline__ bool tile_of_workgroup(int wg, int tiles_m, int tiles_n, int &tm, int &tn) {
    const int ntiles = tiles_m * tiles_n;
    const int per_xcd = (ntiles + 7) >> 3;
    const int t = (wg & 7) * per_xcd + (wg >> 3);
    if ((wg >> 3) >= per_xcd || t >= ntiles) return false;
    const int band = t / (8 * tiles_n);
    const int rows_in_band = tiles_m - band * 8 < 8 ? tiles_m - band * 8 : 8;
    const int r = t - band * 8 * tiles_n;
    tn = r / rows_in_band;
    tm = band * 8 + r % rows_in_band;
    return true;
}

// SPB: k-steps of 32 per exponent block: 1, 2, or 0 = a multiple of 4 (blocks span whole stages)
template <int SPB, bool DUMP>
__global__ __launch_bounds__(kThreads, 2) void gemm_i8_kernel(const GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    int tm, tn;
    if (!tile_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn)) return;   // whole workgroup, before any barrier
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
    const int split = blockIdx.y;
    const int st_begin = split * p.stages_per_split;
    int st_end = st_begin + p.stages_per_split;
    if (st_end > p.nstage) st_end = p.nstage;

    // ---- staging roles: 4 x 16 bytes of A and of B per thread and stage; one exponent row per thread
    const int srow = t >> 3, schunk = t & 7;
    const uint8_t *gA[4], *gB[4];
    int ldsoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = srow + 32 * i;
        int64_t ra = row0 + r, rb = col0 + r;
        ra = ra < p.M ? ra : p.M - 1;   // rows past the edge re-read the last row; their results are never stored
        rb = rb < p.N ? rb : p.N - 1;
        gA[i] = p.A + ra * p.kpad + schunk * 16;
        gB[i] = p.B + rb * p.kpad + schunk * 16;
        ldsoff[i] = r * BK + ((schunk ^ (r & 7)) * 16);   // 16-byte chunks XOR-swizzled by row
    }
    const bool exp_is_a = t < 128;
    const int erow = t & 127;
    const uint8_t *gE;
    {
        int64_t r = (exp_is_a ? row0 : col0) + erow;
        const int64_t lim = exp_is_a ? p.M : p.N;
        r = r < lim ? r : lim - 1;
        gE = exp_is_a ? p.eA + r * p.eA_ld : p.eB + r * p.eB_ld;
    }
    const int stages_per_block = SPB == 0 ? p.spb / 4 : 1;

    // fragment addresses inside a stage buffer (k-step s adds 32 bytes before the swizzle)
    int offA[2], offB[2], swzA[2], swzB[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r_a = wm * 64 + i * 32 + l32, r_b = wn * 64 + i * 32 + l32;
        offA[i] = r_a * BK;
        swzA[i] = r_a & 7;
        offB[i] = kMantBytes + r_b * BK;
        swzB[i] = r_b & 7;
    }
    const int offW = 2 * kMantBytes + (wm * 64 + 4 * lh) * 4;          // + (slot*128 + mi*32 + 8g) * 4
    const int offS = 2 * kMantBytes + kWordBytes + (wn * 64 + l32) * 4;  // + (slot*128 + ni*32) * 4

    float acc[2][2][16];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
    v16i d[2][2];
    if (SPB != 1) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) d[mi][ni][v] = 0;
    }

    StageRegs regs;
    if (st_begin < st_end) {
        load_stage<SPB>(regs, gA, gB, gE, st_begin, stages_per_block);
        store_stage<SPB, DUMP>(regs, lds, ldsoff, exp_is_a, erow);
    }
    __syncthreads();

    for (int st = st_begin; st < st_end; ++st) {
        const int buf = (st - st_begin) & 1;
        const bool more = st + 1 < st_end;
        if (more) load_stage<SPB>(regs, gA, gB, gE, st + 1, stages_per_block);

        const uint8_t *base = lds + buf * kStageBytes;

#pragma unroll 1
        for (int s = 0; s < 4; ++s) {
            bool first, last;
            int slot;
            if (SPB == 1) { first = true; last = true; slot = s; }
            else if (SPB == 2) { first = (s & 1) == 0; last = (s & 1) == 1; slot = s >> 1; }
            else {
                first = s == 0 && (st % stages_per_block) == 0;
                last = s == 3 && ((st + 1) % stages_per_block) == 0;
                slot = 0;
            }
            v4i a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = *reinterpret_cast<const v4i *>(base + offA[i] + (((2 * s + lh) ^ swzA[i]) * 16));
                b[i] = *reinterpret_cast<const v4i *>(base + offB[i] + (((2 * s + lh) ^ swzB[i]) * 16));
            }
            v16i cin[2];
            if (first || last) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const v4i c4 = *reinterpret_cast<const v4i *>(base + offW + (slot * 128 + mi * 32 + 8 * g) * 4);
                        cin[mi][4 * g + 0] = c4[0];
                        cin[mi][4 * g + 1] = c4[1];
                        cin[mi][4 * g + 2] = c4[2];
                        cin[mi][4 * g + 3] = c4[3];
                    }
            }
            float sb[2] = {0.0f, 0.0f};
            if (last && !DUMP) {
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    sb[ni] = *reinterpret_cast<const float *>(base + offS + (slot * 128 + ni * 32) * 4);
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    v16i r;
                    if (first) r = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], b[ni], cin[mi], 0, 0, 0);
                    else r = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], b[ni], d[mi][ni], 0, 0, 0);
                    if (SPB != 1) d[mi][ni] = r;
                    if (!last) continue;
                    if (!DUMP) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const float x = __int_as_float(r[v]) - __int_as_float(cin[mi][v]);
                            acc[mi][ni][v] = fmaf(x, sb[ni], acc[mi][ni][v]);
                        }
                    } else {
                        const int64_t blk = SPB == 0 ? st / stages_per_block : ((int64_t)st * 4 + s) / SPB;
                        if (blk < p.nblk) {
#pragma unroll
                            for (int v = 0; v < 16; ++v) {
                                const int64_t i = row0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                                const int64_t j = col0 + wn * 64 + ni * 32 + l32;
                                if (i < p.M && j < p.N) p.P[(i * p.N + j) * p.nblk + blk] = r[v];
                            }
                        }
                    }
                    // keep each matrix instruction next to its own scaling and the LDS reads of a
                    // k-step next to that step: left alone, the scheduler hoists all of a stage's
                    // operands and results at once, which does not fit the register file
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        if (more) store_stage<SPB, DUMP>(regs, lds + (buf ^ 1) * kStageBytes, ldsoff, exp_is_a, erow);
        __syncthreads();
    }

    if (DUMP) return;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t i = row0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                const int64_t j = col0 + wn * 64 + ni * 32 + l32;
                if (i < p.M && j < p.N) {
                    const float val = acc[mi][ni][v] * p.final_scale;
                    if (p.splits > 1) p.partial[((int64_t)split * p.M + i) * p.N + j] = val;
                    else if (p.beta) p.C[i * p.ldc + j] += val;
                    else p.C[i * p.ldc + j] = val;
                }
            }
}

// ------------------------------------------------------------------------------------------------
// Blocks of at most 32 elements (one matrix instruction per exponent block): the hot case, where the
// FP32 scale-and-accumulate, not the matrix core, sets the pace.  Same tiling as above, but laid out so
// that nothing except the two vector instructions per output and block lands on the vector ALU:
//   - LDS holds a stage as [k-step][row][32 bytes], so every fragment address is a per-thread base
//     plus an immediate; the two 16-byte halves of a row swap on every eighth row, which spreads 16
//     consecutive rows over all LDS banks;
//   - global loads use a scalar base that advances by 128 bytes per stage and a per-thread 32-bit
//     offset that never changes;
//   - the k-step loop is unrolled and each matrix instruction is issued one scaling block ahead of
//     the instructions that consume it.
__device__ __forceinline__ void scale_accumulate(float (&acc)[16], const v16i &d, const v16i &cin, float sb) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const float x = __int_as_float(d[v]) - __int_as_float(cin[v]);   // exact: P * 2^(Ea - 150)
        acc[v] = fmaf(x, sb, acc[v]);
    }
    // pin the results here: without it the compiler sinks all of a stage's scaling below the matrix
    // instructions and spills every block sum on the way
#pragma unroll
    for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(acc[v]));
}

__device__ __forceinline__ v16i read_cin(const uint8_t *w) {
    v16i c;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const v4i c4 = *reinterpret_cast<const v4i *>(w + g * 32);
        c[4 * g + 0] = c4[0];
        c[4 * g + 1] = c4[1];
        c[4 * g + 2] = c4[2];
        c[4 * g + 3] = c4[3];
    }
    return c;
}

// One k-step of one operand tile in LDS: 128 rows x 32 bytes, plus 64 bytes so that the four k-steps a
// staging thread group writes land on different banks.  LDS has 64 banks of 4 bytes: a 16-byte access is
// conflict free when every 16 consecutive lanes cover 256 different bytes modulo 256, hence the two halves
// of a row swap on every eighth row.
constexpr int kStepBytes = 128 * 32 + 64;
constexpr int kTileBytes = 4 * kStepBytes;                 // one operand tile of one stage
constexpr int kB32StageBytes = 2 * kTileBytes + 2 * kWordBytes;
constexpr int kB32LdsBytes = 2 * kB32StageBytes;

__global__ __launch_bounds__(kThreads, 2) void gemm_i8_b32_kernel(const GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // wave w owns rows 32 w .. 32 w + 31 of the tile and all 128 columns (1 x 4 matrix tiles): the row
    // constants of a k-step are read from LDS once per four matrix instructions
    const int t = threadIdx.x, lane = t & 63, wm = t >> 6;
    const int l32 = lane & 31, lh = lane >> 5;

    int tm, tn;
    if (!tile_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn)) return;   // whole workgroup, before any barrier
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
    const int split = blockIdx.y;
    const int st_begin = split * p.stages_per_split;
    int st_end = st_begin + p.stages_per_split;
    if (st_end > p.nstage) st_end = p.nstage;

    // Staging: mantissas go from global memory straight into LDS (global_load_lds, 16 bytes per lane,
    // consecutive lanes fill consecutive LDS bytes).  Wave w moves rows 32 w .. 32 w + 31 of A and of B, one
    // k-step plane (32 rows x 32 bytes = 1 KB) per instruction: lane l fills 16-byte slot l & 1 of row l >> 1
    // and therefore fetches the half of the row that the swapped layout keeps in that slot.
    const int wave_u = __builtin_amdgcn_readfirstlane(wm);
    const int drow = wm * 32 + (lane >> 1);
    const int dhalf = (lane & 1) ^ ((drow >> 3) & 1);
    const int rows_a = (int)((p.M - row0) < BM ? (p.M - row0) : BM), rows_b = (int)((p.N - col0) < BN ? (p.N - col0) : BN);
    // rows past the edge re-read the last row; their results are never stored
    const uint32_t dmaA = (uint32_t)(drow < rows_a ? drow : rows_a - 1) * (uint32_t)p.kpad + dhalf * 16;
    const uint32_t dmaB = (uint32_t)(drow < rows_b ? drow : rows_b - 1) * (uint32_t)p.kpad + dhalf * 16;
    const uint8_t *tileA = p.A + row0 * p.kpad, *tileB = p.B + col0 * p.kpad;   // uniform
    const bool exp_is_a = t < 128;
    const int erow = t & 127;
    const uint8_t *gE;
    {
        int64_t r = (exp_is_a ? row0 : col0) + erow;
        const int64_t lim = exp_is_a ? p.M : p.N;
        r = r < lim ? r : lim - 1;
        gE = exp_is_a ? p.eA + r * p.eA_ld : p.eB + r * p.eB_ld;
    }
    const int word_off = 2 * kTileBytes + (exp_is_a ? 0 : kWordBytes) + erow * 4;

    // per-thread LDS bases of the fragments (k-step s and column tile ni add immediates)
    const int r_a = wm * 32 + l32;
    const int fragA = r_a * 32 + ((lh ^ ((r_a >> 3) & 1)) * 16);
    const int fragB = kTileBytes + l32 * 32 + ((lh ^ ((l32 >> 3) & 1)) * 16);   // + ni * 1024: (32 ni) >> 3 is even
    const int offW = 2 * kTileBytes + (wm * 32 + 4 * lh) * 4;
    const int offS = 2 * kTileBytes + kWordBytes + l32 * 4;

    float acc[4][16];
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[ni][v] = 0.0f;

    uint32_t gexp = 0;
    typedef __attribute__((address_space(1))) const void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;

    // request stage st: this thread's exponent bytes into a register, the mantissa planes into LDS buffer `buf`
#define HBFP_REQUEST_STAGE(st, buf)                                                                       \
    {                                                                                                     \
        gexp = *reinterpret_cast<const uint32_t *>(gE + (st) * 4);                                        \
        const uint8_t *sa = tileA + (int64_t)(st) * BK, *sbp = tileB + (int64_t)(st) * BK;                \
        uint8_t *la = (buf) + wave_u * 1024;                                                              \
        _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                                   \
            __builtin_amdgcn_global_load_lds((gptr_t)(sa + s * 32 + dmaA), (lptr_t)(la + s * kStepBytes), 16, 0, 0); \
            __builtin_amdgcn_global_load_lds((gptr_t)(sbp + s * 32 + dmaB), (lptr_t)(la + kTileBytes + s * kStepBytes), 16, 0, 0); \
        }                                                                                                 \
    }
    // exponent bytes -> the 32-bit words the matrix core (A side) and the FMA (B side) use
#define HBFP_STORE_WORDS(base)                                                                \
    {                                                                                         \
        _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                       \
            uint32_t e = (gexp >> (8 * s)) & 0xffu;                                           \
            e = e > 254u ? 254u : e;                                                          \
            uint32_t word = e << 23;                                                          \
            if (exp_is_a) word |= 0x400000u;                                                  \
            *reinterpret_cast<uint32_t *>((base) + word_off + s * 512) = word;                \
        }                                                                                     \
    }

    // Software pipeline of one stage (4 k-steps) - everything that has latency is requested a step or more
    // before it is needed, and there is one barrier per stage:
    //   step 0, step 1            each step fetches the next step's operands from LDS before its last two
    //                             scaling blocks (the fragment registers are free by then)
    //   words of stage st+1       exponent bytes (requested a stage ago) -> LDS words of the other buffer
    //   step 2, wait, barrier     this wave's LDS accesses and its global->LDS loads of stage st+1 are complete
    //   request stage st+2        into the buffer this stage used: nobody reads it any more
    //   step 3                    fetches step 0 of stage st+1 from the other buffer
    v4i a, b[4];
    v16i cin[2];
    float sb[2][4];
#define HBFP_READ_STEP(base, s, set)                                                                    \
    {                                                                                                   \
        a = *reinterpret_cast<const v4i *>((base) + fragA + (s) * kStepBytes);                          \
        _Pragma("unroll") for (int ni = 0; ni < 4; ++ni)                                                \
            b[ni] = *reinterpret_cast<const v4i *>((base) + fragB + (s) * kStepBytes + ni * 1024);      \
        cin[set] = read_cin((base) + offW + ((s) * 128) * 4);                                           \
        _Pragma("unroll") for (int ni = 0; ni < 4; ++ni)                                                \
            sb[set][ni] = *reinterpret_cast<const float *>((base) + offS + ((s) * 128 + ni * 32) * 4);  \
    }
#define HBFP_STEP(cur, NEXT_READ)                                                                       \
    {                                                                                                   \
        v16i d0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[0], cin[cur], 0, 0, 0);                    \
        v16i d1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[1], cin[cur], 0, 0, 0);                    \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        scale_accumulate(acc[0], d0, cin[cur], sb[cur][0]);                                             \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        d0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[2], cin[cur], 0, 0, 0);                         \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        scale_accumulate(acc[1], d1, cin[cur], sb[cur][1]);                                             \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        d1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[3], cin[cur], 0, 0, 0);                         \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        NEXT_READ;                                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        scale_accumulate(acc[2], d0, cin[cur], sb[cur][2]);                                             \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        scale_accumulate(acc[3], d1, cin[cur], sb[cur][3]);                                             \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }

    if (st_begin < st_end) {
        HBFP_REQUEST_STAGE(st_begin, lds);
        HBFP_STORE_WORDS(lds);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (st_begin + 1 < st_end) HBFP_REQUEST_STAGE(st_begin + 1, lds + kB32StageBytes);
    if (st_begin < st_end) HBFP_READ_STEP(lds, 0, 0);

    for (int st = st_begin; st < st_end; ++st) {
        const bool more = st + 1 < st_end;
        uint8_t *base = lds + ((st - st_begin) & 1) * kB32StageBytes;
        uint8_t *other = lds + (((st - st_begin) & 1) ^ 1) * kB32StageBytes;

        HBFP_STEP(0, HBFP_READ_STEP(base, 1, 1));
        HBFP_STEP(1, HBFP_READ_STEP(base, 2, 0));
        if (more) HBFP_STORE_WORDS(other);
        __builtin_amdgcn_sched_barrier(0);
        HBFP_STEP(0, HBFP_READ_STEP(base, 3, 1));
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (st + 2 < st_end) HBFP_REQUEST_STAGE(st + 2, base);
        HBFP_STEP(1, if (more) HBFP_READ_STEP(other, 0, 0));
    }
#undef HBFP_READ_STEP
#undef HBFP_STEP
#undef HBFP_REQUEST_STAGE
#undef HBFP_STORE_WORDS

#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t i = row0 + wm * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
            const int64_t j = col0 + ni * 32 + l32;
            if (i < p.M && j < p.N) {
                const float val = acc[ni][v] * p.final_scale;
                if (p.splits > 1) p.partial[((int64_t)split * p.M + i) * p.N + j] = val;
                else if (p.beta) p.C[i * p.ldc + j] += val;
                else p.C[i * p.ldc + j] = val;
            }
        }
}

// fixed-order sum over the split-K slices: deterministic, no float atomics
__global__ __launch_bounds__(kThreads) void splitk_reduce_kernel(const float *partial, float *C, int64_t M, int64_t N,
                                                                  int64_t ldc, int splits, int beta) {
    const int64_t n = M * N;
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kThreads) {
        const int64_t i = e / N, j = e % N;
        float s = beta ? C[i * ldc + j] : 0.0f;
        for (int z = 0; z < splits; ++z) s += partial[(int64_t)z * n + e];
        C[i * ldc + j] = s;
    }
}

template <int SPB, bool DUMP>
int launch_t(const GemmParams &p, dim3 grid, hipStream_t s) {
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_i8_kernel<SPB, DUMP>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
            return HBFP_ERR_LAUNCH;
        configured = true;
    }
    hipLaunchKernelGGL((gemm_i8_kernel<SPB, DUMP>), grid, dim3(kThreads), kLdsBytes, s, p);
    return launch_status();
}

}  // namespace

// Split K when the tile grid alone cannot fill the chip (the weight-gradient shape: small
// M x N, very long K).  Pure function of the shapes so that the workspace query agrees.
static int choose_splits(int64_t M, int64_t N, int64_t nstage, int64_t stages_per_block) {
    const int64_t tiles = ceil_div(M, BM) * ceil_div(N, BN);
    const int64_t units = nstage / stages_per_block;   // whole exponent blocks (or stages) that can be dealt out
    if (tiles >= 256 || units < 8) return 1;
    int64_t s = ceil_div(512, tiles);
    if (s > units / 4) s = units / 4;
    if (s > 128) s = 128;
    return s < 1 ? 1 : (int)s;
}

size_t gemm_i8_workspace(int64_t M, int64_t N, int64_t kpad, int64_t kbp) {
    const int64_t nstage = kpad / BK, spb = kbp / 32;
    const int splits = choose_splits(M, N, nstage, spb >= 4 ? spb / 4 : 1);
    if (splits <= 1) return 0;
    return ((size_t)splits * (size_t)M * (size_t)N * 4 + 255) & ~(size_t)255;
}

int launch_gemm_i8(const GemmArgs &a, void *workspace, hipStream_t s) {
    GemmParams p;
    p.A = (const uint8_t *)a.mantA;
    p.B = (const uint8_t *)a.mantB;
    p.eA = a.expA;
    p.eB = a.expB;
    p.C = a.C;
    p.P = a.P;
    p.partial = (float *)workspace;
    p.M = a.M;
    p.N = a.N;
    p.kpad = a.kpad;
    p.eA_ld = a.expA_ld;
    p.eB_ld = a.expB_ld;
    p.ldc = a.ldc;
    p.nblk = a.nblk;
    p.nstage = (int32_t)(a.kpad / BK);
    p.spb = (int32_t)(a.kbp / 32);
    const int64_t tm = ceil_div(a.M, BM), tn = ceil_div(a.N, BN);
    if (tm * tn > 0x7ffffff0 || a.kpad / BK > 0x7fffffff) return HBFP_ERR_ARG;
    p.tiles_m = (int32_t)tm;
    p.tiles_n = (int32_t)tn;
    p.beta = a.beta != 0.0f;
    p.final_scale = ldexpf(1.0f, 27 - a.mA - a.mB);
    const int stages_per_block = p.spb >= 4 ? p.spb / 4 : 1;
    p.splits = a.P ? 1 : choose_splits(a.M, a.N, p.nstage, stages_per_block);
    {
        const int64_t units = p.nstage / stages_per_block;
        p.stages_per_split = (int32_t)(ceil_div(units, p.splits) * stages_per_block);
        p.splits = (int32_t)ceil_div(p.nstage, p.stages_per_split);
    }
    const dim3 grid((unsigned)(ceil_div(tm * tn, 8) * 8), (unsigned)p.splits);
    int rc;
    if (a.P) {
        rc = p.spb == 1 ? launch_t<1, true>(p, grid, s) : p.spb == 2 ? launch_t<2, true>(p, grid, s) : launch_t<0, true>(p, grid, s);
    } else {
        if (p.spb == 1 && (uint64_t)127 * (uint64_t)a.kpad + 128 < ((uint64_t)1 << 32)) {
            static bool configured = false;
            if (!configured) {
                if (hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_i8_b32_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kB32LdsBytes) != hipSuccess)
                    return HBFP_ERR_LAUNCH;
                configured = true;
            }
            hipLaunchKernelGGL(gemm_i8_b32_kernel, grid, dim3(kThreads), kB32LdsBytes, s, p);
            rc = launch_status();
        } else {
            rc = p.spb == 1 ? launch_t<1, false>(p, grid, s) : p.spb == 2 ? launch_t<2, false>(p, grid, s) : launch_t<0, false>(p, grid, s);
        }
    }
    if (rc != HBFP_OK) return rc;
    if (!a.P && p.splits > 1) {
        int64_t nb = ceil_div(a.M * a.N, kThreads);
        if (nb > 8192) nb = 8192;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)nb), dim3(kThreads), 0, s, p.partial, p.C, p.M, p.N,
                           p.ldc, p.splits, p.beta);
        rc = launch_status();
    }
    return rc;
}

}  // namespace hbfp
