// BFP matrix product for gfx950, Eq. (2) of Sec. 4 with per-block FP accumulation
// (Sec. 4 "tiled" products, Sec. 4.2 Tiling):
//     C[i][j] = sum_b 2^(eA[i][b] + eB[j][b]) * sum_{k in b} mA[i][k] * mB[j][k]
//
// Both operands are stored with k contiguous (public header), so this is an "NT"
// product over 128 x 128 tiles of C.  Two kernels:
//   gemm_i8_w8_kernel   the product itself, every block length: 8 waves per workgroup, asynchronous
//                       global -> LDS copies through a ring of LDS buffers (described where it starts);
//   gemm_i8_kernel      4 waves, 2 x 2 matrix tiles per wave, operands staged through registers: kept for
//                       the dump of the integer block sums (hbfp_gemm_partials) and for operands too
//                       long for 32-bit tile offsets.
//
// The per-block scaling is the expensive part on this chip (one FP32 operation per 2*B
// integer operations is cheap next to 8-bit multipliers in the paper's accelerator,
// Sec. 4.2; here one matrix instruction covers 32 x 32 outputs of a block in 32 clocks while
// scaling them takes 32 vector instructions).  It is kept to two vector instructions per output and block:
//   1. the matrix core starts from a constant C input whose int32 bit pattern is the
//      float 1.5 * 2^(Ea - 127): adding the integer block sum P (|P| < 2^22) to those
//      bits gives the float (1.5 * 2^23 + P) * 2^(Ea - 150), so the int->float
//      conversion and the row exponent cost nothing;
//   2. one subtraction removes the constant (exact), one FMA multiplies by the column
//      scale 2^(Eb - 127) and accumulates.
// The remaining constant 2^(27 - mA - mB) is applied once when C is stored.
#include "bfp_device.h"
#include "gemm_common.h"

namespace hbfp {
namespace {


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
    int32_t chain_limit;         // gemm_i8_w8_kernel<3>: most k-steps chained before their sum is scaled
    int32_t stages_per_split;
    int32_t splits;
    int32_t tiles_m, tiles_n;
    int32_t beta;
    float final_scale;
    const int *run_a, *run_b;    // non-null: do nothing unless a packed operand is marked out of range
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

// SPB: k-steps of 32 per exponent block: 1, 2, or 0 = a multiple of 4 (blocks span whole stages)
template <int SPB, bool DUMP>
__global__ __launch_bounds__(kThreads, 2) void gemm_i8_kernel(const GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    if (stands_down(p.run_a, p.run_b)) return;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;

    // 8 and more k ranges are dealt to the XCDs (few tiles, very long k); fewer ride in blockIdx.y while the tiles are
    // dealt to the XCDs as in an unsplit product
    int tm, tn, split = blockIdx.y;
    if (p.splits >= 8 ? !tile_and_split_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, p.splits, tm, tn, split)
                      : !tile_of_workgroup(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn))
        return;                                                                  // whole workgroup, before any barrier
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
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
                // The product kernel closes the chain every 256 elements of k (two stages) as well as at the end of
                // the block: 256 * 127 * 127 < 2^22 keeps the block sum inside the range in which adding it to the bit
                // pattern of the row constant is exact, however long the block.  The dump keeps whole-block int32 sums.
                const int in_block = st % stages_per_block;
                first = s == 0 && (DUMP ? in_block == 0 : (in_block & 1) == 0);
                last = s == 3 && (in_block + 1 == stages_per_block || (!DUMP && (in_block & 1) == 1));
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
// FP32 scale-and-accumulate, not the matrix core, sets the pace: 64 vector instructions per wave and
// k-step against two matrix instructions.  Measured on this chip, one wave issues at most one vector
// instruction every 5 clocks whatever else it does, a SIMD with four such waves retires close to one per
// clock, and a wave that stages operands itself (global loads, LDS stores, the waits between them)
// issues nothing else meanwhile.  So this kernel
//   - runs 4 waves per SIMD: workgroups of 8 waves, a wave owns 32 x 64 of the 128 x 128 tile and stays
//     within 128 registers; it relies on the other waves, not on software pipelining, to cover the
//     latency of its matrix instructions and LDS reads;
//   - moves operands global -> LDS with the asynchronous copy instruction (no registers, no LDS stores,
//     no wait in the wave), three copies per wave and stage, issued right after a hand-over;
//   - stages 64 bytes of k at a time through a ring of four LDS buffers, handed over two at a time, so a
//     copy has two stages of compute to land and there is one barrier per four k-steps;
//   - does not read the C input of a k-step (the row constant 1.5 * 2^(Ea - 127), the same in all 32
//     columns) from LDS, where it would be 16 registers per wave and step: one bf16 matrix instruction
//     spreads one register of row constants over the 32 x 32 output layout (the constant has a 2-bit
//     significand, so bf16 holds it exactly, and the second operand is a single one per column);
//   - takes the scale words (row constants as bf16, column scales as FP32) from arrays a small kernel
//     derives from the exponent bytes beforehand, stored [block][row] so that a copy reads them
//     contiguously;
//   - does all 32 subtractions of a k-step before its 32 multiply-adds: a wave issues back-to-back
//     dependent vector instructions every 7 clocks instead of 5.
// LDS tile of one operand and stage: [128 rows][64 bytes]; the four 16-byte chunks of a row are XORed
// with (row >> 2) & 3, which makes both the copy (16 rows x 64 bytes per wave) and the fragment reads
// (16 consecutive rows, one chunk) cover all 64 banks.
constexpr int kW8Threads = 512;
constexpr int kHalfK = 64;                                  // bytes of k per stage
constexpr int kHalfTile = 128 * kHalfK;                     // 8 KB: one operand
constexpr int kHalfWords = 2 * 128 * 4;                     // 1 KB: two blocks x 128 rows
constexpr int kHalfStage = 2 * kHalfTile + 2 * kHalfWords;  // 18 KB
constexpr int kW8Ring = 4;
constexpr int kW8LdsBytes = kW8Ring * kHalfStage;           // 72 KB: two workgroups per CU

// Operand A gathered from an encoded image instead of read as a stored matrix (a convolution executed as a matrix
// product, Sec. 5.1): operand row = output position (img, oy, ox), k = (filter row, filter column, channel).  The
// image is an operand of its own, [pixels][channels] with blocks of 32 channels; a stage of 64 bytes of k is 64
// channels of one filter tap, i.e. of one pixel, so the gather is one address per lane and stage.  Taps that fall
// outside the image read a page of zeros.
// DIL: the image stands for one with dil - 1 rows and columns of zeros between its pixels (the output gradient of a
// strided convolution, whose data gradient is a stride-1 convolution of exactly that, Sec. 5.1); positions of the
// dilated image that are not a multiple of dil read the page of zeros as well, and the others divide by dil (in FP32:
// exact while coordinates stay below 2^21, which the host checks).
struct ConvA {
    const uint8_t *zeros;        // at least 64 zero bytes; behind them, at +64, one row-constant word for them
    const uint32_t *words;       // row constants of the image [channel block][pixel pitch]
    int64_t word_pitch;
    int32_t H, W, Ho, Wo, S, ntaps, spt;   // image, output, filter columns, taps, stages (64 channels) per tap
    int32_t pad_h, pad_w, str_h, str_w;
    int32_t pix_bytes;           // bytes between pixels of the encoded image
    int32_t dil_h, dil_w;        // DIL only
    float inv_dh, inv_dw;
    int32_t ncb, R, cb_order, nslots;   // SLOT only: stored blocks per pixel, filter rows, order of k, r * s * ncb
};

// SLOT: the general gather.  The image is stored in blocks of at most 32 channels, each padded to 32 bytes (a slot), so
// any channel count that is a multiple of the block length works, and k runs over slots either tap by tap
// (k = (tap, channel block, channel): cb_order 0) or channel block by channel block (k = (channel block, tap, channel):
// cb_order 1, the order in which a filter tile spans the whole window, Sec. 5.1).  A stage of 64 bytes is two consecutive
// slots, in general of two different pixels: the lanes that copy its upper half take the second slot's tap and block.
// PHASE: the data gradient of a strided convolution, output phase by output phase.  The input positions
// (yy * sh + py, xx * sw + px) of one phase (py, px) meet only the filter taps fr0 + j * sh, fs0 + i * sw, and under tap
// (j, i) they read the stored gradient at (yy + oy0 + j, xx + ox0 + i): a stride-1 gather without any zeros in between.
// Operand B stays the whole mirrored filter; the kernel steps through the taps of its phase in it.  blockIdx.y names the
// phase, and a row of the phase is stored to the row of its input position.
struct ConvPhase {
    int32_t Hp, Wp;              // input positions of the phase
    int32_t py, px;
    int32_t oy0, ox0;            // may be negative
    int32_t fr0, fs0;
    int32_t Rp, Sp;              // taps of the phase
    int32_t tiles_m;
    int32_t nst;                 // stages of 64 bytes of k: Rp * Sp * stages per tap, rounded up to an even number
};
constexpr int kConvPhases = 16;
struct ConvPhases {
    ConvPhase p[kConvPhases];
    int32_t sh, sw;              // strides of the forward convolution
    int32_t h, w;                // input extents: where the rows of a phase are stored
    int32_t s_full;              // filter columns of the whole filter
    int32_t n;                   // images
};

// floor(i / d) for a coordinate i of the dilated image (may be negative), inv = 1 / d rounded
__device__ __forceinline__ int conv_undilate(int i, float inv) { return (int)__builtin_floorf(((float)i + 0.5f) * inv); }

// ENC: the product leaves the kernel as an encoded operand (the FP->BFP conversion of Sec. 4.1 / Sec. 5.3 applied to the
// accumulators): rows of C, blocks of 32 along its columns - for a convolution, the next layer's image.
struct W8Enc {
    uint8_t *mant, *exps;
    int64_t kpad, exp_ld;
    int32_t nblk, m, rounding, relu;
    uint32_t s0, s1;
};

struct W8Params {
    GemmParams g;
    const uint32_t *wA, *wB;     // scale words [kpad / 32][rows_pad]
    int64_t mpad, npad;
    ConvA cv;                    // CONV only
    ConvPhases ph;               // PHASE only
    W8Enc enc;                   // ENC only
};

// The same kernel multiplies 9..12-bit mantissas stored as FP16 numbers (F16): an 11-bit magnitude is an FP16
// significand, so the mantissa itself is an FP16 value, v_mfma_f32_32x32x16_f16 multiplies two of them exactly (22 bits)
// and accumulates in FP32, and a k-step of 32 bytes is 16 elements.  A block's chain then starts from zero, its FP32 sum
// (exact below 2^24, rounded to nearest beyond: the same rounding the int32 -> FP32 conversion of the limb kernels
// applies once) is multiplied by the row scale 2^(Ea - 127), spread over the output layout by the same bf16 matrix
// instruction, and by the column scale: again two vector instructions per output and block.
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
template <bool F16>
struct W8Ops;
template <>
struct W8Ops<false> {
    typedef v16i acc_t;
    static __device__ __forceinline__ acc_t mma(const v4i &a, const v4i &b, const acc_t &c) { return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }
    // what a block's chain of matrix instructions starts from: the row constants
    static __device__ __forceinline__ acc_t start(const acc_t &row) { return row; }
    // the block sum with its row scale applied: the constant removed
    static __device__ __forceinline__ float scaled(int d, int row) { return __int_as_float(d) - __int_as_float(row); }
    static __device__ __forceinline__ acc_t rows(uint32_t rowc, const v2i &one_hot) { return row_constants(rowc, one_hot); }
    // keeps both results in vector registers at this point of the schedule
    static __device__ __forceinline__ void pin(const acc_t &d0, const acc_t &d1) { asm volatile("" ::"v"(d0), "v"(d1)); }
};
template <>
struct W8Ops<true> {
    typedef v16f acc_t;
    static __device__ __forceinline__ acc_t mma(const v4i &a, const v4i &b, const acc_t &c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ acc_t start(const acc_t &) { return acc_t{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}; }   // zero
    static __device__ __forceinline__ float scaled(float d, float row) { return d * row; }                    // the scale multiplied in
    static __device__ __forceinline__ acc_t rows(uint32_t rowc, const v2i &one_hot) { return __builtin_bit_cast(v16f, row_constants(rowc, one_hot)); }
    static __device__ __forceinline__ void pin(const acc_t &d0, const acc_t &d1) { asm volatile("" ::"v"(d0), "v"(d1)); }
};

// ENC epilogue.  The accumulators hold a column per lane and rows across registers, the conversion wants the 32 columns
// of a block side by side: the tile goes through LDS (the ring is free by then) as [128 rows][132 floats], and each of the
// 512 threads converts one row's block of 32 - largest magnitude, shared exponent, rounding with the index of the
// element in C, 32 mantissas in two 16-byte stores, one exponent byte - with the arithmetic of the conversion kernels,
// so the result is what converting the FP32 product would give.  A wave that computed nothing writes nothing (its columns
// lie past N and count as zeros) but keeps both barriers.
constexpr int kEncStride = 132;
template <int ROUND>
__device__ __forceinline__ void w8_encode_block(const W8Enc &o, const float *row, int64_t grow, int64_t gcol0, int64_t N) {
    float x[32];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float4 d = *reinterpret_cast<const float4 *>(row + 4 * j);
        x[4 * j] = d.x, x[4 * j + 1] = d.y, x[4 * j + 2] = d.z, x[4 * j + 3] = d.w;
    }
    uint32_t amax = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        if (gcol0 + j >= N) x[j] = 0.0f;
        amax = max(amax, __float_as_uint(x[j]) & 0x7fffffffu);
    }
    const uint32_t Eb = block_exponent<ROUND>(amax, o.m);
    uint32_t w[8];
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        int qv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t idx = (uint64_t)grow * (uint64_t)N + (uint64_t)(gcol0 + 4 * g + e);
            qv[e] = quantise<ROUND>(x[4 * g + e], Eb, o.m, (uint32_t)idx, (uint32_t)(idx >> 32), o.s0, o.s1);
        }
        w[g] = (uint32_t)(qv[0] & 0xff) | ((uint32_t)(qv[1] & 0xff) << 8) | ((uint32_t)(qv[2] & 0xff) << 16) | ((uint32_t)qv[3] << 24);
    }
    uint4 *dst = reinterpret_cast<uint4 *>(o.mant + grow * o.kpad + gcol0);
    dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
    dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
    const int64_t b = gcol0 >> 5;
    if (b < o.exp_ld) o.exps[grow * o.exp_ld + b] = b < o.nblk ? (uint8_t)Eb : (uint8_t)1;
}

// first half, for a wave that computed: its 32 x 64 results into the tile
__device__ __forceinline__ void w8_tile_to_lds(const W8Enc &o, uint8_t *lds, const float (&acc)[2][16], float final_scale) {
    // (its place in the tile recomputed from the thread index: the kernels that call this have no register to keep it in)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave & 3, wn = wave >> 2, l32 = lane & 31, lh = lane >> 5;
    float *tile = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float val = acc[ni][v] * final_scale;
            if (o.relu && val < 0.0f) val = 0.0f;
            tile[(wm * 32 + 8 * (v >> 2) + 4 * lh + (v & 3)) * kEncStride + wn * 64 + ni * 32 + l32] = val;
        }
}
// second half, for every thread: one row's block of 32
__device__ __forceinline__ void w8_encode_from_lds(const W8Enc &o, const uint8_t *lds, int64_t row0, int64_t col0, int64_t M, int64_t N) {
    const float *tile = reinterpret_cast<const float *>(lds);
    const int r = threadIdx.x >> 2, qb = threadIdx.x & 3;
    const int64_t grow = row0 + r, gcol0 = col0 + qb * 32;
    if (grow < M && gcol0 < o.kpad) {
        if (o.rounding) w8_encode_block<1>(o, tile + r * kEncStride + qb * 32, grow, gcol0, N);
        else w8_encode_block<0>(o, tile + r * kEncStride + qb * 32, grow, gcol0, N);
    }
}

// SPB: k-steps of 32 per exponent block: 1, 2, or 0 = a multiple of 4 (a block is spb / 2 whole stages).  A block
// that spans several k-steps chains its matrix instructions through the C input and is scaled at its last
// k-step, and, when it is longer than 256 elements, after every 256 (four stages) with the same scales: the
// chained sum then stays below 256 * 127 * 127 < 2^22, the range in which adding it to the bit pattern of the
// row constant is exact.  The longer the block, the closer the kernel gets to the matrix core's own pace.
// GATHER (CONV only): 0 the image as it is (64 channels of one tap per stage), 1 = DIL, 2 = PHASE, 3 = SLOT, 4 = SLOT + DIL
// SPB = 3: stored blocks of one k-step whose exponents repeat over runs of p.spb consecutive blocks in BOTH operands
// (an image with one exponent per training input against filter tiles that span the whole window, Sec. 5.1): the scale
// words are staged per k-step as for SPB = 1, but a run is chained like a long block and scaled once, at its last
// k-step, after p.chain_limit k-steps (the range in which the row constant trick is exact) and at the end of the k range.
template <int SPB, bool CONV = false, bool F16 = false, int GATHER = 0, bool ENC = false>
__global__ __launch_bounds__(kW8Threads, 4) void gemm_i8_w8_kernel(const W8Params q) {
    constexpr bool STEPW = SPB == 1 || SPB == 3;     // scale words per k-step
    constexpr bool CHAIN = SPB == 0 || SPB == 3;     // the matrix instructions of a block (run) chain through their C input
    constexpr bool DIL = GATHER == 1 || GATHER == 4, PHASE = GATHER == 2, SLOT = GATHER == 3 || GATHER == 4;
    typedef W8Ops<F16> ops;
    typedef typename ops::acc_t acc_t;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const GemmParams &p = q.g;
    if (stands_down(p.run_a, p.run_b)) return;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave & 3, wn = wave >> 2;
    const int l32 = lane & 31, lh = lane >> 5;

    // 8 and more k ranges are dealt to the XCDs (few tiles, very long k); fewer ride in blockIdx.y while the tiles are
    // dealt to the XCDs as in an unsplit product
    int tm, tn, split = PHASE ? 0 : blockIdx.y;
    // geometry of the gather: the convolution's own, or that of this workgroup's phase (uniform)
    int64_t M = p.M;
    int gHo = q.cv.Ho, gWo = q.cv.Wo, gS = q.cv.S, gtaps = q.cv.ntaps;
    int gstr_h = q.cv.str_h, gstr_w = q.cv.str_w, gpad_h = q.cv.pad_h, gpad_w = q.cv.pad_w;
    int tiles_m = p.tiles_m, ph_nst = 0, ph_py = 0, ph_px = 0, ph_fr0 = 0, ph_fs0 = 0;
    if (PHASE) {
        const ConvPhase &f = q.ph.p[blockIdx.y];
        gHo = f.Hp, gWo = f.Wp, gS = f.Sp, gtaps = f.Rp * f.Sp;
        gstr_h = gstr_w = 1, gpad_h = -f.oy0, gpad_w = -f.ox0;
        tiles_m = f.tiles_m, ph_nst = f.nst, ph_py = f.py, ph_px = f.px, ph_fr0 = f.fr0, ph_fs0 = f.fs0;
        M = (int64_t)q.ph.n * f.Hp * f.Wp;
    }
    if (p.splits >= 8 && !PHASE ? !tile_and_split_of_workgroup(blockIdx.x, tiles_m, p.tiles_n, p.splits, tm, tn, split)
                                : !tile_of_workgroup(blockIdx.x, tiles_m, p.tiles_n, tm, tn))
        return;                                                                  // whole workgroup, before any barrier
    const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
    const int st_begin = 2 * split * p.stages_per_split;                         // in 64-byte stages
    int st_end = st_begin + 2 * p.stages_per_split;
    if (st_end > 2 * p.nstage) st_end = 2 * p.nstage;
    if (PHASE) st_end = ph_nst;
    const int nst = st_end - st_begin;

    // ---- copy roles.  Mantissas: wave w moves rows 16 w .. 16 w + 15 of A and of B, lane -> (row, LDS chunk).
    // Words: waves 0..3 move the row words of A, waves 4..7 the column words of B, 64 rows of one block each.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    uint32_t voffA, voffB, voffW;
    {
        const int r = 16 * wave + (lane >> 2);
        const int chunk = (lane & 3) ^ ((r >> 2) & 3);
        const int rows_a = (int)((M - row0) < BM ? (M - row0) : BM), rows_b = (int)((p.N - col0) < BN ? (p.N - col0) : BN);
        const int ra = r < rows_a ? r : rows_a - 1;   // rows past the edge re-read the last row; never stored
        const int rb = r < rows_b ? r : rows_b - 1;
        voffA = (uint32_t)ra * (uint32_t)p.kpad + chunk * 16;
        voffB = (uint32_t)rb * (uint32_t)p.kpad + chunk * 16;
        voffW = lane * 4;
    }
    // CONV: where this lane's operand rows sit in the image.  cy / cx: input row and column under filter tap (0, 0) of
    // the row whose mantissas the lane copies; wy / wx the same for the row whose row constants it copies (waves 0..3).
    int cy = 0, cx = 0, wy = 0, wx = 0;
    int64_t cpix = 0, wpix = 0;                                                  // pixel index of that corner (may lie outside)
    int cchunk = 0;
    if (CONV) {
        const int rows_a = (int)((M - row0) < BM ? (M - row0) : BM);
        const int rm = 16 * wave + (lane >> 2), rw = 64 * (wave & 1) + lane;
        const int64_t pm = row0 + (rm < rows_a ? rm : rows_a - 1), pw = row0 + (rw < rows_a ? rw : rows_a - 1);
        const int64_t per_img = (int64_t)gHo * gWo;
        const int64_t im = pm / per_img, iw = pw / per_img;
        const int remm = (int)(pm - im * per_img), remw = (int)(pw - iw * per_img);
        cy = remm / gWo * gstr_h - gpad_h;
        cx = remm % gWo * gstr_w - gpad_w;
        wy = remw / gWo * gstr_h - gpad_h;
        wx = remw % gWo * gstr_w - gpad_w;
        cchunk = ((lane & 3) ^ ((rm >> 2) & 3)) * 16;
        cpix = ((im * q.cv.H + cy) * q.cv.W + cx) * q.cv.pix_bytes + cchunk;     // byte offset of that corner's chunk in the image
        wpix = (iw * q.cv.H + wy) * q.cv.W + wx;
        if (DIL) {                                                               // corners are in dilated coordinates: keep the image only
            cpix = im * q.cv.H * q.cv.W * q.cv.pix_bytes + cchunk;
            wpix = iw * q.cv.H * q.cv.W;
        }
        if (SLOT) cpix -= cchunk & 32;                                           // the half of the stage selects the slot, not an offset
    }
    const uint8_t *tileA = p.A + row0 * p.kpad, *tileB = p.B + col0 * p.kpad;   // uniform
    const int wc = wave_u & 3;                                                   // word copy: block wc >> 1, rows 64 (wc & 1) ..
    const uint32_t *wordsrc = wave_u < 4 ? q.wA + row0 + 64 * (wc & 1) : q.wB + col0 + 64 * (wc & 1);
    const int64_t wordpitch = wave_u < 4 ? q.mpad : q.npad;
    const uint32_t ldsM = wave_u * 1024;
    const uint32_t ldsW = 2 * kHalfTile + (wave_u < 4 ? 0 : kHalfWords) + (wc >> 1) * 512 + (wc & 1) * 256;
    const int spb64 = SPB == 0 ? p.spb / 2 : 1;                                  // stages per block when blocks span stages

    // stages are requested in order, so the three source pointers of this wave just advance
    const uint8_t *nextA = tileA + (int64_t)st_begin * kHalfK, *nextB = tileB + (int64_t)st_begin * kHalfK;
    const uint32_t *nextW = wordsrc + (STEPW ? 2 * (int64_t)st_begin + (wc >> 1) : SPB == 2 ? (int64_t)st_begin : (int64_t)st_begin / spb64) * wordpitch;
    const int64_t stepW = (STEPW ? 2 : 1) * wordpitch;                           // words per stage (long blocks: per block)
    int req_pos = 0;                                                             // SPB == 0: stage within its block
    // CONV: filter tap and 64-channel piece of the stage requested next (uniform)
    int ctap = CONV ? st_begin / q.cv.spt : 0, csub = CONV ? st_begin % q.cv.spt : 0;
    int cfr = CONV ? ctap / gS : 0, cfs = CONV ? ctap % gS : 0;
    // SLOT: filter row, filter column and channel block of the first slot of the stage requested next, and its number
    int sidx = 2 * st_begin, scb = 0;
    if (SLOT) {
        const int tap = q.cv.cb_order ? sidx % q.cv.ntaps : sidx / q.cv.ncb;
        scb = q.cv.cb_order ? sidx / q.cv.ntaps : sidx % q.cv.ncb;
        cfr = tap / gS, cfs = tap % gS;
    }
    // the slot after (fr, fs, cb) in the order of k
#define HBFP_NEXT_SLOT(fr, fs, cb)                                                                      \
    {                                                                                                   \
        if (q.cv.cb_order) {                                                                            \
            if (++fs == gS) { fs = 0; if (++fr == q.cv.R) { fr = 0; ++cb; } }                           \
        } else if (++cb == q.cv.ncb) {                                                                  \
            cb = 0;                                                                                     \
            if (++fs == gS) { fs = 0; ++fr; }                                                           \
        }                                                                                               \
    }
#define HBFP_COPY_NEXT(ring)                                                                            \
    {                                                                                                   \
        const uint32_t lb = (ring) * kHalfStage;                                                        \
        int fr1 = cfr, fs1 = cfs, cb1 = scb;                /* SLOT: the second slot of the stage (uniform) */ \
        if (SLOT) HBFP_NEXT_SLOT(fr1, fs1, cb1);                                                        \
        if (SLOT) {                                                                                     \
            const bool upper = (cchunk & 32) != 0;                                                      \
            const int fr = upper ? fr1 : cfr, fs = upper ? fs1 : cfs, cb = upper ? cb1 : scb;           \
            bool in_m = sidx + (upper ? 1 : 0) < q.cv.nslots;                                           \
            int py = cy + fr, px = cx + fs;                 /* DIL: in the spread-out image; cpix holds the image only */ \
            if (DIL) {                                                                                  \
                const int qy = conv_undilate(py, q.cv.inv_dh), qx = conv_undilate(px, q.cv.inv_dw);     \
                in_m = in_m && qy * q.cv.dil_h == py && qx * q.cv.dil_w == px;                          \
                py = qy, px = qx;                                                                       \
            }                                                                                           \
            in_m = in_m && (unsigned)py < (unsigned)q.cv.H && (unsigned)px < (unsigned)q.cv.W;          \
            const uint8_t *srcA = p.A + cpix + (int64_t)((DIL ? py : fr) * q.cv.W + (DIL ? px : fs)) * q.cv.pix_bytes + cb * 32; \
            async_copy16_at(in_m ? srcA : q.cv.zeros, lb + ldsM);                                       \
        } else if (CONV) {                                                                              \
            const bool tap_ok = ctap < gtaps;                                                           \
            const uint8_t *tapA = p.A + ((int64_t)cfr * q.cv.W + cfs) * q.cv.pix_bytes + csub * kHalfK;  /* uniform */ \
            bool in_m = tap_ok && (unsigned)(cy + cfr) < (unsigned)q.cv.H && (unsigned)(cx + cfs) < (unsigned)q.cv.W; \
            const uint8_t *srcA = tapA + cpix;                                                          \
            if (DIL) {                                                                                  \
                const int iy = cy + cfr, ix = cx + cfs;                                                 \
                const int qy = conv_undilate(iy, q.cv.inv_dh), qx = conv_undilate(ix, q.cv.inv_dw);     \
                in_m = tap_ok && qy * q.cv.dil_h == iy && qx * q.cv.dil_w == ix && (unsigned)qy < (unsigned)q.cv.H && \
                       (unsigned)qx < (unsigned)q.cv.W;                                                 \
                srcA = p.A + cpix + (int64_t)(qy * q.cv.W + qx) * q.cv.pix_bytes + csub * kHalfK;       \
            }                                                                                           \
            async_copy16_at(in_m ? srcA : q.cv.zeros, lb + ldsM);                                       \
        } else {                                                                                        \
            async_copy16(nextA, voffA, lb + ldsM);                                                      \
        }                                                                                               \
        /* PHASE: where this stage's tap lies along k in the whole filter (uniform); past the last tap A reads zeros */ \
        const int64_t kphase = PHASE && ctap < gtaps ? ((int64_t)(ph_fr0 + cfr * q.ph.sh) * q.ph.s_full + (ph_fs0 + cfs * q.ph.sw)) * (q.cv.spt * kHalfK) + csub * kHalfK : 0; \
        async_copy16(PHASE ? tileB + kphase : nextB, voffB, lb + kHalfTile + ldsM);                     \
        if (SLOT && wave_u < 4) {                           /* the wave's slot of the stage: uniform */ \
            const bool upper = (wc >> 1) != 0;                                                          \
            const int fr = upper ? fr1 : cfr, fs = upper ? fs1 : cfs, cb = upper ? cb1 : scb;           \
            bool in_w = sidx + (upper ? 1 : 0) < q.cv.nslots;                                           \
            int py = wy + fr, px = wx + fs;                                                             \
            if (DIL) {                                                                                  \
                const int qy = conv_undilate(py, q.cv.inv_dh), qx = conv_undilate(px, q.cv.inv_dw);     \
                in_w = in_w && qy * q.cv.dil_h == py && qx * q.cv.dil_w == px;                          \
                py = qy, px = qx;                                                                       \
            }                                                                                           \
            in_w = in_w && (unsigned)py < (unsigned)q.cv.H && (unsigned)px < (unsigned)q.cv.W;          \
            const uint32_t *srcW = q.cv.words + (int64_t)cb * q.cv.word_pitch + (wpix + ((DIL ? py : fr) * q.cv.W + (DIL ? px : fs))); \
            const uint32_t *outW = reinterpret_cast<const uint32_t *>(q.cv.zeros + 64);                  \
            if (SPB == 3) {                                 /* a chain has one exponent: a tap outside takes that of the nearest pixel of the image */ \
                const int ny = py < 0 ? 0 : (py >= q.cv.H ? q.cv.H - 1 : py), nx = px < 0 ? 0 : (px >= q.cv.W ? q.cv.W - 1 : px); \
                outW = q.cv.words + (int64_t)(cb < q.cv.ncb ? cb : 0) * q.cv.word_pitch + (wpix + ((ny - wy) * q.cv.W + (nx - wx))); \
            }                                                                                           \
            async_copy4_at(in_w ? srcW : outW, lb + ldsW);                                              \
        } else if (CONV && wave_u < 4) {                                                                \
            const bool tap_ok = ctap < gtaps;                                                           \
            const uint32_t *tapW = q.cv.words + (int64_t)(2 * csub + (wc >> 1)) * q.cv.word_pitch + ((int64_t)cfr * q.cv.W + cfs);  /* uniform */ \
            bool in_w = tap_ok && (unsigned)(wy + cfr) < (unsigned)q.cv.H && (unsigned)(wx + cfs) < (unsigned)q.cv.W; \
            const uint32_t *srcW = tapW + wpix;                                                         \
            if (DIL) {                                                                                  \
                const int iy = wy + cfr, ix = wx + cfs;                                                 \
                const int qy = conv_undilate(iy, q.cv.inv_dh), qx = conv_undilate(ix, q.cv.inv_dw);     \
                in_w = tap_ok && qy * q.cv.dil_h == iy && qx * q.cv.dil_w == ix && (unsigned)qy < (unsigned)q.cv.H && \
                       (unsigned)qx < (unsigned)q.cv.W;                                                 \
                srcW = q.cv.words + (int64_t)(2 * csub + (wc >> 1)) * q.cv.word_pitch + (wpix + (qy * q.cv.W + qx)); \
            }                                                                                           \
            async_copy4_at(in_w ? srcW : reinterpret_cast<const uint32_t *>(q.cv.zeros + 64), lb + ldsW); \
        } else {                                                                                        \
            async_copy4(PHASE ? wordsrc + (kphase / 32 + (wc >> 1)) * wordpitch : nextW, voffW, lb + ldsW); \
        }                                                                                               \
        nextA += kHalfK;                                                                                \
        nextB += kHalfK;                                                                                \
        if (SPB != 0) nextW += stepW;                                                                   \
        else if (++req_pos == spb64) { req_pos = 0; nextW += stepW; }                                   \
        if (SLOT) {                                                                                     \
            cfr = fr1, cfs = fs1, scb = cb1;                                                            \
            HBFP_NEXT_SLOT(cfr, cfs, scb);                                                              \
            sidx += 2;                                                                                  \
        } else if (CONV && ++csub == q.cv.spt) {                                                        \
            csub = 0;                                                                                   \
            ++ctap;                                                                                     \
            if (++cfs == gS) { cfs = 0; ++cfr; }                                                        \
        }                                                                                               \
    }
#define HBFP_WAIT_COPIES(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")

    // ---- fragment addresses in ring buffer 0 (k-step 1 flips the 32-byte half of the row)
    const int r_a = wm * 32 + l32, r_b = wn * 64 + l32;            // second column tile: + 32 rows = + 2048 bytes
    const int fragA0 = r_a * 64 + (((2 * 0 + lh) ^ ((r_a >> 2) & 3)) * 16);
    const int fragB0 = kHalfTile + r_b * 64 + (((2 * 0 + lh) ^ ((r_b >> 2) & 3)) * 16);
    const int fragA1 = fragA0 ^ 32, fragB1 = ((fragB0 - kHalfTile) ^ 32) + kHalfTile;
    const int offW = 2 * kHalfTile + r_a * 4;                      // + 512 for k-step 1
    const int offS = 2 * kHalfTile + kHalfWords + r_b * 4;         // + 512 for k-step 1, + 128 for the second column tile
    const v2i one_hot = {lh ? 0 : 0x3F80, 0};

    float acc[2][16];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[ni][v] = 0.0f;

    v4i a, b[2];
    acc_t cin, d0, d1;
    uint32_t rowc = 0;
    float sb[2][2];
#define HBFP_READ_STEP(ring, s_, set)                                                                         \
    {                                                                                                         \
        constexpr int s = STEPW ? (s_) : 0;              /* slot of the words */                              \
        const uint8_t *base_ = lds + (ring) * kHalfStage;                                                     \
        rowc = *reinterpret_cast<const uint32_t *>(base_ + offW + (s) * 512);                                 \
        a = *reinterpret_cast<const v4i *>(base_ + ((s_) ? fragA1 : fragA0));                                 \
        b[0] = *reinterpret_cast<const v4i *>(base_ + ((s_) ? fragB1 : fragB0));                              \
        b[1] = *reinterpret_cast<const v4i *>(base_ + ((s_) ? fragB1 : fragB0) + 2048);                       \
        sb[set][0] = *reinterpret_cast<const float *>(base_ + offS + (s) * 512);                              \
        sb[set][1] = *reinterpret_cast<const float *>(base_ + offS + (s) * 512 + 128);                        \
    }
    // One k-step: both matrix instructions, then whatever has to happen between issue and use (MIDDLE:
    // the stage hand-over and the next step's LDS reads), then 32 subtractions, the next step's row
    // constants on the matrix core, and 32 multiply-adds that cover its latency.
#define HBFP_STEP(cur, FIRST, LAST, MIDDLE)                                                             \
    {                                                                                                   \
        if (FIRST) {                                                                                    \
            d0 = ops::mma(a, b[0], ops::start(cin));                                                    \
            d1 = ops::mma(a, b[1], ops::start(cin));                                                    \
        } else {                                                                                        \
            d0 = ops::mma(a, b[0], d0);                                                                 \
            d1 = ops::mma(a, b[1], d1);                                                                 \
        }                                                                                               \
        /* both results live at once: the second matrix instruction runs while the first is scaled */   \
        ops::pin(d0, d1);                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        MIDDLE;                                                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        if (LAST) {                                                                                     \
            float x0[16], x1[16];                                                                       \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) x0[v] = ops::scaled(d0[v], cin[v]);          \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) x1[v] = ops::scaled(d1[v], cin[v]);          \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(x0[v]));              \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(x1[v]));              \
            __builtin_amdgcn_sched_barrier(0);                                                          \
            cin = ops::rows(rowc, one_hot);                                                             \
            if (CHAIN) {                  /* long blocks always chain: the next block starts from its constants */ \
                if (F16) {                                                                              \
                    d0 = ops::start(cin);                                                               \
                    d1 = ops::start(cin);                                                               \
                } else {                                                                                \
                    d0 = ops::rows(rowc, one_hot);                                                      \
                    d1 = ops::rows(rowc, one_hot);                                                      \
                }                                                                                       \
            }                                                                                           \
            __builtin_amdgcn_sched_barrier(0);                                                          \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[0][v] = fmaf(x0[v], sb[cur][0], acc[0][v]); \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[1][v] = fmaf(x1[v], sb[cur][1], acc[1][v]); \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(acc[0][v]));          \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(acc[1][v]));          \
        }                                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                              \
    }
    // Stages come in pairs (a stage is 64 bytes of k, the stored k extent and every split-K range are
    // multiples of 128); the pair starting at stage st lives in ring buffers {0, 1} or {2, 3}.  There is one
    // hand-over per pair, in its last k-step right after the matrix instructions are issued: by then this
    // wave has consumed every LDS read of the pair, so after the barrier both buffers are free for the pair
    // after next, and the next pair - requested a pair earlier - has landed for everyone.  One barrier per
    // four k-steps instead of two was worth 5 % although a copy now has two stages instead of three to land.
    // SPB = 3: whether the k-step that comes now ends a chain; moves on to the next k-step
#define HBFP_CHAIN_ENDS(flag)                                                                           \
    bool flag = false;                                                                                  \
    if (SPB == 3) {                                                                                     \
        flag = cpos == p.spb - 1 || crun == p.chain_limit - 1 || cstep == 2 * nst - 1;                  \
        cpos = cpos == p.spb - 1 ? 0 : cpos + 1;                                                        \
        crun = flag ? 0 : crun + 1;                                                                     \
        ++cstep;                                                                                        \
    }
#define HBFP_PAIR(ring)                                                                                 \
    {                                                                                                   \
        {                                                                                               \
            const bool first0 = !CHAIN, last1 = SPB == 1 || SPB == 2 || (SPB == 0 && (pos == spb64 - 1 || (!F16 && (pos & 3) == 3))); \
            pos = pos == spb64 - 1 ? 0 : pos + 1;                                                       \
            HBFP_CHAIN_ENDS(end0);                                                                      \
            HBFP_CHAIN_ENDS(end1);                                                                      \
            HBFP_STEP(0, first0, SPB == 1 || end0, HBFP_READ_STEP(ring, 1, 1));                         \
            HBFP_STEP(1, SPB == 1, last1 || end1, HBFP_READ_STEP((ring) + 1, 0, 0));                    \
        }                                                                                               \
        {                                                                                               \
            const bool first0 = !CHAIN, last1 = SPB == 1 || SPB == 2 || (SPB == 0 && (pos == spb64 - 1 || (!F16 && (pos & 3) == 3))); \
            pos = pos == spb64 - 1 ? 0 : pos + 1;                                                       \
            HBFP_CHAIN_ENDS(end0);                                                                      \
            HBFP_CHAIN_ENDS(end1);                                                                      \
            HBFP_STEP(0, first0, SPB == 1 || end0, HBFP_READ_STEP((ring) + 1, 1, 1));                   \
            HBFP_STEP(1, SPB == 1, last1 || end1, {                                                     \
                const int rem = st_end - 2 - st;                 /* stages after this pair */           \
                if (rem > 0) {                                                                          \
                    HBFP_WAIT_COPIES(0);                                                                \
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                  \
                    __builtin_amdgcn_s_barrier();                                                       \
                    asm volatile("" ::: "memory");                                                      \
                    if (rem >= 4) { HBFP_COPY_NEXT(ring); HBFP_COPY_NEXT((ring) + 1); }                 \
                    HBFP_READ_STEP(((ring) + 2) & 3, 0, 0);                                             \
                }                                                                                       \
            });                                                                                         \
        }                                                                                               \
    }

    if (nst > 0) {
        HBFP_COPY_NEXT(0);
        HBFP_COPY_NEXT(1);
        if (nst > 2) { HBFP_COPY_NEXT(2); HBFP_COPY_NEXT(3); }
        if (nst > 2) HBFP_WAIT_COPIES(6); else HBFP_WAIT_COPIES(0);
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // A wave whose 64 columns lie past the last column of the product (the second column half of a tile over at most 64
    // remaining columns) has nothing to multiply: it keeps its part of the copies and every hand-over of the loop below,
    // and leaves its SIMD to the waves that compute (the kernel is bound by their vector instructions).
    if (col0 + (wave_u >> 2) * 64 >= p.N) {
        for (int st = st_begin; st < st_end; st += 2) {
            const int ring = ((st - st_begin) & 2);
            const int rem = st_end - 2 - st;
            if (rem > 0) {
                HBFP_WAIT_COPIES(0);
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (rem >= 4) { HBFP_COPY_NEXT(ring); HBFP_COPY_NEXT(ring + 1); }
            }
        }
        if (ENC) {
            __syncthreads();                                 // as below, without results of its own
            __syncthreads();
            w8_encode_from_lds(q.enc, lds, row0, col0, M, p.N);
        }
        return;
    }
    if (nst > 0) {
        HBFP_READ_STEP(0, 0, 0);
        cin = ops::rows(rowc, one_hot);
        if (CHAIN) {
            if (F16) {
                d0 = ops::start(cin);
                d1 = ops::start(cin);
            } else {
                d0 = ops::rows(rowc, one_hot);
                d1 = ops::rows(rowc, one_hot);
            }
        }
    }
    int pos = 0;
    // SPB = 3: k-step within its run of equal exponents, k-steps since the last scaling, k-step of this workgroup's range
    int cpos = SPB == 3 ? (2 * st_begin) % p.spb : 0, crun = 0, cstep = 0;
    for (int st = st_begin; st < st_end;) {
        HBFP_PAIR(0);
        st += 2;
        if (st >= st_end) break;
        HBFP_PAIR(2);
        st += 2;
    }
#undef HBFP_PAIR
#undef HBFP_CHAIN_ENDS
#undef HBFP_READ_STEP
#undef HBFP_STEP
#undef HBFP_COPY_NEXT
#undef HBFP_NEXT_SLOT
#undef HBFP_WAIT_COPIES

    if (ENC) {
        __syncthreads();                                     // every wave has read the last stage of the ring
        w8_tile_to_lds(q.enc, lds, acc, p.final_scale);
        __syncthreads();
        w8_encode_from_lds(q.enc, lds, row0, col0, M, p.N);
        return;
    }
    if (PHASE) {
        // a row of the phase goes to the row of its input position; the 16 rows of a lane are 4 runs of 4
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int64_t i0 = row0 + wm * 32 + 8 * g + 4 * lh;
            const uint32_t per_img = (uint32_t)(gHo * gWo);
            uint32_t img = (uint32_t)i0 / per_img, rem = (uint32_t)i0 % per_img;
            uint32_t yy = rem / (uint32_t)gWo, xx = rem % (uint32_t)gWo;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int v = 4 * g + u;
                const int64_t orow = ((int64_t)img * q.ph.h + (yy * q.ph.sh + ph_py)) * q.ph.w + (xx * q.ph.sw + ph_px);
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    const int64_t j = col0 + wn * 64 + ni * 32 + l32;
                    if (i0 + u < M && j < p.N) {
                        const float val = acc[ni][v] * p.final_scale;
                        if (p.beta) p.C[orow * p.ldc + j] += val;
                        else __builtin_nontemporal_store(val, p.C + orow * p.ldc + j);
                    }
                }
                if (++xx == (uint32_t)gWo) {
                    xx = 0;
                    if (++yy == (uint32_t)gHo) yy = 0, ++img;
                }
            }
        }
        return;
    }
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t i = row0 + wm * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
            const int64_t j = col0 + wn * 64 + ni * 32 + l32;
            if (i < p.M && j < p.N) {
                const float val = acc[ni][v] * p.final_scale;
                if (p.splits > 1) p.partial[((int64_t)split * p.M + i) * p.N + j] = val;
                else if (p.beta) p.C[i * p.ldc + j] += val;
                else __builtin_nontemporal_store(val, p.C + i * p.ldc + j);   // written once, not read again here
            }
        }
}

// fixed-order sum over the split-K slices: deterministic, no float atomics.  The slices of one output are
// requested eight at a time and added in slice order, so the result does not depend on the unrolling.
__global__ __launch_bounds__(kThreads) void splitk_reduce_kernel(const float *partial, float *C, int64_t M, int64_t N,
                                                                  int64_t ldc, int splits, int beta, const int *run_a,
                                                                  const int *run_b) {
    if (stands_down(run_a, run_b)) return;
    const int64_t n = M * N;
    for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < n; e += (int64_t)gridDim.x * kThreads) {
        const int64_t i = e / N, j = e % N;
        float s = beta ? C[i * ldc + j] : 0.0f;
        int z = 0;
        for (; z + 8 <= splits; z += 8) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = partial[(int64_t)(z + u) * n + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += t[u];
        }
        for (; z < splits; ++z) s += partial[(int64_t)z * n + e];
        C[i * ldc + j] = s;
    }
}

template <int SPB, bool DUMP>
int launch_t(const GemmParams &p, dim3 grid, hipStream_t s) {
    static std::atomic<bool> configured{false};
    if (allow_dynamic_lds(configured, reinterpret_cast<const void *>(&gemm_i8_kernel<SPB, DUMP>), kLdsBytes) != HBFP_OK) return HBFP_ERR_LAUNCH;
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
    if (s > 8) s -= s % 8;                             // the k ranges are dealt to the 8 XCDs in turn: keep them level
    return s < 1 ? 1 : (int)s;
}

// the asynchronous-copy kernel addresses an operand tile with 32-bit offsets
static bool use_w8(int64_t kpad) { return (uint64_t)127 * (uint64_t)kpad + 128 < ((uint64_t)1 << 32); }
static size_t split_bytes(int64_t M, int64_t N, int splits) {
    return splits <= 1 ? 0 : ((size_t)splits * (size_t)M * (size_t)N * 4 + 255) & ~(size_t)255;
}

// workspace: [split-K slices][row words of A][column words of B]
size_t gemm_i8_workspace(int64_t M, int64_t N, int64_t kpad, int64_t kbp, int64_t exp_ld) {
    const int64_t nstage = kpad / BK, spb = kbp / 32;
    const int splits = choose_splits(M, N, nstage, spb >= 4 ? spb / 4 : 1);
    size_t n = split_bytes(M, N, splits);
    if (use_w8(kpad)) n += word_bytes(M, exp_ld) + word_bytes(N, exp_ld);
    return n;
}

// ------------------------------------------------------------------------------------------------
// Convolution as a matrix product whose activation operand is gathered from the encoded image by the product
// kernel's own copies (Sec. 5.1).  Row constants of the image [channel block][pixels], column scales of the filter
// matrix [k block][filters] and the page of zeros that out-of-image taps read, all in one small kernel.
namespace {
__global__ __launch_bounds__(256) void conv_words_kernel(const uint8_t *eimg, int64_t eimg_ld, int64_t pixels, int cblocks, int64_t pitch,
                                                         uint32_t *wimg, const uint8_t *eflt, int64_t eflt_ld, int64_t N, int kblocks,
                                                         int64_t npad, uint32_t *wflt, uint32_t *zeros) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.y == 0) {
        if (i < pixels) {
            for (int b = 0; b < cblocks; ++b) {
                uint32_t e = eimg[i * eimg_ld + b];
                e = e > 254u ? 254u : e;
                wimg[(int64_t)b * pitch + i] = (e << 7) | 0x40u;            // bf16 pattern of 1.5 * 2^(E - 127)
            }
        }
        if (i < 64) zeros[i] = i == 16 ? 0xC0u : 0u;                        // 64 zero bytes, then the row constant of E = 1
    } else if (i < npad) {
        for (int b = 0; b < kblocks; ++b) {
            uint32_t e = i < N ? eflt[i * eflt_ld + b] : 1u;
            e = e > 254u ? 254u : e;
            wflt[(int64_t)b * npad + i] = e << 23;                         // the float 2^(E - 127)
        }
    }
}
}  // namespace

// whether the gathering kernel can deliver this product as the encoded operand `out` (no split along k)
bool conv_encoded_output_ok(int64_t M, int64_t N, int64_t kpad, const hbfp_tensor &out) {
    return out.contract_axis == 1 && out.kblock == 32 && out.kblock_pad == 32 && out.rblock == 1 && out.kshare == 1 && out.mant_bits <= 8 &&
           out.rows == M && out.kdim == N && choose_splits(M, N, kpad / BK, 1) == 1;
}

size_t gemm_conv_workspace(int64_t M, int64_t N, int64_t kpad, int64_t pixels, int cblocks) {
    const int splits = choose_splits(M, N, kpad / BK, 1);
    return split_bytes(M, N, splits) + (size_t)cblocks * (size_t)(ceil_div(pixels, 128) * 128) * 4 + word_bytes(N, kpad / 32) + 256;
}

// a: M = output positions, N = filters, mantB/expB = the filter matrix, kpad = its stored k extent (r * s * c rounded up to
// 128); mantA/expA = the encoded image [pixels][pix_bytes], expA_ld its exponent pitch.
// Whether the data gradient of a convolution with these strides and this window runs phase by phase: every phase must
// meet at least one filter tap in each direction.
bool conv_dgrad_by_phase(int r, int s, int stride_h, int stride_w) {
    return (stride_h > 1 || stride_w > 1) && stride_h * stride_w <= kConvPhases && r >= stride_h && s >= stride_w;
}

// dil_h, dil_w > 1: the image stands for its zero-dilated form (c.h, c.w are the stored extents; c.pad_* and the taps
// count in dilated positions); ho x wo is then whatever the caller wants computed.  by_phase: the same result computed
// output phase by output phase (conv_dgrad_by_phase must hold), without multiplying the zeros.  slot_order >= 0: the
// general gather from an image stored in blocks of kblock channels (c.c a multiple of it), k tap by tap (0) or channel
// block by channel block (1); it combines with the dilation, not with the phases.  chain > 1 (slot_order 1, no dilation):
// both operands repeat their exponents over runs of `chain` consecutive stored blocks, which are then scaled once.
// enc: the product leaves as this encoded operand (rows of C, blocks of 32 along its columns, at most 8 bits; the caller
// has checked conv_encoded_output_ok), with ReLU first if asked for; a.C is then unused.
int launch_gemm_conv_i8(const GemmArgs &a, const hbfp_conv2d &c, int64_t ho, int64_t wo, int64_t pix_bytes, void *workspace,
                        hipStream_t s, int dil_h, int dil_w, bool by_phase, int slot_order, int kblock, int chain, const hbfp_tensor *enc,
                        int relu) {
    GemmParams p = {};
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
    p.nblk = a.nblk;
    p.nstage = (int32_t)(a.kpad / BK);
    p.spb = 1;
    const int64_t tm = ceil_div(a.M, BM), tn = ceil_div(a.N, BN);
    if (tm * tn > 0x7ffffff0 || a.kpad / BK > 0x7fffffff || !use_w8(a.kpad)) return HBFP_ERR_ARG;
    p.tiles_m = (int32_t)tm;
    p.tiles_n = (int32_t)tn;
    p.beta = a.beta != 0.0f;
    p.final_scale = ldexpf(1.0f, 27 - a.mA - a.mB);
    p.splits = choose_splits(a.M, a.N, p.nstage, 1);
    p.stages_per_split = (int32_t)ceil_div(p.nstage, p.splits);
    p.splits = (int32_t)ceil_div(p.nstage, p.stages_per_split);
    p.partial = (float *)workspace;
    const int64_t pixels = c.n * c.h * c.w;
    const bool slots = slot_order >= 0;
    if (slots && (kblock < 1 || kblock > 32 || c.c % kblock || by_phase)) return HBFP_ERR_ARG;
    const int cblocks = (int)(slots ? c.c / kblock : c.c / 32);
    W8Params q = {};
    q.g = p;
    q.mpad = ceil_div(a.M, 128) * 128;
    q.npad = ceil_div(a.N, 128) * 128;
    uint8_t *w = (uint8_t *)workspace + split_bytes(a.M, a.N, p.splits);
    const int64_t pitch = ceil_div(pixels, 128) * 128;
    uint32_t *wimg = (uint32_t *)w;
    uint32_t *wflt = wimg + (size_t)cblocks * pitch;
    uint32_t *zeros = wflt + word_bytes(a.N, a.kpad / 32) / 4;
    q.wA = wimg;                 // unused by the gathering kernel
    q.wB = wflt;
    q.cv.zeros = (const uint8_t *)zeros;
    q.cv.words = wimg;
    q.cv.word_pitch = pitch;
    q.cv.H = (int32_t)c.h;
    q.cv.W = (int32_t)c.w;
    q.cv.Ho = (int32_t)ho;
    q.cv.Wo = (int32_t)wo;
    q.cv.S = c.s;
    q.cv.ntaps = c.r * c.s;
    q.cv.spt = slots ? 1 : (int32_t)(c.c / 64);
    q.cv.ncb = cblocks;
    q.cv.R = c.r;
    q.cv.cb_order = slot_order > 0;
    q.cv.nslots = c.r * c.s * cblocks;
    q.cv.pad_h = c.pad_h;
    q.cv.pad_w = c.pad_w;
    q.cv.str_h = c.stride_h;
    q.cv.str_w = c.stride_w;
    q.cv.pix_bytes = (int32_t)pix_bytes;
    q.cv.dil_h = dil_h;
    q.cv.dil_w = dil_w;
    q.cv.inv_dh = 1.0f / (float)dil_h;
    q.cv.inv_dw = 1.0f / (float)dil_w;
    const bool dilated = dil_h > 1 || dil_w > 1;
    if (dil_h < 1 || dil_w < 1) return HBFP_ERR_ARG;
    // the kernel divides dilated coordinates in FP32
    if (dilated && (ho * c.stride_h + c.r + (c.pad_h < 0 ? -c.pad_h : c.pad_h) >= (1 << 21) ||
                    wo * c.stride_w + c.s + (c.pad_w < 0 ? -c.pad_w : c.pad_w) >= (1 << 21)))
        return HBFP_ERR_ARG;
    {
        const int64_t most = pixels > q.npad ? pixels : q.npad;
        if (ceil_div(most, 256) > 0x7fffffff) return HBFP_ERR_ARG;
        hipLaunchKernelGGL(conv_words_kernel, dim3((unsigned)ceil_div(most, 256), 2), dim3(256), 0, s, a.expA, a.expA_ld, pixels, cblocks,
                           pitch, wimg, a.expB, a.expB_ld, a.N, (int)(a.kpad / 32), q.npad, wflt, zeros);
        if (launch_status() != HBFP_OK) return HBFP_ERR_LAUNCH;
    }
    static std::atomic<bool> configured{false}, configured_dil{false};
    if (allow_dynamic_lds(configured, reinterpret_cast<const void *>(&gemm_i8_w8_kernel<1, true>), kW8LdsBytes) != HBFP_OK) return HBFP_ERR_LAUNCH;
    if (allow_dynamic_lds(configured_dil, reinterpret_cast<const void *>(&gemm_i8_w8_kernel<1, true, false, 1>), kW8LdsBytes) != HBFP_OK)
        return HBFP_ERR_LAUNCH;
    if (by_phase) {
        if (!conv_dgrad_by_phase(c.r, c.s, dil_h, dil_w) || c.stride_h != 1 || c.stride_w != 1) return HBFP_ERR_ARG;
        static std::atomic<bool> configured_phase{false};
        if (allow_dynamic_lds(configured_phase, reinterpret_cast<const void *>(&gemm_i8_w8_kernel<1, true, false, 2>), kW8LdsBytes) != HBFP_OK)
            return HBFP_ERR_LAUNCH;
        q.g.splits = 1;
        q.ph.sh = dil_h, q.ph.sw = dil_w, q.ph.h = (int32_t)ho, q.ph.w = (int32_t)wo, q.ph.s_full = c.s, q.ph.n = (int32_t)c.n;
        const auto mod = [](int x, int m) { return ((x % m) + m) % m; };
        int64_t most = 0;
        for (int py = 0; py < dil_h; ++py)
            for (int px = 0; px < dil_w; ++px) {
                ConvPhase &f = q.ph.p[py * dil_w + px];
                f.py = py, f.px = px;
                f.Hp = ho > py ? (int32_t)((ho - py + dil_h - 1) / dil_h) : 0;
                f.Wp = wo > px ? (int32_t)((wo - px + dil_w - 1) / dil_w) : 0;
                f.fr0 = mod(c.pad_h - py, dil_h), f.fs0 = mod(c.pad_w - px, dil_w);
                f.Rp = (c.r - f.fr0 + dil_h - 1) / dil_h, f.Sp = (c.s - f.fs0 + dil_w - 1) / dil_w;
                f.oy0 = (py - c.pad_h + f.fr0) / dil_h, f.ox0 = (px - c.pad_w + f.fs0) / dil_w;   // exact divisions
                const int64_t rows = c.n * f.Hp * f.Wp;
                f.tiles_m = (int32_t)ceil_div(rows, BM);
                f.nst = (int32_t)(ceil_div((int64_t)f.Rp * f.Sp * q.cv.spt, 2) * 2);
                most = f.tiles_m > most ? f.tiles_m : most;
            }
        hipLaunchKernelGGL((gemm_i8_w8_kernel<1, true, false, 2>), dim3((unsigned)(ceil_div(most * tn, 8) * 8), (unsigned)(dil_h * dil_w)),
                           dim3(kW8Threads), kW8LdsBytes, s, q);
        return launch_status();
    }
    const dim3 grid = p.splits >= 8 ? dim3((unsigned)(8 * tm * tn * ceil_div(p.splits, 8)))
                                    : dim3((unsigned)(ceil_div(tm * tn, 8) * 8), (unsigned)p.splits);
    if (enc) {
        if (dilated || p.splits != 1 || p.beta) return HBFP_ERR_ARG;
        q.enc.mant = (uint8_t *)enc->mant;
        q.enc.exps = enc->exps;
        q.enc.kpad = enc->kpad;
        q.enc.exp_ld = enc->exp_ld;
        q.enc.nblk = (int32_t)enc->nblk;
        q.enc.m = enc->mant_bits;
        q.enc.rounding = enc->rounding;
        q.enc.relu = relu;
        q.enc.s0 = (uint32_t)enc->seed;
        q.enc.s1 = (uint32_t)(enc->seed >> 32);
        // (the variant that scales runs of blocks once has no registers left for this epilogue: the caller converts behind it)
        if (chain > 1) return HBFP_ERR_ARG;
        static std::atomic<bool> c0{false}, c1{false};
        if (allow_dynamic_lds(c0, reinterpret_cast<const void *>(&gemm_i8_w8_kernel<1, true, false, 0, true>), kW8LdsBytes) != HBFP_OK ||
            allow_dynamic_lds(c1, reinterpret_cast<const void *>(&gemm_i8_w8_kernel<1, true, false, 3, true>), kW8LdsBytes) != HBFP_OK)
            return HBFP_ERR_LAUNCH;
        if (slots) hipLaunchKernelGGL((gemm_i8_w8_kernel<1, true, false, 3, true>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
        else hipLaunchKernelGGL((gemm_i8_w8_kernel<1, true, false, 0, true>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
        return launch_status();
    }
    const int64_t chain_limit = (((int64_t)1 << 22) - 1) / ((int64_t)kblock * (((int64_t)1 << (a.mA - 1)) - 1) * (((int64_t)1 << (a.mB - 1)) - 1));
    if (slots && !dilated && slot_order == 1 && chain > 1 && chain_limit > 1) {
        static std::atomic<bool> configured_chain{false};
        if (allow_dynamic_lds(configured_chain, reinterpret_cast<const void *>(&gemm_i8_w8_kernel<3, true, false, 3>), kW8LdsBytes) != HBFP_OK)
            return HBFP_ERR_LAUNCH;
        q.g.spb = chain;
        q.g.chain_limit = (int32_t)(chain_limit < chain ? chain_limit : chain);
        hipLaunchKernelGGL((gemm_i8_w8_kernel<3, true, false, 3>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
    } else if (slots) {
        static std::atomic<bool> configured_slot{false}, configured_slot_dil{false};
        if (allow_dynamic_lds(configured_slot, reinterpret_cast<const void *>(&gemm_i8_w8_kernel<1, true, false, 3>), kW8LdsBytes) != HBFP_OK ||
            allow_dynamic_lds(configured_slot_dil, reinterpret_cast<const void *>(&gemm_i8_w8_kernel<1, true, false, 4>), kW8LdsBytes) != HBFP_OK)
            return HBFP_ERR_LAUNCH;
        if (dilated) hipLaunchKernelGGL((gemm_i8_w8_kernel<1, true, false, 4>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
        else hipLaunchKernelGGL((gemm_i8_w8_kernel<1, true, false, 3>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
    } else if (dilated) hipLaunchKernelGGL((gemm_i8_w8_kernel<1, true, false, 1>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
    else hipLaunchKernelGGL((gemm_i8_w8_kernel<1, true>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
    int rc = launch_status();
    if (rc != HBFP_OK) return rc;
    if (p.splits > 1) {
        int64_t nb = ceil_div(a.M * a.N, kThreads);
        if (nb > 8192) nb = 8192;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)nb), dim3(kThreads), 0, s, p.partial, p.C, p.M, p.N, p.ldc, p.splits,
                           p.beta, (const int *)nullptr, (const int *)nullptr);
        rc = launch_status();
    }
    return rc;
}

// ------------------------------------------------------------------------------------------------
// 9..12-bit mantissas on the FP16 matrix instruction: the int16 mantissas become FP16 planes (exact: |m| <= 2047) in
// the workspace, then the kernel above runs on them with F16 set.  workspace: [split-k slices][A plane][B plane]
// [row words of A][column words of B].
namespace {
__global__ __launch_bounds__(256) void mant_to_f16_kernel(const int16_t *src, _Float16 *dst, int64_t n8) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        const v4i x = reinterpret_cast<const v4i *>(src)[i];
        v8h y;
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] = (_Float16)(float)(int16_t)((uint32_t)x[e >> 1] >> (16 * (e & 1)));
        reinterpret_cast<v8h *>(dst)[i] = y;
    }
}
size_t f16_plane_bytes(int64_t rows, int64_t kpad) { return ((size_t)rows * (size_t)kpad * 2 + 255) & ~(size_t)255; }
int f16_splits(int64_t M, int64_t N, int64_t kpad, int64_t kbp) {
    const int64_t spb = kbp / 16;                       // k-steps of 32 bytes per block
    return choose_splits(M, N, kpad * 2 / BK, spb >= 4 ? spb / 4 : 1);
}
}  // namespace

bool gemm_f16_possible(const GemmArgs &a) {
    return !a.P && a.mA > 8 && a.mB > 8 && a.mA <= 12 && a.mB <= 12 && (a.kbp == 32 || a.kbp == 64 || a.kbp % 128 == 0) &&
           use_w8(a.kpad * 2) && ceil_div(a.M, BM) * ceil_div(a.N, BN) <= 0x7ffffff0 && a.kpad * 2 / BK <= 0x7fffffff;
}

size_t gemm_f16_workspace(int64_t M, int64_t N, int64_t kpad, int64_t kbp, int64_t exp_ld) {
    return split_bytes(M, N, f16_splits(M, N, kpad, kbp)) + f16_plane_bytes(M, kpad) + f16_plane_bytes(N, kpad) + word_bytes(M, exp_ld) +
           word_bytes(N, exp_ld);
}

int launch_gemm_f16(const GemmArgs &a, void *workspace, hipStream_t s) {
    if (!gemm_f16_possible(a) || !workspace) return HBFP_ERR_FORMAT;
    GemmParams p = {};
    p.splits = f16_splits(a.M, a.N, a.kpad, a.kbp);
    uint8_t *w = (uint8_t *)workspace;
    p.partial = (float *)w;
    w += split_bytes(a.M, a.N, p.splits);
    _Float16 *planeA = (_Float16 *)w;
    w += f16_plane_bytes(a.M, a.kpad);
    _Float16 *planeB = (_Float16 *)w;
    w += f16_plane_bytes(a.N, a.kpad);
    {
        const int64_t na = a.M * a.kpad / 8, nb = a.N * a.kpad / 8;       // kpad is a multiple of 128
        int64_t ga = ceil_div(na, 256), gb = ceil_div(nb, 256);
        ga = ga > 65536 ? 65536 : ga;
        gb = gb > 65536 ? 65536 : gb;
        hipLaunchKernelGGL(mant_to_f16_kernel, dim3((unsigned)ga), dim3(256), 0, s, (const int16_t *)a.mantA, planeA, na);
        hipLaunchKernelGGL(mant_to_f16_kernel, dim3((unsigned)gb), dim3(256), 0, s, (const int16_t *)a.mantB, planeB, nb);
        if (launch_status() != HBFP_OK) return HBFP_ERR_LAUNCH;
    }
    p.A = (const uint8_t *)planeA;
    p.B = (const uint8_t *)planeB;
    p.eA = a.expA;
    p.eB = a.expB;
    p.C = a.C;
    p.M = a.M;
    p.N = a.N;
    p.kpad = a.kpad * 2;                                  // bytes of k per operand row
    p.eA_ld = a.expA_ld;
    p.eB_ld = a.expB_ld;
    p.ldc = a.ldc;
    p.nblk = a.nblk;
    p.nstage = (int32_t)(p.kpad / BK);
    p.spb = (int32_t)(a.kbp / 16);                        // k-steps of 32 bytes (16 elements) per exponent block
    const int64_t tm = ceil_div(a.M, BM), tn = ceil_div(a.N, BN);
    p.tiles_m = (int32_t)tm;
    p.tiles_n = (int32_t)tn;
    p.beta = a.beta != 0.0f;
    p.final_scale = ldexpf(1.0f, 4 - a.mA - a.mB);        // scales are 2^(E - 127) each, one mantissa unit 2^(E - 125 - m)
    const int stages_per_block = p.spb >= 4 ? p.spb / 4 : 1;
    {
        const int64_t units = p.nstage / stages_per_block;
        p.stages_per_split = (int32_t)(ceil_div(units, p.splits) * stages_per_block);
        p.splits = (int32_t)ceil_div(p.nstage, p.stages_per_split);
    }
    W8Params q = {};
    q.g = p;
    q.mpad = ceil_div(a.M, 128) * 128;
    q.npad = ceil_div(a.N, 128) * 128;
    q.wA = (const uint32_t *)w;
    q.wB = (const uint32_t *)(w + word_bytes(a.M, a.expA_ld));
    int rc = launch_scale_words(a.expA, a.expA_ld, a.M, a.expB, a.expB_ld, a.N, (int)a.expA_ld, 0u, const_cast<uint32_t *>(q.wA),
                                const_cast<uint32_t *>(q.wB), nullptr, nullptr, s);
    if (rc != HBFP_OK) return rc;
    static std::atomic<bool> configured[2];
    const void *const kernels[2] = {reinterpret_cast<const void *>(&gemm_i8_w8_kernel<2, false, true>),
                                    reinterpret_cast<const void *>(&gemm_i8_w8_kernel<0, false, true>)};
    for (int i = 0; i < 2; ++i)
        if (allow_dynamic_lds(configured[i], kernels[i], kW8LdsBytes) != HBFP_OK) return HBFP_ERR_LAUNCH;
    const dim3 grid = p.splits >= 8 ? dim3((unsigned)(8 * tm * tn * ceil_div(p.splits, 8)))
                                    : dim3((unsigned)(ceil_div(tm * tn, 8) * 8), (unsigned)p.splits);
    if (p.spb == 2) hipLaunchKernelGGL((gemm_i8_w8_kernel<2, false, true>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
    else hipLaunchKernelGGL((gemm_i8_w8_kernel<0, false, true>), grid, dim3(kW8Threads), kW8LdsBytes, s, q);
    rc = launch_status();
    if (rc != HBFP_OK) return rc;
    if (p.splits > 1) {
        int64_t nb = ceil_div(a.M * a.N, kThreads);
        if (nb > 8192) nb = 8192;
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)nb), dim3(kThreads), 0, s, p.partial, p.C, p.M, p.N, p.ldc, p.splits,
                           p.beta, (const int *)nullptr, (const int *)nullptr);
        rc = launch_status();
    }
    return rc;
}

// split-K plan of the int8 kernels for product `a`
static void split_plan(const GemmArgs &a, int32_t *splits, int32_t *stages_per_split) {
    const int32_t nstage = (int32_t)(a.kpad / BK), spb = (int32_t)(a.kbp / 32);
    const int stages_per_block = spb >= 4 ? spb / 4 : 1;
    int32_t sp = a.P ? 1 : choose_splits(a.M, a.N, nstage, stages_per_block);
    const int64_t units = nstage / stages_per_block;
    *stages_per_split = (int32_t)(ceil_div(units, sp) * stages_per_block);
    *splits = (int32_t)ceil_div(nstage, *stages_per_split);
}

bool gemm_i8_standby_words(const GemmArgs &a, void *workspace, StandbyWords *w) {
    if (!workspace || a.P || a.mA > 8 || a.mB > 8 || !use_w8(a.kpad)) return false;
    if (a.wide ? gemm_wide_possible(a) : gemm_wide_ok(a)) return false;                  // that kernel reads exponent bytes itself
    if (ceil_div(a.M, BM) * ceil_div(a.N, BN) > 0x7ffffff0 || a.kpad / BK > 0x7fffffff) return false;
    int32_t splits, sps;
    split_plan(a, &splits, &sps);
    uint8_t *base = (uint8_t *)workspace + split_bytes(a.M, a.N, splits);
    w->eA = a.expA; w->eB = a.expB;
    w->ldA = a.expA_ld; w->ldB = a.expB_ld;
    w->M = a.M; w->N = a.N;
    w->slots = (int32_t)a.expA_ld;
    w->a_or = 0x40u;
    w->wA = (uint32_t *)base;
    w->wB = (uint32_t *)(base + word_bytes(a.M, a.expA_ld));
    return true;
}

int launch_gemm_i8(const GemmArgs &a, void *workspace, hipStream_t s) {
    if (a.wide ? gemm_wide_possible(a) : gemm_wide_ok(a)) return launch_gemm_wide(a, s);
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
    p.run_a = a.run_a;
    p.run_b = a.run_b;
    split_plan(a, &p.splits, &p.stages_per_split);
    const dim3 grid = p.splits >= 8 ? dim3((unsigned)(8 * tm * tn * ceil_div(p.splits, 8)))
                                    : dim3((unsigned)(ceil_div(tm * tn, 8) * 8), (unsigned)p.splits);
    int rc;
    if (a.P) {
        rc = p.spb == 1 ? launch_t<1, true>(p, grid, s) : p.spb == 2 ? launch_t<2, true>(p, grid, s) : launch_t<0, true>(p, grid, s);
    } else {
        // behind the block-scaled kernel the product almost never runs: one launch, no scale-word kernel in front of it;
        // it is the 8-wave kernel when the product kernel has prepared its scale words (words_ready), else the 4-wave one
        if (use_w8(a.kpad) && (!a.run_a || a.words_ready)) {
            static std::atomic<bool> configured[3];
            const void *const kernels[3] = {reinterpret_cast<const void *>(&gemm_i8_w8_kernel<1>), reinterpret_cast<const void *>(&gemm_i8_w8_kernel<2>),
                                            reinterpret_cast<const void *>(&gemm_i8_w8_kernel<0>)};
            for (int i = 0; i < 3; ++i)
                if (allow_dynamic_lds(configured[i], kernels[i], kW8LdsBytes) != HBFP_OK) return HBFP_ERR_LAUNCH;
            if (!workspace) return HBFP_ERR_WORKSPACE;
            W8Params q;
            q.g = p;
            q.mpad = ceil_div(a.M, 128) * 128;
            q.npad = ceil_div(a.N, 128) * 128;
            uint8_t *w = (uint8_t *)workspace + split_bytes(a.M, a.N, p.splits);
            q.wA = (const uint32_t *)w;
            q.wB = (const uint32_t *)(w + word_bytes(a.M, a.expA_ld));
            if (!a.words_ready) {
                rc = launch_scale_words(a.expA, a.expA_ld, a.M, a.expB, a.expB_ld, a.N, (int)a.expA_ld, 0x40u,
                                        const_cast<uint32_t *>(q.wA), const_cast<uint32_t *>(q.wB), a.run_a, a.run_b, s);
                if (rc != HBFP_OK) return rc;
            }
            if (p.spb == 1) hipLaunchKernelGGL(gemm_i8_w8_kernel<1>, grid, dim3(kW8Threads), kW8LdsBytes, s, q);
            else if (p.spb == 2) hipLaunchKernelGGL(gemm_i8_w8_kernel<2>, grid, dim3(kW8Threads), kW8LdsBytes, s, q);
            else hipLaunchKernelGGL(gemm_i8_w8_kernel<0>, grid, dim3(kW8Threads), kW8LdsBytes, s, q);
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
                           p.ldc, p.splits, p.beta, p.run_a, p.run_b);
        rc = launch_status();
    }
    return rc;
}

}  // namespace hbfp
