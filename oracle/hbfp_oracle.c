/*
 * CPU oracle for the block-floating-point (BFP) hot path of HBFP
 * ("Training DNNs with Hybrid Block Floating Point", arXiv 1804.01526).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from the product path.
 *
 * What it follows in the paper:
 *   - Eq. (1), Sec. 4:  a_i = m_i * 2^e  (one exponent e shared by a block).
 *   - Sec. 4.1 / Sec. 5.3: the shared exponent is the exponent of the largest
 *     magnitude in the block; mantissas are normalised to it.
 *   - Eq. (2), Sec. 4:  a.b = 2^(ea+eb) * (m^a . m^b), the mantissa dot product
 *     being a pure fixed-point (integer) sum.
 *   - Sec. 4 (tiled matmul) / Sec. 4.2 "Tiling": per-tile fixed-point results
 *     are accumulated in floating point.
 *   - Sec. 5.3: stochastic rounding during mantissa truncation.
 *   - Sec. 4.2 "Wide weight storage" / Sec. 5.1 (optimizer shell): weights live in
 *     BFP with wide mantissas; an update is computed in FP32 and converted to a
 *     wide and a narrow BFP tensor.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - "m-bit mantissa" counts the sign: two's complement, symmetric range
 *     +-(2^(m-1)-1).
 *   - The largest magnitude of a block occupies the top magnitude bit; if
 *     rounding it would reach 2^(m-1) the shared exponent is raised by one.
 *   - Round-to-nearest-even or stochastic rounding act on the magnitude, the
 *     sign is applied afterwards.
 *   - The random numbers of stochastic rounding come from a counter hash of
 *     (seed, logical element index r*cols+c); the hash is specified in prose in
 *     the public header and typed independently here ("parity unpinned" as to
 *     the choice of hash; its statistics are pinned by tests).
 *   - The stored exponent byte Eb is the IEEE-754 biased exponent of the block
 *     maximum (after the possible raise), at least 1; an element's value is
 *     mant * 2^(Eb - 125 - m).
 *
 * Everything is integer arithmetic on FP32 bit patterns except the GEMM, which
 * is the plain FP64 triple loop over the dequantised operands.
 */
#include <stdint.h>
#include <string.h>
#include <math.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static uint32_t bits_of(float x) {
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    return u;
}

int hbfp_ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Counter hash for stochastic rounding (Sec. 5.3 names a xorshift generator:
 * three shifts, three xors; that triple is the first mixing stage here, and a
 * two-multiply avalanche stage follows so that consecutive counters decorrelate).
 */
uint32_t hbfp_ref_hash32(uint64_t seed, uint64_t idx) {
    uint32_t x = (uint32_t)idx ^ (uint32_t)seed;
    x ^= x << 13;
    x ^= x >> 17;
    x ^= x << 5;
    x += (uint32_t)(idx >> 32) ^ (uint32_t)(seed >> 32);
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}

/* number of blocks along an extent n for block length b (b == 0: one block) */
static int64_t nblocks(int64_t n, int64_t b) {
    if (b <= 0 || b >= n) return 1;
    return (n + b - 1) / b;
}

/*
 * FP32 -> BFP (Sec. 4.1: convert before every dot product, using the exponent
 * of the largest value; Sec. 5.3: detect the maximum exponent, normalise).
 *
 * src   [rows][ld]   FP32, finite
 * block = br x bc elements of src share one exponent (0 = whole extent);
 *         edge blocks are short.
 * m     mantissa bits including the sign, 2..16
 * rounding 0 = round to nearest even, 1 = stochastic
 * mant  [rows][cols] int32 (value range +-(2^(m-1)-1))
 * exps  [nbr][nbc]   stored exponent byte of each block
 * returns 0, or -1 on a bad argument.
 */
int hbfp_ref_encode(const float *src, int64_t rows, int64_t cols, int64_t ld,
                    int64_t br, int64_t bc, int m, int rounding, uint64_t seed,
                    int32_t *mant, uint8_t *exps) {
    if (!src || !mant || !exps || rows <= 0 || cols <= 0 || ld < cols) return -1;
    if (m < 2 || m > 16 || (rounding != 0 && rounding != 1)) return -1;
    if (br <= 0 || br > rows) br = rows;
    if (bc <= 0 || bc > cols) bc = cols;
    const int64_t nbr = nblocks(rows, br), nbc = nblocks(cols, bc);
    const int sh0 = 25 - m; /* shift that leaves m-1 magnitude bits of a 24-bit significand */

#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t tb = 0; tb < nbr; ++tb) {
        for (int64_t cb = 0; cb < nbc; ++cb) {
            const int64_t r0 = tb * br, r1 = (r0 + br < rows) ? r0 + br : rows;
            const int64_t c0 = cb * bc, c1 = (c0 + bc < cols) ? c0 + bc : cols;

            /* step 1: largest magnitude (bit patterns of finite floats order like magnitudes) */
            uint32_t amax = 0;
            for (int64_t r = r0; r < r1; ++r)
                for (int64_t c = c0; c < c1; ++c) {
                    uint32_t a = bits_of(src[r * ld + c]) & 0x7fffffffu;
                    if (a > amax) amax = a;
                }

            /* step 2: shared exponent = exponent of the maximum, raised by one exactly
               when rounding the maximum could carry out of its m-1 magnitude bits */
            const uint32_t rb = rounding ? ((1u << sh0) - 1u) : (1u << (sh0 - 1));
            uint32_t Eb = (uint32_t)(((uint64_t)amax + rb) >> 23);
            if (Eb < 1) Eb = 1;
            if (Eb > 255) Eb = 255; /* only reachable with non-finite input */
            exps[tb * nbc + cb] = (uint8_t)Eb;

            /* step 3: align every significand to the shared exponent and round */
            for (int64_t r = r0; r < r1; ++r)
                for (int64_t c = c0; c < c1; ++c) {
                    const uint32_t u = bits_of(src[r * ld + c]);
                    const uint32_t a = u & 0x7fffffffu;
                    const uint32_t be = a >> 23;
                    const uint32_t bep = be ? be : 1;                    /* subnormals: exponent 1, no hidden bit */
                    const uint32_t sig = (a & 0x7fffffu) | (be ? 0x800000u : 0u);
                    const int sh = sh0 + (int)Eb - (int)bep;             /* |x| = sig * 2^(bep-150) */
                    uint32_t q;
                    if (rounding == 0) {
                        if (sh >= 26) q = 0;
                        else q = (uint32_t)(((uint64_t)sig + (1u << (sh - 1)) - 1u + ((sig >> sh) & 1u)) >> sh);
                    } else {
                        if (sh > 32) q = 0;
                        else {
                            const uint64_t idx = (uint64_t)r * (uint64_t)cols + (uint64_t)c;
                            const uint32_t h = hbfp_ref_hash32(seed, idx);
                            const uint64_t rnd = (sh == 32) ? (uint64_t)h : (uint64_t)(h >> (32 - sh));
                            q = (uint32_t)(((uint64_t)sig + rnd) >> sh);
                        }
                    }
                    const uint32_t qmax = (1u << (m - 1)) - 1u;
                    if (q > qmax) q = qmax; /* only reachable with non-finite input */
                    mant[r * cols + c] = (u >> 31) ? -(int32_t)q : (int32_t)q;
                }
        }
    }
    return 0;
}

/* BFP -> FP32, Eq. (1): value = mant * 2^(Eb - 125 - m); exact in FP32. */
int hbfp_ref_decode(const int32_t *mant, const uint8_t *exps, int64_t rows, int64_t cols,
                    int64_t br, int64_t bc, int m, float *dst, int64_t ld) {
    if (!mant || !exps || !dst || rows <= 0 || cols <= 0 || ld < cols) return -1;
    if (m < 2 || m > 16) return -1;
    if (br <= 0 || br > rows) br = rows;
    if (bc <= 0 || bc > cols) bc = cols;
    const int64_t nbc = nblocks(cols, bc);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            const int e = (int)exps[(r / br) * nbc + (c / bc)] - 125 - m;
            dst[r * ld + c] = (float)ldexp((double)mant[r * cols + c], e);
        }
    return 0;
}

/*
 * Fixed-point part of Eq. (2) per exponent block along the contraction axis:
 *   P[i][j][b] = sum over k in block b of mA[i][k] * mB[k][j]
 * mA [M][K], mB [K][N] int32 mantissas, kb = block length along K (0 = K).
 * Sums are taken in int64 and must fit int32 ("wide accumulators", Sec. 5.3);
 * returns -2 if any does not, -1 on a bad argument, else 0.
 */
int hbfp_ref_block_dots(const int32_t *mA, const int32_t *mB, int64_t M, int64_t N, int64_t K,
                        int64_t kb, int32_t *P) {
    if (!mA || !mB || !P || M <= 0 || N <= 0 || K <= 0) return -1;
    if (kb <= 0 || kb > K) kb = K;
    const int64_t nb = nblocks(K, kb);
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j)
            for (int64_t b = 0; b < nb; ++b) {
                const int64_t k0 = b * kb, k1 = (k0 + kb < K) ? k0 + kb : K;
                int64_t s = 0;
                for (int64_t k = k0; k < k1; ++k) s += (int64_t)mA[i * K + k] * (int64_t)mB[k * N + j];
                if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
                P[(i * N + j) * nb + b] = (int32_t)s;
            }
    return bad ? -2 : 0;
}

/*
 * The BFP matrix product by its definition: C = A * B over the dequantised
 * operands, every product and sum in FP64 (a product of two FP32 values is
 * exact in FP64).  A [M][lda], B [K][ldb], C [M][N].
 */
int hbfp_ref_gemm(const float *A, int64_t lda, const float *B, int64_t ldb,
                  int64_t M, int64_t N, int64_t K, double *C) {
    if (!A || !B || !C || M <= 0 || N <= 0 || K <= 0 || lda < K || ldb < N) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *c = C + i * N;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = (double)A[i * lda + k];
            const float *b = B + k * ldb;
            for (int64_t j = 0; j < N; ++j) c[j] += a * (double)b[j];
        }
    }
    return 0;
}

/* Same definition, only for the listed rows of A: C [nsel][N]. */
int hbfp_ref_gemm_rows(const float *A, int64_t lda, const float *B, int64_t ldb,
                       int64_t M, int64_t N, int64_t K,
                       const int64_t *sel, int64_t nsel, double *C) {
    if (!A || !B || !C || !sel || M <= 0 || N <= 0 || K <= 0 || nsel <= 0) return -1;
    for (int64_t s = 0; s < nsel; ++s)
        if (sel[s] < 0 || sel[s] >= M) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < nsel; ++s) {
        const int64_t i = sel[s];
        double *c = C + s * N;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = (double)A[i * lda + k];
            const float *b = B + k * ldb;
            for (int64_t j = 0; j < N; ++j) c[j] += a * (double)b[j];
        }
    }
    return 0;
}

/*
 * Eq. (2) with the tile results accumulated in floating point (Sec. 4):
 *   C[i][j] = sum_b P[i][j][b] * 2^(eA[i][b] + eB[b][j])
 * where eX = Eb - 125 - m is the exponent of one mantissa unit.  Accumulation
 * in FP64.  eA [M][nb], eB [nb][N] are stored exponent bytes per (row, block)
 * and (block, column).  Used for the closed-form pins and as a second way to
 * reach the same C as hbfp_ref_gemm.
 */
int hbfp_ref_scale_accumulate(const int32_t *P, const uint8_t *eA, const uint8_t *eB,
                              int64_t M, int64_t N, int64_t nb, int mA, int mB, double *C) {
    if (!P || !eA || !eB || !C || M <= 0 || N <= 0 || nb <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t b = 0; b < nb; ++b) {
                const int e = ((int)eA[i * nb + b] - 125 - mA) + ((int)eB[b * N + j] - 125 - mB);
                s += ldexp((double)P[(i * N + j) * nb + b], e);
            }
            C[i * N + j] = s;
        }
    return 0;
}

/*
 * One update of weights stored with wide mantissas (Sec. 4.2 "Wide weight storage";
 * Sec. 5.1: the update is done in FP32, then the weights are converted to two BFP
 * formats, wide for later updates and narrow for the forward/backward products).
 * Steps, in the paper's order:
 *   1. w  = mant * 2^(Eb - 125 - m_wide)                      Eq. (1), exact in FP32
 *   2. w' = alpha * delta + w in FP32                          the FP32 update
 *   3. wide' = encode(w', m_wide), narrow' = encode(w', m_narrow), same br x bc blocks
 * Reading where the paper is silent: step 2 is one fused multiply-add (a single
 * FP32 rounding); both conversions start from w' (as the optimizer shell of Sec. 5.1
 * does), so the narrow mantissas are the wide ones rounded, not truncated.
 * w_new (optional, [rows][cols]) receives w'.
 */
int hbfp_ref_weight_update(const int32_t *wide_mant, const uint8_t *wide_exps, int64_t rows, int64_t cols,
                           int64_t br, int64_t bc, int m_wide, int rounding_wide, uint64_t seed_wide,
                           const float *delta, int64_t ld, float alpha,
                           int m_narrow, int rounding_narrow, uint64_t seed_narrow,
                           int32_t *wide_mant_out, uint8_t *wide_exps_out,
                           int32_t *narrow_mant, uint8_t *narrow_exps, float *w_new) {
    if (!wide_mant || !wide_exps || !delta || !wide_mant_out || !wide_exps_out || rows <= 0 || cols <= 0 || ld < cols)
        return -1;
    float *w = w_new ? w_new : (float *)malloc((size_t)rows * (size_t)cols * sizeof(float));
    if (!w) return -1;
    int rc = hbfp_ref_decode(wide_mant, wide_exps, rows, cols, br, bc, m_wide, w, cols);
    if (rc == 0) {
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t c = 0; c < cols; ++c) w[r * cols + c] = fmaf(alpha, delta[r * ld + c], w[r * cols + c]);
        rc = hbfp_ref_encode(w, rows, cols, cols, br, bc, m_wide, rounding_wide, seed_wide, wide_mant_out, wide_exps_out);
    }
    if (rc == 0 && narrow_mant && narrow_exps)
        rc = hbfp_ref_encode(w, rows, cols, cols, br, bc, m_narrow, rounding_narrow, seed_narrow, narrow_mant, narrow_exps);
    if (!w_new) free(w);
    return rc;
}
