/*
 * hbfp.h - C ABI of the MI355X (gfx950) block-floating-point library.
 *
 * The library implements the dot-product path of Hybrid Block Floating Point
 * (arXiv 1804.01526): FP32 tensors are converted to BFP right before a dot
 * product, the product runs on fixed-point mantissas, and the result returns to
 * FP32 (Sec. 4.1).  Everything else in the paper stays in floating point and is
 * not part of this library.
 *
 * Conventions
 *   - Every pointer named `src`, `dst`, `C`, `P`, `workspace`, and the `mant`
 *     and `exps` members of an hbfp_tensor are DEVICE pointers.  Format and
 *     tensor descriptors are HOST structs, read during the call.
 *   - The caller owns every buffer.  No entry point allocates or frees device
 *     memory; sizes come from the pure host functions (hbfp_plan, hbfp_*_workspace).
 *   - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls are
 *     asynchronous with respect to the host and ordered on that stream.
 *   - Every function returns an int status: HBFP_OK or a negative HBFP_ERR_*.
 *     Arguments are validated before any work is queued; on an error nothing
 *     has been launched (HBFP_ERR_LAUNCH excepted: the runtime refused a launch).
 *   - Results are deterministic: the same inputs and seed give the same bytes.
 *
 * The BFP tensor (Eq. (1), Sec. 4:  a_i = m_i * 2^e)
 *   - Mantissas are two's complement integers of `mant_bits` bits, the sign
 *     included, in the symmetric range +-(2^(mant_bits-1) - 1).
 *   - A block of elements shares one exponent, stored as one byte Eb in 1..255:
 *     the IEEE-754 biased exponent of the block's largest magnitude (the exponent
 *     rule of Sec. 4.1 and Sec. 5.3), raised by one when rounding
 *     that largest value would reach 2^(mant_bits-1).  One mantissa unit is worth
 *     2^(Eb - 125 - mant_bits); an all-zero or subnormal-only block has Eb = 1.
 *   - Rounding acts on the magnitude, then the sign is applied: round to
 *     nearest even, or stochastic rounding (Sec. 5.3) with the counter hash below.
 *   - Inputs must be finite.  NaN/Inf are not trapped; their blocks hold
 *     unspecified mantissas.
 *
 * Stored ("operand") layout.  A tensor is always encoded FOR a dot product, i.e.
 * with a contraction axis (the k of Eq. (2)).  The other axis indexes operand
 * rows.  With R operand rows and K contraction elements:
 *     kblock      elements of one stored block along k: the exponent block, or a shorter
 *                 stretch of it when hbfp_format.k_slot is used (kshare consecutive stored
 *                 blocks then repeat one exponent)
 *     kblock_pad  stored length of a block: 32 if kblock <= 32, 64 if <= 64,
 *                 otherwise kblock rounded up to a multiple of 128
 *     nblk        ceil(K / kblock)           (the last block may be short)
 *     kpad        nblk * kblock_pad rounded up to a multiple of 128
 *     mant        [R][kpad]  int8 (mant_bits <= 8) or int16; element k of block b
 *                 of row r sits at r*kpad + b*kblock_pad + k; all padding is 0
 *     exp_ld      nblk rounded up to a multiple of 4
 *     exps        [R][exp_ld] uint8; exps[r][b] is the exponent byte of the block
 *                 holding (r, b).  With 2-D blocks several rows repeat the same
 *                 byte.  Bytes b >= nblk are written as 1.
 * k is contiguous for both operands of a product, whatever the source layout,
 * so one GEMM kernel serves the forward, data-gradient and weight-gradient shapes.
 *
 * Stochastic rounding (Sec. 5.3 uses a xorshift generator).  Here the random word
 * of an element is a counter hash, so that any launch geometry draws the same
 * bits.  With idx = r*cols + c the element's logical position in the source
 * matrix (independent of ld), lo/hi the 32-bit halves of idx and s0/s1 those of
 * the seed, all arithmetic modulo 2^32:
 *     x = lo ^ s0;  x ^= x << 13;  x ^= x >> 17;  x ^= x << 5;   x += hi ^ s1;
 *     x ^= x >> 16; x *= 0x85EBCA6B; x ^= x >> 13; x *= 0xC2B2AE35; x ^= x >> 16;
 * An element whose significand must be shifted right by sh bits to align with
 * the block exponent adds the top sh bits of x below the kept bits before
 * truncating (sh > 32: the element becomes 0).
 */
#ifndef HBFP_H
#define HBFP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    HBFP_OK = 0,
    HBFP_ERR_ARG = -1,       /* null pointer, non-positive size, ld too small, bad flag */
    HBFP_ERR_FORMAT = -2,    /* unsupported mantissa width, block shape or rounding mode */
    HBFP_ERR_LAYOUT = -3,    /* descriptor does not match hbfp_plan, or operands do not fit each other */
    HBFP_ERR_RANGE = -4,     /* a block dot product could overflow the int32 accumulator */
    HBFP_ERR_LAUNCH = -5,    /* the HIP runtime reported an error (no device, bad launch) */
    HBFP_ERR_WORKSPACE = -6  /* workspace missing, too small or misaligned (256 bytes) */
};

enum { HBFP_RNE = 0, HBFP_STOCHASTIC = 1 };

/* How a source matrix [rows][cols] is cut into exponent blocks. */
typedef struct hbfp_format {
    int32_t mant_bits;   /* 2..16, sign included */
    int32_t rounding;    /* HBFP_RNE or HBFP_STOCHASTIC */
    int64_t block_rows;  /* block extent along the source rows; 0 = all rows */
    int64_t block_cols;  /* block extent along the source columns; 0 = all columns */
    uint64_t seed;       /* stochastic rounding only */
    int64_t k_slot;      /* 0, or the length of the stored blocks along the contraction axis when the exponent
                            block is longer: the operand is then stored (and scaled in the product) in blocks
                            of k_slot elements that repeat the exponent of the block_rows x block_cols block
                            they lie in.  The block extent along the contraction axis must be a multiple of
                            k_slot or the whole extent.  This is how an operand with one exponent per row
                            (activations with one exponent per training input, Sec. 5.1) meets an operand cut
                            into tiles (24 x 24 weight tiles): both are stored in blocks of 24. */
} hbfp_format;

/* An encoded operand.  hbfp_plan fills everything but the two pointers. */
typedef struct hbfp_tensor {
    void *mant;            /* device, mant_bytes, 16-byte aligned */
    uint8_t *exps;         /* device, exp_bytes, 4-byte aligned */
    int64_t rows;          /* R: operand rows (extent of the non-contraction axis) */
    int64_t kdim;          /* K: contraction extent */
    int64_t kblock;        /* exponent block length along k */
    int64_t kblock_pad;
    int64_t nblk;
    int64_t kpad;
    int64_t exp_ld;
    int64_t rblock;        /* operand rows that share one exponent (block extent across k) */
    int64_t kshare;        /* consecutive k blocks that repeat one exponent (1 unless hbfp_format.k_slot is used) */
    int64_t src_rows, src_cols; /* shape of the source matrix */
    int32_t contract_axis; /* 0: k runs down the source rows, 1: along the source columns */
    int32_t mant_bits;
    int32_t rounding;
    int32_t hints;         /* HBFP_HINT_*: set by the caller after hbfp_plan (which leaves 0); results never depend on it */
    uint64_t seed;
    uint64_t mant_bytes, exp_bytes;
} hbfp_tensor;
/* The values of this operand are heavy-tailed (gradients often are).  It matters for mantissas of at most 5 bits, whose
 * packed form (limb planes with group exponents) will then usually be marked (see hbfp_pack): products on packed operands
 * prepare the faster of the int8 kernels as their stand-by.  That costs about 2 us per product when the stand-by turns out
 * not to be needed and saves a quarter of the time of a product when it is.  Mantissas of 6..9 bits are packed as bf16
 * numbers, which heavy tails do not mark; the hint changes nothing for them. */
#define HBFP_HINT_HEAVY_TAILS 1

/* Library version and a short text for a status code (host, never NULL). */
int hbfp_version(void);
const char *hbfp_status_string(int status);

/*
 * hbfp_plan (host only): geometry and byte sizes of the operand that encoding a
 * source matrix [rows][cols] along `contract_axis` produces (layout above).
 * Sets out->mant = out->exps = NULL.
 * Errors: HBFP_ERR_ARG (null, sizes <= 0, axis not 0/1), HBFP_ERR_FORMAT
 * (mant_bits outside 2..16, negative block extents, unknown rounding).
 */
int hbfp_plan(const hbfp_format *fmt, int64_t rows, int64_t cols, int contract_axis, hbfp_tensor *out);

/*
 * hbfp_sizes (host only): the three numbers a caller needs to allocate an operand, without the descriptor:
 * bytes of mantissas, bytes of exponents and the stored contraction length kpad of the operand that encoding a source
 * matrix [rows][cols] along contract_axis produces.  A thin wrapper over hbfp_plan (same errors); any of the three
 * output pointers may be NULL.
 */
int hbfp_sizes(const hbfp_format *fmt, int64_t rows, int64_t cols, int contract_axis, size_t *mant_bytes, size_t *exp_bytes,
               int64_t *kpad);

/*
 * hbfp_encode_workspace (host only): bytes of scratch hbfp_encode needs for this
 * plan: 0 for blocks of at most 64 elements along k and at most 64 across it (128 and
 * 32 when k is the contiguous source axis); otherwise (long blocks, one exponent per row
 * or column, large tiles, one exponent for the matrix) the conversion takes two passes
 * and needs 4 bytes per exponent block, rounded up to 256.
 */
int hbfp_encode_workspace(const hbfp_tensor *plan, size_t *bytes);

/*
 * hbfp_encode: FP32 -> BFP (the conversion rule of Sec. 4.1, applied to the inputs
 * of every dot product; Sec. 5.3, FP-to-BFP unit: the block's largest exponent is
 * found and the mantissas are aligned to it).
 *   src   device FP32 source matrix, element (r, c) at src[r*ld + c], ld >= cols
 *   out   descriptor from hbfp_plan for the same (fmt, rows, cols, contract_axis),
 *         with mant/exps set by the caller; fully overwritten, padding included
 *   workspace  device scratch of hbfp_encode_workspace bytes (may be NULL when 0)
 * Errors: HBFP_ERR_ARG, HBFP_ERR_FORMAT, HBFP_ERR_LAYOUT (descriptor differs from the
 * plan), HBFP_ERR_WORKSPACE, HBFP_ERR_LAUNCH.
 */
int hbfp_encode(const float *src, int64_t rows, int64_t cols, int64_t ld, int contract_axis,
                const hbfp_format *fmt, hbfp_tensor *out, void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_encode_static: hbfp_encode for callers that cannot allocate device memory or pass scratch of their own (code
 * under HIP graph capture, serving loops with a fixed memory plan, harnesses that forbid hipMalloc).  Same arguments,
 * result and errors as hbfp_encode, without the workspace: the table of block maxima that the two-pass conversions
 * need (hbfp_encode_workspace bytes: 4 per exponent block; one exponent per row or column, per image, per matrix,
 * long blocks, large tiles) lives in a device array inside the library of hbfp_encode_static_limit() = 1 MiB bytes,
 * i.e. up to 262144 exponent blocks, which every GPU the library runs on holds until the process ends.
 * HBFP_ERR_WORKSPACE if the format needs more.  The call allocates nothing and frees nothing.  The first call on a
 * device looks the array's address up (make that call outside a graph capture).  All calls on one GPU share the
 * array: calls that overlap on one GPU (different streams) race; calls ordered on one stream do not, because each
 * call clears the entries it uses before using them.  Formats that need no table (hbfp_encode_workspace = 0) do
 * not touch the array.
 */
size_t hbfp_encode_static_limit(void);
int hbfp_encode_static(const float *src, int64_t rows, int64_t cols, int64_t ld, int contract_axis,
                       const hbfp_format *fmt, hbfp_tensor *out, void *stream);

/*
 * hbfp_decode: BFP -> FP32, Eq. (1): dst[r*ld + c] = mant * 2^(Eb - 125 - mant_bits),
 * written in the SOURCE orientation [src_rows][src_cols] of the tensor.  Exact,
 * subnormal results included.
 */
int hbfp_decode(const hbfp_tensor *t, float *dst, int64_t ld, void *stream);

/*
 * hbfp_encode_im2col: the activation operand of a convolution executed as a matrix product (Sec. 5.1: convolutions
 * and their backward passes get the treatment of matrix multiplications), converted straight from the image
 * tensor, so the lowered FP32 matrix (R*S times the size of the input) never exists in memory.
 *   x     device FP32 tensor [n][h][w][c] (channels innermost), 16-byte aligned
 *   conv  geometry: filter r x s, zero padding pad_h / pad_w on each side, strides; output size
 *         ho = (h + 2 pad_h - r) / stride_h + 1, wo likewise
 *   out   descriptor from hbfp_plan(fmt, rows = n*ho*wo, cols = r*s*c, contract_axis) with mant/exps set.  The
 *         lowered matrix has one row per output position (img, oy, ox) holding the values under the filter
 *         window, column (fr * s + fs) * c + ch, zero where the window leaves the image.  contract_axis 1 gives
 *         the operand of the forward product (k runs along the window), contract_axis 0 that of the weight
 *         gradient (operand rows = window entries, k runs over the output positions).  The result is bit for
 *         bit what hbfp_encode gives for the materialised lowered matrix (same logical indices for stochastic
 *         rounding).
 * Supported formats: 1-D blocks along k; contract_axis 1: at most 128 elements, block length, c and c_block
 * multiples of 8; contract_axis 0: at most 64 elements (HBFP_ERR_FORMAT otherwise).
 * One exponent per training input (Sec. 5.1: the x tensor gets one exponent per training input), contract_axis 1:
 * a format with block_rows = ho*wo (the rows of one image), block_cols = 0 and k_slot = the stored block length
 * (a multiple of 8, at most 128); ho*wo must exceed 1 (with one output position per image the format reads as one
 * exponent per lowered row, which this entry point does not produce: HBFP_ERR_FORMAT).  The exponent is that of the
 * largest value of the whole image x[img] (also of
 * pixels no window reaches when the stride exceeds the filter), each value is converted as if the image had been
 * converted once and lowered afterwards (stochastic rounding draws by the index in x, so a pixel gets the same
 * mantissa in every window), and `workspace` must hold hbfp_encode_im2col_workspace bytes (4 per image, rounded up to 256;
 * HBFP_ERR_WORKSPACE); the other formats need no workspace (NULL, 0).  Errors as hbfp_encode; HBFP_ERR_LAYOUT if the descriptor's shape is not the
 * convolution's.
 */
typedef struct hbfp_conv2d {
    int64_t n, h, w, c;
    int32_t r, s;
    int32_t pad_h, pad_w;
    int32_t stride_h, stride_w;
    int32_t c_block;   /* 0 (or >= c): window entries in the order k = (fr * s + fs) * c + ch.  Otherwise the channels are
                          cut into blocks of c_block (the last may be shorter) and k runs block by block:
                          k = (cb * r * s + fr * s + fs) * c_block + ci for channel ch = cb * c_block + ci (with the last
                          block's width in its own range).  The r * s * c_block entries of a channel block are then
                          consecutive, so a filter matrix [k][filters] in the same order, cut into tiles of
                          (r * s * c_block) x (filter block) with k_slot = c_block, shares one exponent over a channel
                          block, a filter block and the whole window: the tiling of the two outer filter dimensions
                          of Sec. 5.1. */
    int32_t reserved;
} hbfp_conv2d;
int hbfp_encode_im2col_workspace(const hbfp_conv2d *conv, const hbfp_tensor *plan, size_t *bytes);   /* host only */
int hbfp_encode_im2col(const float *x, const hbfp_conv2d *conv, const hbfp_tensor *out, void *workspace, size_t ws_bytes,
                       void *stream);

/*
 * hbfp_gemm_conv2d: a convolution executed as a BFP matrix product (Sec. 5.1) whose activation operand is never
 * lowered at all: the image is converted ONCE, as the matrix [n*h*w pixels][c channels] with blocks along the channels
 * (hbfp_encode, contraction axis 1), and the product kernel gathers every filter tap from it while it stages its
 * operand (one address per operand row and stage; taps outside the image read zeros).
 *     Y[(img, oy, ox)][f] = beta * Y + sum over (fr, fs, ch) of x[img][oy*stride_h - pad_h + fr][ox*stride_w - pad_w + fs][ch]
 *                                                             * w[(fr * s + fs) * c + ch][f]
 * with both factors as their BFP values and the sum taken as Eq. (2) takes it (integer sums over the channels of one
 * stored block of one tap, scaled by the two block exponents, accumulated in FP32).  Because a block of the lowered
 * matrix is a block of the image, the result equals hbfp_gemm_select(HBFP_KERNEL_INT8) on hbfp_encode_im2col's operand bit for bit (with
 * round to nearest; stochastic rounding draws by position in the image here, by position in the lowered matrix there).
 * The data gradient of a stride-1 convolution is the same call on the output gradient (as the image, with padding
 * r - 1 - pad) and the mirrored filter with its channel axes exchanged; hbfp_gemm_conv2d_dgrad does that for any stride.
 *   image    encoded [n*h*w][c], contraction axis 1, stored blocks of B <= 32 channels (block_cols = B, or k_slot = B
 *            with exponents shared more widely: block_rows = h*w and block_cols = 0 is one exponent per training input,
 *            Sec. 5.1), c a multiple of B, <= 8 bits
 *   conv     geometry; c_block 0: window entries in the order (fr, fs, ch); c_block = B: channel block by channel
 *            block (see hbfp_conv2d), the order in which a filter tile of (r*s*B) x (filter block) with k_slot = B
 *            shares one exponent over B channels, a block of filters and the whole window (Sec. 5.1)
 *   filters  encoded filter matrix [r*s*c][filters] in the same order, contraction axis 0, stored blocks of B down its
 *            rows (block_rows = B or k_slot = B; any sharing of exponents), <= 8 bits
 *   Y        device FP32 [n*ho*wo][ldy], ldy >= filters; beta 0 or 1
 *   workspace  hbfp_gemm_conv2d_workspace bytes (scale words of both operands, split-k slices), 256-byte aligned
 * Where both operands repeat their exponents over the r*s taps of a channel block (c_block = B, the image with one
 * exponent per training input, filter tiles over the whole window), the integer sums of such a run of blocks are added
 * up before they are scaled (as Sec. 4 has it: one FP operation per tile, not per block; at most as many blocks as keep
 * the sum below 2^22): fewer FP32 roundings than block by block, so that case equals the product on the lowered operand
 * to rounding, not bit for bit.
 * With B = 32, c a multiple of 64 and c_block = 0 a stage of the product is 64 channels of one tap; otherwise it is two
 * consecutive stored blocks, in general of two different pixels (5 % slower at equal sizes).  Blocks shorter than 32 are
 * stored as 32 and cost as much.  A channel count that is no multiple of B is handled by the caller: zero channels
 * appended to the image tensor and zero rows to the filter change neither exponents nor sums.
 * Errors: HBFP_ERR_ARG, HBFP_ERR_LAYOUT (operands do not match the geometry), HBFP_ERR_FORMAT (stored blocks longer
 * than 32 or different in the two operands, c no multiple of them, c_block neither 0 nor the block length, mantissas
 * wider than 8 bits), HBFP_ERR_WORKSPACE, HBFP_ERR_LAUNCH.
 */
int hbfp_gemm_conv2d_workspace(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, size_t *bytes);
int hbfp_gemm_conv2d(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, float *Y, int64_t ldy, float beta,
                     void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_gemm_conv2d_bfp: hbfp_gemm_conv2d whose result arrives as an encoded operand (Sec. 5.3: an FP-to-BFP unit converts
 * what the MatMul unit produces for the next product; an activation unit sits in between): out = encode(relu ? max(Y, 0) : Y)
 * with Y the convolution of hbfp_gemm_conv2d, as hbfp_gemm_bfp does it for a matrix product.  With `out` planned as the
 * next layer's image - [n*ho*wo][filters], contraction axis 1, blocks of 32 filters, at most 8 bits, round to nearest or
 * stochastic (drawn by the position in Y) - and a product that is not split along k, the product kernel converts its own
 * accumulators (the tile passes through LDS to bring the 32 filters of a block side by side): the FP32 result, four
 * times the bytes, is neither written nor read back, and the next layer needs no conversion call.  Any other output
 * format: the FP32 product in the workspace, then the conversion kernels.  Either way the bytes are those of
 * hbfp_encode on the FP32 result of hbfp_gemm_conv2d.
 *   out    planned and allocated by the caller (hbfp_plan: rows n*ho*wo, columns filters)
 *   relu   0 or 1
 *   workspace  hbfp_gemm_conv2d_bfp_workspace bytes, 256-byte aligned
 * Errors: as hbfp_gemm_conv2d; HBFP_ERR_LAYOUT if `out` has another shape.
 */
int hbfp_gemm_conv2d_bfp_workspace(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, const hbfp_tensor *out,
                                   size_t *bytes);
int hbfp_gemm_conv2d_bfp(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, const hbfp_tensor *out, int relu,
                         void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_gemm_conv2d_dgrad: the data gradient of a convolution of any stride, executed like the forward pass (Sec. 5.1
 * treats the backward pass of a convolution as it treats the forward pass: as a BFP matrix product).  With
 *     y[img][oy][ox][f] = sum over (fr, fs, ch) of x[img][oy*stride_h - pad_h + fr][ox*stride_w - pad_w + fs][ch] * w[fr][fs][ch][f]
 * the gradient is the adjoint sum
 *     dX[(img, iy, ix)][ch] = beta * dX + sum over (fr, fs, f) and the (oy, ox) with oy*stride_h - pad_h + fr = iy,
 *                             ox*stride_w - pad_w + fs = ix of dy[img][oy][ox][f] * w[fr][fs][ch][f],
 * which is a stride-1 convolution, with padding (r - 1 - pad_h, s - 1 - pad_w), of dy with stride - 1 rows and columns of
 * zeros put between its pixels, against the filter mirrored in both window axes with its channel axes exchanged.  The
 * zeros are never stored: the product kernel gathers each tap from dy as converted once ([n*ho*wo][filters], blocks along
 * the filters) and reads a page of zeros for the positions in between; all h x w input positions are computed, also those
 * that only part of a window reaches.  Both factors count as their BFP values and the sum is taken as Eq. (2) takes it.
 * With stride 1 this is hbfp_gemm_conv2d on dy with that padding.
 *   dy       encoded [n*ho*wo][filters] (ho, wo: the output extents of conv), contraction axis 1, in any of the formats
 *            hbfp_gemm_conv2d takes for its image, with the filters in the place of the channels: stored blocks of
 *            B <= 32 filters, filters a multiple of B, any sharing of exponents beyond (one per training input), <= 8 bits
 *   conv     geometry of the FORWARD convolution (n, h, w, c describe x).  c_block 0: k = (mirrored tap, filter);
 *            c_block = B: filter block by filter block, k = (filter block, mirrored tap, filter in the block)
 *   filters  encoded matrix [r*s*filters][c] in that order - with c_block 0, row ((r-1-fr) * s + (s-1-fs)) * filters + f,
 *            column ch = w[fr][fs][ch][f] -, contraction axis 0, stored blocks of B down its rows, <= 8 bits
 *   dX       device FP32 [n*h*w][ldx], ldx >= c; beta 0 or 1
 *   workspace  hbfp_gemm_conv2d_dgrad_workspace bytes, 256-byte aligned
 * With blocks of 32 filters, a multiple of 64 filters and c_block 0, where the window is at least as large as the stride
 * in both directions (and stride_h * stride_w <= 16), the zeros are not multiplied either: the input positions fall
 * into stride_h * stride_w phases (iy mod stride_h, ix mod stride_w), a phase meets only every stride-th filter tap and reads dy without gaps, and one launch walks all phases, each storing
 * to the rows of its input positions.  The taps that do contribute are accumulated in the same order both ways, so the
 * result is bit for bit that of hbfp_gemm_conv2d on a dy whose zeros are stored.  Otherwise (a window smaller than the
 * stride, the other formats) every tap of the spread-out dy is multiplied, zeros included: stride_h * stride_w times the
 * work the sum needs.
 * Errors: as hbfp_gemm_conv2d; HBFP_ERR_ARG also for extents from 2^21 on.
 */
int hbfp_gemm_conv2d_dgrad_workspace(const hbfp_tensor *dy, const hbfp_conv2d *conv, const hbfp_tensor *filters, size_t *bytes);
int hbfp_gemm_conv2d_dgrad(const hbfp_tensor *dy, const hbfp_conv2d *conv, const hbfp_tensor *filters, float *dX, int64_t ldx, float beta,
                           void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_gemm: the BFP matrix product, Eq. (2) with per-block FP accumulation
 * (Sec. 4, tiled matrix multiplication):
 *     C[i][j] = beta*C[i][j] + sum_b 2^(eA[i][b] + eB[j][b]) * sum_{k in b} mA[i][k]*mB[j][k]
 * The inner sum is exact integer arithmetic (int8 matrix cores with int32
 * accumulators, or exact limb products in the block-scaled matrix instruction, see
 * hbfp_gemm_select); the outer sum is FP32.  A has M = A->rows operand rows, B has
 * N = B->rows; both must have the same kdim, kblock and mantissa class (both
 * <= 8 bits, or both 9..12 bits, which run as two int8 limbs per mantissa).
 *   C     device FP32 [M][ldc], ldc >= N
 *   beta  0 (overwrite; C is not read) or 1 (accumulate)
 *   workspace  hbfp_gemm_workspace bytes: scale words of both operands (4 bytes per row and
 *              block), one FP32 slice of C per split when the shape is split along k (few
 *              output tiles, long k), two int8 limb planes per operand for mantissas wider
 *              than 8 bits, and the limb planes of both operands when the block-scaled
 *              kernel is chosen
 * Domain: block exponent bytes up to 254 (magnitudes below 2^127).
 * Errors: HBFP_ERR_ARG, HBFP_ERR_LAYOUT (kdim/kblock mismatch), HBFP_ERR_FORMAT
 * (mantissa classes differ or exceed 12 bits), HBFP_ERR_RANGE (kblock * max|mA| *
 * max|mB| >= 2^31), HBFP_ERR_WORKSPACE, HBFP_ERR_LAUNCH.
 */
int hbfp_gemm_workspace(const hbfp_tensor *A, const hbfp_tensor *B, size_t *bytes);
int hbfp_gemm(const hbfp_tensor *A, const hbfp_tensor *B, float *C, int64_t ldc, float beta,
              void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_gemm_select: hbfp_gemm with the kernel family named by the caller.  The library has two ways to
 * evaluate Eq. (2) with its per-block FP accumulation (Sec. 4):
 *   HBFP_KERNEL_INT8    int8 matrix instructions, int32 block sums, one FP32 scale-and-accumulate per
 *                       output and block on the vector unit;
 *   HBFP_KERNEL_SCALED  the block-scaled matrix instruction: mantissas cut into sign-magnitude limbs of
 *                       4 bits (one limb up to 5-bit mantissas, two up to 9, three up to 12), every
 *                       32-element group multiplied exactly and scaled by its two exponent bytes inside
 *                       the instruction, FP32 accumulation in the matrix core.  Needs block exponents
 *                       in 3..253 for 8-bit mantissas (7..253 for 12-bit); when an operand holds a
 *                       non-zero block outside that range the call computes the product with the int8
 *                       kernels instead, inside the same call and without host synchronisation;
 *   HBFP_KERNEL_INT8_WIDE  the member of the int8 family for one exponent per operand row (a single block
 *                       along k, the basic scheme of Sec. 4) and mantissas of at most 8 bits: 256 x 256 tiles,
 *                       one uninterrupted chain of matrix instructions, exponents applied when C is stored.
 *                       HBFP_KERNEL_INT8 and HBFP_KERNEL_AUTO take it by themselves when at least 128 such
 *                       tiles are at least 75 % full; naming it runs it on any shape (HBFP_ERR_FORMAT if the
 *                       operands have more than one block or wider mantissas);
 *   HBFP_KERNEL_FP16    9..12-bit mantissas as FP16 numbers (an 11-bit magnitude is an FP16 significand): one FP16 matrix
 *                       instruction multiplies them exactly and sums in FP32, then the per-block scale-and-accumulate runs
 *                       on the vector unit as in the int8 family.  A block sum beyond 2^24 is rounded to nearest once per
 *                       16 products of the chain instead of once per block; blocks of 32, 64 or a multiple of 128
 *                       (HBFP_ERR_FORMAT otherwise, and for 8-bit operands);
 *   HBFP_KERNEL_BF16    6..9-bit mantissas as bf16 numbers: such a mantissa times its block's power of two has at most
 *                       8 significant bits and the exponent range of the exponent byte, so Eq. (1) is exact in bf16; one
 *                       bf16 matrix instruction per 16 k multiplies the significands, adds the exponents and accumulates in
 *                       FP32, and nothing is scaled per block (any block length, any spread of exponents; a non-zero block
 *                       with an exponent byte above 253 is computed with plain arithmetic inside the same kernel).  The
 *                       operands are packed into bf16 planes in the workspace first.  HBFP_ERR_FORMAT for other widths;
 *   HBFP_KERNEL_FP16_PLANES  9..12-bit mantissas as FP16 numbers on the kernel of HBFP_KERNEL_BF16: FP16 has the 11-bit
 *                       significand but not the exponent range, so every operand row is taken relative to the largest
 *                       exponent byte Eref of its blocks: an element becomes mant * 2^(E - Eref + 4), exact in FP16
 *                       (subnormals included) when its block lies at most 28 binades below the row's largest, the FP16
 *                       matrix instruction multiplies and accumulates in FP32 with nothing scaled per block, and the
 *                       factors 2^(Eref ...) of the row of A and the row of B are applied once, at the store.  A non-zero
 *                       block further down is computed with plain arithmetic inside the same kernel, as for BF16.  The
 *                       operands are packed in the workspace first.  HBFP_ERR_FORMAT for other widths;
 *   HBFP_KERNEL_AUTO    what hbfp_gemm does, in this order: BF16 when both operands have 6..9-bit mantissas and the shape is
 *                       one where 256 x 256 tiles pay (at least 144 output tiles, a stored contraction length of at least
 *                       2048, or 1024 from 512 tiles on, blocks of at most 32 elements); FP16_PLANES when both have 9..12-bit
 *                       mantissas and the shape is such a one (any block length); FP16 when both operands have
 *                       9..12-bit mantissas in blocks it takes (measured ahead of the int8 and block-scaled families from
 *                       2048^3 to 8192^3); SCALED for the same shapes as BF16 when an operand has at most 5 bits; else INT8.
 * All satisfy the same bound against the FP64 product of the decoded operands.
 * Arguments, domain and errors as hbfp_gemm, plus HBFP_ERR_ARG for an unknown kernel; the workspace
 * size depends on the kernel: hbfp_gemm_select_workspace.
 */
#define HBFP_KERNEL_AUTO 0
#define HBFP_KERNEL_INT8 1
#define HBFP_KERNEL_SCALED 2
#define HBFP_KERNEL_INT8_WIDE 3
#define HBFP_KERNEL_FP16 4
#define HBFP_KERNEL_BF16 5
#define HBFP_KERNEL_FP16_PLANES 6
int hbfp_gemm_select_workspace(const hbfp_tensor *A, const hbfp_tensor *B, int kernel, size_t *bytes);
int hbfp_gemm_select(const hbfp_tensor *A, const hbfp_tensor *B, float *C, int64_t ldc, float beta, int kernel,
                     void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_gemm_batch: up to HBFP_BATCH_MAX independent products C[i] (+)= A[i] . B[i]^T in one call (the data-gradient
 * and weight-gradient products of a layer, Sec. 5.1; the products of several layers or micro-batches).  Every
 * product is what hbfp_gemm_select computes for it (bit for bit with HBFP_KERNEL_BF16, HBFP_KERNEL_SCALED and
 * HBFP_KERNEL_INT8; with HBFP_KERNEL_AUTO within the same bound, because the choice of kernel may differ, see below).
 * Products whose mantissa classes agree can share one launch of the bf16 kernel (6..9-bit mantissas) or of the
 * block-scaled kernel (workgroup ranges of one grid), so that products too small to fill the chip alone fill it
 * together.  They do with HBFP_KERNEL_BF16 and HBFP_KERNEL_SCALED, and with HBFP_KERNEL_AUTO when every product would
 * take that kernel anyway or when the group has at least 256 output tiles of 256 x 256, contraction lengths of at
 * least 1024 within a factor of two of each other, and a format these kernels are ahead in; otherwise the products
 * run one after the other, each as hbfp_gemm_select runs it.
 *   A, B, C, ldc   host arrays of n descriptors / device pointers / leading dimensions
 *   kernel         HBFP_KERNEL_* as for hbfp_gemm_select, applied to every product
 *   workspace      hbfp_gemm_batch_workspace bytes (the sum of the products' own workspaces)
 * Errors: as hbfp_gemm_select for the first product that fails a check (nothing has been launched then).
 */
#define HBFP_BATCH_MAX 4
int hbfp_gemm_batch_workspace(int n, const hbfp_tensor *const *A, const hbfp_tensor *const *B, int kernel, size_t *bytes);
int hbfp_gemm_batch(int n, const hbfp_tensor *const *A, const hbfp_tensor *const *B, float *const *C, const int64_t *ldc,
                    float beta, int kernel, void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_gemm_bfp: the product A . B^T delivered as an encoded operand instead of FP32: out = encode(relu?(A . B^T)),
 * the FP -> BFP conversion of Sec. 4.1 (with the rounding of Sec. 5.3 that `out` names) applied where the product
 * is produced, so that the next product's operand never makes the trip through an FP32 matrix in memory.
 *   out      planned with hbfp_plan for a source matrix of A->rows x B->rows (either contraction axis, any format);
 *            out->mant / out->exps device, written; stochastic rounding draws by position in the product matrix
 *   relu     0 or 1: max(x, 0) on the FP32 values before the conversion (the one floating-point operation between two
 *            products that needs no other operand)
 *   kernel   HBFP_KERNEL_* as for hbfp_gemm_select
 * The result equals hbfp_gemm_select followed by hbfp_encode of its output, bit for bit.  When the bf16 or the block-scaled
 * kernel computes the product and out has k along the columns of the product in blocks of 32 or 64 (one exponent per block
 * and row), the kernel converts its accumulators itself; otherwise the FP32 product goes through the workspace.
 *   workspace  hbfp_gemm_bfp_workspace bytes (includes A->rows * B->rows floats), 256-byte aligned
 * Errors: as hbfp_gemm_select; HBFP_ERR_LAYOUT if out is not the plan of an A->rows x B->rows matrix.
 */
int hbfp_gemm_bfp_workspace(const hbfp_tensor *A, const hbfp_tensor *B, const hbfp_tensor *out, int kernel, size_t *bytes);
int hbfp_gemm_bfp(const hbfp_tensor *A, const hbfp_tensor *B, const hbfp_tensor *out, int relu, int kernel, void *workspace,
                  size_t ws_bytes, void *stream);

/*
 * hbfp_pack / hbfp_gemm_packed: the product in two steps, for operands that take part in many products (weights
 * between two optimizer steps: Sec. 5.1 converts them once per update).  hbfp_pack reorders an encoded operand
 * (mantissas of at most 12 bits) into the form the product kernels read.  The form depends on the operand's mantissa
 * width alone: 6..9 bits -> the bf16 values of its elements (Eq. (1), exact: at most 8 significant bits) in the
 * register order of the bf16 matrix instruction; 10..12 bits -> FP16 elements relative to the largest exponent byte of
 * their row, behind one scale word per row (HBFP_KERNEL_FP16_PLANES); at most 5 bits -> planes of 4-bit limbs with scale
 * bytes for the block-scaled matrix instruction.
 *   packed  device buffer of hbfp_pack_bytes bytes, 256-byte aligned, owned by the caller; its contents are
 *           opaque and stay valid until the operand is encoded again (then pack it again).  The first 256 bytes
 *           hold a mark that differs from pack to pack (it lets a pack signal "cannot be expressed" without
 *           anything having to be cleared first), so two packs of the same operand agree from byte 256 on, not
 *           before: the rule "same inputs, same bytes" holds for every result except this header.  Its first two
 *           32-bit words are equal exactly when the operand is marked: bf16 planes, a non-zero block with an exponent
 *           byte above 253 (values from 2^127 on); FP16 planes, a non-zero block more than 28 binades below the largest
 *           of its row; limb planes, an exponent byte outside the range of the scale bytes,
 *           or neighbouring blocks of a densely packed group more than 3 binades apart, as heavy-tailed values produce
 *           them.  A caller may read the words once the pack has completed.  Products on a marked operand are still
 *           computed inside the same call: from the stored operands by the bf16 / FP16 kernel itself (slowly; such values
 *           do not occur in training data), or by the older int8 kernel behind the block-scaled kernel (by the faster one
 *           if the operand carries HBFP_HINT_HEAVY_TAILS; hbfp_gemm_select with HBFP_KERNEL_INT8 on the stored operands
 *           is the fastest way to that product).
 *           The buffer is
 *           sized for blocks stored padded to 32; blocks of 8, 16 and 24 elements are packed without their
 *           padding and leave its tail unwritten.
 * hbfp_gemm_packed is hbfp_gemm_select on operands packed beforehand, with HBFP_KERNEL_BF16 when both are bf16 planes,
 * HBFP_KERNEL_FP16_PLANES when both are FP16 planes and HBFP_KERNEL_SCALED when both are limb planes (a pair of different
 * forms is multiplied by the int8 kernels from the stored operands): C and beta as in hbfp_gemm; A and B are the descriptors the buffers were packed from (their
 * mantissas and exponents are read only in the cases just named); workspace: hbfp_gemm_packed_workspace bytes (what the
 * int8 kernels need; nothing for a pair of bf16 planes or of FP16 planes).
 * Errors: HBFP_ERR_ARG (null or misaligned pointers, beta, ldc), HBFP_ERR_FORMAT (mantissas wider than 12 bits,
 * mixed classes), HBFP_ERR_LAYOUT, HBFP_ERR_RANGE as hbfp_gemm, HBFP_ERR_WORKSPACE (packed buffer or workspace too
 * small), HBFP_ERR_LAUNCH.
 */
int hbfp_pack_bytes(const hbfp_tensor *t, size_t *bytes);
int hbfp_pack(const hbfp_tensor *t, void *packed, size_t bytes, void *stream);
int hbfp_gemm_packed_workspace(const hbfp_tensor *A, const hbfp_tensor *B, size_t *bytes);
int hbfp_gemm_packed(const hbfp_tensor *A, const void *packed_a, const hbfp_tensor *B, const void *packed_b, float *C,
                     int64_t ldc, float beta, void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_gemm_packed_batch: hbfp_gemm_batch for operands packed beforehand: up to HBFP_BATCH_MAX independent products
 * (the data-gradient and weight-gradient products of a layer, Sec. 5.1, which both wait for the same gradient) in one
 * launch of the bf16 or the block-scaled kernel, so that the output tiles of one product are stored while the next product's
 * tiles are being multiplied.  Every product is bit for bit what hbfp_gemm_packed computes for it.
 *   A, packed_a, B, packed_b, C, ldc   host arrays of n entries, each as the arguments of hbfp_gemm_packed
 *   workspace                          hbfp_gemm_packed_batch_workspace bytes, 256-byte aligned
 * Errors: as hbfp_gemm_packed for the first product that fails a check (nothing has been launched then);
 * HBFP_ERR_FORMAT if the products do not all have the same packed forms and limb counts (mantissas of up to 5, 6..9 or
 * 10..12 bits, operand by operand).
 */
int hbfp_gemm_packed_batch_workspace(int n, const hbfp_tensor *const *A, const hbfp_tensor *const *B, size_t *bytes);
int hbfp_gemm_packed_batch(int n, const hbfp_tensor *const *A, const void *const *packed_a, const hbfp_tensor *const *B,
                           const void *const *packed_b, float *const *C, const int64_t *ldc, float beta, void *workspace,
                           size_t ws_bytes, void *stream);

/*
 * hbfp_gemm_partials: the fixed-point half of Eq. (2) alone, for checking:
 *     P[(i*N + j)*nblk + b] = sum_{k in block b} mA[i][k] * mB[j][k]     (int32, exact)
 * computed with the int8 matrix instruction (v_mfma_i32_32x32x32_i8) by the member of the int8 kernel family
 * that can write its int32 accumulators out: a kernel of its own, not one that hbfp_gemm launches (those keep
 * the block sums in registers and scale them at once).  The kernels hbfp_gemm runs are checked separately, on
 * inputs for which the FP32 result itself is exact.  Same operand rules; workspace: what hbfp_gemm_select_workspace
 * returns for HBFP_KERNEL_INT8.
 *   row0, rows / col0, cols (hbfp_gemm_partials_window): only the block sums of that window of the product are
 *   computed and written, P[((i - row0) * cols + (j - col0)) * nblk + b]: a few tiles of a product whose full
 *   dump would not fit in memory.  HBFP_ERR_ARG if the window is empty or leaves the product.
 */
int hbfp_gemm_partials(const hbfp_tensor *A, const hbfp_tensor *B, int32_t *P,
                       void *workspace, size_t ws_bytes, void *stream);
int hbfp_gemm_partials_window(const hbfp_tensor *A, const hbfp_tensor *B, int64_t row0, int64_t rows, int64_t col0, int64_t cols,
                              int32_t *P, void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_gemm_f32: convert-multiply-convert in one call (Sec. 4.1), BLAS style,
 * row-major:  C[M][N] = op(A) * op(B),  op(A) is M x K, op(B) is K x N.
 *   transA = 0: A is [M][lda];  1: A is [K][lda] (used as its transpose)
 *   transB = 0: B is [K][ldb];  1: B is [N][ldb]
 * (0,0) is the forward product, (0,1) the data gradient dX = dY * W^T,
 * (1,0) the weight gradient dW = X^T * dY.  fa/fb give each operand's exponent
 * blocks in the orientation the matrix is stored in; both must cut the
 * contraction axis into blocks of the same length.
 * workspace: hbfp_gemm_f32_workspace bytes (holds both encoded operands).
 */
int hbfp_gemm_f32_workspace(int transA, int transB, int64_t M, int64_t N, int64_t K,
                            const hbfp_format *fa, const hbfp_format *fb, size_t *bytes);
int hbfp_gemm_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
                  const float *A, int64_t lda, const float *B, int64_t ldb, float *C, int64_t ldc,
                  const hbfp_format *fa, const hbfp_format *fb,
                  void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_encode_multi: convert one FP32 matrix into up to three operand tensors in
 * one call.  A tensor that takes part in the forward and in a backward product is
 * contracted along a different axis in each (Sec. 5.1: the inputs of both passes are
 * converted), so it is needed in two layouts, possibly with different exponent
 * blocks (e.g. 1 x 24 along its rows and 24 x 1 down its columns).
 * src: device FP32 [src_rows][ld].  outs[i]: descriptors from hbfp_plan for the same
 * source shape with both device buffers set; each output is what hbfp_encode gives
 * for its own axis and format, bit for bit.  When all outputs are cut into the same
 * 2-D tiles of at most 32 x 32 (width a multiple of 4, equal rounding mode) the
 * source is read once; otherwise the outputs are produced one after the other (for
 * 1-D blocks the separate row and column kernels are faster than a shared read).
 * workspace: hbfp_encode_multi_workspace bytes (0 for the one-pass case).
 * Errors: HBFP_ERR_ARG (n outside 1..3, null/misaligned pointers, ld < src_cols),
 * HBFP_ERR_LAYOUT (different source shapes, inconsistent descriptor), HBFP_ERR_WORKSPACE.
 */
int hbfp_encode_multi_workspace(int n, const hbfp_tensor *const *outs, size_t *bytes);
int hbfp_encode_multi(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs,
                      void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_encode_packed: hbfp_encode_multi followed by hbfp_pack of its outputs, in one call: every output is converted
 * (Sec. 4.1) and, where packed[i] is not NULL, also written as the limb planes the block-scaled kernel reads, so that
 * hbfp_gemm_packed can multiply it without a pass in between.  A training step converts each of its three FP32
 * matrices (input, weights, output gradient) into the two operand layouts its products need (Sec. 5.1), and each
 * operand is multiplied once: this is the conversion for that case.
 *   outs, n, src, ld, workspace   as hbfp_encode_multi (workspace: hbfp_encode_packed_workspace bytes)
 *   packed[i]        NULL, or a device buffer of at least hbfp_pack_bytes(outs[i]) bytes, 256-byte aligned
 *   packed_bytes[i]  its size
 * Both results are what the two separate calls produce, bit for bit (the packed buffer from its byte 256 on; the
 * words before are a per-call mark).  When the outputs (at most two) have exponent blocks of 24 along k - 1 x 24 or
 * 24 x 1 blocks, or 24 x 24 tiles - with mantissas of at most 8 bits, equal limb counts and rounding, a source aligned
 * to 16 bytes with ld and the number of columns multiples of 4, and all are packed, one kernel reads the source once
 * and writes everything; any other combination runs the separate kernels one after the other.
 * Errors: as hbfp_encode_multi and hbfp_pack.
 */
int hbfp_encode_packed_workspace(int n, const hbfp_tensor *const *outs, size_t *bytes);
int hbfp_encode_packed(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs, void *const *packed,
                       const size_t *packed_bytes, void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_encode_packed_batch: hbfp_encode_packed of up to HBFP_BATCH_MAX independent sources in one call (the input and
 * the weights of a layer before its forward product, Sec. 5.1: neither conversion waits for the other).  Sources that
 * the one-kernel case of hbfp_encode_packed takes, with equal rounding and limb counts, share one launch, so that the
 * conversion of one source fills the compute units that the tail of another leaves idle; the remaining ones are
 * converted one after the other.  Every output is bit for bit what hbfp_encode_packed writes for it.
 *   jobs[j]     the arguments of hbfp_encode_packed for source j (host struct, host arrays; read during the call only)
 *   workspace   hbfp_encode_packed_batch_workspace bytes, 256-byte aligned
 * The outputs of different jobs must not overlap.
 * Errors: as hbfp_encode_packed for the first job that fails a check (nothing has been launched then); HBFP_ERR_ARG
 * if njobs is outside 1..HBFP_BATCH_MAX or a job's reserved field is not 0.
 */
typedef struct hbfp_encode_job {
    const float *src;                  /* device, FP32, row-major                     */
    int64_t ld;                        /* elements between its rows                    */
    int32_t n;                         /* outputs of this source                       */
    int32_t reserved;                  /* 0                                            */
    const hbfp_tensor *const *outs;    /* host array of n planned tensors              */
    void *const *packed;               /* host array of n device buffers (or NULL)     */
    const size_t *packed_bytes;        /* host array of their sizes                    */
} hbfp_encode_job;
int hbfp_encode_packed_batch_workspace(int njobs, const hbfp_encode_job *jobs, size_t *bytes);
int hbfp_encode_packed_batch(int njobs, const hbfp_encode_job *jobs, void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_weight_update: one step on weights kept in BFP with wide mantissas
 * (Sec. 4.2 "Wide weight storage"; Sec. 5.1, the optimizer shell: the update is
 * computed in FP32 and the result is converted to two BFP formats, the wide one
 * for later updates and the narrow one for the forward and backward products).
 *   w   = value of `wide` (Eq. (1); exact in FP32 for mantissas of up to 16 bits)
 *   w'  = fma(alpha, delta, w)            FP32, one rounding, element by element
 *   wide     <- encode(w') in wide's own format, layout and rounding (in place)
 *   narrow_a <- encode(w') in narrow_a's format and layout   (may be NULL)
 *   narrow_b <- encode(w') in narrow_b's format and layout   (may be NULL)
 * delta: device FP32 [src_rows][ld], the same orientation as the matrix the
 * tensors were planned for (e.g. alpha = -learning rate, delta = gradient).
 * wide, narrow_a, narrow_b: descriptors from hbfp_plan with both device buffers
 * set, all of the same source shape; any orientation, block shape, mantissa width
 * and rounding each (typically wide = 16 bits, narrow_a/narrow_b = the forward and
 * the transposed operand of 8 or 12 bits).  wide must hold an encoded tensor; the
 * narrow tensors are outputs only.  Every output is what hbfp_encode would give for
 * the FP32 matrix w', bit for bit.  The workspace contents afterwards are unspecified
 * (when all tensors share a 2-D tile shape of at most 32 x 32, as the paper's 24 x 24,
 * w' only ever exists in registers).
 * workspace: hbfp_weight_update_workspace bytes, 256-byte aligned.
 * Errors: HBFP_ERR_ARG (null/misaligned pointer, ld < src_cols), HBFP_ERR_LAYOUT
 * (descriptors of different source shapes or inconsistent), HBFP_ERR_WORKSPACE.
 */
int hbfp_weight_update_workspace(const hbfp_tensor *wide, const hbfp_tensor *narrow_a, const hbfp_tensor *narrow_b,
                                 size_t *bytes);
int hbfp_weight_update(const hbfp_tensor *wide, const float *delta, int64_t ld, float alpha,
                       const hbfp_tensor *narrow_a, const hbfp_tensor *narrow_b,
                       void *workspace, size_t ws_bytes, void *stream);

/*
 * hbfp_probe_matrix_rate: measurement aid, not part of the path.  Runs a register-only loop of one matrix instruction
 * (no memory traffic inside the loop) on every compute unit, so that a caller can time what the matrix core sustains
 * for given operand bits: the chip lowers its clock under its power limit, and how far depends on the bits.
 *   instruction  0: v_mfma_i32_32x32x32_i8;  1: v_mfma_scale_f32_32x32x64_f8f6f4 with FP6 (E2M3) operands;
 *                2: v_mfma_f32_32x32x16_bf16 (four registers per operand: every half word a finite bf16 number)
 *   words        device, 64 x 64 ints: register r of lane l at words[r * 64 + l]; registers 0..31 feed the first
 *                operands of the 4 x 4 independent chains of a wave, 32..63 the second operands
 *   workgroups   workgroups of 4 waves (8 .. 65536); iters: loop trips, 16 matrix instructions per wave each
 *   sink         device, workgroups * 256 floats (written, so that the loop is not removed)
 *   clocks       device, 2 x int64: shader cycles and 100 MHz wall-clock ticks of the loop of workgroup 7
 * One trip is 16 instructions of 2 * 32 * 32 * 32 (int8), 2 * 32 * 32 * 64 (FP6) or 2 * 32 * 32 * 16 (bf16) operations per wave.
 * Errors: HBFP_ERR_ARG, HBFP_ERR_LAUNCH.
 */
int hbfp_probe_matrix_rate(int instruction, const int *words, int workgroups, int iters, float *sink, long long *clocks,
                           void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HBFP_H */
