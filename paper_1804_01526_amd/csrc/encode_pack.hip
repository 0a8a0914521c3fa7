// FP32 -> BFP conversion that also writes the packed form that the product kernels read (Sec. 4.1: operands are
// converted right before every dot product; Sec. 5.1: forward and backward products both take converted inputs, so an
// activation or weight matrix is needed in two operand layouts).  One read of the FP32 matrix produces, for up to two
// outputs with exponent blocks of 24 along their contraction axes (1 x 24 / 24 x 1 blocks, or 24 x 24 tiles, the
// paper's tile size, Sec. 4.2), the stored operand (int8 mantissas, exponent bytes: what hbfp_encode writes) and its
// packed form (what hbfp_pack writes: bf16 planes for mantissas of 6 to 8 bits, densely packed limb planes for
// narrower ones), so that a product can start without a pack pass.  Several source matrices can share a launch.
//
// A workgroup of 8 waves owns a 192 x 192 region of the source: 8 x 8 tiles of 24 x 24, which is 3 k-steps of 64 and
// 6 row tiles of 32 in either orientation, the smallest region whose packed output consists of whole chunks.  It
// converts the region in two halves of 96 rows; a wave holds 4 tiles of one tile row in registers (16 lanes per tile:
// lane (h, j) owns columns 4 j .. 4 j + 3 of rows 12 h .. 12 h + 11, all loads of a half issued before the first
// use); block maxima are DPP reductions over the lanes of a tile (tiles), of a tile's row (1 x 24 blocks) or a register
// maximum and one exchange (24 x 1 blocks).  The mantissas of each output go to an LDS tile [operand row][k] without
// padding; after one barrier the workgroup streams the stored operand out in 16-byte pieces and writes the packed
// planes from the same tile with the arithmetic of the pack kernels (bf_pack.h, mx_pack.h).  Two workgroups share a
// compute unit (2 x 78 KB of LDS, 128 registers), so one converts while the other loads or stores.
#include "bf_pack.h"
#include "bfp_device.h"
#include "mx_pack.h"

namespace hbfp {
namespace {

constexpr int kEpThreads = 512;
constexpr int kEpRegion = 192;                   // source rows and columns per workgroup
constexpr int kEpStride = 200;                   // bytes between operand rows of an LDS mantissa tile (conflict-free tile writes)
constexpr int kEpTileBytes = kEpRegion * kEpStride;
constexpr int kEpExpBytes = kEpRegion * 8;       // exponent byte of every (operand row, block of the region)
constexpr int kEpLds = 2 * (kEpTileBytes + kEpExpBytes);

struct EpOut {
    uint8_t *mant, *exps;        // stored operand
    uint8_t *planes;             // planes of the packed operand (behind its 256-byte header)
    int *header;
    int64_t kpad, exp_ld, R;
    int32_t m, axis, tiled, present, mark;
    int32_t nb_stored, ksteps, row_tiles;   // stored 32-element blocks per row, k-steps and 32-row tiles of the packed operand
    uint32_t s0, s1;
};

struct EpParams {
    const float *src;
    int64_t ld, rows, cols;
    int32_t gx, gy;              // regions along the columns and the rows that this source needs
    EpOut o[2];
};
// several source matrices in one launch (blockIdx.z picks the source): the workgroups of the second start as those of the
// first retire, which a kernel boundary would not allow
constexpr int kEpBatch = 4;
struct EpBatch {
    EpParams p[kEpBatch];
};

template <int CTRL>
__device__ __forceinline__ uint32_t ep_dpp(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
// low bytes of four values into one word with three byte permutes
__device__ __forceinline__ uint32_t ep_pack4(int a, int b, int c, int d) {
    const uint32_t ab = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);    // bytes: a.0, b.0, 0, 0
    const uint32_t cd = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
}

template <int ROUND, int L>
__global__ __launch_bounds__(kEpThreads, 4) void encode_pack_kernel(const EpBatch batch) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const EpParams &p = batch.p[blockIdx.z];
    if ((int)blockIdx.x >= p.gx || (int)blockIdx.y >= p.gy) return;       // the grid is that of the largest source
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int j = lane & 7, h = (lane >> 3) & 1, tw = lane >> 4;
    const int tcl = (wave & 1) * 4 + tw;                                  // tile column of the region
    for (int half = 0; half < 1024 / kEpThreads; ++half) {
    const int trl = half * (kEpThreads / 128) + (wave >> 1);                               // tile row of the region
    const int64_t tc = (int64_t)blockIdx.x * 8 + tcl, tr = (int64_t)blockIdx.y * 8 + trl;
    const int64_t row0 = tr * 24 + h * 12, col0 = tc * 24 + 4 * j;
    float v[12][4];
    const int64_t tc_wave = (int64_t)blockIdx.x * 8 + (wave & 1) * 4;    // first of the wave's four tile columns
    if ((tr + 1) * 24 <= p.rows && (tc_wave + 4) * 24 <= p.cols) {
        // the wave's tiles lie inside the matrix: one uniform base, a 32-bit lane offset, rows a fixed stride apart.
        // Lanes 6 and 7 of a half tile own no columns; they load those of lane 5 again, which leaves every maximum as
        // it is, and write nothing.
        const float *wbase = p.src + tr * 24 * p.ld + tc_wave * 24;
        const uint32_t loff = (uint32_t)(h * 12) * (uint32_t)p.ld + (uint32_t)(tw * 24 + 4 * (j < 6 ? j : 5));
        float4 d[12];
#pragma unroll
        for (int r = 0; r < 12; ++r) d[r] = *reinterpret_cast<const float4 *>(wbase + r * p.ld + loff);
#pragma unroll
        for (int r = 0; r < 12; ++r) {
            v[r][0] = d[r].x; v[r][1] = d[r].y; v[r][2] = d[r].z; v[r][3] = d[r].w;
        }
    } else {
        const bool col_ok = j < 6 && col0 < p.cols;                       // the number of columns is a multiple of 4
        int rows_here = 0;
        {
            const int64_t left = p.rows - row0;
            rows_here = left <= 0 ? 0 : (left < 12 ? (int)left : 12);
        }
        // every load before the first use; rows that do not exist read the lane's first row again and are zeroed afterwards
        const bool any = col_ok && rows_here > 0;
        const float *sbase = any ? p.src + row0 * p.ld + col0 : p.src;
        float4 d[12];
#pragma unroll
        for (int r = 0; r < 12; ++r) d[r] = *reinterpret_cast<const float4 *>(sbase + (r < rows_here ? r : 0) * p.ld);
#pragma unroll
        for (int r = 0; r < 12; ++r) {
            const bool there = any && r < rows_here;
            v[r][0] = there ? d[r].x : 0.0f;
            v[r][1] = there ? d[r].y : 0.0f;
            v[r][2] = there ? d[r].z : 0.0f;
            v[r][3] = there ? d[r].w : 0.0f;
        }
    }
    // largest magnitudes: of each of this lane's rows, of each of its columns, of everything
    uint32_t ar[12], ac[4] = {0, 0, 0, 0}, at = 0;
#pragma unroll
    for (int r = 0; r < 12; ++r) {
        ar[r] = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t a = __float_as_uint(v[r][e]) & 0x7fffffffu;
            ar[r] = max(ar[r], a);
            ac[e] = max(ac[e], a);
        }
        at = max(at, ar[r]);
    }

#pragma unroll
    for (int oi = 0; oi < 2; ++oi) {
        const EpOut o = p.o[oi];
        if (!o.present) continue;
        uint8_t *T = lds + oi * (kEpTileBytes + kEpExpBytes);
        uint8_t *E = T + kEpTileBytes;
        // exponent of every element of this lane: per row (1 x 24 blocks), per column (24 x 1) or one (tiles)
        uint32_t eb_r[12], eb_c[4];
        if (o.tiled) {
            uint32_t a = at;
            a = max(a, ep_dpp<0xB1>(a));     // quad_perm [1,0,3,2]
            a = max(a, ep_dpp<0x4E>(a));     // quad_perm [2,3,0,1]
            a = max(a, ep_dpp<0x141>(a));    // row_half_mirror
            a = max(a, ep_dpp<0x140>(a));    // row_mirror
            const uint32_t eb = block_exponent<ROUND>(a, o.m);
#pragma unroll
            for (int r = 0; r < 12; ++r) eb_r[r] = eb;
#pragma unroll
            for (int e = 0; e < 4; ++e) eb_c[e] = eb;
        } else if (o.axis == 1) {
#pragma unroll
            for (int r = 0; r < 12; ++r) {   // the 8 lanes j of this half tile hold the row (lanes 6 and 7 hold zeros)
                uint32_t a = ar[r];
                a = max(a, ep_dpp<0xB1>(a));
                a = max(a, ep_dpp<0x4E>(a));
                a = max(a, ep_dpp<0x141>(a));
                eb_r[r] = block_exponent<ROUND>(a, o.m);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {    // the other half of the column is 8 lanes away
                const uint32_t a = max(ac[e], ep_dpp<0x128>(ac[e]));     // row_ror:8
                eb_c[e] = block_exponent<ROUND>(a, o.m);
            }
        }
        const bool per_col = !o.tiled && o.axis == 0;
        if (j < 6) {
            if (o.axis == 1) {
                // operand row = source row, k = source column
#pragma unroll
                for (int r = 0; r < 12; ++r) {
                    int q[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint64_t idx = (uint64_t)(row0 + r) * (uint64_t)p.cols + (uint64_t)(col0 + e);
                        q[e] = quantise<ROUND>(v[r][e], per_col ? eb_c[e] : eb_r[r], o.m, (uint32_t)idx, (uint32_t)(idx >> 32), o.s0, o.s1);
                    }
                    *reinterpret_cast<uint32_t *>(T + (trl * 24 + h * 12 + r) * kEpStride + tcl * 24 + 4 * j) = ep_pack4(q[0], q[1], q[2], q[3]);
                }
                if (j == 0) {
#pragma unroll
                    for (int r = 0; r < 12; ++r) E[(trl * 24 + h * 12 + r) * 8 + tcl] = (uint8_t)eb_r[r];
                }
            } else {
                // operand row = source column, k = source row
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int k = 0; k < 3; ++k) {
                        int q[4];
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            const int r = 4 * k + x;
                            const uint64_t idx = (uint64_t)(row0 + r) * (uint64_t)p.cols + (uint64_t)(col0 + e);
                            q[x] = quantise<ROUND>(v[r][e], per_col ? eb_c[e] : eb_r[r], o.m, (uint32_t)idx, (uint32_t)(idx >> 32), o.s0, o.s1);
                        }
                        *reinterpret_cast<uint32_t *>(T + (tcl * 24 + 4 * j + e) * kEpStride + trl * 24 + h * 12 + 4 * k) = ep_pack4(q[0], q[1], q[2], q[3]);
                    }
                    if (h == 0) E[(tcl * 24 + 4 * j + e) * 8 + trl] = (uint8_t)eb_c[e];
                }
            }
        }
    }
    }
    __syncthreads();

#pragma unroll
    for (int oi = 0; oi < 2; ++oi) {
        const EpOut o = p.o[oi];
        if (!o.present) continue;
        const uint8_t *T = lds + oi * (kEpTileBytes + kEpExpBytes);
        const uint8_t *E = T + kEpTileBytes;
        // Everything that depends only on the workgroup, the wave or the loop trip stays on the scalar unit; a lane adds
        // 32-bit offsets of its own (the host checks that 192 rows of an operand span less than 2^31 bytes).
        const int64_t orow0 = (int64_t)(o.axis == 1 ? blockIdx.y : blockIdx.x) * kEpRegion;   // first operand row of the region
        const int64_t kreg = o.axis == 1 ? blockIdx.x : blockIdx.y;                           // region index along k
        if (blockIdx.x == 0 && blockIdx.y == 0 && t == 0) o.header[1] = o.mark;
        const int rows_left = (int)(o.R - orow0 < kEpRegion ? (o.R - orow0 < 0 ? 0 : o.R - orow0) : kEpRegion);
        // ---- stored operand: 16-byte pieces, two per stored block of 32 (24 mantissas and 8 bytes of padding);
        // a thread keeps its block and half and walks down the rows, 32 at a time
        {
            const int b = (t >> 1) & 7, sh = t & 1, r0 = t >> 4;
            const bool blk_ok = kreg * 8 + b < o.nb_stored;
            uint8_t *dst0 = o.mant + orow0 * o.kpad + kreg * 256;                              // uniform
            const uint32_t goff = (uint32_t)r0 * (uint32_t)o.kpad + (uint32_t)(b * 32 + 16 * sh);
            const uint32_t gstep = 32u * (uint32_t)o.kpad;
            const uint8_t *src0 = T + r0 * kEpStride + 24 * b + 16 * sh;
#pragma unroll
            for (int i = 0; i < 16 * kEpRegion / kEpThreads; ++i) {
                if (blk_ok && r0 + 32 * i < rows_left) {
                    const v2i lo = *reinterpret_cast<const v2i *>(src0 + 32 * i * kEpStride);
                    v2i hi = {0, 0};
                    if (sh == 0) hi = *reinterpret_cast<const v2i *>(src0 + 32 * i * kEpStride + 8);
                    typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
                    const v4u_t w = {(unsigned)lo[0], (unsigned)lo[1], (unsigned)hi[0], (unsigned)hi[1]};
                    __builtin_nontemporal_store(w, reinterpret_cast<v4u_t *>(dst0 + (goff + (uint32_t)i * gstep)));
                }
            }
        }
        if (t < 2 * kEpRegion) {
            const int rl = t >> 1, half = t & 1;
            if (rl < rows_left && kreg * 8 + 4 * half < o.exp_ld)                              // exp_ld is a multiple of 4
                *reinterpret_cast<uint32_t *>(o.exps + orow0 * o.exp_ld + kreg * 8 + ((uint32_t)rl * (uint32_t)o.exp_ld + 4u * half)) =
                    *reinterpret_cast<const uint32_t *>(E + rl * 8 + 4 * half);
        }
        // ---- packed planes: a wave takes 16 operand rows of one k-step of 64 at a time (lane = row, quarter of the k-step)
        bool bad = false;
        const int q = lane & 3, r4 = lane >> 2;
        const uint8_t *tl = T + r4 * kEpStride + q * 16;     // this lane's 16 mantissas of k-step 0 of rows 0..15
        const uint8_t *el = E + r4 * 8;
#pragma unroll
        for (int i = 0; i < (36 + kEpThreads / 64 - 1) / (kEpThreads / 64); ++i) {
            const int unit = wave + (kEpThreads / 64) * i;   // 12 groups of 16 rows x 3 k-steps
            if (unit >= 36) break;
            const int r16 = unit / 3, ksl = unit - 3 * r16;
            const int64_t rt = (orow0 >> 5) + (r16 >> 1), ks = kreg * 3 + ksl;
            if (rt >= o.row_tiles || ks >= o.ksteps) continue;                                 // uniform over the wave
            v2i raw[2];
            int ex[2];
#pragma unroll
            for (int oc = 0; oc < 2; ++oc) {
                raw[oc] = *reinterpret_cast<const v2i *>(tl + r16 * 16 * kEpStride + ksl * 64 + 8 * oc);
                const int jl = ksl * 8 + q * 2 + oc;         // octet of the region's k axis: block jl / 3
                const int e = el[r16 * 128 + (jl * 43 >> 7)];    // jl / 3 for jl < 24
                ex[oc] = (raw[oc][0] | raw[oc][1]) ? (e > 254 ? 254 : e) : 255;
            }
            if constexpr (L == 2) {
                // 6..8-bit mantissas: bf16 planes (bf_pack.h), an octet of one row is 16 bytes of one half k-step of 32
#pragma unroll
                for (int oc = 0; oc < 2; ++oc) {
                    const int jl = ksl * 8 + q * 2 + oc;
                    const int e = el[r16 * 128 + (jl * 43 >> 7)];
                    bad |= ex[oc] != 255 && !bf_exponent_ok(e);
                    *reinterpret_cast<v4u *>(o.planes + bf_piece_offset(rt, 2 * ks + (q >> 1), 2 * (int64_t)o.ksteps, q & 1, oc,
                                                                        (r16 & 1) * 16 + r4)) = bf_octet_i8(raw[oc], e, o.m);
                }
            } else {
                uint8_t *chunk = o.planes + (((rt >> 3) * o.ksteps + ks) * kRowTiles + (rt & 7)) * (int64_t)chunk_bytes(L);
                bad |= pack_half_group_dense<L>(raw, ex, o.m, chunk, (r16 & 1) * 16 + r4 + 32 * (q >> 1), q);
            }
        }
        if (bad) o.header[0] = o.mark;
    }
}

}  // namespace

// Outputs the kernel above covers: blocks of 24 along k stored as blocks of 32, one exponent per operand row and block
// or per 24 x 24 tile, 8-bit storage, the same limb count and rounding for all, every output with a packed buffer.
bool encode_pack_ok(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs, void *const *packed) {
    if (n < 1 || n > 2 || ((uintptr_t)src & 15) || (ld & 3) || ld >= ((int64_t)1 << 27)) return false;
    const hbfp_tensor *f = outs[0];
    if (f->src_cols & 3) return false;
    if (ceil_div(f->src_rows + 256, kEpRegion) + 2 > 65535 || ceil_div(f->src_cols + 256, kEpRegion) + 2 > 0x7fffffff) return false;
    for (int i = 0; i < n; ++i) {
        const hbfp_tensor *t = outs[i];
        if (!packed[i] || t->kblock != 24 || t->kblock_pad != 32 || t->kshare != 1 || (t->rblock != 1 && t->rblock != 24)) return false;
        if (t->mant_bits > 8 || limbs_of(t->mant_bits) != limbs_of(f->mant_bits) || t->rounding != f->rounding) return false;
        if (t->src_rows != f->src_rows || t->src_cols != f->src_cols) return false;
        if (t->kpad * (kEpRegion + 32) >= ((int64_t)1 << 31) || t->rows > ((int64_t)1 << 36)) return false;
    }
    return true;
}

// fills the parameters of one source; marks its packed buffers
static int ep_params_of(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs, void *const *packed, hipStream_t s,
                        EpParams *out) {
    const hbfp_tensor *f = outs[0];
    EpParams p = {};
    p.src = src;
    p.ld = ld;
    p.rows = f->src_rows;
    p.cols = f->src_cols;
    int64_t ext_rows = 0, ext_cols = 0;
    for (int i = 0; i < n; ++i) {
        const hbfp_tensor *t = outs[i];
        EpOut &o = p.o[i];
        o.present = 1;
        o.mant = (uint8_t *)t->mant;
        o.exps = t->exps;
        o.header = (int *)packed[i];
        o.planes = (uint8_t *)packed[i] + 256;
        o.kpad = t->kpad;
        o.exp_ld = t->exp_ld;
        o.R = t->rows;
        o.m = t->mant_bits;
        o.axis = t->contract_axis;
        o.tiled = t->rblock == 24;
        o.nb_stored = (int32_t)(t->kpad / 32);
        {   // the packed k axis ends with the last octet that holds an element (as mx_ksteps counts it)
            const int64_t all = t->nblk * 3, used = ceil_div(t->kdim, 8);
            o.ksteps = (int32_t)(round_up((used < all ? used : all) * 8, 128) / 64);
        }
        o.row_tiles = (int32_t)(ceil_div(t->rows, 256) * 8);
        o.s0 = (uint32_t)t->seed;
        o.s1 = (uint32_t)(t->seed >> 32);
        int rc = mx_pack_begin(packed[i], s, &o.mark);
        if (rc != HBFP_OK) return rc;
        // the region grid must reach every stored block, every k-step and every row tile of the packed operand
        const int64_t kext = ((int64_t)o.nb_stored * 24 > (int64_t)o.ksteps * 64 ? (int64_t)o.nb_stored * 24 : (int64_t)o.ksteps * 64);
        const int64_t rext = (int64_t)o.row_tiles * 32;
        if (o.axis == 1) {
            ext_cols = kext > ext_cols ? kext : ext_cols;
            ext_rows = rext > ext_rows ? rext : ext_rows;
        } else {
            ext_rows = kext > ext_rows ? kext : ext_rows;
            ext_cols = rext > ext_cols ? rext : ext_cols;
        }
    }
    p.gx = (int32_t)ceil_div(ext_cols, kEpRegion);
    p.gy = (int32_t)ceil_div(ext_rows, kEpRegion);
    *out = p;
    return HBFP_OK;
}

// the instantiation that a source's outputs need: rounding and limb count
static int ep_which(const hbfp_tensor *f) { return (f->rounding ? 2 : 0) + (limbs_of(f->mant_bits) - 1); }

bool encode_pack_batch_ok(int nsrc, const hbfp_tensor *const *const *outs) {
    if (nsrc < 1 || nsrc > kEpBatch) return false;
    for (int i = 1; i < nsrc; ++i)
        if (ep_which(outs[i][0]) != ep_which(outs[0][0])) return false;
    return true;
}

// nsrc sources, each of which encode_pack_ok accepts, with equal rounding and limb counts (encode_pack_batch_ok)
int launch_encode_pack_batch(int nsrc, const float *const *src, const int64_t *ld, const int *n, const hbfp_tensor *const *const *outs,
                             void *const *const *packed, hipStream_t s) {
    EpBatch b = {};
    int gx = 0, gy = 0;
    for (int i = 0; i < nsrc; ++i) {
        const int rc = ep_params_of(src[i], ld[i], n[i], outs[i], packed[i], s, &b.p[i]);
        if (rc != HBFP_OK) return rc;
        gx = b.p[i].gx > gx ? b.p[i].gx : gx;
        gy = b.p[i].gy > gy ? b.p[i].gy : gy;
    }
    const dim3 grid((unsigned)gx, (unsigned)gy, (unsigned)nsrc);
    static std::atomic<bool> configured[4];
    const void *const kernels[4] = {reinterpret_cast<const void *>(&encode_pack_kernel<0, 1>), reinterpret_cast<const void *>(&encode_pack_kernel<0, 2>),
                                    reinterpret_cast<const void *>(&encode_pack_kernel<1, 1>), reinterpret_cast<const void *>(&encode_pack_kernel<1, 2>)};
    const int which = ep_which(outs[0][0]);
    if (allow_dynamic_lds(configured[which], kernels[which], kEpLds) != HBFP_OK) return HBFP_ERR_LAUNCH;
    switch (which) {
        case 0: hipLaunchKernelGGL((encode_pack_kernel<0, 1>), grid, dim3(kEpThreads), kEpLds, s, b); break;
        case 1: hipLaunchKernelGGL((encode_pack_kernel<0, 2>), grid, dim3(kEpThreads), kEpLds, s, b); break;
        case 2: hipLaunchKernelGGL((encode_pack_kernel<1, 1>), grid, dim3(kEpThreads), kEpLds, s, b); break;
        default: hipLaunchKernelGGL((encode_pack_kernel<1, 2>), grid, dim3(kEpThreads), kEpLds, s, b); break;
    }
    return launch_status();
}

int launch_encode_pack(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs, void *const *packed, hipStream_t s) {
    return launch_encode_pack_batch(1, &src, &ld, &n, &outs, &packed, s);
}

}  // namespace hbfp
