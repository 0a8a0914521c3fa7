// FP32 -> BFP conversion kernels for gfx950 (Sec. 4.1: convert before every dot
// product with the exponent of the largest value; Sec. 5.3: FP-to-BFP unit).
//
// Three paths, all writing the operand layout described in the public header:
//   row   1-D blocks along contiguous source columns (k contiguous in the source):
//         each lane owns 8 consecutive elements, a block is 4/8/16 neighbouring
//         lanes, the block maximum is a DPP reduction, one pass over HBM.
//   col   1-D blocks down the source rows (k strided in the source): each lane owns
//         one operand row and a whole block in registers, the k-contiguous output is
//         transposed through LDS so that global stores are full 128-byte lines.
//   tile  everything else (2-D tiles, very long blocks): a max pass into a small
//         per-tile array, then a quantise pass.
#include "bfp_device.h"
#include "hbfp_internal.h"

namespace hbfp {
namespace {

constexpr int kThreads = 256;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

// max over groups of GP neighbouring lanes (GP = 4, 8, 16), result in every lane of the group
template <int GP>
__device__ __forceinline__ uint32_t group_max(uint32_t v) {
    v = max(v, dpp_u32<0xB1>(v));                 // quad_perm [1,0,3,2]
    v = max(v, dpp_u32<0x4E>(v));                 // quad_perm [2,3,0,1]
    if (GP >= 8) v = max(v, dpp_u32<0x141>(v));   // row_half_mirror: the other quad of the 8
    if (GP >= 16) v = max(v, dpp_u32<0x140>(v));  // row_mirror: the other half of the 16
    return v;
}

// low bytes of four values into one word: two byte permutes gather pairs, the third joins them (the mask-shift-or
// form takes seven instructions)
__device__ __forceinline__ uint32_t pack4_i8(int a, int b, int c, int d) {
    const uint32_t ab = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);    // bytes: a.0, b.0, 0, 0
    const uint32_t cd = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(cd, ab, 0x05040100u);                                    // ab.0, ab.1, cd.0, cd.1
}
__device__ __forceinline__ uint32_t pack2_i16(int a, int b) {
    return (uint32_t)(a & 0xffff) | ((uint32_t)b << 16);
}

// streaming stores: an encoded operand is written once and not read again by the kernel that writes it
typedef unsigned v2u_t __attribute__((ext_vector_type(2)));
typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_stream(uint8_t *dst, uint2 v) {
    const v2u_t w = {v.x, v.y};
    __builtin_nontemporal_store(w, reinterpret_cast<v2u_t *>(dst));
}
__device__ __forceinline__ void store_stream(uint8_t *dst, uint4 v) {
    const v4u_t w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<v4u_t *>(dst));
}

// ------------------------------------------------------------------------------------------
// n / d for 0 <= n < 2^31 as a multiplication: with l = ceil(log2 d) and m = ceil(2^(31 + l) / d) (fits 32 bits),
// floor(n * m / 2^(31 + l)) = floor(n / d) for every such n (round-up method of Granlund and Montgomery).
// magic[0] = m, magic[1] = l - 1; d = 1 is stored as m = 0.
__device__ __forceinline__ uint32_t div_magic(uint32_t n, const uint32_t (&magic)[2]) {
    return magic[0] ? __umulhi(n, magic[0]) >> magic[1] : n;
}

// A convolution's lowered activation matrix, never materialised: row = output position (img, oy, ox), column k =
// an entry of the filter window.  The channels are cut into blocks of cbs (the last may be shorter) and k runs
// block by block: k = (cb * R * S + fr * S + fs) * cbs + ci inside full blocks, the same with the last block's
// width after them; one block of all channels gives the plain order (fr * S + fs) * C + c.  With this order
// the R * S * cbs values of a channel block are consecutive, so a filter matrix cut into tiles of
// (R * S * cbs) x (output channels) shares exponents over the two outer filter dimensions (Sec. 5.1).
struct ConvGeom {
    int32_t H, W, C, S, Ho, Wo, pad_h, pad_w, str_h, str_w;
    int32_t cbs, per_blk, c_last, k_last;   // channel block, R*S*cbs, width of the last block, first k of the last block
    uint32_t dPer[2], dCb[2], dCl[2], dS[2], dP[2], dW[2];   // divisions by per_blk, cbs, c_last, S, Ho*Wo, Wo
};

// window entry k -> filter row, filter column, channel
__device__ __forceinline__ void conv_window_entry(const ConvGeom &c, uint32_t k, int &fr, int &fs, int &ch) {
    uint32_t base, off, tap, width;
    if (k < (uint32_t)c.k_last) {
        const uint32_t cb = div_magic(k, c.dPer);
        off = k - cb * (uint32_t)c.per_blk;
        tap = div_magic(off, c.dCb);
        width = (uint32_t)c.cbs;
        base = cb * (uint32_t)c.cbs;
    } else {
        off = k - (uint32_t)c.k_last;
        tap = div_magic(off, c.dCl);
        width = (uint32_t)c.c_last;
        base = (uint32_t)(c.C - c.c_last);
    }
    ch = (int)(base + off - tap * width);
    fr = (int)div_magic(tap, c.dS);
    fs = (int)(tap - (uint32_t)fr * (uint32_t)c.S);
}

// output position -> image, top-left corner of its window
__device__ __forceinline__ void conv_position(const ConvGeom &c, uint32_t pos, uint32_t &img, int &y0, int &x0, int &oy, int &ox) {
    img = div_magic(pos, c.dP);
    const uint32_t rem = pos - img * (uint32_t)(c.Ho * c.Wo);
    oy = (int)div_magic(rem, c.dW);
    ox = (int)rem - oy * c.Wo;
    y0 = oy * c.str_h - c.pad_h;
    x0 = ox * c.str_w - c.pad_w;
}
__device__ __forceinline__ void conv_position(const ConvGeom &c, uint32_t pos, uint32_t &img, int &y0, int &x0) {
    int oy, ox;
    conv_position(c, pos, img, y0, x0, oy, ox);
}

// row path
struct RowParams {
    const float *src;
    uint8_t *mant;
    uint8_t *exps;
    int64_t ld, R, K, kpad, exp_ld, src_cols;
    int32_t kblock, nblk, nb_stored, m;
    int32_t lpr_log2;   // log2 of the chunks per row when that is a power of two, else -1
    int32_t chunks;     // 8-element chunks per stored row = kpad / 8
    int32_t nseg;       // segments per row = ceil(chunks / lanes-per-row)
    int32_t vec_ok;     // 16-byte vector loads are aligned
    int32_t sr_aligned; // the stochastic-rounding counter of every chunk's first element is a multiple of 8
    int32_t one_row;    // every workgroup's chunks lie in one row and 32-bit offsets reach anywhere inside a row
    uint32_t s0, s1;
    // GP = 0 (second pass of the two-pass conversion): the largest magnitude of every exponent block has been
    // computed already, table[(row / rblock) * ntk + block / kshare]; a stored block is gp chunks long
    const uint32_t *table;
    int64_t rblock, ntk;
    int32_t gp, kshare;
    // CONV: the source is an NHWC image tensor and the operand is its lowered form, never materialised: operand row
    // (n, ho, wo) holds the values under the filter window, k = (r * S + s) * C + c, zero outside the image
    ConvGeom cv;
    uint32_t dChunks[2];                         // likewise by the chunks per row (when that is no power of two)
    uint32_t dGp[2], dR[2], dK[2];               // and by gp, rblock and kshare (GP = 0 only)
};


template <int GP, bool WIDE, int ROUND, int U, bool CONV = false>
__global__ __launch_bounds__(kThreads) void enc_row_kernel(const RowParams p) {
    // The (row, chunk) pairs of the whole operand form one flat index space: a workgroup takes U * 256
    // consecutive chunks.  A row holds a multiple of 16 chunks, so the 4/8/16 lanes of a block never
    // straddle rows; rows need not be a power of two long.
    const uint64_t total = (uint64_t)p.R * (uint64_t)p.chunks;
    const uint64_t g0 = (uint64_t)blockIdx.x * (kThreads * U) + threadIdx.x;
    // Long rows (a workgroup's chunks inside one row, the usual case): the row and everything that is a multiple of it
    // stay on the scalar unit and a lane adds 32-bit offsets; the flat 64-bit index space is for the general case.
    // Only stochastic rounding, which is bound by its vector instructions, takes this path (nearest-even rounding
    // waits for memory, and its short workgroups lose more to the longer scalar prologue than they gain: 60 against 57 us
    // on 2^26 elements).
    const bool one_row = !CONV && GP != 0 && ROUND == 1 && p.one_row;
    uint64_t wg_row = 0;
    uint32_t wg_cl = 0;
    if (one_row) {
        const uint64_t gw = (uint64_t)blockIdx.x * (kThreads * U);
        wg_row = p.lpr_log2 >= 0 ? gw >> p.lpr_log2 : gw / (uint64_t)(uint32_t)p.chunks;
        wg_cl = (uint32_t)(gw - wg_row * (uint64_t)(uint32_t)p.chunks);
        if (wg_row >= (uint64_t)p.R) return;         // the grid is rounded up to whole workgroups of four chunks per thread
    }

    float v[U][8];
    int n[U], cl[U];
    int64_t rows[U];
    int64_t at[U];        // CONV with one exponent per image: index of the chunk's first value in the image tensor, else -1
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (one_row) {
            cl[u] = (int)(wg_cl + threadIdx.x + u * kThreads);
            rows[u] = (int64_t)wg_row;
            const uint32_t blk = (uint32_t)cl[u] / (uint32_t)(GP ? GP : 1), j = (uint32_t)cl[u] % (uint32_t)(GP ? GP : 1);
            const uint32_t kb = blk * (uint32_t)p.kblock, k0 = kb + 8u * j;     // K < 2^30 here
            uint32_t cnt = 0;
            if (blk < (uint32_t)p.nblk) {
                const uint32_t K = (uint32_t)p.K, blen = K - kb < (uint32_t)p.kblock ? K - kb : (uint32_t)p.kblock;
                cnt = blen > 8u * j ? (blen - 8u * j < 8u ? blen - 8u * j : 8u) : 0u;
            }
            n[u] = (int)cnt;
            const char *s = reinterpret_cast<const char *>(p.src + wg_row * (uint64_t)p.ld) + (cnt ? k0 * 4u : 0u);
            if (cnt == 8) {
                const float4 a = *reinterpret_cast<const float4 *>(s);
                const float4 b = *reinterpret_cast<const float4 *>(s + 16);
                v[u][0] = a.x; v[u][1] = a.y; v[u][2] = a.z; v[u][3] = a.w;
                v[u][4] = b.x; v[u][5] = b.y; v[u][6] = b.z; v[u][7] = b.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[u][e] = ((uint32_t)e < cnt) ? reinterpret_cast<const float *>(s)[e] : 0.0f;
            }
            continue;
        }
        const uint64_t g = g0 + (uint64_t)u * kThreads;
        const bool in = g < total;
        int64_t row;
        if (p.lpr_log2 >= 0) {                       // chunks per row is a power of two
            row = (int64_t)(g >> p.lpr_log2);
            cl[u] = (int)(g & (uint64_t)(p.chunks - 1));
        } else if (total <= 0x7fffffffull) {
            const uint32_t q = div_magic((uint32_t)g, p.dChunks);
            row = q;
            cl[u] = (int)((uint32_t)g - q * (uint32_t)p.chunks);
        } else if (total <= 0xffffffffull) {
            const uint32_t q = (uint32_t)g / (uint32_t)p.chunks;
            row = q;
            cl[u] = (int)((uint32_t)g - q * (uint32_t)p.chunks);
        } else {
            row = (int64_t)(g / (uint64_t)p.chunks);
            cl[u] = (int)(g - (uint64_t)row * (uint64_t)p.chunks);
        }
        rows[u] = in ? row : -1;
        const int blk = GP ? cl[u] / (GP ? GP : 1) : (int)div_magic((uint32_t)cl[u], p.dGp);
        const int j = cl[u] - blk * (GP ? GP : p.gp);
        int cnt = 0;
        if (in && blk < p.nblk) {
            const int64_t k0 = (int64_t)blk * p.kblock;
            const int64_t blen = (p.K - k0 < p.kblock) ? (p.K - k0) : p.kblock;
            const int64_t left = blen - 8 * j;
            cnt = left <= 0 ? 0 : (left >= 8 ? 8 : (int)left);
        }
        n[u] = cnt;
        const float *s;
        if (!CONV) {
            s = p.src + (in ? row : 0) * p.ld + (int64_t)blk * p.kblock + 8 * j;
        } else {
            // a chunk of 8 never leaves its filter tap (channel blocks and the block length are multiples of 8)
            const uint32_t k0 = (uint32_t)blk * (uint32_t)p.kblock + 8u * (uint32_t)j;
            int fr, fs, c0, y0, x0;
            uint32_t img;
            conv_window_entry(p.cv, cnt ? k0 : 0u, fr, fs, c0);
            conv_position(p.cv, in ? (uint32_t)row : 0u, img, y0, x0);
            const int hi = y0 + fr, wi = x0 + fs;
            const bool inside = hi >= 0 && hi < p.cv.H && wi >= 0 && wi < p.cv.W;
            if (!inside) cnt = 0;                                        // zeros; they still count as elements of the block
            const int64_t off = inside ? (((int64_t)img * p.cv.H + hi) * p.cv.W + wi) * p.cv.C + c0 : 0;
            s = p.src + off;
            at[u] = (p.table && inside) ? off : -1;
        }
        if (cnt == 8 && p.vec_ok) {
            const float4 a = *reinterpret_cast<const float4 *>(s);
            const float4 b = *reinterpret_cast<const float4 *>(s + 4);
            v[u][0] = a.x; v[u][1] = a.y; v[u][2] = a.z; v[u][3] = a.w;
            v[u][4] = b.x; v[u][5] = b.y; v[u][6] = b.z; v[u][7] = b.w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[u][e] = (e < cnt) ? s[e] : 0.0f;
        }
    }
    // Second half, per chunk: exponent, rounding, stores.  It is expanded twice, once with the row as the workgroup's
    // (scalar) value and once with the lane's, so that in the long-row case every multiple of the row stays scalar.
    auto finish = [&](const int u, const int64_t row, const bool row_is_uniform) {
        const int blk = GP ? cl[u] / (GP ? GP : 1) : (int)div_magic((uint32_t)cl[u], p.dGp);
        const int j = cl[u] - blk * (GP ? GP : p.gp);
        uint32_t amax = 0;
        if (GP) {
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = max(amax, __float_as_uint(v[u][e]) & 0x7fffffffu);
            amax = group_max<(GP ? GP : 4)>(amax);
        } else if (row >= 0 && blk < p.nblk) {
            amax = p.table[(int64_t)div_magic((uint32_t)row, p.dR) * p.ntk + div_magic((uint32_t)blk, p.dK)];   // rows fit 31 bits here
        }
        const uint32_t Eb = block_exponent<ROUND>(amax, p.m);
        int q[8];
        uint32_t pairs[4];            // the same mantissas as 16-bit halves, where the rounding step produces them that way
        bool have_pairs = false;
        // stochastic rounding draws by logical index: of the (lowered) source matrix, or, when a whole image shares one
        // exponent, of the image tensor: a pixel is then rounded the same way in every window it appears in, as if
        // the image had been converted once and lowered afterwards
        uint64_t idx0;
        if (row_is_uniform) idx0 = (uint64_t)row * (uint64_t)p.src_cols + (uint32_t)(blk * p.kblock + 8 * j);
        else idx0 = (uint64_t)row * (uint64_t)p.src_cols + (uint64_t)((int64_t)blk * p.kblock + 8 * j);
        if (CONV && GP == 0 && at[u] >= 0) idx0 = (uint64_t)at[u];
        if (ROUND == 1 && p.sr_aligned) {
            // the eight counters are idx0 | e: the xorshift steps of the hash, linear over GF(2), run once on the common
            // part and the elements differ by compile-time constants
            const uint32_t common = sr_triple((uint32_t)idx0 ^ p.s0), high = (uint32_t)(idx0 >> 32) ^ p.s1;
            const uint32_t small = sr_small_bits(Eb, p.m);
            const int unit = 125 + p.m - (int)Eb;
            uint32_t mag[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) mag[e] = quant_sr_magnitude(v[u][e], unit, small, sr_hash_tail(common ^ sr_triple((uint32_t)e), high));
            // signs two at a time; the pairs are the stored 16-bit mantissas, or give their low bytes to the 8-bit ones
#pragma unroll
            for (int e = 0; e < 8; e += 2) pairs[e / 2] = signed_pair16(mag[e], mag[e + 1], v[u][e], v[u][e + 1]);
            have_pairs = true;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint64_t idx = idx0 + e;
                q[e] = quantise<ROUND>(v[u][e], Eb, p.m, (uint32_t)idx, (uint32_t)(idx >> 32), p.s0, p.s1);
            }
        }
        if (row >= 0) {
            // destination of this chunk's mantissas: row base (uniform in the long-row case) plus the lane's chunk
            uint8_t *mrow = p.mant + row * p.kpad * (WIDE ? 2 : 1), *erow = p.exps + row * p.exp_ld;
            if (!WIDE) {
                uint2 o;
                if (have_pairs) {
                    o.x = __builtin_amdgcn_perm(pairs[1], pairs[0], 0x06040200u);     // the low byte of each half
                    o.y = __builtin_amdgcn_perm(pairs[3], pairs[2], 0x06040200u);
                } else {
                    o.x = pack4_i8(q[0], q[1], q[2], q[3]);
                    o.y = pack4_i8(q[4], q[5], q[6], q[7]);
                }
                // streaming stores: the mantissas are not read again by this kernel (about 1 % on a 2^26-element encode)
                typedef unsigned v2u __attribute__((ext_vector_type(2)));
                const v2u o2 = {o.x, o.y};
                __builtin_nontemporal_store(o2, reinterpret_cast<v2u *>(mrow + (uint32_t)cl[u] * 8u));
            } else {
                uint4 o;
                if (have_pairs) {
                    o.x = pairs[0]; o.y = pairs[1]; o.z = pairs[2]; o.w = pairs[3];
                } else {
                    o.x = pack2_i16(q[0], q[1]);
                    o.y = pack2_i16(q[2], q[3]);
                    o.z = pack2_i16(q[4], q[5]);
                    o.w = pack2_i16(q[6], q[7]);
                }
                typedef unsigned v4u __attribute__((ext_vector_type(4)));
                const v4u o4 = {o.x, o.y, o.z, o.w};
                __builtin_nontemporal_store(o4, reinterpret_cast<v4u *>(mrow + (uint32_t)cl[u] * 16u));
            }
            if (j == 0) {
                uint8_t *e = erow;
                e[blk] = blk < p.nblk ? (uint8_t)Eb : (uint8_t)1;
                if (blk == p.nb_stored - 1)
                    for (int64_t b = p.nb_stored; b < p.exp_ld; ++b) e[b] = 1;
            }
        }
    };
    if (one_row) {
#pragma unroll
        for (int u = 0; u < U; ++u) finish(u, (int64_t)wg_row, true);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) finish(u, rows[u], false);
    }
}

// 2-D tiles whose k axis is contiguous in the source: a workgroup owns the rblock source rows of one
// row of tiles and 256 chunk lanes of them.  Pass 1 takes the maximum down the rows in each lane and
// across the lanes of a block; pass 2 reads the same (cache-resident) rows again and quantises.
template <int GP, bool WIDE, int ROUND>
__global__ __launch_bounds__(kThreads) void enc_row_tiled_kernel(const RowParams p, int rblock) {
    const int t = threadIdx.x;
    const int64_t rfirst = (int64_t)blockIdx.x * rblock;
    int64_t rlast = rfirst + rblock;
    rlast = rlast < p.R ? rlast : p.R;
    for (int seg = blockIdx.y; seg < p.nseg; seg += gridDim.y) {
        const int cl = seg * kThreads + t;
        const bool lane_ok = cl < p.chunks;
        const int blk = cl / GP, j = cl % GP;
        int cnt = 0;
        if (lane_ok && blk < p.nblk) {
            const int64_t k0 = (int64_t)blk * p.kblock;
            const int64_t blen = (p.K - k0 < p.kblock) ? (p.K - k0) : p.kblock;
            const int64_t left = blen - 8 * j;
            cnt = left <= 0 ? 0 : (left >= 8 ? 8 : (int)left);
        }
        const int64_t col = (int64_t)blk * p.kblock + 8 * j;
        uint32_t amax = 0;
        for (int64_t row = rfirst; row < rlast; ++row) {
            const float *s = p.src + row * p.ld + col;
            if (cnt == 8 && p.vec_ok) {
                const float4 a = *reinterpret_cast<const float4 *>(s);
                const float4 b = *reinterpret_cast<const float4 *>(s + 4);
                amax = max(amax, max(max(__float_as_uint(a.x) & 0x7fffffffu, __float_as_uint(a.y) & 0x7fffffffu),
                                     max(__float_as_uint(a.z) & 0x7fffffffu, __float_as_uint(a.w) & 0x7fffffffu)));
                amax = max(amax, max(max(__float_as_uint(b.x) & 0x7fffffffu, __float_as_uint(b.y) & 0x7fffffffu),
                                     max(__float_as_uint(b.z) & 0x7fffffffu, __float_as_uint(b.w) & 0x7fffffffu)));
            } else {
                for (int e = 0; e < cnt; ++e) amax = max(amax, __float_as_uint(s[e]) & 0x7fffffffu);
            }
        }
        amax = group_max<GP>(amax);
        const uint32_t Eb = block_exponent<ROUND>(amax, p.m);
        for (int64_t row = rfirst; row < rlast; ++row) {
            const float *s = p.src + row * p.ld + col;
            float v[8];
            if (cnt == 8 && p.vec_ok) {
                const float4 a = *reinterpret_cast<const float4 *>(s);
                const float4 b = *reinterpret_cast<const float4 *>(s + 4);
                v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
                v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = (e < cnt) ? s[e] : 0.0f;
            }
            int q[8];
            const uint64_t idx0 = (uint64_t)row * (uint64_t)p.src_cols + (uint64_t)col;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint64_t idx = idx0 + e;
                q[e] = quantise<ROUND>(v[e], Eb, p.m, (uint32_t)idx, (uint32_t)(idx >> 32), p.s0, p.s1);
            }
            if (lane_ok) {
                if (!WIDE) {
                    uint2 o;
                    o.x = pack4_i8(q[0], q[1], q[2], q[3]);
                    o.y = pack4_i8(q[4], q[5], q[6], q[7]);
                    store_stream(p.mant + row * p.kpad + (int64_t)cl * 8, o);
                } else {
                    uint4 o;
                    o.x = pack2_i16(q[0], q[1]);
                    o.y = pack2_i16(q[2], q[3]);
                    o.z = pack2_i16(q[4], q[5]);
                    o.w = pack2_i16(q[6], q[7]);
                    store_stream(p.mant + (row * p.kpad + (int64_t)cl * 8) * 2, o);
                }
                if (j == 0) {
                    uint8_t *e = p.exps + row * p.exp_ld;
                    e[blk] = blk < p.nblk ? (uint8_t)Eb : (uint8_t)1;
                    if (blk == p.nb_stored - 1)
                        for (int64_t b = p.nb_stored; b < p.exp_ld; ++b) e[b] = 1;
                }
            }
        }
    }
}

template <int GP>
void launch_row_tiled_g(const RowParams &p, int rblock, dim3 grid, bool wide, int rounding, hipStream_t s) {
    if (!wide && rounding == 0) hipLaunchKernelGGL((enc_row_tiled_kernel<GP, false, 0>), grid, dim3(kThreads), 0, s, p, rblock);
    else if (!wide) hipLaunchKernelGGL((enc_row_tiled_kernel<GP, false, 1>), grid, dim3(kThreads), 0, s, p, rblock);
    else if (rounding == 0) hipLaunchKernelGGL((enc_row_tiled_kernel<GP, true, 0>), grid, dim3(kThreads), 0, s, p, rblock);
    else hipLaunchKernelGGL((enc_row_tiled_kernel<GP, true, 1>), grid, dim3(kThreads), 0, s, p, rblock);
}

template <int GP, bool WIDE, int ROUND>
void launch_row_t(const RowParams &p, dim3 grid, hipStream_t s) {
    // stochastic rounding is bound by its vector instructions and holds more registers: two chunks per thread instead of
    // four keep more waves on a SIMD (config 2, 8-bit: 67 us against 71-75 us)
    if (ROUND) hipLaunchKernelGGL((enc_row_kernel<GP, WIDE, ROUND, 2>), dim3(grid.x * 2), dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((enc_row_kernel<GP, WIDE, ROUND, 4>), grid, dim3(kThreads), 0, s, p);
}

template <int GP>
void launch_row_conv_g(const RowParams &p, dim3 grid, bool wide, int rounding, hipStream_t s) {
    if (!wide && rounding == 0) hipLaunchKernelGGL((enc_row_kernel<GP, false, 0, 4, true>), grid, dim3(kThreads), 0, s, p);
    else if (!wide) hipLaunchKernelGGL((enc_row_kernel<GP, false, 1, 4, true>), grid, dim3(kThreads), 0, s, p);
    else if (rounding == 0) hipLaunchKernelGGL((enc_row_kernel<GP, true, 0, 4, true>), grid, dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((enc_row_kernel<GP, true, 1, 4, true>), grid, dim3(kThreads), 0, s, p);
}

template <int GP>
void launch_row_g(const RowParams &p, dim3 grid, bool wide, int rounding, hipStream_t s) {
    if (!wide && rounding == 0) launch_row_t<GP, false, 0>(p, grid, s);
    else if (!wide) launch_row_t<GP, false, 1>(p, grid, s);
    else if (rounding == 0) launch_row_t<GP, true, 0>(p, grid, s);
    else launch_row_t<GP, true, 1>(p, grid, s);
}

// ------------------------------------------------------------------------------------------
// col path
struct ColParams {
    const float *src;
    uint8_t *mant;
    uint8_t *exps;
    int64_t ld, R, K, kpad, exp_ld, src_cols;
    int32_t kblock, nblk, nb_stored, m;
    int32_t rblock;     // operand rows (lanes) sharing one exponent: 1 for 1-D blocks, up to 64 for 2-D tiles
    int32_t lanes;      // lanes of a wave that carry operand rows: the largest multiple of rblock <= 64
    uint32_t row_groups;   // workgroups per group of blocks (the grid is flat: block group = blockIdx.x / row_groups)
    uint32_t s0, s1;
    // TABLE (second pass of the two-pass conversion): the largest magnitude of every exponent block has been computed
    // already, table[(block / kshare) * ntc + row / rblock_t]; the kernel then walks stored pieces of KBP elements,
    // spb of which make up one stored block
    const uint32_t *table;
    int64_t rblock_t, ntc;
    int32_t spb, kshare;
    // CONV: the source is an NHWC image tensor; operand row = (fr * S + fs) * C + ch of the lowered matrix, k = the
    // output position (img, oy, ox): the operand of the weight-gradient product, never materialised
    ConvGeom cv;
};

constexpr int kColRowBytes = 512;   // bytes of one operand row in an LDS tile
constexpr int kColStride = 528;     // padded LDS row stride: 16-byte writes of 16 lanes hit 16 bank groups

// CONV: the KBP values of one piece for the lane's window entry (fr, fs, channel; off = its offset from the corner pixel
// of a window) at the consecutive output positions from (img, oy, ox) on.  The position is the wave's: it walks on the
// scalar unit, and only the end of an output row costs more than a compare there - the row's corner pixel is then a new
// uniform base address and the lane's row check a new mask.  Inside a row the lane steps its own column and offset.
// FULL: all KBP positions exist.
template <int KBP, bool FULL>
__device__ __forceinline__ void conv_col_gather(const ColParams &p, uint32_t img, int y0, int x0, int oy, int ox, int blen, bool r_ok,
                                                int fr, int fs, int off, float (&v)[KBP]) {
    const int step = p.cv.str_w * p.cv.C;                                                 // elements per output column
    const float *corner = p.src + (((int64_t)img * p.cv.H + y0) * p.cv.W + x0) * p.cv.C; // may lie outside the tensor; uniform
    bool row_ok = r_ok && (unsigned)(y0 + fr) < (unsigned)p.cv.H;
    int xl = x0 + fs, offl = off;                                                         // the lane's input column and offset
#pragma unroll
    for (int kk = 0; kk < KBP; ++kk) {
        const bool inside = (FULL || kk < blen) && row_ok && (unsigned)xl < (unsigned)p.cv.W;
        v[kk] = inside ? corner[offl] : 0.0f;
        xl += p.cv.str_w;
        offl += step;
        if (++ox == p.cv.Wo) {                                                            // next output row, or next image
            ox = 0, y0 += p.cv.str_h;
            if (++oy == p.cv.Ho) oy = 0, y0 = -p.cv.pad_h, ++img;
            corner = p.src + (((int64_t)img * p.cv.H + y0) * p.cv.W - p.cv.pad_w) * p.cv.C;
            row_ok = r_ok && (unsigned)(y0 + fr) < (unsigned)p.cv.H;
            xl = fs - p.cv.pad_w, offl = off;
        }
    }
}

template <int KBP, bool WIDE, int ROUND, bool TABLE, bool CONV = false>
__global__ __launch_bounds__(kThreads) void enc_col_kernel(const ColParams p) {
    constexpr int ESZ = WIDE ? 2 : 1;
    constexpr int NBT = kColRowBytes / (KBP * ESZ);  // exponent blocks per tile row: 16, 8, 8 or 4
    __shared__ __attribute__((aligned(16))) uint8_t tile[64 * kColStride];
    __shared__ __attribute__((aligned(4))) uint8_t etile[64 * NBT];
    __shared__ uint32_t lane_amax[4][64];

    // the wave index as a scalar: block indices, block lengths and (CONV) output positions stay on the scalar unit
    const int t = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;
    const int64_t r = (int64_t)(blockIdx.x % p.row_groups) * p.lanes + lane;
    const int64_t blk0 = (int64_t)(blockIdx.x / p.row_groups) * NBT;
    const bool r_ok = lane < p.lanes && r < p.R;
    const int group0 = (lane / p.rblock) * p.rblock;   // first lane of this lane's 2-D tile
    int conv_fr = 0, conv_fs = 0, conv_ch = 0;          // CONV: this lane's filter tap and channel
    if (CONV) conv_window_entry(p.cv, r_ok ? (uint32_t)r : 0u, conv_fr, conv_fs, conv_ch);
    const int conv_off = CONV ? (conv_fr * p.cv.W + conv_fs) * p.cv.C + conv_ch : 0;    // of the lane's window entry from the corner

    for (int bi = wave; bi < NBT; bi += 4) {
        const int64_t piece = blk0 + bi;                                  // stored piece of KBP elements
        const int64_t blk = TABLE ? piece / p.spb : piece;                // exponent block
        const int sub = TABLE ? (int)(piece % p.spb) * KBP : 0;           // the piece's offset in its block
        int blen = 0;
        if (blk < p.nblk) {
            int64_t left = p.K - blk * p.kblock;
            left = (left < p.kblock ? left : p.kblock) - sub;
            blen = left < 0 ? 0 : (left < KBP ? (int)left : KBP);
        }
        const int64_t kfirst = (blk < p.nblk ? blk : 0) * p.kblock + (blen ? sub : 0);
        const float *s = p.src + kfirst * p.ld + (r_ok ? r : 0);
        float v[KBP];
        if (!CONV) {
#pragma unroll
            for (int kk = 0; kk < KBP; ++kk) v[kk] = (kk < blen && r_ok) ? s[(int64_t)kk * p.ld] : 0.0f;
        } else {
            // The output position is the same for the whole wave and walks on by one per element: it is decoded once
            // per piece and advanced on the scalar unit, and its corner pixel is a uniform base address; the lane adds
            // the offset of its own window entry, so the vector unit only checks the two coordinates.
            uint32_t img;
            int y0, x0, oy, ox;
            conv_position(p.cv, (uint32_t)kfirst, img, y0, x0, oy, ox);
            if (blen == KBP) conv_col_gather<KBP, true>(p, img, y0, x0, oy, ox, blen, r_ok, conv_fr, conv_fs, conv_off, v);
            else conv_col_gather<KBP, false>(p, img, y0, x0, oy, ox, blen, r_ok, conv_fr, conv_fs, conv_off, v);
        }
        uint32_t amax = 0;
#pragma unroll
        for (int kk = 0; kk < KBP; ++kk) amax = max(amax, __float_as_uint(v[kk]) & 0x7fffffffu);
        if (TABLE) {
            amax = (blk < p.nblk && r_ok)
                       ? p.table[(int64_t)((uint32_t)blk / (uint32_t)p.kshare) * p.ntc + (uint32_t)r / (uint32_t)p.rblock_t]
                       : 0u;                                              // rows and blocks fit 31 bits here
        } else if (p.rblock > 1) {
            // 2-D tile: the maximum also runs over the rblock neighbouring operand rows (lanes of this wave)
            lane_amax[wave][lane] = amax;
            __builtin_amdgcn_wave_barrier();
            for (int i = 0; i < p.rblock; ++i) amax = max(amax, lane_amax[wave][(group0 + i) & 63]);
            __builtin_amdgcn_wave_barrier();
        }
        const uint32_t Eb = block_exponent<ROUND>(amax, p.m);
        if (!TABLE) etile[lane * NBT + bi] = blk < p.nblk ? (uint8_t)Eb : (uint8_t)1;
        else if (sub == 0 && r_ok && blk < p.nblk) p.exps[r * p.exp_ld + blk] = (uint8_t)Eb;
        uint8_t *out = tile + lane * kColStride + bi * KBP * ESZ;
#pragma unroll
        for (int kk = 0; kk < KBP; kk += 8) {
            int q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint64_t idx = (uint64_t)(kfirst + kk + e) * (uint64_t)p.src_cols + (uint64_t)r;
                q[e] = quantise<ROUND>(v[kk + e], Eb, p.m, (uint32_t)idx, (uint32_t)(idx >> 32), p.s0, p.s1);
            }
            if (!WIDE) {
                uint2 o;
                o.x = pack4_i8(q[0], q[1], q[2], q[3]);
                o.y = pack4_i8(q[4], q[5], q[6], q[7]);
                *reinterpret_cast<uint2 *>(out + kk) = o;
            } else {
                uint4 o;
                o.x = pack2_i16(q[0], q[1]);
                o.y = pack2_i16(q[2], q[3]);
                o.z = pack2_i16(q[4], q[5]);
                o.w = pack2_i16(q[6], q[7]);
                *reinterpret_cast<uint4 *>(out + kk * 2) = o;
            }
        }
    }
    __syncthreads();

    // stored blocks of this tile that exist in the operand row
    const int64_t left_blocks = p.nb_stored - blk0;
    const int valid_bytes = (int)((left_blocks < NBT ? left_blocks : NBT) * KBP * ESZ);
    const int piece = t & 31;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
        const int rl = pass * 8 + (t >> 5);
        const int64_t rr = (int64_t)(blockIdx.x % p.row_groups) * p.lanes + rl;
        if (rl < p.lanes && rr < p.R && piece * 16 < valid_bytes) {
            const uint4 d = *reinterpret_cast<const uint4 *>(tile + rl * kColStride + piece * 16);
            typedef unsigned v4u __attribute__((ext_vector_type(4)));
            const v4u d4 = {d.x, d.y, d.z, d.w};
            __builtin_nontemporal_store(d4, reinterpret_cast<v4u *>(p.mant + (rr * p.kpad + blk0 * KBP) * ESZ + piece * 16));
        }
    }
    if (TABLE) {
        if (blk0 == 0 && t < 64 && r_ok)                                 // exponent bytes past the last block
            for (int64_t b = p.nblk; b < p.exp_ld; ++b) p.exps[r * p.exp_ld + b] = 1;
    } else if (t < 64 && r_ok) {
#pragma unroll
        for (int w = 0; w < NBT / 4; ++w) {
            const int64_t b = blk0 + 4 * w;
            if (b < p.exp_ld)
                *reinterpret_cast<uint32_t *>(p.exps + r * p.exp_ld + b) =
                    *reinterpret_cast<const uint32_t *>(etile + t * NBT + 4 * w);
        }
    }
}

template <int KBP>
void launch_col_k(const ColParams &p, dim3 grid, bool wide, int rounding, hipStream_t s) {
    if (!wide && rounding == 0) hipLaunchKernelGGL((enc_col_kernel<KBP, false, 0, false>), grid, dim3(kThreads), 0, s, p);
    else if (!wide) hipLaunchKernelGGL((enc_col_kernel<KBP, false, 1, false>), grid, dim3(kThreads), 0, s, p);
    else if (rounding == 0) hipLaunchKernelGGL((enc_col_kernel<KBP, true, 0, false>), grid, dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((enc_col_kernel<KBP, true, 1, false>), grid, dim3(kThreads), 0, s, p);
}

template <int KBP>
void launch_col_conv_k(const ColParams &p, dim3 grid, bool wide, int rounding, hipStream_t s) {
    if (!wide && rounding == 0) hipLaunchKernelGGL((enc_col_kernel<KBP, false, 0, false, true>), grid, dim3(kThreads), 0, s, p);
    else if (!wide) hipLaunchKernelGGL((enc_col_kernel<KBP, false, 1, false, true>), grid, dim3(kThreads), 0, s, p);
    else if (rounding == 0) hipLaunchKernelGGL((enc_col_kernel<KBP, true, 0, false, true>), grid, dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((enc_col_kernel<KBP, true, 1, false, true>), grid, dim3(kThreads), 0, s, p);
}

void launch_col_table(const ColParams &p, dim3 grid, bool wide, int rounding, hipStream_t s) {
    if (!wide && rounding == 0) hipLaunchKernelGGL((enc_col_kernel<32, false, 0, true>), grid, dim3(kThreads), 0, s, p);
    else if (!wide) hipLaunchKernelGGL((enc_col_kernel<32, false, 1, true>), grid, dim3(kThreads), 0, s, p);
    else if (rounding == 0) hipLaunchKernelGGL((enc_col_kernel<32, true, 0, true>), grid, dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((enc_col_kernel<32, true, 1, true>), grid, dim3(kThreads), 0, s, p);
}

// ------------------------------------------------------------------------------------------
// two-pass path: any block shape
struct TileParams {
    const float *src;
    uint32_t *tile_amax;   // [nbr][nbc] largest magnitude bit pattern per exponent block
    int64_t ld, src_rows, src_cols, br, bc, nbr, nbc;
};

__global__ __launch_bounds__(kThreads) void fill_u32_kernel(uint32_t *p, int64_t n, uint32_t v) {
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) p[i] = v;
}

// First pass of the two-pass conversion: the largest magnitude of every exponent block, any block shape.
// A workgroup covers kAmaxRows source rows x 1024 columns; a lane keeps the maxima of its 4 columns in
// registers down the rows of one row of blocks.  When all columns of a wave fall into one block the wave
// combines its lanes first and touches the table once; the max over unsigned bit patterns is order
// independent, so the atomics leave a deterministic result.
constexpr int kAmaxRows = 64;

// strip height: 64 rows; 8 when every row is a block of its own (no more atomics than with 64, more workgroups)
int amax_strip_rows(int64_t block_rows) { return block_rows == 1 ? 8 : kAmaxRows; }

__device__ __forceinline__ void amax_flush_wave(uint32_t v, uint32_t *slot) {
    v = group_max<16>(v);
    v = max(v, (uint32_t)__shfl_xor((int)v, 16));
    v = max(v, (uint32_t)__shfl_xor((int)v, 32));
    if ((threadIdx.x & 63) == 0 && v) atomicMax(slot, v);
}

__global__ __launch_bounds__(kThreads) void tile_amax_kernel(const TileParams p, int vec_ok, int strip_rows) {
    const int64_t c0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    int64_t tc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) tc[e] = ((c0 + e < p.src_cols) ? c0 + e : p.src_cols - 1) / p.bc;
    const int ncol = c0 >= p.src_cols ? 0 : (p.src_cols - c0 >= 4 ? 4 : (int)(p.src_cols - c0));
    const int64_t wave_tc = __shfl(tc[0], 0);
    const bool wave_one = __all(tc[0] == wave_tc && tc[3] == wave_tc);
    for (int64_t r0 = (int64_t)blockIdx.y * strip_rows; r0 < p.src_rows; r0 += (int64_t)gridDim.y * strip_rows) {
        const int64_t r1 = r0 + strip_rows < p.src_rows ? r0 + strip_rows : p.src_rows;
        if (p.br == 1 && wave_one && vec_ok && __all(ncol == 4)) {
            // one exponent block per row (and per wave): 8 rows in flight at a time instead of a load, a reduction
            // and an atomic in turn for every row
            for (int64_t r = r0; r < r1; r += 8) {
                float4 d[8];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    d[i] = *reinterpret_cast<const float4 *>(p.src + (r + i < r1 ? r + i : r1 - 1) * p.ld + c0);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if (r + i >= r1) break;
                    const uint32_t v = max(max(__float_as_uint(d[i].x) & 0x7fffffffu, __float_as_uint(d[i].y) & 0x7fffffffu),
                                           max(__float_as_uint(d[i].z) & 0x7fffffffu, __float_as_uint(d[i].w) & 0x7fffffffu));
                    amax_flush_wave(v, p.tile_amax + (r + i) * p.nbc + wave_tc);
                }
            }
            continue;
        }
        int64_t r = r0;
        int64_t tr = r0 / p.br, tile_end = (tr + 1) * p.br;              // one division per strip, none per row
        while (r < r1) {
            const int64_t rend = tile_end < r1 ? tile_end : r1;
            uint32_t a[4] = {0u, 0u, 0u, 0u};
            if (ncol == 4 && vec_ok) {
#pragma unroll 8
                for (int64_t rr = r; rr < rend; ++rr) {
                    const float4 d = *reinterpret_cast<const float4 *>(p.src + rr * p.ld + c0);
                    a[0] = max(a[0], __float_as_uint(d.x) & 0x7fffffffu);
                    a[1] = max(a[1], __float_as_uint(d.y) & 0x7fffffffu);
                    a[2] = max(a[2], __float_as_uint(d.z) & 0x7fffffffu);
                    a[3] = max(a[3], __float_as_uint(d.w) & 0x7fffffffu);
                }
            } else {
                for (int64_t rr = r; rr < rend; ++rr)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (e < ncol) a[e] = max(a[e], __float_as_uint(p.src[rr * p.ld + c0 + e]) & 0x7fffffffu);
            }
            r = rend;
            uint32_t *row_of_table = p.tile_amax + tr * p.nbc;
            if (rend == tile_end) {
                ++tr;
                tile_end += p.br;
            }
            if (wave_one) {
                amax_flush_wave(max(max(a[0], a[1]), max(a[2], a[3])), row_of_table + wave_tc);
            } else if (ncol) {
                // merge neighbours that fall into the same block before touching memory
                uint32_t run = a[0];
#pragma unroll
                for (int e = 1; e < 4; ++e) {
                    if (tc[e] == tc[e - 1]) {
                        run = max(run, a[e]);
                    } else {
                        if (run) atomicMax(row_of_table + tc[e - 1], run);
                        run = a[e];
                    }
                }
                if (run) atomicMax(row_of_table + tc[3], run);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// One wave per (operand row, exponent block), k contiguous in the source: exponent blocks of up to 64 * 8 * NV
// stored elements (one exponent per row of a matrix a few thousand columns wide, Sec. 4; with k_slot the stored
// blocks are shorter than the exponent block and repeat its exponent).  The wave holds the whole exponent block
// in registers, so the source is read once: all loads first, maximum across the wave, quantise, store.
struct WaveParams {
    const float *src;
    uint8_t *mant;
    uint8_t *exps;
    int64_t ld, R, K, kpad, exp_ld, src_cols;
    int32_t kblock, nblk, nb_stored, m;
    int32_t gp;            // 8-element chunks per stored block
    int32_t kshare;        // stored blocks per exponent block
    int32_t nreg;          // exponent blocks per row
    int32_t chunks;        // chunks per stored row
    int32_t vec_ok;
    uint32_t s0, s1;
};

template <bool WIDE, int ROUND, int NV>
__global__ __launch_bounds__(kThreads) void enc_rowwave_kernel(const WaveParams p) {
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);    // (row, exponent block)
    if (item >= p.R * p.nreg) return;                                                   // whole waves leave together
    const int64_t row = item / p.nreg;
    const int reg = (int)(item - row * p.nreg);
    // chunks of this exponent block; the last one also covers the padding blocks at the end of the stored row
    const int c_first = reg * p.kshare * p.gp;
    const int c_end = reg == p.nreg - 1 ? p.chunks : c_first + p.kshare * p.gp;
    const float *srow = p.src + row * p.ld;
    float v[NV][8];
    int cnt[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int cl = c_first + lane + 64 * i;
        const int blk = cl / p.gp, j = cl - blk * p.gp;
        int c = 0;
        if (cl < c_end && blk < p.nblk) {
            const int k0 = blk * p.kblock;
            const int blen = (p.K - k0 < p.kblock) ? (int)(p.K - k0) : p.kblock;
            const int left = blen - 8 * j;
            c = left <= 0 ? 0 : (left >= 8 ? 8 : left);
        }
        cnt[i] = c;
        const float *s = srow + (c ? (int64_t)blk * p.kblock + 8 * j : 0);
        if (c == 8 && p.vec_ok) {
            const float4 a = *reinterpret_cast<const float4 *>(s);
            const float4 b = *reinterpret_cast<const float4 *>(s + 4);
            v[i][0] = a.x; v[i][1] = a.y; v[i][2] = a.z; v[i][3] = a.w;
            v[i][4] = b.x; v[i][5] = b.y; v[i][6] = b.z; v[i][7] = b.w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[i][e] = (e < c) ? s[e] : 0.0f;
        }
    }
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) amax = max(amax, __float_as_uint(v[i][e]) & 0x7fffffffu);
    amax = group_max<16>(amax);
    amax = max(amax, (uint32_t)__shfl_xor((int)amax, 16));
    amax = max(amax, (uint32_t)__shfl_xor((int)amax, 32));
    const uint32_t Eb = block_exponent<ROUND>(amax, p.m);
    uint8_t *erow = p.exps + row * p.exp_ld;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int cl = c_first + lane + 64 * i;
        if (cl >= c_end) continue;
        const int blk = cl / p.gp, j = cl - blk * p.gp;
        int q[8];
        const uint64_t idx0 = (uint64_t)row * (uint64_t)p.src_cols + (uint64_t)((int64_t)blk * p.kblock + 8 * j);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint64_t idx = idx0 + e;
            q[e] = quantise<ROUND>(v[i][e], Eb, p.m, (uint32_t)idx, (uint32_t)(idx >> 32), p.s0, p.s1);
        }
        if (!WIDE) {
            uint2 o;
            o.x = pack4_i8(q[0], q[1], q[2], q[3]);
            o.y = pack4_i8(q[4], q[5], q[6], q[7]);
            store_stream(p.mant + row * p.kpad + (int64_t)cl * 8, o);
        } else {
            uint4 o;
            o.x = pack2_i16(q[0], q[1]);
            o.y = pack2_i16(q[2], q[3]);
            o.z = pack2_i16(q[4], q[5]);
            o.w = pack2_i16(q[6], q[7]);
            store_stream(p.mant + (row * p.kpad + (int64_t)cl * 8) * 2, o);
        }
        if (j == 0) {
            if (blk < p.exp_ld) erow[blk] = blk < p.nblk ? (uint8_t)Eb : (uint8_t)1;
            if (blk == p.nb_stored - 1)
                for (int64_t b = p.nb_stored; b < p.exp_ld; ++b) erow[b] = 1;
        }
    }
}

template <int NV>
void launch_rowwave_n(const WaveParams &p, dim3 grid, bool wide, int rounding, hipStream_t s) {
    if (!wide && rounding == 0) hipLaunchKernelGGL((enc_rowwave_kernel<false, 0, NV>), grid, dim3(kThreads), 0, s, p);
    else if (!wide) hipLaunchKernelGGL((enc_rowwave_kernel<false, 1, NV>), grid, dim3(kThreads), 0, s, p);
    else if (rounding == 0) hipLaunchKernelGGL((enc_rowwave_kernel<true, 0, NV>), grid, dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((enc_rowwave_kernel<true, 1, NV>), grid, dim3(kThreads), 0, s, p);
}

void magic_of(uint32_t d, uint32_t (&magic)[2]) {
    if (d == 1) {
        magic[0] = magic[1] = 0;
        return;
    }
    int l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    const unsigned __int128 two = (unsigned __int128)1 << (31 + l);
    magic[0] = (uint32_t)((two + d - 1) / d);
    magic[1] = (uint32_t)(l - 1);
}

// The same pass when one exponent block spans all columns (one exponent per row of a long row, per image, per band of
// rows, or for the whole matrix): a workgroup walks up to 16 chunks of 1024 columns, keeps one maximum per row of
// blocks and combines its four waves through LDS, so the table sees one atomic per workgroup and block row.
constexpr int kAmaxChunks = 16;

__global__ __launch_bounds__(kThreads) void tile_amax_wide_kernel(const TileParams p, int vec_ok, int strip_rows, int cpw) {
    __shared__ uint32_t wave_max[kThreads / 64];
    __shared__ uint32_t wave_max8[kThreads / 64][8];
    const int64_t cbase = ((int64_t)blockIdx.x * cpw * kThreads + threadIdx.x) * 4;
    for (int64_t r0 = (int64_t)blockIdx.y * strip_rows; r0 < p.src_rows; r0 += (int64_t)gridDim.y * strip_rows) {
        const int64_t r1 = r0 + strip_rows < p.src_rows ? r0 + strip_rows : p.src_rows;
        if (p.br == 1 && vec_ok) {
            // every row is a block row: 8 rows at a time, all of their loads in flight together, one exchange
            // through LDS for the 8 maxima
            for (int64_t r = r0; r < r1; r += 8) {
                uint32_t a8[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) a8[i] = 0;
                for (int cc = 0; cc < cpw; ++cc) {
                    const int64_t c0 = cbase + (int64_t)cc * kThreads * 4;
                    if (c0 + 3 < p.src_cols) {
                        float4 d[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            d[i] = *reinterpret_cast<const float4 *>(p.src + (r + i < r1 ? r + i : r1 - 1) * p.ld + c0);
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            a8[i] = max(a8[i], max(max(__float_as_uint(d[i].x) & 0x7fffffffu, __float_as_uint(d[i].y) & 0x7fffffffu),
                                                   max(__float_as_uint(d[i].z) & 0x7fffffffu, __float_as_uint(d[i].w) & 0x7fffffffu)));
                    } else {
                        for (int i = 0; i < 8 && r + i < r1; ++i)
                            for (int e = 0; e < 4; ++e)
                                if (c0 + e < p.src_cols) a8[i] = max(a8[i], __float_as_uint(p.src[(r + i) * p.ld + c0 + e]) & 0x7fffffffu);
                    }
                }
                __syncthreads();                               // the previous group's maxima have been read
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    uint32_t v = group_max<16>(a8[i]);
                    v = max(v, (uint32_t)__shfl_xor((int)v, 16));
                    v = max(v, (uint32_t)__shfl_xor((int)v, 32));
                    if ((threadIdx.x & 63) == 0) wave_max8[threadIdx.x >> 6][i] = v;
                }
                __syncthreads();
                if (threadIdx.x < 8 && r + threadIdx.x < r1) {
                    const int i = threadIdx.x;
                    const uint32_t v = max(max(wave_max8[0][i], wave_max8[1][i]), max(wave_max8[2][i], wave_max8[3][i]));
                    if (v) atomicMax(p.tile_amax + r + i, v);
                }
            }
            continue;
        }
        int64_t r = r0;
        int64_t tr = r0 / p.br, tile_end = (tr + 1) * p.br;
        while (r < r1) {
            const int64_t rend = tile_end < r1 ? tile_end : r1;
            uint32_t a = 0;
            for (int64_t rr = r; rr < rend; ++rr) {
                const float *srow = p.src + rr * p.ld;
#pragma unroll 4
                for (int cc = 0; cc < cpw; ++cc) {
                    const int64_t c0 = cbase + (int64_t)cc * kThreads * 4;
                    if (c0 + 3 < p.src_cols && vec_ok) {
                        const float4 d = *reinterpret_cast<const float4 *>(srow + c0);
                        a = max(a, max(max(__float_as_uint(d.x) & 0x7fffffffu, __float_as_uint(d.y) & 0x7fffffffu),
                                       max(__float_as_uint(d.z) & 0x7fffffffu, __float_as_uint(d.w) & 0x7fffffffu)));
                    } else {
                        for (int e = 0; e < 4; ++e)
                            if (c0 + e < p.src_cols) a = max(a, __float_as_uint(srow[c0 + e]) & 0x7fffffffu);
                    }
                }
            }
            r = rend;
            a = group_max<16>(a);
            a = max(a, (uint32_t)__shfl_xor((int)a, 16));
            a = max(a, (uint32_t)__shfl_xor((int)a, 32));
            __syncthreads();                                   // the previous block row's maxima have been read
            if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = a;
            __syncthreads();
            if (threadIdx.x == 0) {
                const uint32_t v = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
                if (v) atomicMax(p.tile_amax + tr, v);
            }
            if (rend == tile_end) {
                ++tr;
                tile_end += p.br;
            }
        }
    }
}

// The same pass once more for blocks that span all columns of a narrow matrix whose rows lie back to back in memory
// (ld = columns; an image tensor seen as [pixels][channels] with one exponent per image, say): a block row is one
// contiguous run of br * columns values.  The kernels above give a lane 4 columns and walk down the rows, which leaves
// most lanes without a column and one load in flight per lane here; this one reduces the run flat, 8 vector loads per
// lane in flight, one atomic per workgroup.  gridDim.x workgroups share a block row, gridDim.y strides over the block rows.
constexpr int kFlatLoads = 8;

__global__ __launch_bounds__(kThreads) void tile_amax_flat_kernel(const TileParams p) {
    __shared__ uint32_t wave_max[kThreads / 64];
    const int64_t per_tile = p.br * p.src_cols, total = p.src_rows * p.src_cols;
    for (int64_t tr = blockIdx.y; tr < p.nbr; tr += gridDim.y) {
        const int64_t begin = tr * per_tile, end = begin + per_tile < total ? begin + per_tile : total;
        uint32_t a = 0;
        for (int64_t base = begin + ((int64_t)blockIdx.x * kFlatLoads * kThreads + threadIdx.x) * 4; base < end;
             base += (int64_t)gridDim.x * kFlatLoads * kThreads * 4) {
            float4 d[kFlatLoads];
#pragma unroll
            for (int u = 0; u < kFlatLoads; ++u) {
                const int64_t i = base + (int64_t)u * kThreads * 4;               // runs are multiples of 4 values long
                d[u] = i < end ? *reinterpret_cast<const float4 *>(p.src + i) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
#pragma unroll
            for (int u = 0; u < kFlatLoads; ++u)
                a = max(a, max(max(__float_as_uint(d[u].x) & 0x7fffffffu, __float_as_uint(d[u].y) & 0x7fffffffu),
                               max(__float_as_uint(d[u].z) & 0x7fffffffu, __float_as_uint(d[u].w) & 0x7fffffffu)));
        }
        a = group_max<16>(a);
        a = max(a, (uint32_t)__shfl_xor((int)a, 16));
        a = max(a, (uint32_t)__shfl_xor((int)a, 32));
        __syncthreads();                                       // the previous block row's maxima have been read
        if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = a;
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t v = max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3]));
            if (v) atomicMax(p.tile_amax + tr, v);
        }
    }
}

// launches the maximum pass (the table has been cleared)
int launch_tile_amax(const TileParams &p, hipStream_t s) {
    const int vec_ok = (((uintptr_t)p.src & 15) == 0 && (p.ld % 4) == 0) ? 1 : 0;
    if (p.nbc == 1 && vec_ok && p.ld == p.src_cols && p.src_cols < kThreads * 4 && p.br >= 8) {
        const int64_t per_wg = (int64_t)kFlatLoads * kThreads * 4;
        int64_t gx = ceil_div(p.br * p.src_cols, per_wg);
        gx = gx > 64 ? 64 : gx;
        const int64_t gy = p.nbr > 65535 ? 65535 : p.nbr;
        hipLaunchKernelGGL(tile_amax_flat_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(kThreads), 0, s, p);
        return HBFP_OK;
    }
    const int strip = amax_strip_rows(p.br);
    int64_t gy = ceil_div(p.src_rows, strip);
    gy = gy > 65535 ? 65535 : gy;
    if (p.nbc == 1) {
        // chunks per workgroup: as many as still leave about a thousand workgroups
        const int64_t chunks = ceil_div(p.src_cols, kThreads * 4);
        int64_t want = chunks * gy / 1024;
        want = want < 1 ? 1 : (want > kAmaxChunks ? kAmaxChunks : want);
        const int cpw = (int)(want < chunks ? want : chunks);
        const int64_t gx = ceil_div(chunks, cpw);
        if (gx > 0x7fffffff) return HBFP_ERR_ARG;
        hipLaunchKernelGGL(tile_amax_wide_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(kThreads), 0, s, p, vec_ok, strip, cpw);
    } else {
        const int64_t gx = ceil_div(p.src_cols, kThreads * 4);
        if (gx > 0x7fffffff) return HBFP_ERR_ARG;
        hipLaunchKernelGGL(tile_amax_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(kThreads), 0, s, p, vec_ok, strip);
    }
    return HBFP_OK;
}

int ilog2_ceil(int64_t x) {
    int l = 0;
    while (((int64_t)1 << l) < x) ++l;
    return l;
}

}  // namespace

int launch_encode_row_fused(const float *src, const EncodeGeom &g, void *mant, uint8_t *exps, hipStream_t s) {
    RowParams p;
    p.src = src;
    p.mant = (uint8_t *)mant;
    p.exps = exps;
    p.ld = g.ld;
    p.R = g.R;
    p.K = g.K;
    p.kpad = g.kpad;
    p.exp_ld = g.exp_ld;
    p.src_cols = g.src_cols;
    p.kblock = (int32_t)g.kblock;
    p.nblk = (int32_t)g.nblk;
    p.nb_stored = (int32_t)(g.kpad / g.kbp);
    p.m = g.m;
    if (g.kpad / 8 > 0x7fffffff || g.nblk > 0x7fffffff) return HBFP_ERR_ARG;
    p.chunks = (int32_t)(g.kpad / 8);
    const int l2 = ilog2_ceil(p.chunks);
    p.lpr_log2 = (((int64_t)1 << l2) == p.chunks) ? l2 : -1;
    p.nseg = 0;
    p.vec_ok = (((uintptr_t)src & 15) == 0 && (g.ld % 4) == 0 && (g.kblock % 4) == 0) ? 1 : 0;
    p.sr_aligned = ((g.src_cols % 8) == 0 && (g.kblock % 8) == 0) ? 1 : 0;
    {
        const int per_wg = kThreads * 2;                                 // chunks of a stochastic-rounding workgroup (launch_row_t)
        p.one_row = (g.rounding && p.vec_ok && g.rblock <= 1 && p.chunks % per_wg == 0 && g.K < ((int64_t)1 << 30) && g.kpad < ((int64_t)1 << 30) &&
                     g.exp_ld < ((int64_t)1 << 31)) ? 1 : 0;
    }
    p.s0 = g.seed_lo;
    p.s1 = g.seed_hi;
    p.table = nullptr;
    p.rblock = 1;
    p.ntk = 0;
    p.gp = 0;
    p.kshare = 1;
    magic_of((uint32_t)p.chunks, p.dChunks);
    if (g.rblock > 1) {
        p.nseg = (int32_t)ceil_div(p.chunks, kThreads);
        const int64_t gx = ceil_div(g.R, g.rblock);
        const int64_t gy = p.nseg > 65535 ? 65535 : p.nseg;
        if (gx > 0x7fffffff || g.rblock > 0x7fffffff) return HBFP_ERR_ARG;
        const dim3 grid((unsigned)gx, (unsigned)gy);
        const bool wide = g.m > 8;
        if (g.kbp == 32) launch_row_tiled_g<4>(p, (int)g.rblock, grid, wide, g.rounding, s);
        else if (g.kbp == 64) launch_row_tiled_g<8>(p, (int)g.rblock, grid, wide, g.rounding, s);
        else if (g.kbp == 128) launch_row_tiled_g<16>(p, (int)g.rblock, grid, wide, g.rounding, s);
        else return HBFP_ERR_FORMAT;
        return launch_status();
    }
    const int64_t gx = ceil_div(g.R * (int64_t)p.chunks, (int64_t)kThreads * 4);
    if (gx > 0x3fffffff) return HBFP_ERR_ARG;                            // the stochastic-rounding launch doubles the grid
    const dim3 grid((unsigned)gx);
    const bool wide = g.m > 8;
    if (g.kbp == 32) launch_row_g<4>(p, grid, wide, g.rounding, s);
    else if (g.kbp == 64) launch_row_g<8>(p, grid, wide, g.rounding, s);
    else if (g.kbp == 128) launch_row_g<16>(p, grid, wide, g.rounding, s);
    else return HBFP_ERR_FORMAT;
    return launch_status();
}

static ConvGeom conv_geom(const hbfp_conv2d &c, int64_t ho, int64_t wo) {
    ConvGeom g;
    g.H = (int32_t)c.h;
    g.W = (int32_t)c.w;
    g.C = (int32_t)c.c;
    g.S = c.s;
    g.Ho = (int32_t)ho;
    g.Wo = (int32_t)wo;
    g.pad_h = c.pad_h;
    g.pad_w = c.pad_w;
    g.str_h = c.stride_h;
    g.str_w = c.stride_w;
    g.cbs = (c.c_block > 0 && c.c_block < c.c) ? c.c_block : (int32_t)c.c;
    g.per_blk = c.r * c.s * g.cbs;
    const int32_t full = g.C / g.cbs;                   // channel blocks of full width
    g.c_last = g.C - full * g.cbs;                      // 0: no shorter block at the end
    g.k_last = full * g.per_blk;
    if (g.c_last == 0) g.c_last = g.cbs;                // never used then (k < k_last always); keeps the division defined
    magic_of((uint32_t)g.per_blk, g.dPer);
    magic_of((uint32_t)g.cbs, g.dCb);
    magic_of((uint32_t)g.c_last, g.dCl);
    magic_of((uint32_t)c.s, g.dS);
    magic_of((uint32_t)(ho * wo), g.dP);
    magic_of((uint32_t)wo, g.dW);
    return g;
}

// The activation operand of a convolution, converted straight from the NHWC tensor (1-D blocks along k).
int launch_encode_im2col(const float *x, const hbfp_conv2d &c, int64_t ho, int64_t wo, const EncodeGeom &g, void *mant,
                         uint8_t *exps, uint32_t *table, hipStream_t s) {
    if (table) {
        // one exponent per image: largest magnitude of each image (the tensor as a matrix [n][h * w * c], one block per
        // row) into table[n]; the gather below then looks its exponent up there
        TileParams t;
        t.src = x;
        t.tile_amax = table;
        t.src_rows = c.n;
        t.src_cols = c.h * c.w * c.c;
        t.ld = t.src_cols;
        t.br = 1;
        t.bc = t.src_cols;
        t.nbr = c.n;
        t.nbc = 1;
        int64_t fb = ceil_div(c.n, kThreads);
        if (fb > 4096) fb = 4096;
        hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)fb), dim3(kThreads), 0, s, table, c.n, 0u);
        const int rc = launch_tile_amax(t, s);
        if (rc != HBFP_OK) return rc;
    }
    if (g.axis == 0) {
        // weight-gradient orientation: operand rows = (filter tap, channel), k = output positions
        ColParams p;
        p.src = x;
        p.mant = (uint8_t *)mant;
        p.exps = exps;
        p.ld = 0;
        p.R = g.R;
        p.K = g.K;
        p.kpad = g.kpad;
        p.exp_ld = g.exp_ld;
        p.src_cols = g.src_cols;
        if (g.nblk > 0x7fffffff || g.R > 0x7fffffff || g.K > 0x7fffffff) return HBFP_ERR_ARG;
        p.kblock = (int32_t)g.kblock;
        p.nblk = (int32_t)g.nblk;
        p.nb_stored = (int32_t)(g.kpad / g.kbp);
        p.m = g.m;
        p.s0 = g.seed_lo;
        p.s1 = g.seed_hi;
        p.rblock = 1;
        p.lanes = 64;
        p.table = nullptr;
        p.rblock_t = 1;
        p.ntc = 0;
        p.spb = 1;
        p.kshare = 1;
        p.cv = conv_geom(c, ho, wo);
        const bool wide = g.m > 8;
        const int nbt = kColRowBytes / ((int)g.kbp * (wide ? 2 : 1));
        const int64_t nb_cover = p.nb_stored > g.exp_ld ? p.nb_stored : g.exp_ld;
        const int64_t gx = ceil_div(g.R, 64), gy = ceil_div(nb_cover, nbt);
        if (gx > 0x7fffffff || gx * gy > 0x7fffffff) return HBFP_ERR_ARG;
        p.row_groups = (uint32_t)gx;
        const dim3 grid((unsigned)(gx * gy));
        if (g.kbp == 32) launch_col_conv_k<32>(p, grid, wide, g.rounding, s);
        else if (g.kbp == 64) launch_col_conv_k<64>(p, grid, wide, g.rounding, s);
        else return HBFP_ERR_FORMAT;
        return launch_status();
    }
    RowParams p;
    p.src = x;
    p.mant = (uint8_t *)mant;
    p.exps = exps;
    p.ld = 0;
    p.R = g.R;
    p.K = g.K;
    p.kpad = g.kpad;
    p.exp_ld = g.exp_ld;
    p.src_cols = g.src_cols;
    if (g.kpad / 8 > 0x7fffffff || g.nblk > 0x7fffffff || g.R > 0x7fffffff || g.K > 0x7fffffff) return HBFP_ERR_ARG;
    p.kblock = (int32_t)g.kblock;
    p.nblk = (int32_t)g.nblk;
    p.nb_stored = (int32_t)(g.kpad / g.kbp);
    p.m = g.m;
    p.chunks = (int32_t)(g.kpad / 8);
    const int l2 = ilog2_ceil(p.chunks);
    p.lpr_log2 = (((int64_t)1 << l2) == p.chunks) ? l2 : -1;
    p.nseg = 0;
    p.vec_ok = (((uintptr_t)x & 15) == 0) ? 1 : 0;                      // C is a multiple of 8
    p.sr_aligned = 0;
    p.one_row = 0;
    p.s0 = g.seed_lo;
    p.s1 = g.seed_hi;
    p.table = table;
    p.rblock = table ? g.rblock : 1;                                     // rows of one image
    p.ntk = 1;
    p.gp = (int32_t)(g.kbp / 8);
    p.kshare = (int32_t)g.nblk;
    magic_of((uint32_t)p.chunks, p.dChunks);
    magic_of((uint32_t)p.gp, p.dGp);
    magic_of((uint32_t)p.rblock, p.dR);
    magic_of((uint32_t)p.kshare, p.dK);
    p.cv = conv_geom(c, ho, wo);
    const int64_t gx = ceil_div(g.R * (int64_t)p.chunks, (int64_t)kThreads * 4);
    if (gx > 0x3fffffff) return HBFP_ERR_ARG;                            // the stochastic-rounding launch doubles the grid
    const dim3 grid((unsigned)gx);
    const bool wide = g.m > 8;
    if (table) launch_row_conv_g<0>(p, grid, wide, g.rounding, s);
    else if (g.kbp == 32) launch_row_conv_g<4>(p, grid, wide, g.rounding, s);
    else if (g.kbp == 64) launch_row_conv_g<8>(p, grid, wide, g.rounding, s);
    else if (g.kbp == 128) launch_row_conv_g<16>(p, grid, wide, g.rounding, s);
    else return HBFP_ERR_FORMAT;
    return launch_status();
}

int launch_encode_col_fused(const float *src, const EncodeGeom &g, void *mant, uint8_t *exps, hipStream_t s) {
    ColParams p;
    p.src = src;
    p.mant = (uint8_t *)mant;
    p.exps = exps;
    p.ld = g.ld;
    p.R = g.R;
    p.K = g.K;
    p.kpad = g.kpad;
    p.exp_ld = g.exp_ld;
    p.src_cols = g.src_cols;
    p.kblock = (int32_t)g.kblock;
    if (g.nblk > 0x7fffffff) return HBFP_ERR_ARG;
    p.nblk = (int32_t)g.nblk;
    p.nb_stored = (int32_t)(g.kpad / g.kbp);
    p.m = g.m;
    p.s0 = g.seed_lo;
    p.s1 = g.seed_hi;
    if (g.rblock < 1 || g.rblock > 64) return HBFP_ERR_FORMAT;
    p.rblock = (int32_t)g.rblock;
    p.lanes = (int32_t)((64 / g.rblock) * g.rblock);
    p.table = nullptr;
    p.rblock_t = 1;
    p.ntc = 0;
    p.spb = 1;
    p.kshare = 1;
    const bool wide = g.m > 8;
    const int nbt = kColRowBytes / ((int)g.kbp * (wide ? 2 : 1));
    // cover every stored block and every exponent byte up to exp_ld
    const int64_t nb_cover = p.nb_stored > g.exp_ld ? p.nb_stored : g.exp_ld;
    const int64_t gx = ceil_div(g.R, p.lanes), gy = ceil_div(nb_cover, nbt);
    if (gx > 0x7fffffff || gx * gy > 0x7fffffff) return HBFP_ERR_ARG;
    p.row_groups = (uint32_t)gx;
    const dim3 grid((unsigned)(gx * gy));
    if (g.kbp == 32) launch_col_k<32>(p, grid, wide, g.rounding, s);
    else if (g.kbp == 64) launch_col_k<64>(p, grid, wide, g.rounding, s);
    else return HBFP_ERR_FORMAT;
    return launch_status();
}

// Two passes for block shapes the single-pass kernels do not cover (long blocks, one exponent per row or column,
// large 2-D tiles, one exponent for the whole matrix): the largest magnitude of every block into a table, then the
// row / column kernels quantise with the exponents of the table (the second read mostly hits the last-level cache).
// Exponent blocks of one operand row each, short enough for the registers of a wave (k contiguous in the source).
static bool rowwave_ok(const EncodeGeom &g) {
    if (g.axis != 1 || g.rblock != 1 || g.kpad > 0x7fffffff || g.R > 0x7fffffff) return false;
    const int64_t gp = g.kbp / 8, nreg = ceil_div(g.nblk, g.kshare);
    // the last exponent block of a row also covers the padding blocks behind it
    const int64_t most = nreg == 1 ? g.kpad / 8 : max(g.kshare * gp, g.kpad / 8 - (nreg - 1) * g.kshare * gp);
    return most <= 64 * 16;
}

static int launch_encode_rowwave(const float *src, const EncodeGeom &g, void *mant, uint8_t *exps, hipStream_t s) {
    WaveParams p;
    p.src = src;
    p.mant = (uint8_t *)mant;
    p.exps = exps;
    p.ld = g.ld;
    p.R = g.R;
    p.K = g.K;
    p.kpad = g.kpad;
    p.exp_ld = g.exp_ld;
    p.src_cols = g.src_cols;
    p.kblock = (int32_t)g.kblock;
    p.nblk = (int32_t)g.nblk;
    p.nb_stored = (int32_t)(g.kpad / g.kbp);
    p.m = g.m;
    p.gp = (int32_t)(g.kbp / 8);
    p.kshare = (int32_t)(g.kshare > g.nblk ? g.nblk : g.kshare);
    p.nreg = (int32_t)ceil_div(g.nblk, g.kshare);
    p.chunks = (int32_t)(g.kpad / 8);
    p.vec_ok = (((uintptr_t)src & 15) == 0 && (g.ld % 4) == 0 && (g.kblock % 4) == 0) ? 1 : 0;
    p.s0 = g.seed_lo;
    p.s1 = g.seed_hi;
    const int64_t most = p.nreg == 1 ? p.chunks : max((int64_t)p.kshare * p.gp, p.chunks - (int64_t)(p.nreg - 1) * p.kshare * p.gp);
    const int64_t items = g.R * p.nreg, gx = ceil_div(items, kThreads / 64);
    if (gx > 0x7fffffff) return HBFP_ERR_ARG;
    const dim3 grid((unsigned)gx);
    const bool wide = g.m > 8;
    if (most <= 64 * 2) launch_rowwave_n<2>(p, grid, wide, g.rounding, s);
    else if (most <= 64 * 4) launch_rowwave_n<4>(p, grid, wide, g.rounding, s);
    else if (most <= 64 * 8) launch_rowwave_n<8>(p, grid, wide, g.rounding, s);
    else launch_rowwave_n<16>(p, grid, wide, g.rounding, s);
    return launch_status();
}

int launch_encode_generic(const float *src, const EncodeGeom &g, void *mant, uint8_t *exps,
                          uint32_t *tile_amax, hipStream_t s) {
    if (rowwave_ok(g)) return launch_encode_rowwave(src, g, mant, exps, s);
    const bool wide = g.m > 8;
    {
        TileParams p;
        p.src = src;
        p.tile_amax = tile_amax;
        p.ld = g.ld;
        p.src_rows = g.src_rows;
        p.src_cols = g.src_cols;
        p.br = g.br;
        p.bc = g.bc;
        p.nbr = g.nbr;
        p.nbc = g.nbc;
        const int64_t ntile = g.nbr * g.nbc;
        int64_t fb = ceil_div(ntile, kThreads);
        if (fb > 4096) fb = 4096;
        hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)fb), dim3(kThreads), 0, s, tile_amax, ntile, 0u);
        const int rc = launch_tile_amax(p, s);
        if (rc != HBFP_OK) return rc;
    }
    if (g.axis == 1) {
        RowParams p;
        p.src = src;
        p.mant = (uint8_t *)mant;
        p.exps = exps;
        p.ld = g.ld;
        p.R = g.R;
        p.K = g.K;
        p.kpad = g.kpad;
        p.exp_ld = g.exp_ld;
        p.src_cols = g.src_cols;
        if (g.kpad / 8 > 0x7fffffff || g.nblk > 0x7fffffff || g.kblock > 0x7fffffff || g.R > 0x7fffffff) return HBFP_ERR_ARG;
        p.kblock = (int32_t)g.kblock;
        p.nblk = (int32_t)g.nblk;
        p.nb_stored = (int32_t)(g.kpad / g.kbp);
        p.m = g.m;
        p.chunks = (int32_t)(g.kpad / 8);
        const int l2 = ilog2_ceil(p.chunks);
        p.lpr_log2 = (((int64_t)1 << l2) == p.chunks) ? l2 : -1;
        p.nseg = 0;
        p.vec_ok = (((uintptr_t)src & 15) == 0 && (g.ld % 4) == 0 && (g.kblock % 4) == 0) ? 1 : 0;
        p.sr_aligned = ((g.src_cols % 8) == 0 && (g.kblock % 8) == 0) ? 1 : 0;
        p.one_row = 0;
        p.s0 = g.seed_lo;
        p.s1 = g.seed_hi;
        p.table = tile_amax;
        p.rblock = g.rblock;
        p.ntk = g.nbc;
        p.gp = (int32_t)(g.kbp / 8);
        p.kshare = (int32_t)(g.kshare > g.nblk ? g.nblk : g.kshare);
        if (g.rblock > 0x7fffffff) return HBFP_ERR_ARG;
        magic_of((uint32_t)p.chunks, p.dChunks);
        magic_of((uint32_t)p.gp, p.dGp);
        magic_of((uint32_t)p.rblock, p.dR);
        magic_of((uint32_t)p.kshare, p.dK);
        const int64_t gx = ceil_div(g.R * (int64_t)p.chunks, (int64_t)kThreads * 4);
        if (gx > 0x3fffffff) return HBFP_ERR_ARG;
        launch_row_g<0>(p, dim3((unsigned)gx), wide, g.rounding, s);
    } else {
        ColParams p;
        p.src = src;
        p.mant = (uint8_t *)mant;
        p.exps = exps;
        p.ld = g.ld;
        p.R = g.R;
        p.K = g.K;
        p.kpad = g.kpad;
        p.exp_ld = g.exp_ld;
        p.src_cols = g.src_cols;
        if (g.nblk > 0x7fffffff || g.kblock > 0x7fffffff || g.kpad / 32 > 0x7fffffff || g.R > 0x7fffffff) return HBFP_ERR_ARG;
        p.kblock = (int32_t)g.kblock;
        p.nblk = (int32_t)g.nblk;
        p.nb_stored = (int32_t)(g.kpad / 32);                       // stored pieces of 32 elements
        p.m = g.m;
        p.s0 = g.seed_lo;
        p.s1 = g.seed_hi;
        p.rblock = 1;
        p.lanes = 64;
        p.table = tile_amax;
        p.rblock_t = g.rblock;
        p.ntc = g.nbc;
        p.spb = (int32_t)(g.kbp / 32);
        p.kshare = (int32_t)(g.kshare > g.nblk ? g.nblk : g.kshare);
        const int nbt = kColRowBytes / (32 * (wide ? 2 : 1));
        const int64_t gx = ceil_div(g.R, 64), gy = ceil_div(p.nb_stored, nbt);
        if (gx > 0x7fffffff || gx * gy > 0x7fffffff) return HBFP_ERR_ARG;
        p.row_groups = (uint32_t)gx;
        launch_col_table(p, dim3((unsigned)(gx * gy)), wide, g.rounding, s);
    }
    return launch_status();
}

}  // namespace hbfp
