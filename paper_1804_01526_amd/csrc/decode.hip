// BFP -> FP32, Eq. (1) of Sec. 4: value = mantissa * 2^(Eb - 125 - mant_bits).
// int -> float of a mantissa of at most 16 bits is exact and so is the power-of-two
// scaling (ldexp, subnormal results included), so decode is exact.
// With AXPY the decoded value is the stored weight of an update step (Sec. 4.2 "Wide weight
// storage"): dst = fma(alpha, delta, value), one FP32 rounding.
#include "hbfp_internal.h"

namespace hbfp {
namespace {

constexpr int kThreads = 256;

struct DecParams {
    const uint8_t *mant;
    const uint8_t *exps;
    float *dst;
    const float *delta;          // AXPY only: FP32 [src_rows][ldd]
    int64_t ldd;
    float alpha;
    int64_t ld, src_rows, src_cols, R, K, kblock, kbp, nblk, kpad, exp_ld;
    int32_t axis, m;
    int32_t chunks, lpr_log2, nseg, vec_ok, gp;
    uint32_t dGp[2];             // division by gp (chunks per stored block) as multiply-high + shift
};

// n / d for 0 <= n < 2^31: with l = ceil(log2 d) and m = ceil(2^(31 + l) / d), floor(n * m / 2^(31 + l)) = floor(n / d)
// (round-up method of Granlund and Montgomery); magic[0] = m, magic[1] = l - 1, d = 1 is stored as m = 0.
__device__ __forceinline__ uint32_t div_magic(uint32_t n, const uint32_t (&magic)[2]) {
    return magic[0] ? __umulhi(n, magic[0]) >> magic[1] : n;
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

// row path: k is contiguous in the destination.  A lane turns 4 stored mantissas into one 16-byte store, so a wave
// writes 1 KB of consecutive floats per instruction; it handles kUnroll such chunks per pass, all of their loads
// issued before the first conversion (chunks that do not exist read chunk 0 of the row and store nothing).
// The output is written once and not read again by this kernel: streaming stores.
constexpr int kUnroll = 4;
typedef float v4f __attribute__((ext_vector_type(4)));

template <bool WIDE, bool AXPY>
__global__ __launch_bounds__(kThreads) void dec_row_kernel(const DecParams p) {
    const int t = threadIdx.x;
    const int lpr = 1 << p.lpr_log2;
    const int64_t row = (int64_t)blockIdx.x * (kThreads >> p.lpr_log2) + (t >> p.lpr_log2);
    if (row >= p.R) return;
    const int lr = t & (lpr - 1);
    const uint8_t *mrow = p.mant + row * p.kpad * (WIDE ? 2 : 1);
    const uint8_t *erow = p.exps + row * p.exp_ld;
    for (int seg0 = blockIdx.y * kUnroll; seg0 < p.nseg; seg0 += gridDim.y * kUnroll) {
        uint32_t raw[kUnroll][2];
        int ue[kUnroll], cnt[kUnroll];
        int64_t at[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t cl = (int64_t)(seg0 + u) * lpr + lr;                  // < 2^31: the launcher checks
            const int64_t blk = div_magic((uint32_t)cl, p.dGp);
            const int j = (int)(cl - blk * p.gp);
            int c = 0;
            if (seg0 + u < p.nseg && cl < p.chunks && blk < p.nblk) {
                const int64_t k0 = blk * p.kblock;
                const int64_t left = ((p.K - k0 < p.kblock) ? (p.K - k0) : p.kblock) - 4 * j;
                c = left >= 4 ? 4 : (left > 0 ? (int)left : 0);
            }
            cnt[u] = c;
            at[u] = blk * p.kblock + 4 * j;
            const int64_t cs = c ? cl : 0, bs = c ? blk : 0;
            if (!WIDE) {
                raw[u][0] = *reinterpret_cast<const uint32_t *>(mrow + cs * 4);
                raw[u][1] = 0;
            } else {
                const uint2 d = *reinterpret_cast<const uint2 *>(mrow + cs * 8);
                raw[u][0] = d.x;
                raw[u][1] = d.y;
            }
            ue[u] = (int)erow[bs] - 125 - p.m;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (cnt[u] == 0) continue;
            int q[4];
            if (!WIDE) {
#pragma unroll
                for (int e = 0; e < 4; ++e) q[e] = (int)(int8_t)(raw[u][0] >> (8 * e));
            } else {
                q[0] = (int)(int16_t)(raw[u][0] & 0xffffu);
                q[1] = (int)(int16_t)(raw[u][0] >> 16);
                q[2] = (int)(int16_t)(raw[u][1] & 0xffffu);
                q[3] = (int)(int16_t)(raw[u][1] >> 16);
            }
            float f[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) f[e] = __builtin_amdgcn_ldexpf((float)q[e], ue[u]);
            float *o = p.dst + row * p.ld + at[u];
            const bool vec = cnt[u] == 4 && p.vec_ok;
            if (AXPY) {
                const float *g = p.delta + row * p.ldd + at[u];
                if (vec) {
                    const float4 g0 = *reinterpret_cast<const float4 *>(g);
                    f[0] = fmaf(p.alpha, g0.x, f[0]);
                    f[1] = fmaf(p.alpha, g0.y, f[1]);
                    f[2] = fmaf(p.alpha, g0.z, f[2]);
                    f[3] = fmaf(p.alpha, g0.w, f[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (e < cnt[u]) f[e] = fmaf(p.alpha, g[e], f[e]);
                }
            }
            if (vec) {
                v4f o4;
                o4.x = f[0]; o4.y = f[1]; o4.z = f[2]; o4.w = f[3];
                __builtin_nontemporal_store(o4, reinterpret_cast<v4f *>(o));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (e < cnt[u]) o[e] = f[e];
            }
        }
    }
}

// column path: k runs down the rows of the destination (operand row r is destination column r).  A workgroup
// takes 64 operand rows x 64 stored positions: whole 64-byte (128-byte for 16-bit mantissas) row pieces are read,
// turned in LDS, and every wave instruction then writes 64 consecutive floats of one destination row.
constexpr int kColTileRows = 64, kColTileK = 64;

template <bool WIDE, bool AXPY>
__global__ __launch_bounds__(kThreads) void dec_col_kernel(const DecParams p) {
    constexpr int ESZ = WIDE ? 2 : 1;
    constexpr int kStride = kColTileK * ESZ + 4;                  // bytes per operand row in LDS: lanes 17 / 33 words apart
    __shared__ __attribute__((aligned(16))) uint8_t tile[kColTileRows * kStride];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int64_t r0 = (int64_t)blockIdx.x * kColTileRows, s0 = (int64_t)blockIdx.y * kColTileK;   // stored position
    {   // load: thread -> (row, 16-byte piece); 4 (8) pieces per row
        constexpr int PPR = kColTileK * ESZ / 16;
#pragma unroll
        for (int i = 0; i < PPR / 4; ++i) {
            const int idx = t + i * kThreads, row = idx / PPR, piece = idx % PPR;
            uint4 d = make_uint4(0u, 0u, 0u, 0u);
            if (r0 + row < p.R) d = *reinterpret_cast<const uint4 *>(p.mant + ((r0 + row) * p.kpad + s0) * ESZ + piece * 16);
            uint32_t *l = reinterpret_cast<uint32_t *>(tile + row * kStride + piece * 16);
            l[0] = d.x; l[1] = d.y; l[2] = d.z; l[3] = d.w;
        }
    }
    __syncthreads();
    const int64_t r = r0 + lane;                                  // this lane's operand row = destination column
    if (r >= p.R) return;
    // wave w converts stored positions 4 (w + 4 i) .. + 3, i = 0..3; a group of 4 never leaves its stored block
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int g4 = 4 * (wave + 4 * i);
        const int64_t sp = s0 + g4;
        const int64_t blk = (uint32_t)sp / (uint32_t)p.kbp;      // stored positions fit 31 bits: the launcher checks
        const int kk = (int)(sp - blk * p.kbp);
        if (blk >= p.nblk || kk >= p.kblock) continue;
        const int ue = (int)p.exps[r * p.exp_ld + blk] - 125 - p.m;
        int q[4];
        if (!WIDE) {
            const uint32_t w = *reinterpret_cast<const uint32_t *>(tile + lane * kStride + g4);
#pragma unroll
            for (int e = 0; e < 4; ++e) q[e] = (int)(int8_t)(w >> (8 * e));
        } else {
            const uint32_t w0 = *reinterpret_cast<const uint32_t *>(tile + lane * kStride + g4 * 2);
            const uint32_t w1 = *reinterpret_cast<const uint32_t *>(tile + lane * kStride + g4 * 2 + 4);
            q[0] = (int)(int16_t)(w0 & 0xffffu);
            q[1] = (int)(int16_t)(w0 >> 16);
            q[2] = (int)(int16_t)(w1 & 0xffffu);
            q[3] = (int)(int16_t)(w1 >> 16);
        }
        const int64_t k = blk * p.kblock + kk;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (kk + e >= p.kblock || k + e >= p.K) break;
            float f = __builtin_amdgcn_ldexpf((float)q[e], ue);
            if (AXPY) f = fmaf(p.alpha, p.delta[(k + e) * p.ldd + r], f);
            __builtin_nontemporal_store(f, p.dst + (k + e) * p.ld + r);      // written once, not read again here
        }
    }
}

// any orientation: one thread per destination element
template <bool WIDE, bool AXPY>
__global__ __launch_bounds__(kThreads) void dec_any_kernel(const DecParams p) {
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (c >= p.src_cols) return;
    for (int64_t r = blockIdx.y; r < p.src_rows; r += gridDim.y) {
        const int64_t ro = p.axis == 1 ? r : c, k = p.axis == 1 ? c : r;
        const int64_t blk = k / p.kblock, kk = k % p.kblock;
        const int64_t off = ro * p.kpad + blk * p.kbp + kk;
        const int q = WIDE ? (int)reinterpret_cast<const int16_t *>(p.mant)[off]
                           : (int)reinterpret_cast<const int8_t *>(p.mant)[off];
        const int ue = (int)p.exps[ro * p.exp_ld + blk] - 125 - p.m;
        float f = __builtin_amdgcn_ldexpf((float)q, ue);
        if (AXPY) f = fmaf(p.alpha, p.delta[r * p.ldd + c], f);
        p.dst[r * p.ld + c] = f;
    }
}

}  // namespace

int launch_decode_axpy(const hbfp_tensor *t, float *dst, int64_t ld, const float *delta, int64_t ldd, float alpha,
                       hipStream_t s) {
    DecParams p;
    p.delta = delta;
    p.ldd = ldd;
    p.alpha = alpha;
    const bool axpy = delta != nullptr;
    p.mant = (const uint8_t *)t->mant;
    p.exps = t->exps;
    p.dst = dst;
    p.ld = ld;
    p.src_rows = t->src_rows;
    p.src_cols = t->src_cols;
    p.R = t->rows;
    p.K = t->kdim;
    p.kblock = t->kblock;
    p.kbp = t->kblock_pad;
    p.nblk = t->nblk;
    p.kpad = t->kpad;
    p.exp_ld = t->exp_ld;
    p.axis = t->contract_axis;
    p.m = t->mant_bits;
    p.chunks = p.lpr_log2 = p.nseg = p.vec_ok = p.gp = 0;
    p.dGp[0] = p.dGp[1] = 0;
    const bool wide = t->mant_bits > 8;
    const bool row_path = t->contract_axis == 1 && t->kpad / 4 + 256 <= 0x7fffffff && t->nblk <= 0x7fffffff;
    const bool col_path = t->contract_axis == 0 && t->kpad <= 0x7fffffff && t->kpad / kColTileK <= 65535 && t->rows <= 0x7fffffff;
    if (row_path) {
        p.chunks = (int32_t)(t->kpad / 4);
        int l2 = 0;
        while (((int64_t)1 << l2) < p.chunks) ++l2;
        l2 = l2 < 4 ? 4 : (l2 > 8 ? 8 : l2);
        p.lpr_log2 = l2;
        p.nseg = (int32_t)ceil_div(p.chunks, (int64_t)1 << l2);
        p.gp = (int32_t)(t->kblock_pad / 4);
        magic_of((uint32_t)p.gp, p.dGp);
        p.vec_ok = (((uintptr_t)dst & 15) == 0 && (ld % 4) == 0 && (t->kblock % 4) == 0) ? 1 : 0;
        if (axpy && (((uintptr_t)delta & 15) != 0 || (ldd % 4) != 0)) p.vec_ok = 0;
        const int64_t gx = ceil_div(t->rows, (int64_t)(kThreads >> l2));
        int64_t gy = ceil_div(p.nseg, kUnroll);
        gy = gy > 65535 ? 65535 : gy;
        if (gx > 0x7fffffff) return HBFP_ERR_ARG;
        const dim3 grid((unsigned)gx, (unsigned)gy);
        if (axpy) {
            if (wide) hipLaunchKernelGGL((dec_row_kernel<true, true>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((dec_row_kernel<false, true>), grid, dim3(kThreads), 0, s, p);
        } else {
            if (wide) hipLaunchKernelGGL((dec_row_kernel<true, false>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((dec_row_kernel<false, false>), grid, dim3(kThreads), 0, s, p);
        }
    } else if (col_path) {
        const int64_t gx = ceil_div(t->rows, kColTileRows), gy = t->kpad / kColTileK;      // kpad is a multiple of 128
        if (gx > 0x7fffffff) return HBFP_ERR_ARG;
        const dim3 grid((unsigned)gx, (unsigned)gy);
        if (axpy) {
            if (wide) hipLaunchKernelGGL((dec_col_kernel<true, true>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((dec_col_kernel<false, true>), grid, dim3(kThreads), 0, s, p);
        } else {
            if (wide) hipLaunchKernelGGL((dec_col_kernel<true, false>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((dec_col_kernel<false, false>), grid, dim3(kThreads), 0, s, p);
        }
    } else {
        const int64_t gx = ceil_div(t->src_cols, kThreads);
        int64_t gy = t->src_rows > 65535 ? 65535 : t->src_rows;
        if (gx > 0x7fffffff) return HBFP_ERR_ARG;
        const dim3 grid((unsigned)gx, (unsigned)gy);
        if (axpy) {
            if (wide) hipLaunchKernelGGL((dec_any_kernel<true, true>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((dec_any_kernel<false, true>), grid, dim3(kThreads), 0, s, p);
        } else {
            if (wide) hipLaunchKernelGGL((dec_any_kernel<true, false>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((dec_any_kernel<false, false>), grid, dim3(kThreads), 0, s, p);
        }
    }
    return launch_status();
}

int launch_decode(const hbfp_tensor *t, float *dst, int64_t ld, hipStream_t s) {
    return launch_decode_axpy(t, dst, ld, nullptr, 0, 0.0f, s);
}

}  // namespace hbfp
