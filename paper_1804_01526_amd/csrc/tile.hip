// 2-D exponent tiles of at most 32 x 32 (Sec. 4.2 "Tiling": weight matrices are cut into tiles that
// share an exponent; the paper uses 24 x 24), converted in one pass with the tile held in registers.
//
// A lane owns 4 neighbouring source columns of one tile and walks down the tile's rows (up to 32 rows:
// up to 128 values in registers); the 8 lanes of a tile combine their maxima with three DPP steps.  From
// there the same values can be written in any of the operand layouts of the public header:
//   contraction along the source rows' direction (axis 1): 4 mantissas per lane and row, one store each;
//   contraction down the source rows (axis 0): a lane's column of a tile is 32 consecutive mantissas of
//   one operand row - the transposition itself is free.  The four tile rows a workgroup covers make up
//   whole 128-byte lines of that layout; 8-bit outputs are gathered in LDS and stored as full lines.
// The input is either an FP32 matrix (plain conversion, Sec. 4.1) or weights stored with wide mantissas
// plus an FP32 step (Sec. 4.2 "Wide weight storage", Sec. 5.1): w' = fma(alpha, step, value(wide)),
// converted to up to three outputs (the wide copy in place and the narrow operand layouts) while w' never
// leaves the registers.
#include "bfp_device.h"
#include "hbfp_internal.h"

namespace hbfp {
namespace {

constexpr int kThreads = 256;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t max_of_8_lanes(uint32_t v) {
    v = max(v, dpp_u32<0xB1>(v));    // quad_perm [1,0,3,2]
    v = max(v, dpp_u32<0x4E>(v));    // quad_perm [2,3,0,1]
    v = max(v, dpp_u32<0x141>(v));   // row_half_mirror: the other quad of the 8
    return v;
}
__device__ __forceinline__ uint32_t pack4_i8(int a, int b, int c, int d) {
    return (uint32_t)(a & 0xff) | ((uint32_t)(b & 0xff) << 8) | ((uint32_t)(c & 0xff) << 16) | ((uint32_t)d << 24);
}
__device__ __forceinline__ uint32_t pack2_i16(int a, int b) { return (uint32_t)(a & 0xffff) | ((uint32_t)b << 16); }

struct TileOut {
    uint8_t *mant;
    uint8_t *exps;
    int64_t kpad, exp_ld;
    int32_t m, axis, present;
    int32_t ntile_k;      // stored 32-element blocks along this output's contraction axis = kpad / 32
    uint32_t s0, s1;
};

struct TileParams {
    const float *src;     // FP32 [rows][ld]: the matrix to convert, or the step of a weight update
    int64_t ld;
    float alpha;
    const uint8_t *w_mant;   // weight update: stored weights, contraction axis 1, same tiles; else null
    const uint8_t *w_exps;
    int64_t w_kpad, w_expld;
    int32_t w_m;
    int64_t rows, cols;
    int32_t br, bc, nbr, nbc;
    TileOut o[3];
};

constexpr int kLineStride = 144;   // a 128-byte line of a transposed output in LDS, padded against bank conflicts

template <int BR, int ROUND>
__global__ __launch_bounds__(kThreads) void tile_kernel(const TileParams p) {
    __shared__ __attribute__((aligned(16))) uint8_t lines[256 * kLineStride];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 7;
    // a workgroup takes 8 tile columns x 4 tile rows (one tile row per wave): the four 32-byte pieces of a
    // 128-byte line of a transposed output are then written at about the same time and merge in L2
    const int64_t tc = (int64_t)blockIdx.x * 8 + (lane >> 3);
    const int64_t tr = (int64_t)blockIdx.y * 4 + wave;
    const int64_t row0 = tr * p.br, col0 = tc * p.bc + 4 * j;
    const bool col_ok = tc < p.nbc && 4 * j < p.bc && col0 < p.cols;       // cols and bc are multiples of 4
    int br_eff = 0;
    if (tr < p.nbr) br_eff = (int)((p.rows - row0) < p.br ? (p.rows - row0) : p.br);

    float v[BR][4];
    int we = 0;
    if (p.w_mant && col_ok && br_eff > 0) we = (int)p.w_exps[row0 * p.w_expld + tc] - 125 - p.w_m;
#pragma unroll
    for (int r = 0; r < BR; ++r) {
        v[r][0] = v[r][1] = v[r][2] = v[r][3] = 0.0f;
        if (r < br_eff && col_ok) {
            const float4 d = *reinterpret_cast<const float4 *>(p.src + (row0 + r) * p.ld + col0);
            if (p.w_mant) {
                const uint32_t *wp = reinterpret_cast<const uint32_t *>(p.w_mant + ((row0 + r) * p.w_kpad + tc * 32 + 4 * j) * 2);
                const uint32_t w01 = wp[0], w23 = wp[1];
                v[r][0] = fmaf(p.alpha, d.x, __builtin_amdgcn_ldexpf((float)(int16_t)(w01 & 0xffffu), we));
                v[r][1] = fmaf(p.alpha, d.y, __builtin_amdgcn_ldexpf((float)(int16_t)(w01 >> 16), we));
                v[r][2] = fmaf(p.alpha, d.z, __builtin_amdgcn_ldexpf((float)(int16_t)(w23 & 0xffffu), we));
                v[r][3] = fmaf(p.alpha, d.w, __builtin_amdgcn_ldexpf((float)(int16_t)(w23 >> 16), we));
            } else {
                v[r][0] = d.x; v[r][1] = d.y; v[r][2] = d.z; v[r][3] = d.w;
            }
        }
    }
    uint32_t amax = 0;
#pragma unroll
    for (int r = 0; r < BR; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) amax = max(amax, __float_as_uint(v[r][e]) & 0x7fffffffu);
    amax = max_of_8_lanes(amax);

    for (int oi = 0; oi < 3; ++oi) {
        const TileOut &o = p.o[oi];
        if (!o.present) continue;
        const uint32_t Eb = block_exponent<ROUND>(amax, o.m);
        const bool wide = o.m > 8;
        // element (row0 + r, col0 + e) of the source; the stochastic-rounding counter is its logical index
        auto q = [&](int r, int e) -> int {
            const uint64_t idx = (uint64_t)(row0 + r) * (uint64_t)p.cols + (uint64_t)(col0 + e);
            return quantise<ROUND>(v[r][e], Eb, o.m, (uint32_t)idx, (uint32_t)(idx >> 32), o.s0, o.s1);
        };
        if (o.axis == 1) {
            // operand row = source row; block tc of it holds this tile's columns (lanes without columns write the zero padding)
            if (tc < o.ntile_k) {
#pragma unroll
                for (int r = 0; r < BR; ++r) {
                    if (r >= br_eff) continue;
                    uint8_t *dst = o.mant + ((row0 + r) * o.kpad + tc * 32 + 4 * j) * (wide ? 2 : 1);
                    if (!wide) *reinterpret_cast<uint32_t *>(dst) = pack4_i8(q(r, 0), q(r, 1), q(r, 2), q(r, 3));
                    else *reinterpret_cast<uint2 *>(dst) = make_uint2(pack2_i16(q(r, 0), q(r, 1)), pack2_i16(q(r, 2), q(r, 3)));
                }
            }
            if (tc < o.exp_ld) {
                const uint8_t eb = tc < p.nbc ? (uint8_t)Eb : (uint8_t)1;
                for (int r = j; r < br_eff; r += 8) o.exps[(row0 + r) * o.exp_ld + tc] = eb;
            }
        } else {
            // operand row = source column; block tr of it holds this tile's rows: 32 consecutive mantissas per column
            if (!wide) {
                // the four waves (tile rows 4 by .. 4 by + 3) fill [column][4 x 32 bytes], then every 8 threads store one line
                const int64_t tr0 = (int64_t)blockIdx.y * 4, tc0 = (int64_t)blockIdx.x * 8;
                __syncthreads();                      // the previous output's lines have been read
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    uint32_t w[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        w[k] = 4 * k < BR ? pack4_i8(4 * k + 0 < BR ? q(4 * k + 0, e) : 0, 4 * k + 1 < BR ? q(4 * k + 1, e) : 0,
                                                     4 * k + 2 < BR ? q(4 * k + 2, e) : 0, 4 * k + 3 < BR ? q(4 * k + 3, e) : 0)
                                          : 0u;
                    uint8_t *l = lines + ((lane >> 3) * 32 + 4 * j + e) * kLineStride + wave * 32;
                    *reinterpret_cast<uint4 *>(l) = make_uint4(w[0], w[1], w[2], w[3]);
                    *reinterpret_cast<uint4 *>(l + 16) = make_uint4(w[4], w[5], w[6], w[7]);
                }
                __syncthreads();
                if (tr0 < o.ntile_k) {                // ntile_k is a multiple of 4: all four tile rows are stored or none
                    for (int g = threadIdx.x; g < 256 * 8; g += kThreads) {
                        const int lc = g >> 3, ch = g & 7;
                        const int64_t tcc = tc0 + (lc >> 5), c = tcc * p.bc + (lc & 31);
                        if (tcc < p.nbc && (lc & 31) < p.bc && c < p.cols)
                            *reinterpret_cast<uint4 *>(o.mant + c * o.kpad + tr0 * 32 + ch * 16) =
                                *reinterpret_cast<const uint4 *>(lines + lc * kLineStride + ch * 16);
                    }
                }
                if (col_ok && tr < o.exp_ld) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) o.exps[(col0 + e) * o.exp_ld + tr] = tr < p.nbr ? (uint8_t)Eb : (uint8_t)1;
                }
            } else if (col_ok) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (tr < o.ntile_k) {
                        uint8_t *dst = o.mant + ((col0 + e) * o.kpad + tr * 32) * 2;
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            uint32_t w[4];
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const int r0 = 8 * g + 2 * k;
                                w[k] = r0 < BR ? pack2_i16(q(r0, e), r0 + 1 < BR ? q(r0 + 1, e) : 0) : 0u;
                            }
                            *reinterpret_cast<uint4 *>(dst + 16 * g) = make_uint4(w[0], w[1], w[2], w[3]);
                        }
                    }
                    if (tr < o.exp_ld) o.exps[(col0 + e) * o.exp_ld + tr] = tr < p.nbr ? (uint8_t)Eb : (uint8_t)1;
                }
            }
        }
    }
}

template <int BR>
void launch_br(const TileParams &p, dim3 grid, int rounding, hipStream_t s) {
    if (rounding) hipLaunchKernelGGL((tile_kernel<BR, 1>), grid, dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((tile_kernel<BR, 0>), grid, dim3(kThreads), 0, s, p);
}

bool fits(const hbfp_tensor *t, int64_t br, int64_t bc) {
    const int64_t tbr = t->contract_axis == 1 ? t->rblock : t->kblock, tbc = t->contract_axis == 1 ? t->kblock : t->rblock;
    return tbr == br && tbc == bc && t->kblock_pad == 32 && ((uintptr_t)t->mant & 15) == 0;
}

}  // namespace

// Can the register-tile kernel produce these outputs (all with the tile shape of the first) from one input?
bool tile_path_ok(const hbfp_tensor *const *outs, int n, const hbfp_tensor *wide_in, const float *src, int64_t ld) {
    const hbfp_tensor *f = outs[0];
    const int64_t br = f->contract_axis == 1 ? f->rblock : f->kblock, bc = f->contract_axis == 1 ? f->kblock : f->rblock;
    if (br < 1 || br > 32 || bc < 4 || bc > 32 || (bc & 3) || (f->src_cols & 3) || (ld & 3) || ((uintptr_t)src & 15)) return false;
    if (ceil_div(f->src_rows, br) / 4 + 4 > 65535 || ceil_div(f->src_cols, bc) / 8 + 2 > 0x7fffffff) return false;
    for (int i = 0; i < n; ++i)
        if (!fits(outs[i], br, bc) || outs[i]->rounding != f->rounding || outs[i]->src_rows != f->src_rows ||
            outs[i]->src_cols != f->src_cols)
            return false;
    if (wide_in && (!fits(wide_in, br, bc) || wide_in->contract_axis != 1 || wide_in->mant_bits <= 8)) return false;
    return true;
}

int launch_tile_encode(const float *src, int64_t ld, float alpha, const hbfp_tensor *wide_in, const hbfp_tensor *const *outs,
                       int n, hipStream_t s) {
    const hbfp_tensor *f = outs[0];
    TileParams p;
    p.src = src;
    p.ld = ld;
    p.alpha = alpha;
    p.w_mant = wide_in ? (const uint8_t *)wide_in->mant : nullptr;
    p.w_exps = wide_in ? wide_in->exps : nullptr;
    p.w_kpad = wide_in ? wide_in->kpad : 0;
    p.w_expld = wide_in ? wide_in->exp_ld : 0;
    p.w_m = wide_in ? wide_in->mant_bits : 0;
    p.rows = f->src_rows;
    p.cols = f->src_cols;
    p.br = (int32_t)(f->contract_axis == 1 ? f->rblock : f->kblock);
    p.bc = (int32_t)(f->contract_axis == 1 ? f->kblock : f->rblock);
    p.nbr = (int32_t)ceil_div(p.rows, p.br);
    p.nbc = (int32_t)ceil_div(p.cols, p.bc);
    int64_t tcs = p.nbc, trs = p.nbr;
    for (int i = 0; i < 3; ++i) {
        TileOut &o = p.o[i];
        o.present = i < n;
        if (!o.present) continue;
        const hbfp_tensor *t = outs[i];
        o.mant = (uint8_t *)t->mant;
        o.exps = t->exps;
        o.kpad = t->kpad;
        o.exp_ld = t->exp_ld;
        o.m = t->mant_bits;
        o.axis = t->contract_axis;
        o.ntile_k = (int32_t)(t->kpad / 32);
        o.s0 = (uint32_t)t->seed;
        o.s1 = (uint32_t)(t->seed >> 32);
        const int64_t ext = o.ntile_k > t->exp_ld ? o.ntile_k : t->exp_ld;
        if (o.axis == 1) tcs = ext > tcs ? ext : tcs;
        else trs = ext > trs ? ext : trs;
    }
    const dim3 grid((unsigned)ceil_div(tcs, 8), (unsigned)ceil_div(trs, 4));
    const int rounding = f->rounding;
    if (p.br <= 8) launch_br<8>(p, grid, rounding, s);
    else if (p.br <= 16) launch_br<16>(p, grid, rounding, s);
    else if (p.br <= 24) launch_br<24>(p, grid, rounding, s);
    else launch_br<32>(p, grid, rounding, s);
    return launch_status();
}

}  // namespace hbfp
