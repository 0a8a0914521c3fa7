// 2-D exponent tiles of at most 32 x 32 (Sec. 4.2 "Tiling": weight matrices are cut into tiles that
// share an exponent; the paper uses 24 x 24), converted in one pass with the tile held in registers.
//
// A lane owns 4 neighbouring source columns of half of a tile's rows (at most 16 x 4 values in
// registers); the 16 lanes of a tile combine their maxima with four DPP steps.  From
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
__device__ __forceinline__ uint32_t max_of_16_lanes(uint32_t v) {
    v = max(v, dpp_u32<0xB1>(v));    // quad_perm [1,0,3,2]
    v = max(v, dpp_u32<0x4E>(v));    // quad_perm [2,3,0,1]
    v = max(v, dpp_u32<0x141>(v));   // row_half_mirror: the other quad of the 8
    v = max(v, dpp_u32<0x140>(v));   // row_mirror: the other half of the 16
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

// BR: tile height rounded up to 8.  A tile is shared by 16 lanes: lane (h, j) owns columns 4j .. 4j + 3 of rows
// h * BR/2 .. (h + 1) * BR/2 - 1 (at most 16 x 4 values in registers), a wave holds 4 tiles, a workgroup 4 tile
// columns x 4 tile rows (one tile row per wave): the four 32-byte pieces of a 128-byte line of a transposed
// output are then produced by one workgroup.
template <int BR, int ROUND>
__global__ __launch_bounds__(kThreads) void tile_kernel(const TileParams p) {
    constexpr int RPL = BR / 2;       // rows per lane
    __shared__ __attribute__((aligned(16))) uint8_t lines[128 * kLineStride];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 7, h = (lane >> 3) & 1, tw = lane >> 4;
    const int64_t tc = (int64_t)blockIdx.x * 4 + tw;
    const int64_t tr = (int64_t)blockIdx.y * 4 + wave;
    const int64_t row0 = tr * p.br + h * RPL, col0 = tc * p.bc + 4 * j;
    const bool col_ok = tc < p.nbc && 4 * j < p.bc && col0 < p.cols;       // cols and bc are multiples of 4
    int rows_here = 0;                                                     // rows of this lane that exist
    if (tr < p.nbr) {
        const int64_t tile_rows = (p.rows - tr * p.br) < p.br ? (p.rows - tr * p.br) : p.br;
        const int64_t mine = tile_rows - h * RPL;
        rows_here = mine <= 0 ? 0 : (mine < RPL ? (int)mine : RPL);
    }

    // Every load is issued before the first value is used: rows that do not exist read the lane's first row again
    // (lanes without any element read the first element of the matrix) and are zeroed afterwards, so no load hides
    // behind a branch and all of a lane's rows are in flight together.
    const bool any = col_ok && rows_here > 0;
    const float *sbase = any ? p.src + row0 * p.ld + col0 : p.src;
    float4 d[RPL];
#pragma unroll
    for (int r = 0; r < RPL; ++r) d[r] = *reinterpret_cast<const float4 *>(sbase + (r < rows_here ? r : 0) * p.ld);
    float v[RPL][4];
    if (p.w_mant) {
        const int we = any ? (int)p.w_exps[row0 * p.w_expld + tc] - 125 - p.w_m : 0;
        const uint8_t *wbase = any ? p.w_mant + (row0 * p.w_kpad + tc * 32 + 4 * j) * 2 : p.w_mant;
        uint2 w[RPL];
#pragma unroll
        for (int r = 0; r < RPL; ++r) w[r] = *reinterpret_cast<const uint2 *>(wbase + (r < rows_here ? r : 0) * p.w_kpad * 2);
#pragma unroll
        for (int r = 0; r < RPL; ++r) {
            v[r][0] = fmaf(p.alpha, d[r].x, __builtin_amdgcn_ldexpf((float)(int16_t)(w[r].x & 0xffffu), we));
            v[r][1] = fmaf(p.alpha, d[r].y, __builtin_amdgcn_ldexpf((float)(int16_t)(w[r].x >> 16), we));
            v[r][2] = fmaf(p.alpha, d[r].z, __builtin_amdgcn_ldexpf((float)(int16_t)(w[r].y & 0xffffu), we));
            v[r][3] = fmaf(p.alpha, d[r].w, __builtin_amdgcn_ldexpf((float)(int16_t)(w[r].y >> 16), we));
        }
    } else {
#pragma unroll
        for (int r = 0; r < RPL; ++r) {
            v[r][0] = d[r].x; v[r][1] = d[r].y; v[r][2] = d[r].z; v[r][3] = d[r].w;
        }
    }
#pragma unroll
    for (int r = 0; r < RPL; ++r)
        if (!(any && r < rows_here)) v[r][0] = v[r][1] = v[r][2] = v[r][3] = 0.0f;
    uint32_t amax = 0;
#pragma unroll
    for (int r = 0; r < RPL; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) amax = max(amax, __float_as_uint(v[r][e]) & 0x7fffffffu);
    amax = max_of_16_lanes(amax);

    for (int oi = 0; oi < 3; ++oi) {
        const TileOut o = p.o[oi];        // by value: its fields stay in scalar registers instead of being fetched at every use
        if (!o.present) continue;
        const uint32_t Eb = block_exponent<ROUND>(amax, o.m);
        const bool wide = o.m > 8;
        // Stochastic rounding: the hashes of a whole tile, computed side by side, need more than 256 registers.
        // `chain` is always zero, but the compiler cannot know: each group of hashes waits for the previous store.
        uint32_t chain = 0;
        if (ROUND) {
            asm volatile("" : "+v"(chain));
            // likewise nothing derived from the values (sign, exponent, significand of each) may be kept across outputs
#pragma unroll
            for (int r = 0; r < RPL; ++r)
#pragma unroll
                for (int e = 0; e < 4; ++e) asm volatile("" : "+v"(v[r][e]));
        }
        // element (row0 + r, col0 + e) of the source; the stochastic-rounding counter is its logical index
        auto q = [&](int r, int e) -> int {
            if (!ROUND) return quantise<0>(v[r][e], Eb, o.m, 0u, 0u, 0u, 0u);
            // index of the row's first element once per row; adding `chain` before the column offset keeps the
            // compiler from holding all of a tile's indices in registers across the three outputs
            const uint64_t rbase = (uint64_t)(row0 + r) * (uint64_t)p.cols + (uint64_t)col0;
            const uint32_t lo = ((uint32_t)rbase + chain) + (uint32_t)e;
            const uint32_t hi = (uint32_t)(rbase >> 32) + (lo < (uint32_t)e ? 1u : 0u);
            float x = v[r][e];
            asm volatile("" : "+v"(x) : "v"(chain));     // the value's decomposition waits for the previous group too
            return quantise<ROUND>(x, Eb, o.m, lo, hi, o.s0, o.s1);
        };
        if (o.axis == 1) {
            // operand row = source row; block tc of it holds this tile's columns (lanes without columns write the zero padding)
            if (tc < o.ntile_k) {
                // one address computation per output; the rows are a fixed stride apart
                const int64_t row_bytes = o.kpad * (wide ? 2 : 1);
                uint8_t *dst = o.mant + (row0 * o.kpad + tc * 32 + 4 * j) * (wide ? 2 : 1);
                if (!wide) {
#pragma unroll
                    for (int r = 0; r < RPL; ++r) {
                        if (r < rows_here) {
                            const uint32_t w0 = pack4_i8(q(r, 0), q(r, 1), q(r, 2), q(r, 3));
                            __builtin_nontemporal_store(w0, reinterpret_cast<uint32_t *>(dst + r * row_bytes));
                            if (ROUND) asm volatile("" : "+v"(chain) : "v"(w0));
                        }
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < RPL; ++r) {
                        if (r < rows_here) {
                            const uint32_t w0 = pack2_i16(q(r, 0), q(r, 1)), w1 = pack2_i16(q(r, 2), q(r, 3));
                            *reinterpret_cast<uint2 *>(dst + r * row_bytes) = make_uint2(w0, w1);
                            if (ROUND) asm volatile("" : "+v"(chain) : "v"(w0), "v"(w1));
                        }
                    }
                }
            }
            if (tc < o.exp_ld) {
                const uint8_t eb = tc < p.nbc ? (uint8_t)Eb : (uint8_t)1;
                for (int r = j; r < rows_here; r += 8) o.exps[(row0 + r) * o.exp_ld + tc] = eb;
            }
        } else if (!wide) {
            // operand row = source column; block tr of it holds this tile's rows: 32 consecutive mantissas per column.
            // The four waves (tile rows 4 by .. 4 by + 3) fill [column][4 x 32 bytes], then every 8 threads store one line.
            const int64_t tr0 = (int64_t)blockIdx.y * 4, tc0 = (int64_t)blockIdx.x * 4;
            __syncthreads();                          // the previous output's lines have been read
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint8_t *l = lines + (tw * 32 + 4 * j + e) * kLineStride + wave * 32;
#pragma unroll
                for (int k = 0; k < RPL / 4; ++k)
                {
                    const uint32_t w0 = pack4_i8(q(4 * k, e), q(4 * k + 1, e), q(4 * k + 2, e), q(4 * k + 3, e));
                    *reinterpret_cast<uint32_t *>(l + h * RPL + 4 * k) = w0;
                    if (ROUND) asm volatile("" : "+v"(chain) : "v"(w0));
                }
                if (h == 1) {                         // rows BR .. 31 of the block are padding
#pragma unroll
                    for (int k = BR / 4; k < 8; ++k) *reinterpret_cast<uint32_t *>(l + 4 * k) = 0u;
                }
            }
            __syncthreads();
            if (tr0 < o.ntile_k) {                    // ntile_k is a multiple of 4: all four tile rows are stored or none
                for (int g = threadIdx.x; g < 128 * 8; g += kThreads) {
                    const int lc = g >> 3, ch = g & 7;
                    const int64_t tcc = tc0 + (lc >> 5), c = tcc * p.bc + (lc & 31);
                    if (tcc < p.nbc && (lc & 31) < p.bc && c < p.cols) {
                        typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
                        const uint4 d = *reinterpret_cast<const uint4 *>(lines + lc * kLineStride + ch * 16);
                        const v4u_t w = {d.x, d.y, d.z, d.w};            // streaming store: written once, not read again here
                        __builtin_nontemporal_store(w, reinterpret_cast<v4u_t *>(o.mant + c * o.kpad + tr0 * 32 + ch * 16));
                    }
                }
            }
            if (col_ok && h == 0 && tr < o.exp_ld) {
#pragma unroll
                for (int e = 0; e < 4; ++e) o.exps[(col0 + e) * o.exp_ld + tr] = tr < p.nbr ? (uint8_t)Eb : (uint8_t)1;
            }
        } else if (col_ok) {
            // 16-bit transposed output: each lane stores its rows of its four columns directly (8 bytes at a time)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (tr < o.ntile_k) {
                    uint8_t *dst = o.mant + ((col0 + e) * o.kpad + tr * 32) * 2;
#pragma unroll
                    for (int k = 0; k < RPL / 4; ++k)
                    {
                        const uint32_t w0 = pack2_i16(q(4 * k, e), q(4 * k + 1, e)), w1 = pack2_i16(q(4 * k + 2, e), q(4 * k + 3, e));
                        *reinterpret_cast<uint2 *>(dst + (h * RPL + 4 * k) * 2) = make_uint2(w0, w1);
                        if (ROUND) asm volatile("" : "+v"(chain) : "v"(w0), "v"(w1));
                    }
                    if (h == 1) {
#pragma unroll
                        for (int k = BR / 4; k < 8; ++k) *reinterpret_cast<uint2 *>(dst + 8 * k) = make_uint2(0u, 0u);
                    }
                }
                if (h == 0 && tr < o.exp_ld) o.exps[(col0 + e) * o.exp_ld + tr] = tr < p.nbr ? (uint8_t)Eb : (uint8_t)1;
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
    return tbr == br && tbc == bc && t->kblock_pad == 32 && t->kshare == 1 && ((uintptr_t)t->mant & 15) == 0;
}

}  // namespace

// Can the register-tile kernel produce these outputs (all with the tile shape of the first) from one input?
bool tile_path_ok(const hbfp_tensor *const *outs, int n, const hbfp_tensor *wide_in, const float *src, int64_t ld) {
    const hbfp_tensor *f = outs[0];
    const int64_t br = f->contract_axis == 1 ? f->rblock : f->kblock, bc = f->contract_axis == 1 ? f->kblock : f->rblock;
    if (br < 1 || br > 32 || bc < 4 || bc > 32 || (bc & 3) || (f->src_cols & 3) || (ld & 3) || ((uintptr_t)src & 15)) return false;
    if (ceil_div(f->src_rows, br) / 4 + 4 > 65535 || ceil_div(f->src_cols, bc) / 4 + 2 > 0x7fffffff) return false;
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
    const dim3 grid((unsigned)ceil_div(tcs, 4), (unsigned)ceil_div(trs, 4));
    const int rounding = f->rounding;
    if (p.br <= 8) launch_br<8>(p, grid, rounding, s);
    else if (p.br <= 16) launch_br<16>(p, grid, rounding, s);
    else if (p.br <= 24) launch_br<24>(p, grid, rounding, s);
    else launch_br<32>(p, grid, rounding, s);
    return launch_status();
}

}  // namespace hbfp
