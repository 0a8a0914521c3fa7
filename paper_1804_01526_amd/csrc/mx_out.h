// The product delivered as an encoded operand: the conversion of Sec. 4.1 / Sec. 5.3 applied to the FP32 accumulators of
// a product kernel whose waves hold 64 x 128 outputs as 2 x 4 results of 32 x 32 matrix instructions, computed with the
// operands of the instruction exchanged (see mx_store_encoded).  Shared by the block-scaled kernel (gemm_mx.hip) and the
// bf16 kernel (gemm_bf.hip); each translation unit gets its own copy.
#pragma once
#include "bfp_device.h"
#include "gemm_common.h"
#include "hbfp_internal.h"

namespace hbfp {
namespace {

// The product written as an encoded operand instead of FP32 (the conversion of Sec. 4.1 / Sec. 5.3 applied to the
// accumulators: the next product's activation operand, k along the columns of C, blocks of 32 or 64).
struct MxOut {
    uint8_t *mant, *exps;        // mant == nullptr: FP32 output
    int64_t kpad, exp_ld;
    int32_t nblk, kblock, m, rounding, wide, relu;
    uint32_t s0, s1;
};

template <int CTRL>
__device__ __forceinline__ uint32_t mx_dpp(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
// maximum over lanes 0..31 and over lanes 32..63, in every lane
__device__ __forceinline__ uint32_t max_of_half_wave(uint32_t v) {
    v = max(v, mx_dpp<0xB1>(v));    // quad_perm [1,0,3,2]
    v = max(v, mx_dpp<0x4E>(v));    // quad_perm [2,3,0,1]
    v = max(v, mx_dpp<0x141>(v));   // row_half_mirror
    v = max(v, mx_dpp<0x140>(v));   // row_mirror
    return max(v, (uint32_t)__shfl_xor((int)v, 16));
}

// Encoded output of a wave's 64 x 128 accumulators.  The kernel variant that produces it multiplies with the operands
// of the matrix instruction exchanged, so that its 32 x 32 results arrive transposed: lane (l32, lh) holds row l32
// of the row tile and, in register v, column 8 * (v / 4) + 4 * lh + v % 4 of the column tile.  The 32 columns of an
// exponent block are then 16 registers of lane l32 and 16 of lane l32 + 32: one maximum over registers and one
// exchange across the wave halves per block (a block of 64 combines two column tiles).  Same arithmetic and the same
// stochastic-rounding index (position in C) as the conversion kernels, so the result equals converting the FP32 product.
template <int ROUND>
__device__ __forceinline__ void mx_store_encoded(const MxOut &o, v16f (&acc)[2][4], int64_t row0, int64_t col0, int64_t M,
                                                 int64_t N, int lane) {
    const int l32 = lane & 31, lh = lane >> 5;
    const bool relu = o.relu != 0;
    // value v of column tile j as it is converted: zero beyond the last column, ReLU if asked for
#define HBFP_MX_VALUE(i, j, v, left) (((8 * ((v) >> 2) + ((v) & 3)) < (left)) ? (relu && acc[i][j][v] < 0.0f ? 0.0f : acc[i][j][v]) : 0.0f)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t row = row0 + i * 32 + l32;
#pragma unroll
        for (int jp = 0; jp < 2; ++jp) {                       // two column tiles at a time: one block of 64 or two of 32
            uint32_t am[2], eb[2];
            int left[2];                                        // columns of this lane's run that exist
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int jj = 2 * jp + h;
                const int64_t c0 = col0 + jj * 32 + 4 * lh;
                const int64_t rest = N - c0;
                left[h] = rest > 32 ? 32 : (rest < 0 ? 0 : (int)rest);
                am[h] = 0;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float f = HBFP_MX_VALUE(i, jj, v, left[h]);
                    acc[i][jj][v] = f;                         // in place: the second pass reads the value as converted
                    am[h] = max(am[h], __float_as_uint(f) & 0x7fffffffu);
                }
                am[h] = max(am[h], (uint32_t)__shfl_xor((int)am[h], 32));
            }
            if (o.kblock == 64) am[0] = am[1] = max(am[0], am[1]);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int jj = 2 * jp + h;
                eb[h] = block_exponent<ROUND>(am[h], o.m);
                const int64_t c0 = col0 + jj * 32 + 4 * lh;
                const uint64_t idx0 = (uint64_t)row * (uint64_t)N + (uint64_t)c0;
                // this lane's 16 mantissas are four runs of 4 (columns 8 g + 4 lh ..); the partner in the other wave half
                // has the runs in between.  One exchange gives each of the two 16 consecutive columns, so a row's 32
                // mantissas leave as two 16-byte stores (32-byte for 16-bit mantissas) instead of eight 4-byte ones.
                int w[4][2];
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    int q[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint64_t idx = idx0 + (uint64_t)(8 * gq + e);
                        q[e] = quantise<ROUND>(acc[i][jj][4 * gq + e], eb[h], o.m, (uint32_t)idx, (uint32_t)(idx >> 32),
                                               o.s0, o.s1);
                    }
                    if (o.wide) {
                        w[gq][0] = (int)((uint32_t)(q[0] & 0xffff) | ((uint32_t)q[1] << 16));
                        w[gq][1] = (int)((uint32_t)(q[2] & 0xffff) | ((uint32_t)q[3] << 16));
                    } else {
                        w[gq][0] = (int)((uint32_t)(q[0] & 0xff) | ((uint32_t)(q[1] & 0xff) << 8) | ((uint32_t)(q[2] & 0xff) << 16) | ((uint32_t)q[3] << 24));
                        w[gq][1] = 0;
                    }
                }
                // lower half keeps runs 0 and 1 and receives the partner's runs 0 and 1; upper half keeps 2 and 3
                const int nw = o.wide ? 2 : 1;
                int got[2][2];
#pragma unroll
                for (int x = 0; x < 2; ++x)
#pragma unroll
                    for (int y = 0; y < 2; ++y) got[x][y] = y < nw ? __shfl_xor(lh ? w[x][y] : w[2 + x][y], 32) : 0;
                const int64_t col = col0 + jj * 32 + 16 * lh;  // first of this lane's 16 consecutive columns
                if (row < M && col0 + jj * 32 < o.kpad) {
                    typedef int v4i_t __attribute__((ext_vector_type(4)));
                    if (o.wide) {
                        const v4i_t a = lh ? v4i_t{got[0][0], got[0][1], w[2][0], w[2][1]} : v4i_t{w[0][0], w[0][1], got[0][0], got[0][1]};
                        const v4i_t b = lh ? v4i_t{got[1][0], got[1][1], w[3][0], w[3][1]} : v4i_t{w[1][0], w[1][1], got[1][0], got[1][1]};
                        v4i_t *dst = reinterpret_cast<v4i_t *>(o.mant + (row * o.kpad + col) * 2);
                        dst[0] = a;
                        dst[1] = b;
                    } else {
                        const v4i_t a = lh ? v4i_t{got[0][0], w[2][0], got[1][0], w[3][0]} : v4i_t{w[0][0], got[0][0], w[1][0], got[1][0]};
                        *reinterpret_cast<v4i_t *>(o.mant + row * o.kpad + col) = a;
                    }
                }
            }
            // exponent bytes of these 64 columns of the row: two blocks of 32 (one half word) or one block of 64
            if (lh == 0 && row < M) {
                if (o.kblock == 32) {
                    const int64_t b0 = (col0 >> 5) + 2 * jp;   // even, like the row length of the exponents
                    const uint32_t w = (b0 < o.nblk ? eb[0] : 1u) | ((b0 + 1 < o.nblk ? eb[1] : 1u) << 8);
                    if (b0 < o.exp_ld) *reinterpret_cast<uint16_t *>(o.exps + row * o.exp_ld + b0) = (uint16_t)w;
                } else {
                    const int64_t b0 = (col0 >> 6) + jp;
                    if (b0 < o.exp_ld) o.exps[row * o.exp_ld + b0] = b0 < o.nblk ? (uint8_t)eb[0] : (uint8_t)1;
                }
            }
            __builtin_amdgcn_sched_barrier(0);                 // the unrolled epilogue must not pile up temporaries
        }
    }
#undef HBFP_MX_VALUE
}

inline MxOut mx_out_of(const hbfp_tensor &t, int relu) {
    MxOut o = {};
    o.mant = (uint8_t *)t.mant;
    o.exps = t.exps;
    o.kpad = t.kpad;
    o.exp_ld = t.exp_ld;
    o.nblk = (int32_t)t.nblk;
    o.kblock = (int32_t)t.kblock;
    o.m = t.mant_bits;
    o.rounding = t.rounding;
    o.wide = t.mant_bits > 8;
    o.relu = relu != 0;
    o.s0 = (uint32_t)t.seed;
    o.s1 = (uint32_t)(t.seed >> 32);
    return o;
}

}  // namespace
}  // namespace hbfp
