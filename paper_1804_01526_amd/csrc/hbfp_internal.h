// Internal declarations shared by the host API and the kernel launchers.
// Nothing here is part of the public ABI (see include/hbfp.h).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "hbfp.h"

namespace hbfp {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

inline int launch_status() { return hipGetLastError() == hipSuccess ? HBFP_OK : HBFP_ERR_LAUNCH; }

// Raises a kernel's dynamic LDS limit the first time it is launched.  `done` is that kernel's own flag; two threads
// that meet here both make the (idempotent) runtime call, which is all a race can do.
inline int allow_dynamic_lds(std::atomic<bool> &done, const void *kernel, int bytes) {
    if (done.load(std::memory_order_acquire)) return HBFP_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return HBFP_ERR_LAUNCH;
    done.store(true, std::memory_order_release);
    return HBFP_OK;
}

// Geometry of one encode/decode call in terms of the SOURCE matrix.
struct EncodeGeom {
    int64_t src_rows, src_cols, ld;   // source matrix
    int64_t br, bc;                   // exponent block extents in the source (already clamped to the matrix)
    int64_t nbr, nbc;                 // blocks along source rows / cols
    int32_t axis;                     // contraction axis in the source
    // operand side
    int64_t R, K, kblock, kbp, nblk, kpad, exp_ld, rblock;
    int64_t kshare;                   // stored blocks along k that repeat one exponent
    int32_t m, rounding;
    uint32_t seed_lo, seed_hi;
};

// encode.hip
int launch_encode_row_fused(const float *src, const EncodeGeom &g, void *mant, uint8_t *exps, hipStream_t s);
int launch_encode_col_fused(const float *src, const EncodeGeom &g, void *mant, uint8_t *exps, hipStream_t s);
int launch_encode_im2col(const float *x, const hbfp_conv2d &c, int64_t ho, int64_t wo, const EncodeGeom &g, void *mant,
                         uint8_t *exps, uint32_t *table, hipStream_t s);
int launch_encode_generic(const float *src, const EncodeGeom &g, void *mant, uint8_t *exps,
                          uint32_t *tile_amax, hipStream_t s);

// decode.hip
int launch_decode(const hbfp_tensor *t, float *dst, int64_t ld, hipStream_t s);
// dst = fma(alpha, delta, decode(t)); delta == nullptr: plain decode
int launch_decode_axpy(const hbfp_tensor *t, float *dst, int64_t ld, const float *delta, int64_t ldd, float alpha,
                       hipStream_t s);

// gemm.hip
struct GemmArgs {
    const void *mantA, *mantB;        // int8 [rows][kpad] (or limb planes)
    const uint8_t *expA, *expB;       // [rows][exp_ld]
    int64_t M, N, kpad, expA_ld, expB_ld, nblk, kbp, kblock;
    int64_t kdim;                     // contraction length without any padding (0: unknown, take nblk * kblock)
    int32_t mA, mB;                   // mantissa bits
    float *C;
    int64_t ldc;
    float beta;
    int32_t *P;                       // non-null: dump block partials instead of C
    // stand-by launches (behind the block-scaled kernel): non-null pointers to the headers of the two packed operands;
    // every kernel of the launch does nothing unless one of them is marked out of range (word 0 == word 1)
    const int *run_a, *run_b;
    int32_t wide;                     // 1: the caller asked for the 256 x 256-tile int8 kernel whatever the shape
    int32_t words_ready;              // stand-by launches: the scale words of the 8-wave int8 kernel are in the workspace already
};
// What the block-scaled product kernel needs in order to prepare the scale words of the int8 stand-by launch behind it
// (extra workgroups of its own grid that do nothing unless an operand is marked)
struct StandbyWords {
    const uint8_t *eA, *eB;
    uint32_t *wA, *wB;
    int64_t ldA, ldB, M, N;
    int32_t slots;
    uint32_t a_or;
};
// true if the int8 stand-by of product `a` is the 8-wave kernel, whose scale words then lie at w->wA / w->wB in `workspace`
bool gemm_i8_standby_words(const GemmArgs &a, void *workspace, StandbyWords *w);
// 2-D tiles of at most 32 x 32 held in registers: one input (FP32 matrix, or stored wide weights + alpha * step),
// up to three outputs of the same tile shape in any orientation
bool tile_path_ok(const hbfp_tensor *const *outs, int n, const hbfp_tensor *wide_in, const float *src, int64_t ld);
int launch_tile_encode(const float *src, int64_t ld, float alpha, const hbfp_tensor *wide_in, const hbfp_tensor *const *outs,
                       int n, hipStream_t s);
int launch_gemm_i8(const GemmArgs &a, void *workspace, hipStream_t s);
size_t gemm_i8_workspace(int64_t M, int64_t N, int64_t kpad, int64_t kbp, int64_t exp_ld);
size_t gemm_conv_workspace(int64_t M, int64_t N, int64_t kpad, int64_t pixels, int cblocks);
int launch_gemm_conv_i8(const GemmArgs &a, const hbfp_conv2d &c, int64_t ho, int64_t wo, int64_t pix_bytes, void *workspace,
                        hipStream_t s, int dil_h = 1, int dil_w = 1, bool by_phase = false, int slot_order = -1,
                        int kblock = 32, int chain = 0, const hbfp_tensor *enc = nullptr, int relu = 0);
bool conv_encoded_output_ok(int64_t M, int64_t N, int64_t kpad, const hbfp_tensor &out);
bool conv_dgrad_by_phase(int r, int s, int stride_h, int stride_w);
// 9..12-bit mantissas as FP16 numbers on the FP16 matrix instruction (blocks of 32, 64 or multiples of 128)
bool gemm_f16_possible(const GemmArgs &a);
size_t gemm_f16_workspace(int64_t M, int64_t N, int64_t kpad, int64_t kbp, int64_t exp_ld);
int launch_gemm_f16(const GemmArgs &a, void *workspace, hipStream_t s);
int launch_gemm_limb(const GemmArgs &a, void *workspace, hipStream_t s);
size_t gemm_limb_workspace(const hbfp_tensor *A, const hbfp_tensor *B);

// gemm_wide.hip: int8 kernel for one exponent per operand row (a single block along k), 256 x 256 tiles
bool gemm_wide_possible(const GemmArgs &a);
bool gemm_wide_ok(const GemmArgs &a);
int launch_gemm_wide(const GemmArgs &a, hipStream_t s);

// gemm_mx.hip: the product on the block-scaled matrix instruction.  A packed operand is a 256-byte header followed
// by the limb planes; the header's first two words are equal when some exponent of the operand could not be
// expressed, in which case the product kernel does not touch C and the int8 path has to run (run_a, run_b).
bool gemm_mx_possible(const GemmArgs &a);   // shapes the kernel can address
bool gemm_mx_ok(const GemmArgs &a);         // shapes and formats for which it is the faster choice
size_t mx_packed_bytes(int64_t rows, int64_t kpad, int mant_bits);   // header + planes, a multiple of 256
// packs operand A (rows a.M) and / or operand B (rows a.N) of `a` in one launch; a null buffer skips that operand
int launch_mx_pack(const GemmArgs &a, void *packed_a, void *packed_b, hipStream_t s);
int mx_pack_begin(void *packed, hipStream_t s, int32_t *mark);
// encode_pack.hip: conversion and packing in one kernel (blocks of 24 along k, up to two outputs from one read)
bool encode_pack_ok(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs, void *const *packed);
int launch_encode_pack(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs, void *const *packed, hipStream_t s);
bool encode_pack_batch_ok(int nsrc, const hbfp_tensor *const *const *outs);
int launch_encode_pack_batch(int nsrc, const float *const *src, const int64_t *ld, const int *n, const hbfp_tensor *const *const *outs,
                             void *const *const *packed, hipStream_t s);
// gemm_bf.hip: mantissas of 6 to 9 bits as bf16 numbers on the bf16 matrix instruction.  A packed operand of that class
// is the same 256-byte header followed by bf16 planes.
bool bf_operand(int mant_bits);
size_t packed_operand_bytes(int64_t rows, int64_t kpad, int mant_bits);   // of either kind of packed operand
bool gemm_bf_possible(const GemmArgs &a);
int launch_bf_pack(const GemmArgs &a, void *packed_a, void *packed_b, hipStream_t s);
int launch_bf_products(int n, const GemmArgs *args, const void *const *packed_a, const void *const *packed_b, hipStream_t s);
// 9..12-bit mantissas as FP16 numbers relative to their rows' largest exponents, on the same kernel with the FP16
// matrix instruction; packed operand: header, one scale word per row, FP16 planes
bool gemm_f16_planes_possible(const GemmArgs &a);
size_t f16_planes_bytes(int64_t rows, int64_t kpad);
int launch_f16_planes_pack(const GemmArgs &a, void *packed_a, void *packed_b, hipStream_t s);
int launch_f16_planes_products(int n, const GemmArgs *args, const void *const *packed_a, const void *const *packed_b, hipStream_t s);
int launch_bf_product_encoded(const GemmArgs &a, const void *packed_a, const void *packed_b, const hbfp_tensor &out, int relu,
                              hipStream_t s);
bool mx_same_limbs(const GemmArgs &a, const GemmArgs &b);
bool gemm_mx_group_ok(int n, const GemmArgs *args);
bool mx_encoded_output_ok(const hbfp_tensor &out);
int launch_mx_product_encoded(const GemmArgs &a, const void *packed_a, const void *packed_b, const hbfp_tensor &out, int relu,
                              hipStream_t s);
int launch_mx_encode_standby(const float *C, int64_t ldc, const hbfp_tensor &out, int relu, const int *run_a, const int *run_b,
                             hipStream_t s);
int launch_relu(float *x, int64_t n, hipStream_t s);
// standby_ws: per product, the workspace its int8 stand-by launch will be given, or null; where that stand-by is the
// 8-wave int8 kernel the launch also prepares its scale words (args[i].words_ready is set then)
int launch_mx_products(int n, GemmArgs *args, const void *const *packed_a, const void *const *packed_b, void *const *standby_ws,
                       hipStream_t s);
int launch_mx_product(GemmArgs &a, const void *packed_a, const void *packed_b, void *standby_ws, hipStream_t s);

}  // namespace hbfp
