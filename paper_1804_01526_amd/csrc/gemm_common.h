// Pieces shared by the matrix-product kernels (each translation unit gets its own copy).
#pragma once
#include "hbfp_internal.h"

namespace hbfp {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Workgroup -> tile.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  XCD x gets
// a contiguous eighth of the tiles, walked in bands of 8 tile rows column by column, so that the 64
// tiles an XCD works on at any time are an 8 x 8 patch: 8 row panels and 8 column panels of the current
// k range stay in that XCD's L2 and each is used 8 times.  Returns false for the padding workgroups.
__device__ __forceinline__ bool tile_of_workgroup(int wg, int tiles_m, int tiles_n, int &tm, int &tn) {
    const int ntiles = tiles_m * tiles_n;
    const int per_xcd = (ntiles + 7) >> 3;
    const int t = (wg & 7) * per_xcd + (wg >> 3);
    if ((wg >> 3) >= per_xcd || t >= ntiles) return false;
    const int band = t / (8 * tiles_n);
    const int rows_in_band = tiles_m - band * 8 < 8 ? tiles_m - band * 8 : 8;
    const int r = t - band * 8 * tiles_n;
    tn = r / rows_in_band;
    tm = band * 8 + r % rows_in_band;
    return true;
}

// Split-K launches with at least 8 k ranges (few tiles, very long k): a one-dimensional grid of
// 8 * tiles * ceil(splits / 8) workgroups.
// XCD x takes the k ranges x, x + 8, ... and, for each, every tile: the tiles of one k range share their operand
// panels in that XCD's L2, and the work is spread over all 8 XCDs however few tiles there are (dealing tiles to
// XCDs as above would leave XCDs idle when there are fewer than 8 tiles).  Returns false for padding workgroups.
__device__ __forceinline__ bool tile_and_split_of_workgroup(int wg, int tiles_m, int tiles_n, int splits, int &tm, int &tn,
                                                            int &split) {
    const int ntiles = tiles_m * tiles_n;
    const int slot = wg >> 3;
    split = (slot / ntiles) * 8 + (wg & 7);
    if (split >= splits) return false;
    const int t = slot % ntiles;
    tn = t / tiles_m;
    tm = t - tn * tiles_m;
    return true;
}

__device__ __forceinline__ void async_copy16(const void *gbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(gbase) : "memory");
}
// the same copies from a full 64-bit address per lane (gathers whose sources do not share one base)
__device__ __forceinline__ void async_copy16_at(const void *addr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(addr) : "memory");
}
__device__ __forceinline__ void async_copy4_at(const void *addr, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(addr) : "memory");
}
__device__ __forceinline__ void async_copy4(const void *gbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_addr), "v"(voff), "s"(gbase) : "memory");
}

// A kernel queued behind the block-scaled product kernel as its stand-in runs only when one of the two packed
// operands is marked out of range (the first two words of its header are equal); without headers it always runs.
__device__ __forceinline__ bool stands_down(const int *run_a, const int *run_b) {
    return run_a && run_a[0] != run_a[1] && run_b[0] != run_b[1];
}

typedef short v4s __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

// rowc holds, in its low half, the bf16 pattern of 1.5 * 2^(Ea - 127) of row (lane % 32); every other
// 16-bit element of the first operand meets a zero of one_hot (a bf16 one at k = 0 of lanes 0..31) and
// only has to be finite.  The product is exact, so the result is the FP32 constant in every column.
__device__ __forceinline__ v16i row_constants(uint32_t rowc, const v2i &one_hot) {
    const v2i a2 = {(int)rowc, 0};
    const v16f zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const v16f c = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(v4s, a2), __builtin_bit_cast(v4s, one_hot), zero, 0, 0, 0);
    return __builtin_bit_cast(v16i, c);
}

// exponent bytes [rows][ld] -> scale words [slots][rows_pad] for both operands in one launch (blockIdx.z
// picks the operand); rows past the end get the smallest scale.  A thread turns four consecutive blocks
// of one row (one 32-bit load: ld and slots are multiples of 4) into four words; consecutive lanes take
// consecutive rows, so the stores are contiguous.
struct WordParams {
    const uint8_t *exps[2];
    uint32_t *words[2];
    int64_t ld[2], rows[2], rows_pad[2];
    int slots, row_blocks;
    uint32_t a_or;               // 0x40: row words are 1.5 * 2^(E - 127) as bf16; 0: 2^(E - 127) as bf16
    const int *run_a, *run_b;
};
// one block of 256 threads of that job: block index, operand, thread
__device__ __forceinline__ void scale_words_block(const WordParams &w, uint32_t block, int z, int thread) {
    const int64_t row = (int64_t)(block % (uint32_t)w.row_blocks) * 256 + thread;
    if (row >= w.rows_pad[z]) return;
    const int s0 = (int)(block / (uint32_t)w.row_blocks) * 4;
    const uint32_t e4 = row < w.rows[z] ? *reinterpret_cast<const uint32_t *>(w.exps[z] + row * w.ld[z] + s0) : 0x01010101u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t e = (e4 >> (8 * i)) & 0xffu;
        e = e > 254u ? 254u : e;
        w.words[z][(int64_t)(s0 + i) * w.rows_pad[z] + row] = z == 0 ? ((e << 7) | w.a_or) : (e << 23);
    }
}
__global__ __launch_bounds__(256) void scale_words_t_kernel(const WordParams w) {
    if (stands_down(w.run_a, w.run_b)) return;
    scale_words_block(w, blockIdx.x, (int)blockIdx.z, (int)threadIdx.x);
}

// bytes of one operand's scale words: [slots][rows rounded up to 128]
inline size_t word_bytes(int64_t rows, int64_t slots) { return (size_t)slots * (size_t)(ceil_div(rows, 128) * 128) * 4; }

// slots must be a multiple of 4 and at most the exponent row pitch of either operand
inline WordParams scale_word_params(const uint8_t *eA, int64_t ldA, int64_t M, const uint8_t *eB, int64_t ldB, int64_t N, int slots,
                                    uint32_t a_or, uint32_t *wA, uint32_t *wB, const int *run_a, const int *run_b) {
    WordParams wp;
    wp.exps[0] = eA; wp.exps[1] = eB;
    wp.words[0] = wA; wp.words[1] = wB;
    wp.ld[0] = ldA; wp.ld[1] = ldB;
    wp.rows[0] = M; wp.rows[1] = N;
    wp.rows_pad[0] = ceil_div(M, 128) * 128; wp.rows_pad[1] = ceil_div(N, 128) * 128;
    wp.slots = slots;
    wp.a_or = a_or;
    wp.run_a = run_a;
    wp.run_b = run_b;
    const int64_t maxpad = wp.rows_pad[0] > wp.rows_pad[1] ? wp.rows_pad[0] : wp.rows_pad[1];
    wp.row_blocks = (int)ceil_div(maxpad, 256);
    return wp;
}
// blocks of 256 threads per operand that the job consists of
inline int64_t scale_word_blocks(const WordParams &wp) { return (int64_t)wp.row_blocks * (wp.slots / 4); }
inline int launch_scale_words(const uint8_t *eA, int64_t ldA, int64_t M, const uint8_t *eB, int64_t ldB, int64_t N, int slots,
                              uint32_t a_or, uint32_t *wA, uint32_t *wB, const int *run_a, const int *run_b,
                              hipStream_t s) {
    const WordParams wp = scale_word_params(eA, ldA, M, eB, ldB, N, slots, a_or, wA, wB, run_a, run_b);
    if (scale_word_blocks(wp) > 0x7fffffff) return HBFP_ERR_ARG;
    hipLaunchKernelGGL(scale_words_t_kernel, dim3((unsigned)scale_word_blocks(wp), 1, 2), dim3(256), 0, s, wp);
    return launch_status();
}

}  // namespace
}  // namespace hbfp
