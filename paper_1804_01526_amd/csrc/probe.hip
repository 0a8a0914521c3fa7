// Measurement aid: what the matrix core sustains on this chip with given operand bits.  A register-only loop of one
// matrix instruction (no memory traffic inside the loop), 4 x 4 independent accumulator chains per wave, and the
// shader clock it ran at (cycle counter against the 100 MHz wall clock over the loop of one workgroup).  The rate
// depends on the operand bits because the chip lowers its clock to stay inside its power limit; the product kernels'
// roofline is judged against the published peak and, for scale, against what this loop reaches on random bits.
#include "hbfp_internal.h"

namespace hbfp {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

// words: [64 registers][64 lanes]; registers 0..31 feed the first operands, 32..63 the second
__global__ __launch_bounds__(256) void probe_scaled_fp6_kernel(const int *words, float *sink, long long *clocks, int iters) {
    v8i a[4], b[4];
    for (int n = 0; n < 4; ++n)
        for (int r = 0; r < 8; ++r) {
            a[n][r] = words[(n * 8 + r) * 64 + (threadIdx.x & 63)];
            b[n][r] = words[(32 + n * 8 + r) * 64 + (threadIdx.x & 63)];
        }
    v16f c[4];
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) c[n][v] = 0.0f;
    const int scale = 127 | (127 << 8);
    const long long t0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int m = 0; m < 4; ++m) c[m] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[n], b[m], c[m], 2, 2, 0, scale, 0, scale);
    }
    const long long t1 = clock64(), w1 = wall_clock64();
    float r = 0.0f;
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) r += c[n][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
    if (threadIdx.x == 0 && blockIdx.x == 7) {
        clocks[0] = t1 - t0;
        clocks[1] = w1 - w0;
    }
}

__global__ __launch_bounds__(256) void probe_int8_kernel(const int *words, float *sink, long long *clocks, int iters) {
    v4i a[4], b[4];
    for (int n = 0; n < 4; ++n)
        for (int r = 0; r < 4; ++r) {
            a[n][r] = words[(n * 8 + r) * 64 + (threadIdx.x & 63)];
            b[n][r] = words[(32 + n * 8 + r) * 64 + (threadIdx.x & 63)];
        }
    v16i c[4];
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) c[n][v] = 0;
    const long long t0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int m = 0; m < 4; ++m) c[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[n], b[m], c[m], 0, 0, 0);
    }
    const long long t1 = clock64(), w1 = wall_clock64();
    int r = 0;
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) r += c[n][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = (float)r;
    if (threadIdx.x == 0 && blockIdx.x == 7) {
        clocks[0] = t1 - t0;
        clocks[1] = w1 - w0;
    }
}

// 16-bit operand words: every half word must be a finite bf16 number for the sums to mean anything (the rate does not care)
__global__ __launch_bounds__(256) void probe_bf16_kernel(const int *words, float *sink, long long *clocks, int iters) {
    typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
    v4i a[4], b[4];
    for (int n = 0; n < 4; ++n)
        for (int r = 0; r < 4; ++r) {
            a[n][r] = words[(n * 8 + r) * 64 + (threadIdx.x & 63)];
            b[n][r] = words[(32 + n * 8 + r) * 64 + (threadIdx.x & 63)];
        }
    v16f c[4];
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) c[n][v] = 0.0f;
    const long long t0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int m = 0; m < 4; ++m)
                c[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a[n]), __builtin_bit_cast(v8bf, b[m]), c[m], 0, 0, 0);
    }
    const long long t1 = clock64(), w1 = wall_clock64();
    float r = 0.0f;
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) r += c[n][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
    if (threadIdx.x == 0 && blockIdx.x == 7) {
        clocks[0] = t1 - t0;
        clocks[1] = w1 - w0;
    }
}

}  // namespace
}  // namespace hbfp

extern "C" int hbfp_probe_matrix_rate(int instruction, const int *words, int workgroups, int iters, float *sink, long long *clocks,
                                      void *stream) {
    if (!words || !sink || !clocks || workgroups < 8 || workgroups > 65536 || iters < 1 || iters > (1 << 20)) return HBFP_ERR_ARG;
    if (instruction < 0 || instruction > 2) return HBFP_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (instruction == 0) hipLaunchKernelGGL(hbfp::probe_int8_kernel, dim3((unsigned)workgroups), dim3(256), 0, s, words, sink, clocks, iters);
    else if (instruction == 2) hipLaunchKernelGGL(hbfp::probe_bf16_kernel, dim3((unsigned)workgroups), dim3(256), 0, s, words, sink, clocks, iters);
    else hipLaunchKernelGGL(hbfp::probe_scaled_fp6_kernel, dim3((unsigned)workgroups), dim3(256), 0, s, words, sink, clocks, iters);
    return hbfp::launch_status();
}
