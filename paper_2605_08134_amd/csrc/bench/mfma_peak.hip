// Register-resident MFMA loop: what the matrix pipe of this chip sustains when
// nothing else (no LDS, no memory) is in the way.  It calibrates the datasheet peak
// that the projection and attention kernels are measured against.  Benchmark aid: built
// into libdare_bench.so, not into the product library.
#include <hip/hip_runtime.h>

#include "dare_bench.h"

namespace {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kChains = 8;  // independent accumulator chains per wave

__global__ void __launch_bounds__(256) mfma_loop_kernel(int n_iter, int pattern, float* out) {
  bf16x8 a, b;
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    // pattern 0: all-zero operands (the data-independent ceiling); 1: values that
    // differ per lane and element, as real operands do (switching power is part of
    // what a real kernel can sustain)
    const float va = pattern ? 0.001f * (float)(((lane * 8 + e) * 37 + blockIdx.x) % 199 - 99) : 0.f;
    const float vb = pattern ? 0.002f * (float)(((lane * 8 + e) * 53 + blockIdx.x) % 211 - 105) : 0.f;
    a[e] = (bf16_t)va;
    b[e] = (bf16_t)vb;
  }
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int i = 0; i < n_iter; ++i) {
#pragma unroll
    for (int c = 0; c < kChains; ++c)
      acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += acc[c][r];
  if (out && sum == 12345.678f) out[0] = sum;  // keeps the loop alive; practically never stores
}

}  // namespace

extern "C" int dare_bench_mfma_loop(int n_blocks, int n_iter, int pattern, float* out, double* flops,
                                    void* hip_stream) {
  if (n_blocks < 0 || n_iter < 0 || (pattern != 0 && pattern != 1)) return 1;
  if (flops) *flops = (double)n_blocks * 4.0 * (double)n_iter * kChains * (2.0 * 32 * 32 * 16);
  if (n_blocks == 0 || n_iter == 0) return 0;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(n_blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), n_iter,
                     pattern, out);
  return hipGetLastError() == hipSuccess ? 0 : 4;
}
