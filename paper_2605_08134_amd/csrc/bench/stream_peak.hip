// Streams from memory into LDS, one workgroup per CU: what ONE CU can pull, and how the
// rate scales with the number of CUs that pull at once.  Every workgroup walks its own
// contiguous span of the source once (global -> LDS loads of 16 bytes per lane, the load the
// projection and attention kernels use), so with a source far larger than the last-level
// cache nothing is re-read.  Benchmark aid: built into libdare_bench.so, not into the
// product library.
#include <hip/hip_runtime.h>

#include "dare_bench.h"

namespace {

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int kWaves = 8;                 // waves per workgroup
constexpr int kBatch = 8;                 // 1 KiB loads a wave issues before it waits
constexpr int kIterBytes = kWaves * kBatch * 1024;

// DEPTH batches of a wave may be in flight (DEPTH * 64 KiB per workgroup).
template <int DEPTH>
__global__ void __launch_bounds__(kWaves * 64) stream_kernel(const unsigned char* __restrict__ src,
                                                              unsigned long long span, int iters, unsigned* out) {
  __shared__ __attribute__((aligned(1024))) unsigned char ring[2 * kIterBytes];
  const unsigned lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned char* base = src + (unsigned long long)blockIdx.x * span + lane * 16;
  for (int it = 0; it < iters; ++it) {
    unsigned char* mine = ring + ((it & 1) * kWaves + wave) * kBatch * 1024;
    const unsigned char* from = base + ((unsigned long long)it * kWaves + wave) * kBatch * 1024;
#pragma unroll
    for (int i = 0; i < kBatch; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(from + i * 1024), (lptr_t)(mine + i * 1024), 16, 0, 0);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DEPTH - 1) * kBatch) : "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  const unsigned v = *reinterpret_cast<const unsigned*>(ring + threadIdx.x * 4);
  if (out && v == 0x12345678u) out[0] = v;  // keeps the loads alive; practically never stores
}

}  // namespace

extern "C" int dare_bench_stream(int n_blocks, unsigned long long bytes_per_block, int depth, const void* src,
                                 unsigned* out, void* hip_stream) {
  if (n_blocks < 0 || !src || bytes_per_block % kIterBytes != 0 || bytes_per_block / kIterBytes > 0x7fffffffULL)
    return 1;
  if (n_blocks == 0 || bytes_per_block == 0) return 0;
  const int iters = (int)(bytes_per_block / kIterBytes);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const unsigned char* p = static_cast<const unsigned char*>(src);
  if (depth == 1)
    hipLaunchKernelGGL(stream_kernel<1>, dim3(n_blocks), dim3(kWaves * 64), 0, s, p, bytes_per_block, iters, out);
  else if (depth == 2)
    hipLaunchKernelGGL(stream_kernel<2>, dim3(n_blocks), dim3(kWaves * 64), 0, s, p, bytes_per_block, iters, out);
  else if (depth == 4)
    hipLaunchKernelGGL(stream_kernel<4>, dim3(n_blocks), dim3(kWaves * 64), 0, s, p, bytes_per_block, iters, out);
  else
    return 1;
  return hipGetLastError() == hipSuccess ? 0 : 4;
}
