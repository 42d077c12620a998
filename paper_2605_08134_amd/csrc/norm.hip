// The block around the layer step: normalisation of the hidden state before the
// projections (Alg. 1/2 line 1: LayerNorm; the root-mean-square variant of
// LLaDA-class models) and the residual sum after the output projection.
// Memory-bound: one read and one write of a [tokens, d] tensor each.
#include "dare_common.h"

namespace dare {
namespace {

__device__ inline float block_sum(float v, float* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();  // sh may still be read from the previous call
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}

// 8 consecutive elements (16-byte aligned groups) to and from fp32
__device__ inline void load8(const bf16_t* p, float* v) {
  const bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)t[e];
}
__device__ inline void load8(const float* p, float* v) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v[e] = a[e];
    v[4 + e] = b[e];
  }
}
__device__ inline void store8(bf16_t* p, const float* v) {
  bf16x8 t;
#pragma unroll
  for (int e = 0; e < 8; ++e) t[e] = (bf16_t)v[e];
  *reinterpret_cast<bf16x8*>(p) = t;
}
__device__ inline void store8(float* p, const float* v) {
  const f32x4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
  *reinterpret_cast<f32x4*>(p) = a;
  *reinterpret_cast<f32x4*>(p + 4) = b;
}

// One workgroup of 256 threads per token row.  Thread t owns the 8-element groups
// t, t + 256, ... of the row (16 B loads for bf16, 2 x 16 B for fp32); up to kHold
// groups are kept in registers, so a row of up to 256 * 8 * kHold channels is read from
// memory once.  kind 1: (x - mean) / sqrt(var + eps) * gain + bias, variance taken around
// the mean in a second pass over the registers; kind 2: x / sqrt(mean(x^2) + eps) * gain.
constexpr int kHold = 4;

template <typename T>
__global__ void __launch_bounds__(256) norm_kernel(const T* __restrict__ x, const T* __restrict__ gain,
                                                   const T* __restrict__ bias, float eps, int d, int kind,
                                                   T* __restrict__ out, int seq, int prefix) {
  __shared__ float sh[4];
  long tok = blockIdx.x;
  if (seq > 0) tok = (tok / (seq - prefix)) * seq + prefix + tok % (seq - prefix);  // skip a frozen prefix
  const T* row = x + tok * d;
  T* orow = out + tok * d;
  const int groups = d >> 3;
  float v[kHold][8];
  float s1 = 0.f;
#pragma unroll
  for (int h = 0; h < kHold; ++h) {
    const int g = threadIdx.x + h * 256;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[h][e] = 0.f;
    if (g < groups) load8(row + g * 8, v[h]);
#pragma unroll
    for (int e = 0; e < 8; ++e) s1 += kind == 1 ? v[h][e] : v[h][e] * v[h][e];
  }
  for (int g = threadIdx.x + kHold * 256; g < groups; g += 256) {  // rows longer than the registers hold
    float a[8];
    load8(row + g * 8, a);
#pragma unroll
    for (int e = 0; e < 8; ++e) s1 += kind == 1 ? a[e] : a[e] * a[e];
  }
  s1 = block_sum(s1, sh);
  float mean = 0.f, scale;
  if (kind == 1) {
    mean = s1 / (float)d;
    float s2 = 0.f;
#pragma unroll
    for (int h = 0; h < kHold; ++h) {
      const int g = threadIdx.x + h * 256;
      if (g < groups) {
#pragma unroll
        for (int e = 0; e < 8; ++e) s2 += (v[h][e] - mean) * (v[h][e] - mean);
      }
    }
    for (int g = threadIdx.x + kHold * 256; g < groups; g += 256) {
      float a[8];
      load8(row + g * 8, a);
#pragma unroll
      for (int e = 0; e < 8; ++e) s2 += (a[e] - mean) * (a[e] - mean);
    }
    s2 = block_sum(s2, sh);
    scale = 1.0f / sqrtf(s2 / (float)d + eps);
  } else {
    scale = 1.0f / sqrtf(s1 / (float)d + eps);
  }
  auto finish = [&](int g, const float* a) {
    float gn[8], y[8];
    load8(gain + g * 8, gn);
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = (a[e] - mean) * scale * gn[e];
    if (bias) {
      float bs[8];
      load8(bias + g * 8, bs);
#pragma unroll
      for (int e = 0; e < 8; ++e) y[e] += bs[e];
    }
    store8(orow + g * 8, y);
  };
#pragma unroll
  for (int h = 0; h < kHold; ++h) {
    const int g = threadIdx.x + h * 256;
    if (g < groups) finish(g, v[h]);
  }
  for (int g = threadIdx.x + kHold * 256; g < groups; g += 256) {
    float a[8];
    load8(row + g * 8, a);
    finish(g, a);
  }
}

// out = x + o, 8 elements per thread and step.
template <typename T>
__global__ void __launch_bounds__(256) residual_add_kernel(const T* __restrict__ x, const T* __restrict__ o,
                                                           T* __restrict__ out, long n_groups) {
  for (long g = (long)blockIdx.x * 256 + threadIdx.x; g < n_groups; g += (long)gridDim.x * 256) {
    float a[8], b[8];
    load8(x + g * 8, a);
    load8(o + g * 8, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] += b[e];
    store8(out + g * 8, a);
  }
}

// x[t, :] <- x[t, :] + o[t, :] (rounded to T as it is stored), h[t, :] <- that row / sqrt(mean of its
// squares + eps) * gain: the residual sum of one block fused with the RMS normalisation that opens
// the next.  One workgroup per row, the row held in registers (d <= 256 * 8 * kHold), rows mapped
// past a frozen prefix as in norm_kernel.
template <typename T>
__global__ void __launch_bounds__(256) residual_norm_kernel(T* __restrict__ x, const T* __restrict__ o,
                                                            const T* __restrict__ gain, float eps, int d,
                                                            T* __restrict__ h, int seq, int prefix) {
  __shared__ float sh[4];
  long tok = blockIdx.x;
  if (seq > 0) tok = (tok / (seq - prefix)) * seq + prefix + tok % (seq - prefix);
  T* xr = x + tok * d;
  const T* orow = o + tok * d;
  T* hr = h + tok * d;
  const int groups = d >> 3;
  float v[kHold][8];
  float s1 = 0.f;
#pragma unroll
  for (int k = 0; k < kHold; ++k) {
    const int g = threadIdx.x + k * 256;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[k][e] = 0.f;
    if (g < groups) {
      float a[8], b[8];
      load8(xr + g * 8, a);
      load8(orow + g * 8, b);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[k][e] = (float)(T)(a[e] + b[e]);  // the stored sum
      store8(xr + g * 8, v[k]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s1 += v[k][e] * v[k][e];
  }
  s1 = block_sum(s1, sh);
  const float scale = 1.0f / sqrtf(s1 / (float)d + eps);
#pragma unroll
  for (int k = 0; k < kHold; ++k) {
    const int g = threadIdx.x + k * 256;
    if (g < groups) {
      float gn[8], y[8];
      load8(gain + g * 8, gn);
#pragma unroll
      for (int e = 0; e < 8; ++e) y[e] = v[k][e] * scale * gn[e];
      store8(hr + g * 8, y);
    }
  }
}

// x[t, :] += f[t, :] for the listed rows (a frozen prefix leaves the other rows alone).
template <typename T>
__global__ void __launch_bounds__(256) residual_rows_kernel(T* __restrict__ x, const T* __restrict__ f, int n_rows,
                                                            int d, const int32_t* __restrict__ idx) {
  const int groups = d >> 3;
  for (int r = blockIdx.x; r < n_rows; r += gridDim.x) {
    const long tok = (long)idx[r];
    for (int g = threadIdx.x; g < groups; g += 256) {
      float a[8], b[8];
      load8(x + tok * d + g * 8, a);
      load8(f + tok * d + g * 8, b);
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] += b[e];
      store8(x + tok * d + g * 8, a);
    }
  }
}

}  // namespace

// returns hipErrorInvalidValue for rows longer than the kernel holds in registers
hipError_t launch_residual_norm(int dtype, void* x, const void* o, const void* gain, float eps, int n_rows, int d,
                                void* h, int seq, int prefix, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  if (d > 256 * 8 * kHold || (d & 7)) return hipErrorInvalidValue;
  if (dtype == DARE_BF16)
    hipLaunchKernelGGL(residual_norm_kernel<bf16_t>, dim3(n_rows), dim3(256), 0, s, static_cast<bf16_t*>(x),
                       static_cast<const bf16_t*>(o), static_cast<const bf16_t*>(gain), eps, d,
                       static_cast<bf16_t*>(h), seq, prefix);
  else
    hipLaunchKernelGGL(residual_norm_kernel<float>, dim3(n_rows), dim3(256), 0, s, static_cast<float*>(x),
                       static_cast<const float*>(o), static_cast<const float*>(gain), eps, d, static_cast<float*>(h),
                       seq, prefix);
  return hipGetLastError();
}

hipError_t launch_residual_rows(int dtype, void* x, const void* f, int n_rows, int d, const int32_t* idx,
                                hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  const int grid = n_rows < 8192 ? n_rows : 8192;
  if (dtype == DARE_BF16)
    hipLaunchKernelGGL(residual_rows_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, static_cast<bf16_t*>(x),
                       static_cast<const bf16_t*>(f), n_rows, d, idx);
  else
    hipLaunchKernelGGL(residual_rows_kernel<float>, dim3(grid), dim3(256), 0, s, static_cast<float*>(x),
                       static_cast<const float*>(f), n_rows, d, idx);
  return hipGetLastError();
}

hipError_t launch_norm(int dtype, int kind, const void* x, const void* gain, const void* bias, float eps,
                       int n_rows, int d, void* out, int seq, int prefix, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  if (dtype == DARE_BF16)
    hipLaunchKernelGGL(norm_kernel<bf16_t>, dim3(n_rows), dim3(256), 0, s, static_cast<const bf16_t*>(x),
                       static_cast<const bf16_t*>(gain), static_cast<const bf16_t*>(bias), eps, d, kind,
                       static_cast<bf16_t*>(out), seq, prefix);
  else
    hipLaunchKernelGGL(norm_kernel<float>, dim3(n_rows), dim3(256), 0, s, static_cast<const float*>(x),
                       static_cast<const float*>(gain), static_cast<const float*>(bias), eps, d, kind,
                       static_cast<float*>(out), seq, prefix);
  return hipGetLastError();
}

hipError_t launch_residual_add(int dtype, const void* x, const void* o, void* out, long n_elems,
                               hipStream_t s) {
  const long groups = n_elems / 8;
  if (groups == 0) return hipSuccess;
  const long want = (groups + 255) / 256;
  const int grid = (int)(want < 8192 ? want : 8192);
  if (dtype == DARE_BF16)
    hipLaunchKernelGGL(residual_add_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, static_cast<const bf16_t*>(x),
                       static_cast<const bf16_t*>(o), static_cast<bf16_t*>(out), groups);
  else
    hipLaunchKernelGGL(residual_add_kernel<float>, dim3(grid), dim3(256), 0, s, static_cast<const float*>(x),
                       static_cast<const float*>(o), static_cast<float*>(out), groups);
  return hipGetLastError();
}

}  // namespace dare
