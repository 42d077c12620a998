// fp32 debug path of the selected-row bidirectional attention (App. E.2; Alg. 1
// line 10; Alg. 2 line 8).  One wave per (query row, head): logits for a chunk of
// keys go to LDS, the running max / sum are rescaled chunk by chunk, and the
// value sum is accumulated with one lane per output channel.
#include "dare_common.h"

namespace dare {
namespace {

constexpr int kKeysPerChunk = 512;

struct AttnF32Dev {
  const float* q;
  const float* k;
  const float* v;
  float* out;
  const int32_t* idx;
  const int32_t* sel_off;
  int seq, d;
  float scale;
};

__device__ inline float wave_max_f(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline float wave_sum_f(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <int DH>
__global__ void __launch_bounds__(256) attn_f32_kernel(AttnF32Dev p) {
  constexpr int R = DH / 64;  // output channels per lane
  __shared__ float zs[4][kKeysPerChunk];
  __shared__ float qs[4][DH];
  const int b = blockIdx.z, h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int T = p.seq;
  int cnt, off;
  if (p.idx) {
    off = p.sel_off[b];
    cnt = p.sel_off[b + 1] - off;
  } else {
    off = b * T;
    cnt = T;
  }
  if (blockIdx.x * 4 >= cnt) return;  // uniform for the workgroup
  const int j = blockIdx.x * 4 + wave;
  const bool valid = j < cnt;
  const int jc = valid ? j : cnt - 1;
  const long tok = p.idx ? (long)p.idx[off + jc] : (long)(off + jc);

  for (int c = lane; c < DH; c += 64) qs[wave][c] = p.q[tok * p.d + h * DH + c];
  __syncthreads();

  const float* kbase = p.k + (long)b * T * p.d + h * DH;
  const float* vbase = p.v + (long)b * T * p.d + h * DH;
  float acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  for (int c0 = 0; c0 < T; c0 += kKeysPerChunk) {
    const int nk = T - c0 < kKeysPerChunk ? T - c0 : kKeysPerChunk;
    float m_loc = -INFINITY;
    for (int jj = lane; jj < nk; jj += 64) {
      const float* kr = kbase + (long)(c0 + jj) * p.d;
      float z = 0.f;
      for (int c = 0; c < DH; c += 4) {
        const f32x4 kv = *reinterpret_cast<const f32x4*>(kr + c);
        z = fmaf(qs[wave][c], kv[0], z);
        z = fmaf(qs[wave][c + 1], kv[1], z);
        z = fmaf(qs[wave][c + 2], kv[2], z);
        z = fmaf(qs[wave][c + 3], kv[3], z);
      }
      z *= p.scale;
      zs[wave][jj] = z;
      m_loc = fmaxf(m_loc, z);
    }
    const float m_new = fmaxf(m_run, wave_max_f(m_loc));
    const float alpha = expf(m_run - m_new);
    m_run = m_new;
    __syncthreads();
    float l_loc = 0.f;
    for (int jj = lane; jj < nk; jj += 64) {
      const float pr = expf(zs[wave][jj] - m_new);
      zs[wave][jj] = pr;
      l_loc += pr;
    }
    l_run = l_run * alpha + wave_sum_f(l_loc);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] *= alpha;
    for (int jj = 0; jj < nk; ++jj) {
      const float pr = zs[wave][jj];
      const float* vr = vbase + (long)(c0 + jj) * p.d;
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] = fmaf(pr, vr[lane + 64 * r], acc[r]);
    }
    __syncthreads();
  }
  if (!valid) return;
  const float inv = 1.0f / l_run;
#pragma unroll
  for (int r = 0; r < R; ++r) p.out[tok * p.d + h * DH + lane + 64 * r] = acc[r] * inv;
}

}  // namespace

hipError_t launch_attn_f32(const AttnArgs& a, hipStream_t s) {
  AttnF32Dev p;
  p.q = static_cast<const float*>(a.q);
  p.k = static_cast<const float*>(a.k);
  p.v = static_cast<const float*>(a.v);
  p.out = static_cast<float*>(a.out);
  p.idx = a.idx;
  p.sel_off = a.sel_off;
  p.seq = a.seq;
  p.d = a.n_heads * a.head_dim;
  p.scale = 1.0f / sqrtf((float)a.head_dim);
  dim3 grid((a.seq + 3) / 4, a.n_heads, a.batch);
  if (a.head_dim == 128)
    hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(256), 0, s, p);
  else if (a.head_dim == 64)
    hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(256), 0, s, p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace dare
