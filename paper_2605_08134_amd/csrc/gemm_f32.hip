// fp32 debug path of the row-selected projection C[t, :] = A[t, :] . W (same
// contract as the bf16 kernel; Alg. 1 lines 2, 6-7, 11, Alg. 2 lines 2, 7, 11).
// Plain LDS-tiled FMA kernel: 64 x 64 tile, k in steps of 16, 4 x 4 outputs per
// thread, every output one fp32 sum in k order.
#include "dare_common.h"

namespace dare {
namespace {

constexpr int FBM = 64, FBN = 64, FBK = 16, FLD = FBM + 4;

struct GemmF32Dev {
  const float* a;
  const float* wt;
  const int32_t* idx;
  const int32_t* m_dev;
  float* c0;
  float* c1;
  float* c2;
  float* c32;
  int lda, n, k, m_max, ldc, seg_n, c32_cols;
  const float* rope;
  int rope_cols, rope_dh, rope_seq;
};

__global__ void __launch_bounds__(256) gemm_f32_kernel(GemmF32Dev p) {
  __shared__ __attribute__((aligned(16))) float As[FBK][FLD];
  __shared__ __attribute__((aligned(16))) float Bs[FBK][FLD];
  const int m = p.m_dev ? *p.m_dev : p.m_max;
  const int m0 = blockIdx.x * FBM, n0 = blockIdx.y * FBN;
  if (m0 >= m) return;
  const int tid = threadIdx.x;
  const int lr = tid >> 2, lk = (tid & 3) * 4;  // staging: row, k offset
  int arow = m0 + lr;
  arow = arow < m ? arow : m - 1;
  const long atok = p.idx ? (long)p.idx[arow] : (long)arow;
  int bcol = n0 + lr;
  bcol = bcol < p.n ? bcol : p.n - 1;
  const float* asrc = p.a + atok * p.lda + lk;
  const float* bsrc = p.wt + (long)bcol * p.k + lk;
  const int ty = tid >> 4, tx = tid & 15;

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < p.k; k0 += FBK) {
    const f32x4 va = *reinterpret_cast<const f32x4*>(asrc + k0);
    const f32x4 vb = *reinterpret_cast<const f32x4*>(bsrc + k0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      As[lk + j][lr] = va[j];
      Bs[lk + j][lr] = vb[j];
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < FBK; ++kk) {
      const f32x4 a4 = *reinterpret_cast<const f32x4*>(&As[kk][ty * 4]);
      const f32x4 b4 = *reinterpret_cast<const f32x4*>(&Bs[kk][tx * 4]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a4[i], b4[j], acc[i][j]);
    }
    __syncthreads();
  }

  const int col = n0 + tx * 4;
  if (col >= p.n) return;
  const int seg = col / p.seg_n;
  float* cbase = seg == 0 ? p.c0 : (seg == 1 ? p.c1 : p.c2);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + ty * 4 + i;
    if (row >= m) continue;
    const long tok = p.idx ? (long)p.idx[row] : (long)row;
    float v0 = acc[i][0], v1 = acc[i][1], v2 = acc[i][2], v3 = acc[i][3];
    if (p.c32 && col < p.c32_cols) {  // the scored columns: before any rotation
      const f32x4 o = {v0, v1, v2, v3};
      *reinterpret_cast<f32x4*>(p.c32 + tok * p.c32_cols + col) = o;
    }
    if (cbase) {
      if (p.rope && col < p.rope_cols) rope_rotate4(p.rope, p.rope_dh, p.rope_seq, tok, col, v0, v1, v2, v3);
      const f32x4 o = {v0, v1, v2, v3};
      *reinterpret_cast<f32x4*>(cbase + tok * p.ldc + (col - seg * p.seg_n)) = o;
    }
  }
}

}  // namespace

hipError_t launch_gemm_f32(const GemmArgs& g, hipStream_t s) {
  GemmF32Dev p;
  p.a = static_cast<const float*>(g.a);
  p.wt = static_cast<const float*>(g.wt);
  p.idx = g.idx;
  p.m_dev = g.m_dev;
  p.c0 = static_cast<float*>(g.c[0]);
  p.c1 = static_cast<float*>(g.c[1]);
  p.c2 = static_cast<float*>(g.c[2]);
  p.c32 = g.c32;
  p.lda = g.lda;
  p.n = g.n;
  p.k = g.k;
  p.m_max = g.m_max;
  p.ldc = g.ldc;
  p.seg_n = g.seg_n;
  p.c32_cols = g.c32_cols;
  p.rope = g.rope;
  p.rope_cols = g.rope_cols;
  p.rope_dh = g.rope_dh;
  p.rope_seq = g.rope_seq;
  const int tm = (g.m_max + FBM - 1) / FBM, tn = (g.n + FBN - 1) / FBN;
  if (tm == 0 || tn == 0) return hipSuccess;
  hipLaunchKernelGGL(gemm_f32_kernel, dim3(tm, tn), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace dare
