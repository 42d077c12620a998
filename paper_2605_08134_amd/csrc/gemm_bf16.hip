// Row-selected bf16 projection on the gfx950 matrix cores:
//     C[t, :] = A[t, :] . W      for t in a device-side row list
// (Alg. 1 lines 2, 6-7, 11 and Alg. 2 lines 2, 7, 11 of the paper: the Q, K, V
// and output projections, for all rows or only for the refreshed rows).
//
// Layout: A rows are k-contiguous; the weight arrives packed as Wt[n, k]
// (k-contiguous), so both MFMA operands are 16-byte loads of 8 consecutive k.
// A workgroup owns a BM x BN output tile and walks k in steps of 64 through a
// double-buffered LDS stage (rows padded to 72 elements: conflict-free 16-byte
// reads).  Each wave computes the TRANSPOSED tile with v_mfma_f32_32x32x16_bf16
// (weight fragment as the first operand): a lane then owns one output row and
// runs of 4 consecutive output columns, which gives 8-byte stores and keeps a
// row's values inside one lane for row reductions.
// Workgroup ids are remapped so that the ids the hardware deals round-robin to
// the 8 XCDs become contiguous tile ranges per XCD (each XCD has its own L2).
#include "dare_common.h"

namespace dare {
namespace {

constexpr int BK = 64;
constexpr int LDS_LD = BK + 8;  // padded row, in elements

struct GemmDev {
  const bf16_t* a;
  const bf16_t* wt;
  const int32_t* idx;
  const int32_t* m_dev;
  bf16_t* c0;
  bf16_t* c1;
  bf16_t* c2;
  float* c32;
  int lda, n, k, m_max, ldc, seg_n, c32_cols;
  int tiles_m, tiles_n, per_xcd;
};

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ void __launch_bounds__(WAVES_M* WAVES_N * 64)
    gemm_bf16_kernel(GemmDev p) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");

  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * LDS_LD];

  // XCD-aware tile order: hardware id -> (xcd, slot) -> contiguous range per XCD.
  const int hw = blockIdx.x;
  const int logical = (hw & 7) * p.per_xcd + (hw >> 3);
  const int total = p.tiles_m * p.tiles_n;
  if (logical >= total) return;
  const int tile_m = logical % p.tiles_m;  // m fastest: neighbours share a weight tile
  const int tile_n = logical / p.tiles_m;
  const int m = p.m_dev ? *p.m_dev : p.m_max;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  if (m0 >= m) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
  const int l32 = lane & 31, half = lane >> 5;

  // global -> register staging pointers
  const bf16_t* a_src[A_CH];
  const bf16_t* b_src[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int ch = tid + i * NT;
    int row = m0 + (ch >> 3);
    row = row < m ? row : m - 1;
    const long tok = p.idx ? (long)p.idx[row] : (long)row;
    a_src[i] = p.a + tok * p.lda + (ch & 7) * 8;
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int ch = tid + i * NT;
    int col = n0 + (ch >> 3);
    col = col < p.n ? col : p.n - 1;
    b_src[i] = p.wt + (long)col * p.k + (ch & 7) * 8;
  }

  uint4 ra[A_CH], rb[B_CH];
  auto load_global = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) ra[i] = *reinterpret_cast<const uint4*>(a_src[i] + kt * BK);
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[i] = *reinterpret_cast<const uint4*>(b_src[i] + kt * BK);
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int ch = tid + i * NT;
      *reinterpret_cast<uint4*>(&As[buf][(ch >> 3) * LDS_LD + (ch & 7) * 8]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int ch = tid + i * NT;
      *reinterpret_cast<uint4*>(&Bs[buf][(ch >> 3) * LDS_LD + (ch & 7) * 8]) = rb[i];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = p.k / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) load_global(kt + 1);
    const bf16_t* as = &As[buf][(wave_m * WM + l32) * LDS_LD + half * 8];
    const bf16_t* bs = &Bs[buf][(wave_n * WN + l32) * LDS_LD + half * 8];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * LDS_LD + ks * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(bs + j * 32 * LDS_LD + ks * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_lds(buf ^ 1);
    __syncthreads();
  }

  // Epilogue.  acc[i][j][r] = C[row, col] with
  //   row = m0 + wave_m*WM + i*32 + l32
  //   col = n0 + wave_n*WN + j*32 + (r/4)*8 + half*4 + r%4
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wave_m * WM + i * 32 + l32;
    if (row >= m) continue;
    const long tok = p.idx ? (long)p.idx[row] : (long)row;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wave_n * WN + j * 32 + g * 8 + half * 4;
        if (col >= p.n) continue;
        const float v0 = acc[i][j][g * 4 + 0], v1 = acc[i][j][g * 4 + 1];
        const float v2 = acc[i][j][g * 4 + 2], v3 = acc[i][j][g * 4 + 3];
        const int seg = col / p.seg_n;
        bf16_t* cbase = seg == 0 ? p.c0 : (seg == 1 ? p.c1 : p.c2);
        if (cbase) {
          bf16x4 o;
          o[0] = (bf16_t)v0;
          o[1] = (bf16_t)v1;
          o[2] = (bf16_t)v2;
          o[3] = (bf16_t)v3;
          *reinterpret_cast<bf16x4*>(cbase + tok * p.ldc + (col - seg * p.seg_n)) = o;
        }
        if (p.c32 && col < p.c32_cols) {
          f32x4 o = {v0, v1, v2, v3};
          *reinterpret_cast<f32x4*>(p.c32 + tok * p.c32_cols + col) = o;
        }
      }
    }
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t s) {
  GemmDev p;
  p.a = static_cast<const bf16_t*>(g.a);
  p.wt = static_cast<const bf16_t*>(g.wt);
  p.idx = g.idx;
  p.m_dev = g.m_dev;
  p.c0 = static_cast<bf16_t*>(g.c[0]);
  p.c1 = static_cast<bf16_t*>(g.c[1]);
  p.c2 = static_cast<bf16_t*>(g.c[2]);
  p.c32 = g.c32;
  p.lda = g.lda;
  p.n = g.n;
  p.k = g.k;
  p.m_max = g.m_max;
  p.ldc = g.ldc;
  p.seg_n = g.seg_n;
  p.c32_cols = g.c32_cols;
  p.tiles_m = (g.m_max + BM - 1) / BM;
  p.tiles_n = (g.n + BN - 1) / BN;
  const int total = p.tiles_m * p.tiles_n;
  p.per_xcd = (total + 7) / 8;
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N>), dim3(p.per_xcd * 8),
                     dim3(WAVES_M * WAVES_N * 64), 0, s, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_bf16(const GemmArgs& g, hipStream_t s) {
  if (g.n % 128 == 0) return launch_cfg<128, 128, 2, 2>(g, s);
  return launch_cfg<128, 64, 4, 1>(g, s);
}

}  // namespace dare
