// Bidirectional multi-head attention for a selected set of query rows on the
// gfx950 matrix cores (App. E.2; Alg. 1 line 10; Alg. 2 line 8):
//     out[t, h] = softmax(q[t, h] . K_b[:, h]^T / sqrt(Dh)) V_b[:, h]
// with t running over all tokens or over the refreshed tokens of each sequence.
//
// One workgroup = 4 waves = 128 query rows of one (sequence, head); each wave
// owns 32 rows.  Keys/values stream through LDS in tiles of 64 rows.  The wave
// computes the TRANSPOSED logits S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so a
// lane holds 32 logits of ONE query row: the running max / sum of the online
// softmax are per-lane scalars (one exchange with lane^32), and the
// probabilities are already in the register layout of the second operand of
// O^T = V^T P^T.  V is transposed on its way into LDS (4 keys x 8 channels per
// thread, 8-byte LDS writes), K is stored as it is.
#include "dare_common.h"

namespace dare {
namespace {

constexpr int BQ = 128;   // query rows per workgroup
constexpr int BKV = 64;   // keys per tile
constexpr float kLog2e = 1.4426950408889634f;

struct AttnDev {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  bf16_t* out;
  const int32_t* idx;
  const int32_t* sel_off;
  int seq, d;
  float scale_log2;
};

template <int DH>
__global__ void __launch_bounds__(256) attn_bf16_kernel(AttnDev p) {
  constexpr int K_LD = DH + 8;     // Ks[key][channel], padded
  constexpr int V_LD = BKV + 8;    // Vt[channel][key], padded
  constexpr int KSTEPS = DH / 16;  // k-steps of the logits product
  constexpr int OT = DH / 32;      // 32-channel tiles of the output
  constexpr int K_CH = BKV * (DH / 8) / 256;  // 16-byte chunks of K per thread
  constexpr int DG = DH / 8;       // channel groups of 8

  __shared__ __attribute__((aligned(16))) bf16_t Ks[BKV * K_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Vt[DH * V_LD];

  const int b = blockIdx.z, h = blockIdx.y, qt = blockIdx.x;
  const int T = p.seq;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;

  // the query row of this lane
  int cnt, off;
  if (p.idx) {
    off = p.sel_off[b];
    cnt = p.sel_off[b + 1] - off;
  } else {
    off = b * T;
    cnt = T;
  }
  if (qt * BQ >= cnt) return;
  const int j = qt * BQ + wave * 32 + l32;
  const bool valid = j < cnt;
  const int jc = valid ? j : cnt - 1;
  const long tok = p.idx ? (long)p.idx[off + jc] : (long)(off + jc);

  bf16x8 qf[KSTEPS];
  {
    const bf16_t* qrow = p.q + tok * p.d + h * DH + half * 8;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
      qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
  }

  const bf16_t* kbase = p.k + (long)b * T * p.d + h * DH;
  const bf16_t* vbase = p.v + (long)b * T * p.d + h * DH;

  // staging assignment
  const int v_dg = tid % DG, v_kg = tid / DG;  // V: 8 channels x 4 keys per thread
  constexpr bool kAllStageV = 256 / DG == BKV / 4;  // every thread has a V unit
  const bool v_active = kAllStageV || v_kg < BKV / 4;
  u32x4 rk[K_CH], rv[4];
  auto load_global = [&](int kv0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < K_CH; ++i) {
      const int ch = tid + i * 256;
      int key = kv0 + ch / DG;
      key = key < T ? key : T - 1;
      rk[i] = *reinterpret_cast<const u32x4*>(kbase + (long)key * p.d + (ch % DG) * 8);
    }
    if (v_active) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        int key = kv0 + v_kg * 4 + r;
        key = key < T ? key : T - 1;
        rv[r] = *reinterpret_cast<const u32x4*>(vbase + (long)key * p.d + v_dg * 8);
      }
    }
  };
  auto store_lds = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < K_CH; ++i) {
      const int ch = tid + i * 256;
      *reinterpret_cast<u32x4*>(&Ks[(ch / DG) * K_LD + (ch % DG) * 8]) = rk[i];
    }
    if (v_active) {
      const u32x4 w0 = rv[0], w1 = rv[1], w2 = rv[2], w3 = rv[3];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // channels 2e (low halves) and 2e+1 (high halves) of the 4 keys
        u32x2 lo, hi;
        lo[0] = (w0[e] & 0xffffu) | (w1[e] << 16);
        lo[1] = (w2[e] & 0xffffu) | (w3[e] << 16);
        hi[0] = (w0[e] >> 16) | (w1[e] & 0xffff0000u);
        hi[1] = (w2[e] >> 16) | (w3[e] & 0xffff0000u);
        *reinterpret_cast<u32x2*>(&Vt[(v_dg * 8 + 2 * e) * V_LD + v_kg * 4]) = lo;
        *reinterpret_cast<u32x2*>(&Vt[(v_dg * 8 + 2 * e + 1) * V_LD + v_kg * 4]) = hi;
      }
    }
  };

  f32x16 acc_o[OT];
#pragma unroll
  for (int t = 0; t < OT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[t][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  load_global(0);
  for (int kv0 = 0; kv0 < T; kv0 += BKV) {
    store_lds();
    __syncthreads();
    // prefetch the next tile; past the end the last tile is fetched again (unused),
    // which keeps the loop body free of a conditional around the staged registers
    load_global(kv0 + BKV < T ? kv0 + BKV : kv0);

    // S^T tile: 64 keys x 32 query rows, as two 32-key MFMA tiles
    f32x16 acc_s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_s[kt][r] = 0.f;
      const bf16_t* ks_row = &Ks[(kt * 32 + l32) * K_LD + half * 8];
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks_row + ks * 16);
        acc_s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[kt], 0, 0, 0);
      }
    }
    // register r of tile kt is key kv0 + kt*32 + (r/4)*8 + half*4 + r%4
    const bool ragged = kv0 + BKV > T;
    float m_tile = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float s = acc_s[kt][r] * p.scale_log2;
        if (ragged) {
          const int key = kv0 + kt * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          if (key >= T) s = -INFINITY;
        }
        acc_s[kt][r] = s;
        m_tile = fmaxf(m_tile, s);
      }
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64));
    const float m_new = fmaxf(m_run, m_tile);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float l_tile = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        // the row sum is taken over the probabilities as rounded for the value
        // product, so numerator and denominator carry the same rounding
        const bf16_t pb = (bf16_t)__builtin_amdgcn_exp2f(acc_s[kt][r] - m_new);
        l_tile += (float)pb;
        pf[kt * 2 + (r >> 3)][r & 7] = pb;
      }
    l_run = l_run * alpha + l_tile;
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[t][r] *= alpha;

    // O^T += V^T P^T.  Slot s of P fragment s4 is key s4*16 + (s/4)*8 + half*4 + s%4.
#pragma unroll
    for (int t = 0; t < OT; ++t) {
      const bf16_t* vt_row = &Vt[(t * 32 + l32) * V_LD + half * 4];
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vt_row + s4 * 16);
        const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vt_row + s4 * 16 + 8);
        const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        acc_o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[s4], acc_o[t], 0, 0, 0);
      }
    }
    __syncthreads();
  }

  const float l_all = l_run + __shfl_xor(l_run, 32, 64);
  if (!valid) return;
  const float inv = 1.0f / l_all;
  bf16_t* orow = p.out + tok * p.d + h * DH + half * 4;
#pragma unroll
  for (int t = 0; t < OT; ++t)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(acc_o[t][g * 4 + e] * inv);
      *reinterpret_cast<bf16x4*>(orow + t * 32 + g * 8) = o;
    }
}

}  // namespace

uint64_t attn_bf16_work_bytes(int, int, int, int) { return 0; }

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t s) {
  AttnDev p;
  p.q = static_cast<const bf16_t*>(a.q);
  p.k = static_cast<const bf16_t*>(a.k);
  p.v = static_cast<const bf16_t*>(a.v);
  p.out = static_cast<bf16_t*>(a.out);
  p.idx = a.idx;
  p.sel_off = a.sel_off;
  p.seq = a.seq;
  p.d = a.n_heads * a.head_dim;
  p.scale_log2 = kLog2e / sqrtf((float)a.head_dim);
  dim3 grid((a.seq + BQ - 1) / BQ, a.n_heads, a.batch);
  if (a.head_dim == 128)
    hipLaunchKernelGGL(attn_bf16_kernel<128>, grid, dim3(256), 0, s, p);
  else if (a.head_dim == 64)
    hipLaunchKernelGGL(attn_bf16_kernel<64>, grid, dim3(256), 0, s, p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace dare
