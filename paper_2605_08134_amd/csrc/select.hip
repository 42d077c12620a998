// The memory-bound stages of the layer step: weight re-packing, per-token drift
// score + reuse decision + score-cache update, ordered compaction of the
// refreshed set, and row copies between token-indexed buffers.
#include "dare_common.h"

namespace dare {
namespace {

// ---------------------------------------------------------------------------
// wt[n, k] = w[k, n]: 32 x 32 tiles through LDS, both sides coalesced.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) pack_weight_kernel(const T* __restrict__ w, int rows_k,
                                                         int cols_n, T* __restrict__ wt,
                                                         int ldwt) {
  __shared__ T tile[32][33];
  const int k0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int r = ty; r < 32; r += 8) {
    const int k = k0 + r, n = n0 + tx;
    if (k < rows_k && n < cols_n) tile[r][tx] = w[(long)k * cols_n + n];
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int n = n0 + r, k = k0 + tx;
    if (k < rows_k && n < cols_n) wt[(long)n * ldwt + k] = tile[tx][r];
  }
}

// ---------------------------------------------------------------------------
// Drift score (Sec. 3.1 eq. 1) and reuse decision (Sec. 3.2 eq. 2): one wave
// per token.  The three sums use the same lane assignment and the same
// butterfly, so a token whose query did not change gets dot == |q|^2 == |p|^2
// bit for bit and a score of exactly 0.
// ---------------------------------------------------------------------------
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__global__ void __launch_bounds__(256) score_kernel(const float* __restrict__ q_new, int ld_new,
                                                   int width, int n_parts, long part_stride,
                                                   float* __restrict__ q_prev,
                                                   int n_tokens, float threshold,
                                                   int force_refresh, float* __restrict__ scores,
                                                   float* __restrict__ scores2,
                                                   uint8_t* __restrict__ mask, int seq, int prefix) {
  const int lane = threadIdx.x & 63;
  const int tok = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (tok >= n_tokens) return;
  if (prefix > 0 && tok % seq < prefix) {  // frozen token: always reused, never scored
    if (lane == 0) {
      if (scores) scores[tok] = 0.f;
      if (scores2) scores2[tok] = 0.f;
      mask[tok] = 1;
    }
    return;
  }
  const float* q = q_new + (long)tok * ld_new;
  float* p = q_prev + (long)tok * width;
  float dot = 0.f, nq = 0.f, np = 0.f;
  if ((width & 1) == 0 && (ld_new & 1) == 0 && (part_stride & 1) == 0) {
    // two neighbouring channels per lane: 8-byte loads, all slabs of a pair in flight at once
    for (int c = lane * 2; c < width; c += 128) {
      f32x2 a = *reinterpret_cast<const f32x2*>(q + c);
      for (int s = 1; s < n_parts; ++s) a += *reinterpret_cast<const f32x2*>(q + c + s * part_stride);  // k-range slabs, in order
      const f32x2 b = *reinterpret_cast<const f32x2*>(p + c);
      dot = fmaf(a[0], b[0], dot);
      nq = fmaf(a[0], a[0], nq);
      np = fmaf(b[0], b[0], np);
      dot = fmaf(a[1], b[1], dot);
      nq = fmaf(a[1], a[1], nq);
      np = fmaf(b[1], b[1], np);
      *reinterpret_cast<f32x2*>(p + c) = a;  // the score cache takes this step's query for every token
    }
  } else {
    for (int c = lane; c < width; c += 64) {
      float a = q[c];
      for (int s = 1; s < n_parts; ++s) a += q[c + s * part_stride];
      const float b = p[c];
      dot = fmaf(a, b, dot);
      nq = fmaf(a, a, nq);
      np = fmaf(b, b, np);
      p[c] = a;
    }
  }
  dot = wave_sum(dot);
  nq = wave_sum(nq);
  np = wave_sum(np);
  if (lane == 0) {
    const float den = fmaxf(sqrtf(nq * np), 1e-30f);
    const float s = 1.0f - dot / den;
    if (scores) scores[tok] = s;
    if (scores2) scores2[tok] = s;
    mask[tok] = (!force_refresh && s <= threshold) ? 1 : 0;
  }
}

// ---------------------------------------------------------------------------
// Ordered compaction (Alg. 1/2 line 5).  One workgroup per chunk of 1024
// tokens of one sequence.  Its base offset is the number of refreshed tokens in
// front of the chunk, counted from the mask bytes; inside the chunk a wave
// ballot and a prefix over the wave counts give each refreshed token its slot.
// No atomics: the list is ascending and identical from run to run.
// ---------------------------------------------------------------------------
constexpr int kChunk = 1024;

__device__ inline int block_sum_256(int v, int* sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}

// refreshed tokens (mask byte 0; the bytes are 0 or 1) in [begin, end), summed over the
// workgroup's threads by the caller: 16 bytes per thread and step between the aligned
// bounds, single bytes at the ragged ends
__device__ inline int count_refreshed(const uint8_t* __restrict__ mask, long begin, long end) {
  int c = 0;
  const long a0 = (begin + 15) & ~15l, a1 = end & ~15l;
  if (a0 >= a1) {
    for (long i = begin + threadIdx.x; i < end; i += 256) c += mask[i] == 0;
    return c;
  }
  for (long i = begin + threadIdx.x; i < a0; i += 256) c += mask[i] == 0;
  for (long i = a1 + threadIdx.x; i < end; i += 256) c += mask[i] == 0;
  const u32x4* v = reinterpret_cast<const u32x4*>(mask + a0);
  const long nv = (a1 - a0) >> 4;
  for (long i = threadIdx.x; i < nv; i += 256) {
    const u32x4 w = v[i];
    c += 16 - __popc(w[0] & 0x01010101u) - __popc(w[1] & 0x01010101u) - __popc(w[2] & 0x01010101u) -
         __popc(w[3] & 0x01010101u);
  }
  return c;
}

__global__ void __launch_bounds__(256) compact_kernel(const uint8_t* __restrict__ mask, int batch,
                                                     int seq, int32_t* __restrict__ sel_idx,
                                                     int32_t* __restrict__ sel_idx2,
                                                     int32_t* __restrict__ sel_count,
                                                     int32_t* __restrict__ sel_count2,
                                                     int32_t* __restrict__ sel_off) {
  __shared__ int sh[4];
  __shared__ int wave_cnt[4];
  const int b = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long seq_begin = (long)b * seq;
  const long begin = seq_begin + (long)chunk * kChunk;
  const long seq_end = seq_begin + seq;
  const long end = begin + kChunk < seq_end ? begin + kChunk : seq_end;

  int base = block_sum_256(count_refreshed(mask, 0, begin), sh);

  if (chunk == 0) {
    if (sel_off) sel_off[b] = base;
    if (sel_count || sel_count2 || (sel_off && b == batch - 1)) {
      const int cnt = block_sum_256(count_refreshed(mask, seq_begin, seq_end), sh);
      if (threadIdx.x == 0) {
        if (sel_count) sel_count[b] = cnt;
        if (sel_count2) sel_count2[b] = cnt;
        if (sel_off && b == batch - 1) sel_off[batch] = base + cnt;
      }
    }
  }
  if (!sel_idx && !sel_idx2) return;

  for (long t0 = begin; t0 < end; t0 += 256) {
    const long t = t0 + threadIdx.x;
    const bool sel = t < end && mask[t] == 0;
    const unsigned long long bal = __ballot(sel);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    __syncthreads();
    if (lane == 0) wave_cnt[wave] = __popcll(bal);
    __syncthreads();
    int off = base;
    for (int w = 0; w < wave; ++w) off += wave_cnt[w];
    if (sel) {
      if (sel_idx) sel_idx[off + before] = (int32_t)t;
      if (sel_idx2) sel_idx2[off + before] = (int32_t)t;
    }
    base += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
  }
}

// ---------------------------------------------------------------------------
// Threshold from a reuse rate (Sec. 3.1, "Reuse rate allocation"): per sequence, tau is
// the k-th smallest of its drift scores, found exactly by a radix select over an
// order-preserving 32-bit key (four passes of 8 bits, most significant first; NaN keys
// sort last).  One workgroup per sequence; it then writes the reuse decision s <= tau of
// its tokens and adds the sequence's score sum and count to slot b of the running drift
// statistics (the layer-wise mean drift of the same section; one slot per sequence, no
// atomics).
//   rank > 0: select and decide; rank = 0: tau = -inf, nothing reused; rank < 0: statistics
//   only (mask and tau untouched).
// ---------------------------------------------------------------------------
__device__ inline unsigned order_key(float s) {
  if (s != s) return 0xffffffffu;
  const unsigned u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float key_value(unsigned key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

constexpr int kSelectThreads = 1024;

__global__ void __launch_bounds__(kSelectThreads) quantile_mask_kernel(
    const float* __restrict__ scores, int stride, int first, int seq, int rank, int force_refresh,
    float* __restrict__ tau_out, uint8_t* __restrict__ mask, double* __restrict__ stat_sum,
    unsigned long long* __restrict__ stat_count) {
  __shared__ unsigned hist[256];
  __shared__ unsigned sh_digit, sh_rank;
  __shared__ double red_sum[kSelectThreads / 64];
  __shared__ unsigned red_cnt[kSelectThreads / 64];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // tokens [first, first + seq) of a sequence of `stride` tokens take part
  const float* s = scores + (long)b * stride + first;
  mask += (long)b * stride + first;

  float tau = -INFINITY;
  if (rank > 0) {
    unsigned prefix = 0, known = 0, want = (unsigned)rank;  // 1-based rank among the keys that match prefix
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      for (int i = tid; i < seq; i += kSelectThreads) {
        const unsigned key = order_key(s[i]);
        if ((key & known) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      if (wave == 0) {  // lane L owns bins 4L .. 4L+3; find the bin that holds the wanted rank
        unsigned c[4], tot = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          c[j] = hist[lane * 4 + j];
          tot += c[j];
        }
        unsigned incl = tot;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const unsigned up = __shfl_up(incl, o, 64);
          if (lane >= o) incl += up;
        }
        unsigned before = incl - tot;
        if (want > before && want <= incl) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (want > before && want <= before + c[j]) {
              sh_digit = (unsigned)(lane * 4 + j);
              sh_rank = want - before;
            }
            before += c[j];
          }
        }
      }
      __syncthreads();
      prefix |= sh_digit << shift;
      known |= 0xffu << shift;
      want = sh_rank;
    }
    tau = key_value(prefix);
    if (tau != tau) tau = INFINITY;  // only NaN scores left at this rank: reuse every real score
  }
  if (rank >= 0) {
    if (tid == 0 && tau_out) tau_out[b] = tau;
    for (int i = tid; i < seq; i += kSelectThreads)
      mask[i] = (!force_refresh && s[i] <= tau) ? 1 : 0;
  }
  if (stat_sum) {
    double sum = 0.0;
    unsigned cnt = 0;
    for (int i = tid; i < seq; i += kSelectThreads) {
      const float v = s[i];
      if (v == v) {
        sum += (double)v;
        ++cnt;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      sum += __shfl_xor(sum, o, 64);
      cnt += __shfl_xor(cnt, o, 64);
    }
    if (lane == 0) {
      red_sum[wave] = sum;
      red_cnt[wave] = cnt;
    }
    __syncthreads();
    if (tid == 0) {
      double t = 0.0;
      unsigned long long n = 0;
      for (int w = 0; w < kSelectThreads / 64; ++w) {
        t += red_sum[w];
        n += red_cnt[w];
      }
      // slot b belongs to this workgroup alone and steps are ordered by the stream: a plain
      // read-modify-write, the same sum from run to run (the reader adds the slots in order)
      stat_sum[b] += t;
      stat_count[b] += n;
    }
  }
}

// ---------------------------------------------------------------------------
// Row list of the tokens that are not frozen: ids b*seq + prefix .. b*seq + seq - 1 of
// every sequence, ascending, and the offsets b * (seq - prefix) of the sequences in it.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) active_list_kernel(int batch, int seq, int prefix, int32_t* __restrict__ act_idx,
                                                         int32_t* __restrict__ act_off) {
  const int ta = seq - prefix;
  const long n = (long)batch * ta;
  for (long r = (long)blockIdx.x * 256 + threadIdx.x; r < n; r += (long)gridDim.x * 256)
    act_idx[r] = (int32_t)((r / ta) * seq + prefix + r % ta);
  if (blockIdx.x == 0)
    for (int b = threadIdx.x; b <= batch; b += 256) act_off[b] = b * ta;
}

// ---------------------------------------------------------------------------
// dst[t] = src[t] for the listed (or all) rows: 16 bytes per lane, a row is a
// contiguous run of full cache lines.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) copy_rows_kernel(const uint4* __restrict__ src,
                                                       uint4* __restrict__ dst, int n_rows,
                                                       int row_vec, const int32_t* __restrict__ idx,
                                                       const int32_t* __restrict__ m_dev) {
  const int m = idx ? (m_dev ? *m_dev : n_rows) : n_rows;
  for (int r = blockIdx.x; r < m; r += gridDim.x) {
    const long tok = idx ? (long)idx[r] : (long)r;
    const uint4* s = src + tok * row_vec;
    uint4* d = dst + tok * row_vec;
    for (int c = threadIdx.x; c < row_vec; c += 256) d[c] = s[c];
  }
}

}  // namespace

hipError_t launch_pack_weight(int dtype, const void* w, int rows_k, int cols_n, void* wt, int ldwt,
                              hipStream_t s) {
  dim3 grid((cols_n + 31) / 32, (rows_k + 31) / 32);
  if (dtype == DARE_BF16)
    hipLaunchKernelGGL(pack_weight_kernel<bf16_t>, grid, dim3(256), 0, s,
                       static_cast<const bf16_t*>(w), rows_k, cols_n, static_cast<bf16_t*>(wt),
                       ldwt);
  else
    hipLaunchKernelGGL(pack_weight_kernel<float>, grid, dim3(256), 0, s,
                       static_cast<const float*>(w), rows_k, cols_n, static_cast<float*>(wt), ldwt);
  return hipGetLastError();
}

hipError_t launch_score(const float* q_new, int ld_new, int width, int n_parts, long part_stride,
                        float* q_prev, int n_tokens, float threshold, int force_refresh, float* scores, float* scores2,
                        uint8_t* mask, int seq, int prefix, hipStream_t s) {
  if (n_tokens == 0) return hipSuccess;
  hipLaunchKernelGGL(score_kernel, dim3((n_tokens + 3) / 4), dim3(256), 0, s, q_new, ld_new, width,
                     n_parts, part_stride, q_prev, n_tokens, threshold, force_refresh, scores, scores2, mask,
                     seq, prefix);
  return hipGetLastError();
}

hipError_t launch_compact(const uint8_t* mask, int batch, int seq, int32_t* sel_idx,
                          int32_t* sel_idx2, int32_t* sel_count, int32_t* sel_count2,
                          int32_t* sel_off, hipStream_t s) {
  dim3 grid((seq + kChunk - 1) / kChunk, batch);
  hipLaunchKernelGGL(compact_kernel, grid, dim3(256), 0, s, mask, batch, seq, sel_idx, sel_idx2,
                     sel_count, sel_count2, sel_off);
  return hipGetLastError();
}

hipError_t launch_quantile_mask(const float* scores, int batch, int stride, int first, int seq, int rank,
                                int force_refresh, float* tau_out, uint8_t* mask, double* stat_sum,
                                unsigned long long* stat_count, hipStream_t s) {
  if (batch == 0 || seq == 0) return hipSuccess;
  hipLaunchKernelGGL(quantile_mask_kernel, dim3(batch), dim3(kSelectThreads), 0, s, scores, stride, first, seq,
                     rank, force_refresh, tau_out, mask, stat_sum, stat_count);
  return hipGetLastError();
}

namespace {
__global__ void zero_words_kernel(unsigned long long* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0ull;
}
}  // namespace

// n 64-bit words <- 0 with a kernel (a memset node does not survive a graph capture)
hipError_t launch_zero_words(void* p, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(zero_words_kernel, dim3((n + 63) / 64), dim3(64), 0, s, static_cast<unsigned long long*>(p), n);
  return hipGetLastError();
}

hipError_t launch_active_list(int batch, int seq, int prefix, int32_t* act_idx, int32_t* act_off, hipStream_t s) {
  const long n = (long)batch * (seq - prefix);
  const int grid = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
  hipLaunchKernelGGL(active_list_kernel, dim3(grid < 1 ? 1 : grid), dim3(256), 0, s, batch, seq, prefix, act_idx,
                     act_off);
  return hipGetLastError();
}

hipError_t launch_copy_rows(const void* src, void* dst, int n_rows, int row_bytes,
                            const int32_t* idx, const int32_t* m_dev, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  const int grid = n_rows < 4096 ? n_rows : 4096;
  hipLaunchKernelGGL(copy_rows_kernel, dim3(grid), dim3(256), 0, s, static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), n_rows, row_bytes / 16, idx, m_dev);
  return hipGetLastError();
}

}  // namespace dare
