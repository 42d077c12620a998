// Bidirectional multi-head attention for a selected set of query rows on the
// gfx950 matrix cores (App. E.2; Alg. 1 line 10; Alg. 2 line 8):
//     out[t, h] = softmax(q[t, h] . K_b[:, h]^T / sqrt(Dh)) V_b[:, h]
// with t running over all tokens or over the refreshed tokens of each sequence.
//
// A workgroup serves 32 * QW query rows of one (sequence, head) with QW * KW waves:
// wave (qw, kw) owns 32 query rows and every KW-th tile of TK keys.  K and V tiles go
// from global memory straight into LDS (global_load_lds_dwordx4) through a ring of
// NST stages, rows kept as they are in memory ([key][channel]); bank conflicts are
// removed by fetching, into the LDS slot a lane owns, the 16-byte chunk that an XOR
// of the key index assigns to it.
//
// Each wave computes the TRANSPOSED logits S^T = K Q^T with
// v_mfma_f32_32x32x16_bf16, so a lane holds the logits of ONE query row: the running
// max / sum of the online softmax are per-lane scalars (one exchange with lane^32),
// and the probabilities are already in the register layout of the second operand of
// O^T = V^T P^T.  The first operand, V^T, is read from the row-major V tile with the
// LDS transpose read ds_read_b64_tr_b16 (a lane receives 4 consecutive keys of one
// channel), so V needs no transposition pass.
//
// With KW > 1 the key-waves of a query block each keep their own running
// (max, sum, O) and are merged once at the end through LDS, in a fixed order.
// Few query rows (the refreshed rows of a step) use narrow query blocks with KW > 1,
// which turns the available waves towards the key axis and fills the chip; many
// rows use wide blocks (128 rows with two key-waves, or 256 rows with none when there are
// enough of them), which re-read K and V less often.
#include "dare_common.h"

namespace dare {
namespace {

constexpr float kLog2e = 1.4426950408889634f;

struct AttnDev {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  bf16_t* out;
  const int32_t* idx;
  const int32_t* sel_off;
  int seq, d;
  int n_heads, n_pairs, n_qt;  // heads, batch*heads, query blocks launched per (sequence, head)
  float scale_log2;
};

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

template <int N>
__device__ __forceinline__ void wait_vmcnt_and_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_all_and_barrier() {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int DH, int KW, int TK, int NST>
constexpr int attn_smem_bytes() {
  return NST * KW * 2 * TK * DH * 2;
}

// XOR applied to the 16-byte chunk index of a K row / V row (see the header).
template <int DH>
__device__ __forceinline__ int k_swizzle(int key) {
  return DH == 128 ? (key & 15) : ((key >> 1) & 7);
}
template <int DH>
__device__ __forceinline__ int v_swizzle(int key) {
  return DH == 128 ? ((key & 3) << 2) : (((key >> 1) & 1) << 2);
}

// One query block.  b, h: sequence and head; qt: query block index inside the row set
// [off, off + cnt) of the sequence.  Called by all QW*KW waves of the workgroup.
template <int DH, int QW, int KW, int TK, int NST>
__device__ __forceinline__ void attn_block(const AttnDev& p, int b, int h, int qt, int cnt, int off,
                                           unsigned char* smem) {
  constexpr int NW = QW * KW;
  constexpr int ROWB = DH * 2;             // bytes per K or V row of one head
  constexpr int CPR = DH / 8;              // 16-byte chunks per row
  constexpr int RPL = 64 / CPR;            // rows covered by one wave load
  constexpr int TILE_BYTES = TK * ROWB;
  constexpr int STAGE_BYTES = KW * 2 * TILE_BYTES;
  constexpr int NL = STAGE_BYTES / 1024;   // wave loads per stage
  constexpr int LPW = NL / NW;
  constexpr int KSTEPS = DH / 16;          // k-steps of the logits product
  constexpr int OT = DH / 32;              // 32-channel tiles of the output
  constexpr int ST = TK / 32;              // 32-key tiles of the logits
  constexpr int PS = TK / 16;              // 16-key slices of the value product
  static_assert(NL % NW == 0, "stage loads must divide among the waves");
  static_assert(LPW * (NST - 1) < 64, "vmcnt range");

  const int T = p.seq;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (a scalar: M0 addressing)
  const int qw = wave % QW, kw = wave / QW;
  const int l32 = lane & 31, half = lane >> 5;

  // the query row of this lane
  const int j = qt * (32 * QW) + qw * 32 + l32;
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

  // ---- global -> LDS: stage rows are, per key-wave tile, TK rows of K then TK of V ----
  const bf16_t* kbase = p.k + (long)b * T * p.d + h * DH;
  const bf16_t* vbase = p.v + (long)b * T * p.d + h * DH;
  int ld_key[LPW];           // key of this lane's row at step 0
  const bf16_t* ld_src[LPW]; // K or V base + chunk offset
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int sr = (wave * LPW + i) * RPL + lane / CPR;  // row within the stage
    const int tile = sr / (2 * TK), within = sr % (2 * TK);
    const bool is_v = within >= TK;
    const int key_local = within % TK;
    const int chunk = (lane % CPR) ^ (is_v ? v_swizzle<DH>(key_local) : k_swizzle<DH>(key_local));
    ld_key[i] = tile * TK + key_local;
    ld_src[i] = (is_v ? vbase : kbase) + chunk * 8;
  }
  auto issue_loads = [&](int step, int buf) __attribute__((always_inline)) {
    unsigned char* base = smem + buf * STAGE_BYTES + wave * LPW * 1024;
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      int key = ld_key[i] + step * (KW * TK);
      key = key < T ? key : T - 1;
      __builtin_amdgcn_global_load_lds((gptr_t)(ld_src[i] + (long)key * p.d),
                                       (lptr_t)(base + i * 1024), 16, 0, 0);
    }
  };

  // ---- per-lane LDS read offsets ----
  // K fragment: row (32 kt + l32), chunk (2 ks + half) ^ k_swizzle(row)
  int k_off[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks)
    k_off[ks] = l32 * ROWB + (((ks * 2 + half) ^ k_swizzle<DH>(l32)) * 16);
  // V^T fragment by transpose read: within each group of 16 lanes, lane r supplies the
  // address of key (r >> 2) of the 4-key run, channels 4 (r & 3) .. +3 of the 16
  // channels the group covers; lane i of the group receives those 4 keys at channel i.
  int v_off[OT];
  {
    const int r = lane & 15, e = r >> 2, jj = r & 3;
    const int key_l = half * 4 + e;                       // + 16 s4 + 8 which
    const int c_lane = 2 * ((lane >> 4) & 1) + (jj >> 1); // chunk within the 32-channel tile
    const int vs = v_swizzle<DH>(key_l) >> 2;
#pragma unroll
    for (int t = 0; t < OT; ++t)
      v_off[t] = key_l * ROWB + (((t ^ vs) * 4 + c_lane) * 16) + (jj & 1) * 8;
  }

  f32x16 acc_o[OT];
#pragma unroll
  for (int t = 0; t < OT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[t][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  auto compute = [&](int buf, int kv0) __attribute__((always_inline)) {
    const unsigned char* kb = smem + buf * STAGE_BYTES + kw * 2 * TILE_BYTES;
    const unsigned char* vb = kb + TILE_BYTES;
    // S^T tile: TK keys x 32 query rows
    f32x16 acc_s[ST];
#pragma unroll
    for (int kt = 0; kt < ST; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_s[kt][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kb + kt * 32 * ROWB + k_off[ks]);
        acc_s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[kt], 0, 0, 0);
      }
    }
    // register r of tile kt is key kv0 + kt*32 + (r/4)*8 + half*4 + r%4
    if (kv0 + TK > T) {  // last, ragged tile only (uniform branch): keys past the end
#pragma unroll
      for (int kt = 0; kt < ST; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + kt * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
          if (key >= T) acc_s[kt][r] = -INFINITY;
        }
    }
    float m_tile = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < ST; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) m_tile = fmaxf(m_tile, acc_s[kt][r]);
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64)) * p.scale_log2;  // scale > 0
    // Lazy rescaling: the reference exponent m_run of a row only moves when the row's
    // maximum has grown by more than 2^8 over it, so probabilities stay below 256 and
    // the accumulator rescale (a pass over all of O) is skipped for almost every tile.
    // The result does not depend on the reference: O and the row sum share it.
    const bool grow = m_tile > m_run + 8.0f;
    if (__any(grow)) {
      const float m_new = grow ? m_tile : m_run;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[t][r] *= alpha;
    }
    const float neg_m = -m_run;
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
    float l_tile = 0.f;
    bf16x8 pf[PS];
#pragma unroll
    for (int kt = 0; kt < ST; ++kt)
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        f32x2 pr;
        pr[0] = __builtin_amdgcn_exp2f(fmaf(acc_s[kt][r], p.scale_log2, neg_m));
        pr[1] = __builtin_amdgcn_exp2f(fmaf(acc_s[kt][r + 1], p.scale_log2, neg_m));
        const bf16x2 pb = __builtin_convertvector(pr, bf16x2);
        // the row sum is taken over the probabilities as rounded for the value product,
        // so numerator and denominator carry the same rounding (v_dot2: += pb[0] + pb[1])
        l_tile = __builtin_amdgcn_fdot2_f32_bf16(pb, ones, l_tile, false);
        pf[kt * 2 + (r >> 3)][r & 7] = pb[0];
        pf[kt * 2 + (r >> 3)][(r & 7) + 1] = pb[1];
      }
    l_run += l_tile;

    // O^T += V^T P^T.  Slot s of P slice s4 is key 16 s4 + 8 (s/4) + 4 half + s%4.
#pragma unroll
    for (int t = 0; t < OT; ++t) {
#pragma unroll
      for (int s4 = 0; s4 < PS; ++s4) {
        const unsigned char* va = vb + s4 * 16 * ROWB + v_off[t];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(va));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(va + 8 * ROWB));
        const bf16x4 blo = __builtin_bit_cast(bf16x4, lo), bhi = __builtin_bit_cast(bf16x4, hi);
        const bf16x8 vf = __builtin_shufflevector(blo, bhi, 0, 1, 2, 3, 4, 5, 6, 7);
        acc_o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[s4], acc_o[t], 0, 0, 0);
      }
    }
  };

  // ---- pipeline over the key tiles ----
  const int n_tiles = (T + TK - 1) / TK;
  const int n_steps = (n_tiles + KW - 1) / KW;
#pragma unroll
  for (int s = 0; s < NST - 1; ++s) issue_loads(s < n_steps ? s : n_steps - 1, s);
  for (int step = 0; step < n_steps; ++step) {
    // step's tiles have landed for every wave, and everybody is done with step-1's
    wait_vmcnt_and_barrier<LPW*(NST - 2)>();
    const int nxt = step + NST - 1;
    issue_loads(nxt < n_steps ? nxt : n_steps - 1, nxt % NST);
    const int tile = step * KW + kw;
    if (tile < n_tiles) compute(step % NST, tile * TK);
  }
  float l_all = l_run + __shfl_xor(l_run, 32, 64);

  // ---- merge the key-waves (fixed order), normalise, store ----
  if (KW > 1) {
    constexpr int REGS = OT * 16 + 2;
    static_assert((KW - 1) * QW * REGS * 64 * 4 <= attn_smem_bytes<DH, KW, TK, NST>(),
                  "the merge area must fit into the stage memory");
    wait_all_and_barrier();  // all loads landed, all tiles consumed: stage memory is free
    float* xch = reinterpret_cast<float*>(smem);
    if (kw > 0) {
      float* mine = xch + ((kw - 1) * QW + qw) * REGS * 64 + lane;
      mine[0] = m_run;
      mine[64] = l_all;
#pragma unroll
      for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(2 + t * 16 + r) * 64] = acc_o[t][r];
    }
    __syncthreads();
    if (kw > 0) return;
#pragma unroll
    for (int o = 1; o < KW; ++o) {
      const float* other = xch + ((o - 1) * QW + qw) * REGS * 64 + lane;
      const float m_o = other[0], l_o = other[64];
      const float m_new = fmaxf(m_run, m_o);
      const float sa = __builtin_amdgcn_exp2f(m_run - m_new), sb = __builtin_amdgcn_exp2f(m_o - m_new);
      m_run = m_new;
      l_all = l_all * sa + l_o * sb;
#pragma unroll
      for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[t][r] = acc_o[t][r] * sa + other[(2 + t * 16 + r) * 64] * sb;
    }
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
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

template <int DH, int QW, int KW, int TK, int NST>
__global__ void __launch_bounds__(QW* KW * 64) attn_bf16_kernel(AttnDev p) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[attn_smem_bytes<DH, KW, TK, NST>()];
  // Workgroup ids are dealt round-robin to the 8 XCDs.  All query blocks of one
  // (sequence, head) are placed on the same XCD, so its K and V are fetched from HBM
  // once and re-read from that XCD's L2 by the other blocks.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int pair = (slot / p.n_qt) * 8 + xcd, qt = slot % p.n_qt;
  if (pair >= p.n_pairs) return;
  const int b = pair / p.n_heads, h = pair % p.n_heads;
  int cnt, off;
  if (p.idx) {
    off = p.sel_off[b];
    cnt = p.sel_off[b + 1] - off;
  } else {
    off = b * p.seq;
    cnt = p.seq;
  }
  if (qt * (32 * QW) >= cnt) return;
  attn_block<DH, QW, KW, TK, NST>(p, b, h, qt, cnt, off, smem);
}

template <int DH, int QW, int KW, int TK, int NST>
hipError_t launch_variant(AttnDev p, const AttnArgs& a, hipStream_t s) {
  p.n_heads = a.n_heads;
  p.n_pairs = a.batch * a.n_heads;
  p.n_qt = (a.seq + 32 * QW - 1) / (32 * QW);
  const long grid = (long)((p.n_pairs + 7) / 8) * p.n_qt * 8;
  if (grid > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_bf16_kernel<DH, QW, KW, TK, NST>), dim3((unsigned)grid), dim3(QW * KW * 64), 0, s, p);
  return hipGetLastError();
}

template <int DH>
hipError_t launch_dh(const AttnDev& p, const AttnArgs& a, hipStream_t s) {
  // measured on MI355X: 8 waves per block.  Full rows take the wide block (128 rows, 2
  // key-waves).  Refreshed rows are few per sequence: with few (sequence, head) pairs
  // the narrow block (64 rows, 4 key-waves) is what fills the chip; with many pairs
  // the wide block already does and re-reads K and V less.
  if (a.idx && !a.many_rows && a.batch * a.n_heads < 128) return launch_variant<DH, 2, 4, 32, 2>(p, a, s);
  // Most rows of every sequence and enough of them for a block of 256 query rows per
  // workgroup (8 query-waves, no key split) to fill the chip: a K/V tile then feeds twice
  // the MFMAs per byte that enters LDS (8 x 2048 tokens: 600-650 us against 750-880;
  // 2 x 1024: 43 against 52 us; with 1 x 1024 tokens there are only 128 such blocks).
  if ((!a.idx || a.many_rows) && (long)a.batch * a.n_heads * ((a.seq + 255) / 256) >= 256)
    return launch_variant<DH, 8, 1, 64, 2>(p, a, s);
  return launch_variant<DH, 4, 2, 64, 2>(p, a, s);
}

}  // namespace

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
  if (a.head_dim == 128) return launch_dh<128>(p, a, s);
  if (a.head_dim == 64) return launch_dh<64>(p, a, s);
  return hipErrorInvalidValue;
}

}  // namespace dare
