// Internal declarations shared by the HIP sources of libdare (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dare.h"
#include "dare_kernels.h"

namespace dare {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// ---- launchers (defined one per .hip file); all return a hipError_t ----------

struct GemmArgs {
  const void* a;      // [*, lda]
  int lda;
  const void* wt;     // [n, k] packed weight
  int n, k;
  int m_max;          // launch bound on the row count
  const int32_t* idx; // optional row ids (gather of A rows = scatter of C rows)
  const int32_t* m_dev; // optional device row count
  void* c[3];         // output column segments
  int ldc;
  int seg_n;
  float* c32;         // optional fp32 copy of columns [0, c32_cols)
  int c32_cols;
  int k_parts;        // > 1: only c32 is written, as k_parts slabs of partial sums
  long c32_part_stride;
  // rotary embedding of output columns [0, rope_cols) (fp32 table [pos][head_dim/2]
  // of (cos, sin) pairs; position of a row = token id % rope_seq); nullptr = none
  const float* rope;
  int rope_cols, rope_dh, rope_seq;
  // 1: the output columns are (gate, up) pairs of a SwiGLU feed-forward (weight rows
  // interleaved gate_0, up_0, gate_1, ...): column pair (2j, 2j+1) gives one output
  // silu(gate_j) * up_j at column j of c[0] (bf16 path, one segment, no c32)
  int swiglu_pairs;
  // Row list derived inside the kernel (bf16, device-count kernel only; replaces idx and
  // m_dev): the rows are the tokens whose byte in sel_mask [sel_batch * sel_seq] is 0, in
  // ascending order.  The first workgroup also writes what a compaction kernel would:
  // sel_idx_out (and optionally sel_idx_out2) [tokens], sel_off_out [sel_batch + 1],
  // optionally sel_count_out [sel_batch].  At most kSelMaxTokens tokens.
  const uint8_t* sel_mask;
  int sel_batch, sel_seq;
  int32_t* sel_idx_out;
  int32_t* sel_idx_out2;
  int32_t* sel_off_out;
  int32_t* sel_count_out;
};
constexpr int kSelMaxTokens = 2048;

// Rotation of the channel pairs (v0, v1) and (v2, v3) of four neighbouring output
// columns col .. col + 3 (col a multiple of 4) of token tok.
__device__ __forceinline__ void rope_rotate4(const float* __restrict__ table, int dh, int seq, long tok,
                                             int col, float& v0, float& v1, float& v2, float& v3) {
  const int pos = (int)(tok % seq);
  const f32x4 cs = *reinterpret_cast<const f32x4*>(table + ((long)pos * (dh >> 1) + ((col % dh) >> 1)) * 2);
  const float a0 = v0 * cs[0] - v1 * cs[1], a1 = v0 * cs[1] + v1 * cs[0];
  const float a2 = v2 * cs[2] - v3 * cs[3], a3 = v2 * cs[3] + v3 * cs[2];
  v0 = a0;
  v1 = a1;
  v2 = a2;
  v3 = a3;
}
hipError_t launch_gemm_bf16(const GemmArgs& g, hipStream_t s);
hipError_t launch_gemm_f32(const GemmArgs& g, hipStream_t s);

struct AttnArgs {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  int batch, seq, n_heads, head_dim;
  const int32_t* idx;      // optional selected rows
  const int32_t* sel_off;  // [batch+1] when idx != nullptr
  bool many_rows;          // the listed rows are most of each sequence (a frozen prefix), not a few
};
hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_f32(const AttnArgs& a, hipStream_t s);

hipError_t launch_pack_weight(int dtype, const void* w, int rows_k, int cols_n, void* wt,
                              int ldwt, hipStream_t s);
hipError_t launch_score(const float* q_new, int ld_new, int width, int n_parts, long part_stride,
                        float* q_prev, int n_tokens, float threshold, int force_refresh, float* scores, float* scores2,
                        uint8_t* mask, int seq, int prefix, hipStream_t s);
hipError_t launch_compact(const uint8_t* mask, int batch, int seq, int32_t* sel_idx,
                          int32_t* sel_idx2, int32_t* sel_count, int32_t* sel_count2,
                          int32_t* sel_off, hipStream_t s);
hipError_t launch_quantile_mask(const float* scores, int batch, int stride, int first, int seq, int rank,
                                int force_refresh, float* tau_out, uint8_t* mask, double* stat_sum,
                                unsigned long long* stat_count, hipStream_t s);
hipError_t launch_zero_words(void* p, int n, hipStream_t s);
hipError_t launch_active_list(int batch, int seq, int prefix, int32_t* act_idx, int32_t* act_off, hipStream_t s);
hipError_t launch_copy_rows(const void* src, void* dst, int n_rows, int row_bytes,
                            const int32_t* idx, const int32_t* m_dev, hipStream_t s);
// rows r = 0 .. n_rows-1; with seq > 0 row r is token (r / (seq - prefix)) * seq + prefix + r % (seq - prefix)
hipError_t launch_norm(int dtype, int kind, const void* x, const void* gain, const void* bias, float eps,
                       int n_rows, int d, void* out, int seq, int prefix, hipStream_t s);
hipError_t launch_residual_add(int dtype, const void* x, const void* o, void* out, long n_elems,
                               hipStream_t s);
hipError_t launch_residual_norm(int dtype, void* x, const void* o, const void* gain, float eps, int n_rows, int d,
                                void* h, int seq, int prefix, hipStream_t s);
hipError_t launch_residual_rows(int dtype, void* x, const void* f, int n_rows, int d, const int32_t* idx,
                                hipStream_t s);
hipError_t launch_gather_rows(const void* src, void* dst, const int32_t* ids, int n_rows, int n_src,
                              int row_bytes, hipStream_t s);
hipError_t launch_swiglu(int dtype, void* gate, const void* up, int n_rows, int width, const int32_t* idx,
                         hipStream_t s);

// The attention block of dare_block_step without its first and last launch, for the model
// runtime, which fuses them with its neighbours: `h` is the hidden state already normalised,
// the block output O goes into o_cache only (no residual sum).  Arguments are checked as
// in dare_layer_step; rotary embedding as attached to the context.
dare_status block_core(dare_ctx* ctx, int mode, float threshold, int batch, int seq, const void* h, float* q_prev,
                       void* k_cache, void* v_cache, void* o_cache, uint8_t* reuse_mask, int32_t* sel_count,
                       void* hip_stream);

}  // namespace dare
