/*
 * Kernel-level entry points of libdare: each one enqueues a single stage of the
 * layer step of dare.h on a HIP stream.  dare_layer_step() is built from exactly
 * these stages; they are exported so that each can be checked against its
 * definition and timed on its own.  All data pointers are DEVICE memory owned by
 * the caller; calls are asynchronous and never synchronise.  dtype is a
 * dare_dtype.  Argument errors return DARE_ERR_INVALID_ARG / UNSUPPORTED before
 * anything is enqueued.
 */
#ifndef DARE_KERNELS_H
#define DARE_KERNELS_H

#include <stdint.h>
#include "dare.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Re-pack a projection weight: wt[n, k] = w[k, n] (w is [rows_k, cols_n]
 * row-major, the Y = X W orientation of Sec. 3.2 eq. 3; wt is [cols_n, rows_k]
 * row-major with leading dimension ldwt >= rows_k).  The GEMM below consumes wt.
 */
dare_status dare_k_pack_weight(int dtype, const void* w, int rows_k, int cols_n,
                               void* wt, int ldwt, void* hip_stream);

/*
 * Row-selected projection (Alg. 1 lines 6-7 and 11; Alg. 2 lines 2, 7, 11):
 *     C[t, 0:n] = A[t, 0:k] . W          for t in rows
 * rows = idx[0 .. m) when idx != NULL (flat token ids; the same id addresses the
 * row of A that is read and the row of C that is written), else 0 .. m-1.
 * m = *m_dev (a device int32, read by the kernel) when m_dev != NULL, else m_max;
 * m_max bounds the launch and must be >= *m_dev.
 *   a    [*, lda] dtype, k contiguous          wt [n, k] dtype (packed weight)
 *   c    column segment s = col / seg_n goes to c[s] (up to 3 segments, each
 *        [*, ldc] dtype); seg_n must divide n; unused entries NULL
 *   c32  optional fp32 copy [*, c32_cols] (leading dimension c32_cols) of output
 *        columns [0, c32_cols), taken from the fp32 accumulators before rounding
 *        to dtype: the input of the drift score.  c may be all NULL when only
 *        c32 is wanted (then n == c32_cols).
 *   k_parts  1, or (bf16, all rows, c all NULL, c32_cols == n) a divisor of k/64: k is
 *        cut into k_parts ranges computed by separate workgroups, and range s writes
 *        its partial products to c32 + s * c32_part_stride (elements).  The sum over s,
 *        taken in order, is the projection; dare_k_score adds the slabs itself.  Meant
 *        for the scored query columns of all rows (few output tiles, long k).
 * k must be a multiple of 64, n of 64 (bf16) / 16 (fp32).
 */
dare_status dare_k_gemm(int dtype, const void* a, int lda, const void* wt, int n,
                        int k, int m_max, const int32_t* idx,
                        const int32_t* m_dev, void* const* c, int ldc, int seg_n,
                        float* c32, int c32_cols, int k_parts, long c32_part_stride,
                        void* hip_stream);

/*
 * Drift score and reuse decision (Sec. 3.1 eq. 1, Sec. 3.2 eq. 2; Alg. 1/2
 * lines 3-5) for n_tokens tokens:
 *   s = 1 - <q, p> / max(sqrt(|q|^2 |p|^2), 1e-30), q = q_new[t, 0:width],
 *   p = q_prev[t, 0:width]; mask = (s <= threshold) unless force_refresh;
 *   then q_prev[t] = q.
 *   q_new [n_tokens, ld_new] fp32, or n_parts such slabs part_stride elements apart
 *   whose sum (taken in slab order) is q; q_prev [n_tokens, width] fp32 in/out;
 *   scores optional [n_tokens] fp32; mask [n_tokens] bytes.
 */
dare_status dare_k_score(const float* q_new, int ld_new, int width, int n_parts,
                         long part_stride, float* q_prev, int n_tokens,
                         float threshold, int force_refresh, float* scores,
                         uint8_t* mask, void* hip_stream);

/*
 * Ordered compaction of the refreshed set (Alg. 1/2 line 5): sel_idx = ascending
 * flat ids b*seq+i with mask == 0; sel_count[b] per sequence; sel_off[b] = number
 * of refreshed tokens in sequences before b, sel_off[batch] = total.
 * sel_idx [batch*seq], sel_count [batch], sel_off [batch+1], all int32; any of
 * the three may be NULL.
 */
dare_status dare_k_compact(const uint8_t* mask, int batch, int seq,
                           int32_t* sel_idx, int32_t* sel_count,
                           int32_t* sel_off, void* hip_stream);

/*
 * Bidirectional multi-head attention for selected query rows (App. E.2; Alg. 1
 * line 10; Alg. 2 line 8):
 *   out[t, h] = softmax(q[t, h] . K_b[:, h]^T / sqrt(head_dim)) V_b[:, h]
 * for every head h and every token t of the row set; b = t / seq is the
 * sequence of t, and keys/values are all seq rows of that sequence.
 * Row set: all tokens when idx == NULL; else idx[sel_off[b] .. sel_off[b+1]) for
 * each sequence b (idx, sel_off as produced by dare_k_compact).
 *   q, k, v, out  [batch*seq, n_heads*head_dim] dtype, token-indexed rows
 */
dare_status dare_k_attention(int dtype, const void* q, const void* k,
                             const void* v, void* out, int batch, int seq,
                             int n_heads, int head_dim, const int32_t* idx,
                             const int32_t* sel_off, void* hip_stream);

/*
 * Row copy between token-indexed buffers: dst[t] = src[t] for t in idx[0..*m_dev)
 * (idx != NULL) or for all n_rows rows (idx == NULL).  row_bytes is a multiple
 * of 16.  Used to mirror the layer output between out and o_cache when they are
 * different buffers (Alg. 2 lines 9-10).
 */
dare_status dare_k_copy_rows(const void* src, void* dst, int n_rows,
                             int row_bytes, const int32_t* idx,
                             const int32_t* m_dev, void* hip_stream);

/*
 * Threshold from a reuse rate and the decision under it (Sec. 3.1 "Reuse rate
 * allocation"; rule as dare_set_threshold_rule in dare.h).  scores [batch, seq] fp32.
 * phi in [0, 1]: per sequence tau = k-th smallest score, k = ceil(phi * seq) in fp32;
 * writes tau_out[batch] (optional) and mask[batch, seq] = (score <= tau), all 0 when
 * force_refresh.  phi < 0: statistics only, mask and tau_out are not touched.
 * stat_sum / stat_count (both or neither): device arrays of [batch] slots; the sum and the
 * number of the non-NaN scores of sequence b are added to slot b (plain read-modify-write by
 * the one workgroup that owns the sequence: no atomics, the same result from run to run).
 */
dare_status dare_k_quantile_mask(const float* scores, int batch, int seq, float phi,
                                 int force_refresh, float* tau_out, uint8_t* mask,
                                 double* stat_sum, uint64_t* stat_count, void* hip_stream);

/*
 * The projection above with the rotary embedding in its epilogue (see dare_block_config
 * in dare.h): output columns [0, rope_cols) are rotated, channel pair (2i, 2i+1) of
 * every head_dim-wide head by the angle whose (cos, sin) is
 * rope_table[(t % seq) * head_dim/2 + i], t the token id of the row; the fp32 copy c32
 * keeps the unrotated values.  rope_table: fp32 [positions, head_dim/2, 2].  rope_cols
 * is a multiple of head_dim; seg_n a multiple of head_dim.  No k_parts.
 */
dare_status dare_k_gemm_rope(int dtype, const void* a, int lda, const void* wt, int n,
                             int k, int m_max, const int32_t* idx,
                             const int32_t* m_dev, void* const* c, int ldc, int seg_n,
                             float* c32, int c32_cols, const float* rope_table,
                             int rope_cols, int head_dim, int seq, void* hip_stream);

/*
 * Rotary table for positions 0 .. n_pos-1: table[p, i] = (cos, sin) of
 * p * base^(-2i / head_dim), computed on the HOST in double precision and copied to
 * the device pointer `table` (fp32 [n_pos, head_dim/2, 2]) with a synchronous copy.
 */
dare_status dare_k_rope_table(float* table, int n_pos, int head_dim, double base);

/*
 * Normalisation of token rows (Alg. 1/2 line 1): kind DARE_NORM_LAYER or
 * DARE_NORM_RMS, formulas as in dare_block_config.  x, out [n_rows, d] dtype (out may
 * be x), gain [d], bias [d] or NULL; d a multiple of 8; fp32 statistics.
 */
dare_status dare_k_norm(int dtype, int kind, const void* x, const void* gain,
                        const void* bias, float eps, int n_rows, int d, void* out,
                        void* hip_stream);

/* Residual sum out = x + o over n_elems elements (a multiple of 8) of dtype. */
dare_status dare_k_residual_add(int dtype, const void* x, const void* o, void* out,
                                long n_elems, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DARE_KERNELS_H */
