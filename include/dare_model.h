/*
 * libdare: a masked-diffusion language model made of DARE layers (the setting of Sec. 5
 * of the paper: DARE-KV / DARE-O applied in every self-attention layer of a LLaDA-class
 * model).  The model around the attention is the standard pre-norm transformer of those
 * models and is not the paper's subject; it is here so that the reuse modes can be run
 * and timed on the activations of a whole network:
 *
 *   x_0 = E[ids];  per layer  x <- x + O(rmsnorm(x))            (dare_block_step)
 *                             x <- x + (silu(n Wg) * (n Wu)) Wd, n = rmsnorm(x)
 *   y = rmsnorm(x_L);  logits = y W_head for the rows asked for.
 *
 * Rotary embedding on Q and K, no biases, weights [d_in, d_out].  All data pointers are
 * device memory unless marked host.  Calls enqueue on the given stream; only create,
 * set_* and destroy synchronise.  Errors as in dare.h; dare_model_last_error gives text.
 */
#ifndef DARE_MODEL_H
#define DARE_MODEL_H

#include "dare.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dare_model dare_model;

typedef struct {
  uint32_t struct_size; /* = sizeof(dare_model_config) */
  int32_t n_layers, hidden, n_heads, head_dim, ffn, vocab;
  int32_t max_batch, max_seq;
  int32_t dtype;        /* DARE_F32 or DARE_BF16 */
  float norm_eps;
  float rope_base;      /* 0: no rotary embedding */
  int32_t device;
  uint32_t flags;       /* reserved, 0 */
} dare_model_config;

/* Allocates the per-layer contexts' scratch, the K/V/O/score caches of every layer
 * ([max_batch, max_seq, hidden] each, zeroed) and the activation buffers.  Weights come
 * with the set_* calls.  hidden, ffn and vocab must be multiples of 64. */
dare_status dare_model_create(const dare_model_config* cfg, void* hip_stream, dare_model** out);

/* Weights of one layer (copied and re-packed; the caller may free them afterwards):
 * gains [hidden]; wq, wk, wv, wo [hidden, hidden]; w_gate, w_up [hidden, ffn];
 * w_down [ffn, hidden]; all of the model's dtype. */
dare_status dare_model_set_layer(dare_model* m, int layer, const void* attn_gain, const void* wq,
                                 const void* wk, const void* wv, const void* wo, const void* ffn_gain,
                                 const void* w_gate, const void* w_up, const void* w_down,
                                 void* hip_stream);

/* Token embedding [vocab, hidden], gain of the final normalisation [hidden], output
 * embedding [hidden, vocab] (NULL: dare_model_logits is not available). */
dare_status dare_model_set_io(dare_model* m, const void* embed, const void* final_gain,
                              const void* head, void* hip_stream);

/* Threshold rule and frozen prefix for every layer (dare_set_threshold_rule,
 * dare_set_prefix).  With a prefix the feed-forward also skips the frozen rows. */
dare_status dare_model_set_rule(dare_model* m, int rule);
dare_status dare_model_set_prefix(dare_model* m, int prefix_len);

/*
 * One denoising step: the forward pass of the whole model on ids, each layer in its own
 * mode with its own threshold (or reuse rate under the quantile rule).
 *   modes, thresholds  host arrays [n_layers] (read during the call)
 *   ids         in   [batch, seq] int32; an id outside [0, vocab) gives a zero embedding
 *   hidden_out  out, optional [batch, seq, hidden] dtype: y, after the final normalisation
 *   refreshed   out, optional [n_layers, batch] int32: refreshed tokens per layer and sequence
 *   trace       out, optional [2 n_layers + 1][batch, seq, hidden] dtype: the residual stream
 *               entering each layer, after its attention block, ..., after the last layer
 * The caches hold the state of the previous step for the same batch and seq; the first
 * step after create (or after a change of batch or seq) must run every layer DENSE.
 */
dare_status dare_model_step(dare_model* m, const int32_t* modes, const float* thresholds, int batch,
                            int seq, const int32_t* ids, void* hidden_out, int32_t* refreshed,
                            void* trace, void* hip_stream);

/* logits[r, :] = hidden[rows[r], :] W_head for n_rows flat token ids (device int32);
 * hidden is dare_model_step's hidden_out; logits [n_rows, vocab] dtype. */
dare_status dare_model_logits(dare_model* m, const void* hidden, const int32_t* rows, int n_rows,
                              void* logits, void* hip_stream);

/* The context of one layer (owned by the model), e.g. for dare_drift_stats_*. */
dare_ctx* dare_model_layer(dare_model* m, int layer);

dare_status dare_model_destroy(dare_model* m);
const char* dare_model_last_error(const dare_model* m);

#ifdef __cplusplus
}
#endif
#endif /* DARE_MODEL_H */
