/*
 * libdare: one bidirectional self-attention layer of a diffusion LLM at one
 * denoising step with token-wise activation reuse (DARE), for AMD MI355X
 * (gfx950).  Plain C ABI: pointers and sizes only.
 *
 * What a step computes (paper Sec. 3; Alg. 1 "DARE-KV"; Alg. 2 "DARE-O";
 * App. E.1/E.2):
 *   Q = X Wq.  For every token i the drift score
 *       s_i = 1 - <q_i, p_i> / (|q_i| |p_i|)                (Sec. 3.1 eq. 1)
 *   of its head-0 query q_i against the head-0 query p_i of the previous step
 *   (Sec. 3.2).  Tokens with s_i <= threshold are reused, the others are
 *   refreshed (Sec. 3.2 eq. 2).
 *   DARE_MODE_KV   K and V rows are projected only for the refreshed tokens and
 *                  written into the K/V caches; attention and Wo over all rows
 *                  (Alg. 1).
 *   DARE_MODE_O    K and V for all rows; attention and Wo only for the
 *                  refreshed rows; reused rows return the cached layer output
 *                  (Alg. 2, with the cache holding rows after Wo as in App. E.1).
 *   DARE_MODE_KVO  both at once.
 *   DARE_MODE_DENSE no reuse: softmax(Q K^T / sqrt(head_dim)) V Wo (App. E.2);
 *                  also the step that fills the caches.
 *
 * Every data pointer below is DEVICE memory owned by the caller unless it says
 * "host".  Calls are asynchronous on the given HIP stream and never
 * synchronise.  No exception crosses this boundary: every failure is a status
 * code, and dare_last_error() gives the text.  Argument errors are detected
 * before anything is enqueued, so they leave all buffers untouched.
 * One context serves one stream at a time (it owns scratch memory).
 */
#ifndef DARE_H
#define DARE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dare_ctx dare_ctx;

typedef enum {
  DARE_OK = 0,
  DARE_ERR_INVALID_ARG = 1, /* null pointer, bad mode, shape out of range, NaN */
  DARE_ERR_UNSUPPORTED = 2, /* a shape the kernels are not built for          */
  DARE_ERR_OOM = 3,         /* device allocation failed                       */
  DARE_ERR_HIP = 4          /* any other HIP runtime error                    */
} dare_status;

typedef enum { DARE_F32 = 0, DARE_BF16 = 1 } dare_dtype;

enum { DARE_MODE_DENSE = 0, DARE_MODE_KV = 1, DARE_MODE_O = 2, DARE_MODE_KVO = 3 };

typedef struct {
  uint32_t struct_size; /* = sizeof(dare_config); anything else is INVALID_ARG  */
  int32_t hidden;       /* d; must equal n_heads * head_dim                     */
  int32_t n_heads;
  int32_t head_dim;     /* 64 or 128                                            */
  int32_t max_batch;    /* scratch is sized for max_batch * max_seq tokens      */
  int32_t max_seq;
  int32_t dtype;        /* DARE_F32: fp32 storage and arithmetic (debug path);
                           DARE_BF16: bf16 storage, fp32 accumulation           */
  int32_t score_head;   /* head whose query is scored: 0 = the paper's choice
                           (Sec. 3.2); -1 = the whole query vector (Sec. 3.1)   */
  int32_t device;       /* HIP device ordinal                                   */
  uint32_t flags;       /* reserved, must be 0                                  */
} dare_config;

/*
 * Create a context.  wq, wk, wv, wo: device pointers to row-major
 * [hidden, hidden] matrices of cfg->dtype laid out [d_in, d_out], so that
 * Y = X W (Sec. 3.2 eq. 3, App. E.1).  They are copied and re-packed inside the
 * call; the caller may free them after the call returns (the call synchronises
 * the stream once, it is the only call that does).
 * Errors: INVALID_ARG (null pointer, bad config), UNSUPPORTED (head_dim not 64
 * or 128, hidden not a multiple of 64), OOM, HIP.  On error *out_ctx is NULL.
 */
dare_status dare_create(const dare_config* cfg, const void* wq, const void* wk,
                        const void* wv, const void* wo, void* hip_stream,
                        dare_ctx** out_ctx);

/*
 * One step of the layer (Alg. 1 / Alg. 2 / App. E.2 depending on mode).
 *
 *   hidden     in     [batch, seq, hidden] dtype; already normalised (line 1 of
 *                     both algorithms is the caller's)
 *   q_prev     in/out [batch, seq, head_dim] fp32 (or [batch, seq, hidden] when
 *                     score_head = -1): the scored query of the previous step;
 *                     replaced by this step's for EVERY token, in every mode
 *   k_cache    in/out [batch, seq, hidden] dtype.  KV, KVO: refreshed rows are
 *   v_cache           overwritten, reused rows are read.  DENSE, O: all rows
 *                     are written.
 *   o_cache    in/out [batch, seq, hidden] dtype: the layer output of the
 *                     previous step (after Wo).  O, KVO: reused rows are read.
 *                     Every mode leaves this step's layer output in it.
 *   out        out    [batch, seq, hidden] dtype: this step's layer output.  May
 *                     be the same pointer as o_cache (then no copy is made);
 *                     partial overlap is an error the call cannot detect.
 *   reuse_mask out    [batch, seq] bytes, 1 = reused, 0 = refreshed (all 0 in
 *                     DENSE; always 1 for the tokens of a frozen prefix, see
 *                     dare_set_prefix)
 *   sel_idx    out, optional (NULL to skip) [batch*seq] int32: ascending flat
 *                     token ids b*seq+i of the refreshed tokens; entries past
 *                     the total count are left as they were
 *   sel_count  out, optional [batch] int32: refreshed tokens per sequence
 *   scores     out, optional [batch, seq] fp32 drift scores
 *   threshold  compared in fp32, reuse iff score <= threshold; ignored in DENSE.
 *              A NaN score refreshes.  NaN threshold is INVALID_ARG.  Under
 *              DARE_RULE_QUANTILE (dare_set_threshold_rule) it is a reuse rate.
 *
 * The call enqueues kernels only (no allocation, no memset, no host synchronisation), so
 * it may be recorded into a HIP graph.
 *
 * Errors: INVALID_ARG (null required pointer, unknown mode, batch or seq < 1,
 * batch > max_batch, seq > max_seq, NaN threshold), HIP (a launch failed).
 */
dare_status dare_layer_step(dare_ctx* ctx, int mode, float threshold, int batch,
                            int seq, const void* hidden, float* q_prev,
                            void* k_cache, void* v_cache, void* o_cache,
                            void* out, uint8_t* reuse_mask, int32_t* sel_idx,
                            int32_t* sel_count, float* scores, void* hip_stream);

/*
 * The attention block around the layer step: the normalisation of the hidden state
 * that both algorithms start with (Alg. 1/2 line 1), rotary position embedding of the
 * projected queries and keys, and the residual sum.  The paper states only line 1;
 * position encoding and residual are what a model built from such layers needs, read
 * as follows: the drift score is taken on the query before the rotation; keys are
 * rotated as they are projected, so the K cache holds rotated keys and a reused row
 * keeps the rotation of its own position; the output cache holds the block output
 * before the residual sum, which is formed for every row from the current x.
 */
enum { DARE_NORM_NONE = 0, DARE_NORM_LAYER = 1, DARE_NORM_RMS = 2 };

typedef struct {
  uint32_t struct_size; /* = sizeof(dare_block_config)                              */
  int32_t norm;         /* DARE_NORM_LAYER: (x - mean) / sqrt(var + eps) * gain + bias
                           (Alg. 1/2 line 1); DARE_NORM_RMS: x / sqrt(mean(x^2) + eps)
                           * gain; DARE_NORM_NONE: the hidden state is used as it is  */
  float eps;
  float rope_base;      /* 0: no rotary embedding.  Else the channel pair (2i, 2i+1)
                           of every head of Q and K is rotated by
                           position * rope_base^(-2i / head_dim), position = index of
                           the token in its sequence                                */
  int32_t residual;     /* 1: out = x + O; 0: out = O                               */
} dare_block_config;

/*
 * Attach a block configuration to a context (replaces an earlier one).  gain, bias:
 * device pointers to [hidden] vectors of the context's dtype (gain required unless
 * norm is NONE; bias optional, LayerNorm only); they are copied.  Builds the rotary
 * table for max_seq positions on the host in double precision and uploads it.
 * Synchronises the stream.  Errors: INVALID_ARG, OOM, HIP.
 */
dare_status dare_block_attach(dare_ctx* ctx, const dare_block_config* cfg,
                              const void* gain, const void* bias, void* hip_stream);

/*
 * One step of the attached block: h = norm(x); the layer step of dare_layer_step on h
 * with the rotary embedding applied to Q and to the K rows projected at this step;
 * out = x + O (residual = 1) or O.  Arguments as dare_layer_step, except:
 *   x        in      [batch, seq, hidden] dtype: the hidden state BEFORE normalisation
 *   o_cache  in/out  the block output O before the residual sum
 *   out      out     with residual = 1 it must not be o_cache (INVALID_ARG); it may be
 *                    x itself (the sum is then formed in place, as the last launch)
 * Errors: as dare_layer_step; INVALID_ARG when no block is attached.
 */
dare_status dare_block_step(dare_ctx* ctx, int mode, float threshold, int batch,
                            int seq, const void* x, float* q_prev, void* k_cache,
                            void* v_cache, void* o_cache, void* out,
                            uint8_t* reuse_mask, int32_t* sel_idx, int32_t* sel_count,
                            float* scores, void* hip_stream);

/*
 * Thresholds from reuse rates (Sec. 3.1, "Reuse rate allocation").
 *
 * Rule DARE_RULE_SCORE (default): the `threshold` argument of the step calls is the
 * drift score tau itself.  Rule DARE_RULE_QUANTILE: it is a reuse rate phi in [0, 1],
 * and each sequence's tau is "the drift score at the phi-quantile" of its own scores at
 * this step: the k-th smallest, k = ceil(phi * seq) with the product formed in fp32
 * (phi = 0: tau = -inf, nothing reused; scores that tie with the k-th are reused too;
 * NaN scores sort last, and if the k-th smallest is NaN tau is +inf).  The selection is
 * exact (radix select on the device); tau never travels to the host.  A phi outside
 * [0, 1] is INVALID_ARG at the step call.
 */
enum { DARE_RULE_SCORE = 0, DARE_RULE_QUANTILE = 1 };
dare_status dare_set_threshold_rule(dare_ctx* ctx, int rule);

/*
 * Copy the tau that each sequence used in the last step under DARE_RULE_QUANTILE into
 * dst (device memory, [batch] fp32, batch <= max_batch); enqueued on the stream, no
 * synchronisation.  INVALID_ARG before the rule was first set.
 */
dare_status dare_get_thresholds(dare_ctx* ctx, float* dst, int batch, void* hip_stream);

/*
 * Running layer-wise drift score s_l = mean over tokens and steps of the drift score
 * (Sec. 3.1 eq. 2 of "Reuse rate allocation").  enable(on = 1) zeroes the
 * accumulators and makes every later step (any mode, any rule) add its scores: one
 * fp64 sum and one count on the device, NaN scores left out.  read() synchronises the
 * stream and returns mean (0 if count is 0) and count.  Costs one small kernel per step
 * while enabled under DARE_RULE_SCORE, nothing extra under DARE_RULE_QUANTILE.
 */
dare_status dare_drift_stats_enable(dare_ctx* ctx, int on, void* hip_stream);
dare_status dare_drift_stats_read(dare_ctx* ctx, double* mean, int64_t* count,
                                  void* hip_stream);

/*
 * Layer-wise reuse rates (same section): phi_out[l] = min(1, n_layers * phi_bar *
 * softmax(-s / eps)[l]).  Host arrays of n_layers doubles; no GPU work.
 * INVALID_ARG for n_layers < 1, eps <= 0, phi_bar outside [0, 1] or a NaN.
 */
dare_status dare_allocate_quantiles(int n_layers, const double* s, double phi_bar,
                                    double eps, double* phi_out);

/*
 * The schedule of Sec. 5 (Fast-dLLM-v2 setting), host only: returns DARE_MODE_DENSE
 * for layers [0, skip_layers) and, when refresh_interval > 0, for every step whose
 * index is a multiple of it; else `mode`.
 */
int dare_policy_mode(int mode, int layer, int step, int skip_layers, int refresh_interval);

/*
 * Frozen prefix (prefix caching composed with the reuse modes; Sec. 1 and Sec. 5 name the
 * combination, the reading is the common one for diffusion LLMs): the first prefix_len
 * tokens of every sequence are never projected, scored or queried by the step calls
 * that follow.  Their K, V and output cache rows are read as they are (the caller
 * filled them with an earlier step at prefix_len = 0), their reuse_mask byte is 1, their
 * score 0, their q_prev row is left alone, and `out` returns their cached row.  In every
 * mode, DENSE included, "all rows" then means all rows that are not frozen; a quantile
 * threshold ranks the other tokens only.  prefix_len = 0 switches it off.
 * INVALID_ARG: prefix_len < 0 or >= max_seq; a later step with seq <= prefix_len.
 */
dare_status dare_set_prefix(dare_ctx* ctx, int prefix_len);

/*
 * dare_layer_step for callers that cannot allocate device memory: code under HIP graph
 * capture that must not meet an allocation, tight serving loops, harnesses that forbid
 * hipMalloc.  It needs no context and calls no hipMalloc, hipFree or any other allocating
 * routine, at the first call or later: the scratch that dare_create would allocate (queries,
 * attention rows, the fp32 scored query, the refreshed-row list) lives in a static device
 * array inside the library, which every GPU the library runs on holds until the process
 * ends.
 *
 *   cfg      as for dare_create; max_batch and max_seq are not used
 *   wqkv_t   device, [3 * hidden, hidden]: Wq, Wk, Wv, each re-packed by
 *            dare_k_pack_weight (ldwt = hidden) and stored one after the other
 *   wo_t     device, [hidden, hidden]: Wo re-packed the same way
 *   the other arguments, the modes and the results are those of dare_layer_step (score
 *   rule; no frozen prefix, no block).
 *
 * Limits (DARE_ERR_UNSUPPORTED with a message naming the limit):
 *   batch * seq * hidden * sizeof(dtype)  <= DARE_STATIC_MAX_ROW_BYTES
 *   batch * seq * scored width            <= DARE_STATIC_MAX_SCORE_ELEMS
 * (scored width = head_dim, or hidden with score_head = -1); 1024 tokens of hidden 4096 in
 * bf16 fit exactly.  The array takes about 20.5 MiB per GPU.
 *
 * All calls on one GPU share that GPU's array: two calls whose kernels overlap (different
 * streams, different threads) race; order them on one stream.  Nothing in the scratch has to
 * start at zero, and nothing is kept between calls: every word a kernel reads was written
 * earlier in the same call.
 *
 * dare_static_init(device) looks up the array's device address ahead of time (the step
 * call does it by itself on first use on a device); call it before a graph capture starts.
 * Errors: as dare_layer_step, plus the config errors of dare_create; the text is read with
 * dare_last_error(NULL) on the calling thread.
 */
#define DARE_STATIC_MAX_ROW_BYTES (8u << 20)
#define DARE_STATIC_MAX_SCORE_ELEMS (1u << 20)
dare_status dare_static_init(int device);
dare_status dare_layer_step_static(const dare_config* cfg, const void* wqkv_t, const void* wo_t,
                                   int mode, float threshold, int batch, int seq,
                                   const void* hidden, float* q_prev, void* k_cache,
                                   void* v_cache, void* o_cache, void* out,
                                   uint8_t* reuse_mask, int32_t* sel_idx, int32_t* sel_count,
                                   float* scores, void* hip_stream);

/* Free a context and its device memory.  NULL is a no-op. */
dare_status dare_destroy(dare_ctx* ctx);

/* Text of the last error on this context (or of the last failed dare_create
 * on this thread when ctx is NULL).  Host pointer, valid until the next call. */
const char* dare_last_error(const dare_ctx* ctx);

/* Library version, "major.minor".  Host pointer, static. */
const char* dare_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DARE_H */
