// C ABI of libdare: context, argument checks and the sequence of kernel launches
// that makes one layer step (Alg. 1, Alg. 2, App. E.2 of the paper).  Host code
// only; every stage runs in the kernels of the other .hip files.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "dare_common.h"

using namespace dare;

struct dare_ctx {
  dare_config cfg;
  size_t esize;        // bytes per element of cfg.dtype
  int score_width;     // head_dim, or hidden when the whole query is scored
  void* wqkv_t;        // [3d, d] packed Wq | Wk | Wv
  void* wo_t;          // [d, d] packed Wo
  void* q_buf;         // [max tokens, d] queries, token-indexed
  void* attn_buf;      // [max tokens, d] attention rows before Wo, token-indexed
  float* q_new;        // fp32 scored query of this step: up to 8 k-range slabs of
                       // [tokens, score_width]
  size_t q_new_elems;
  int32_t* sel_idx;    // [max tokens]
  int32_t* sel_off;    // [max_batch + 1]
  // the block around the layer (dare_block_attach)
  bool has_block, has_bias;
  dare_block_config block;
  void* gain;          // [d] copies of the caller's vectors
  void* bias;          // [d] or nullptr
  void* h_buf;         // [max tokens, d] normalised hidden state
  float* rope_table;   // [max_seq, head_dim / 2, 2] (cos, sin), or nullptr
  // thresholds from reuse rates and drift statistics
  int rule;            // DARE_RULE_SCORE or DARE_RULE_QUANTILE
  bool stats_on;
  float* tau_dev;      // [max_batch] thresholds of the last quantile step
  float* scores_buf;   // [max tokens] scores when the caller passes none
  double* stat_sum;    // [max_batch] fp64 sums followed by [max_batch] 64-bit counts, one slot per sequence
  // frozen prefix
  int prefix;          // tokens [0, prefix) of every sequence are frozen
  int32_t* act_idx;    // [max tokens] ids of the tokens that are not frozen
  int32_t* act_off;    // [max_batch + 1] offsets of the sequences in act_idx
  std::string err;
};

// what the block adds to a layer step (all null / zero for dare_layer_step)
struct BlockExtras {
  const float* rope;   // rotary table or nullptr
  const void* x_resid; // hidden state before normalisation when out = x + O, else nullptr
};

namespace {

thread_local std::string g_create_err;

dare_status fail(dare_ctx* ctx, dare_status st, const char* what) {
  if (ctx) ctx->err = what; else g_create_err = what;
  return st;
}

dare_status fail_hip(dare_ctx* ctx, hipError_t e, const char* where) {
  std::string m = std::string(where) + ": " + hipGetErrorString(e);
  if (ctx) ctx->err = m; else g_create_err = m;
  return e == hipErrorOutOfMemory ? DARE_ERR_OOM : DARE_ERR_HIP;
}

struct DeviceGuard {
  int prev = -1;
  bool changed = false;
  hipError_t enter(int dev) {
    hipError_t e = hipGetDevice(&prev);
    if (e != hipSuccess) return e;
    if (prev != dev) {
      e = hipSetDevice(dev);
      changed = e == hipSuccess;
    }
    return e;
  }
  ~DeviceGuard() {
    if (changed) (void)hipSetDevice(prev);
  }
};

void free_ctx(dare_ctx* c) {
  if (!c) return;
  void* bufs[] = {c->wqkv_t, c->wo_t, c->q_buf, c->attn_buf, c->q_new, c->sel_idx, c->sel_off, c->gain, c->bias, c->h_buf, c->rope_table, c->tau_dev, c->scores_buf,
                  c->stat_sum, c->act_idx, c->act_off};
  for (void* b : bufs)
    if (b) (void)hipFree(b);
  delete c;
}

hipError_t gemm(const dare_ctx* c, const GemmArgs& g, hipStream_t s) {
  return c->cfg.dtype == DARE_BF16 ? launch_gemm_bf16(g, s) : launch_gemm_f32(g, s);
}
hipError_t attn(const dare_ctx* c, const AttnArgs& a, hipStream_t s) {
  return c->cfg.dtype == DARE_BF16 ? launch_attn_bf16(a, s) : launch_attn_f32(a, s);
}

}  // namespace

extern "C" {

const char* dare_version(void) { return "0.2"; }

const char* dare_last_error(const dare_ctx* ctx) {
  return ctx ? ctx->err.c_str() : g_create_err.c_str();
}

dare_status dare_create(const dare_config* cfg, const void* wq, const void* wk, const void* wv,
                        const void* wo, void* hip_stream, dare_ctx** out_ctx) {
  if (out_ctx) *out_ctx = nullptr;
  if (!cfg || !out_ctx) return fail(nullptr, DARE_ERR_INVALID_ARG, "null config or out_ctx");
  if (cfg->struct_size != sizeof(dare_config))
    return fail(nullptr, DARE_ERR_INVALID_ARG, "struct_size does not match this library");
  if (!wq || !wk || !wv || !wo) return fail(nullptr, DARE_ERR_INVALID_ARG, "null weight pointer");
  if (cfg->flags != 0) return fail(nullptr, DARE_ERR_INVALID_ARG, "flags must be 0");
  if (cfg->dtype != DARE_F32 && cfg->dtype != DARE_BF16)
    return fail(nullptr, DARE_ERR_INVALID_ARG, "unknown dtype");
  if (cfg->hidden < 1 || cfg->n_heads < 1 || cfg->head_dim < 1 || cfg->max_batch < 1 ||
      cfg->max_seq < 1 || cfg->device < 0)
    return fail(nullptr, DARE_ERR_INVALID_ARG, "non-positive size");
  if ((long)cfg->n_heads * cfg->head_dim != cfg->hidden)
    return fail(nullptr, DARE_ERR_INVALID_ARG, "hidden != n_heads * head_dim");
  if (cfg->score_head != 0 && cfg->score_head != -1)
    return fail(nullptr, DARE_ERR_UNSUPPORTED, "score_head must be 0 or -1");
  if (cfg->head_dim != 64 && cfg->head_dim != 128)
    return fail(nullptr, DARE_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
  if (cfg->hidden % 64 != 0) return fail(nullptr, DARE_ERR_UNSUPPORTED, "hidden must be a multiple of 64");
  const long max_tok = (long)cfg->max_batch * cfg->max_seq;
  if (max_tok > (1l << 30) / 2) return fail(nullptr, DARE_ERR_UNSUPPORTED, "max_batch * max_seq too large");

  DeviceGuard guard;
  hipError_t e = guard.enter(cfg->device);
  if (e != hipSuccess) return fail_hip(nullptr, e, "hipSetDevice");

  dare_ctx* c = new (std::nothrow) dare_ctx();
  if (!c) return fail(nullptr, DARE_ERR_OOM, "host allocation failed");
  c->cfg = *cfg;
  c->esize = cfg->dtype == DARE_BF16 ? 2 : 4;
  c->score_width = cfg->score_head < 0 ? cfg->hidden : cfg->head_dim;
  c->wqkv_t = c->wo_t = c->q_buf = c->attn_buf = nullptr;
  c->q_new = nullptr;
  c->sel_idx = c->sel_off = nullptr;
  c->has_block = c->has_bias = false;
  c->gain = c->bias = c->h_buf = nullptr;
  c->rope_table = nullptr;
  c->rule = DARE_RULE_SCORE;
  c->stats_on = false;
  c->tau_dev = c->scores_buf = nullptr;
  c->stat_sum = nullptr;
  c->prefix = 0;
  c->act_idx = c->act_off = nullptr;
  const size_t d = cfg->hidden;
  // room for 8 k-range slabs of the scored columns up to 4096 tokens (beyond that the
  // projection has enough tiles without cutting k)
  c->q_new_elems = (size_t)max_tok * c->score_width;
  if (max_tok <= 4096) c->q_new_elems *= 8;
  struct { void** p; size_t bytes; } allocs[] = {
      {&c->wqkv_t, 3 * d * d * c->esize},
      {&c->wo_t, d * d * c->esize},
      {&c->q_buf, (size_t)max_tok * d * c->esize},
      {&c->attn_buf, (size_t)max_tok * d * c->esize},
      {(void**)&c->q_new, c->q_new_elems * sizeof(float)},
      {(void**)&c->sel_idx, (size_t)max_tok * sizeof(int32_t)},
      {(void**)&c->sel_off, ((size_t)cfg->max_batch + 1) * sizeof(int32_t)},
  };
  for (auto& a : allocs) {
    if (a.bytes == 0) continue;
    e = hipMalloc(a.p, a.bytes);
    if (e != hipSuccess) {
      *a.p = nullptr;
      dare_status st = fail_hip(nullptr, e, "hipMalloc");
      free_ctx(c);
      return st;
    }
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const void* w3[3] = {wq, wk, wv};
  for (int i = 0; i < 3 && e == hipSuccess; ++i)
    e = launch_pack_weight(cfg->dtype, w3[i], cfg->hidden, cfg->hidden,
                           static_cast<char*>(c->wqkv_t) + (size_t)i * d * d * c->esize, cfg->hidden, s);
  if (e == hipSuccess) e = launch_pack_weight(cfg->dtype, wo, cfg->hidden, cfg->hidden, c->wo_t, cfg->hidden, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) {
    dare_status st = fail_hip(nullptr, e, "weight packing");
    free_ctx(c);
    return st;
  }
  *out_ctx = c;
  return DARE_OK;
}

dare_status dare_destroy(dare_ctx* ctx) {
  if (!ctx) return DARE_OK;
  DeviceGuard guard;
  (void)guard.enter(ctx->cfg.device);
  free_ctx(ctx);
  return DARE_OK;
}

namespace {

dare_status check_step_args(dare_ctx* ctx, int mode, float threshold, int batch, int seq, const void* hidden,
                            const float* q_prev, const void* k_cache, const void* v_cache,
                            const void* o_cache, const void* out, const uint8_t* reuse_mask) {
  if (mode != DARE_MODE_DENSE && mode != DARE_MODE_KV && mode != DARE_MODE_O && mode != DARE_MODE_KVO)
    return fail(ctx, DARE_ERR_INVALID_ARG, "unknown mode");
  if (!hidden || !q_prev || !k_cache || !v_cache || !o_cache || !out || !reuse_mask)
    return fail(ctx, DARE_ERR_INVALID_ARG, "null required pointer");
  if (batch < 1 || seq < 1) return fail(ctx, DARE_ERR_INVALID_ARG, "batch and seq must be >= 1");
  if (batch > ctx->cfg.max_batch || seq > ctx->cfg.max_seq)
    return fail(ctx, DARE_ERR_INVALID_ARG, "batch or seq exceeds the context's maximum");
  if (std::isnan(threshold)) return fail(ctx, DARE_ERR_INVALID_ARG, "threshold is NaN");
  if (ctx->rule == DARE_RULE_QUANTILE && !(threshold >= 0.f && threshold <= 1.f))
    return fail(ctx, DARE_ERR_INVALID_ARG, "under the quantile rule the threshold is a reuse rate in [0, 1]");
  if (ctx->prefix >= seq) return fail(ctx, DARE_ERR_INVALID_ARG, "the frozen prefix covers the whole sequence");
  return DARE_OK;
}

// The launches of one layer step on already-normalised hidden states (arguments checked
// by the caller).
dare_status step_impl(dare_ctx* ctx, int mode, float threshold, int batch, int seq, const void* hidden,
                      float* q_prev, void* k_cache, void* v_cache, void* o_cache, void* out,
                      uint8_t* reuse_mask, int32_t* sel_idx, int32_t* sel_count, float* scores,
                      const BlockExtras& bx, void* hip_stream) {
  const dare_config& cf = ctx->cfg;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int d = cf.hidden, n_tok = batch * seq, sw = ctx->score_width;
  const size_t es = ctx->esize;
  const char* wq_t = static_cast<const char*>(ctx->wqkv_t);
  const char* wkv_t = wq_t + (size_t)d * d * es;
  const bool sel_kv = mode == DARE_MODE_KV || mode == DARE_MODE_KVO;
  const bool sel_o = mode == DARE_MODE_O || mode == DARE_MODE_KVO;
  const int32_t* n_sel = ctx->sel_off + batch;  // device count of refreshed tokens
  hipError_t e;
  int k_parts = 1;

  // Frozen prefix: "all rows" below means the rows of this list, and their results go into
  // the caches at their token index as the refreshed rows' do.
  const int P = ctx->prefix;
  const bool pre = P > 0;
  const int n_act = batch * (seq - P);
  // (written by every step that has a prefix: a list cached across calls would be wrong as
  // soon as a step is recorded into a graph and replayed between eager steps of another shape)
  if (pre && (e = launch_active_list(batch, seq, P, ctx->act_idx, ctx->act_off, s)) != hipSuccess)
    return fail_hip(ctx, e, "active-row list");
  const int32_t* act_idx = pre ? ctx->act_idx : nullptr;

  // 1. Query projection feeding the score (Alg. 1/2 line 2), together with whatever
  //    else this mode projects for all rows.
  GemmArgs g{};
  g.a = hidden;
  g.lda = d;
  g.k = d;
  g.m_max = n_act;
  g.idx = act_idx;
  g.ldc = d;
  g.seg_n = d;
  g.c32 = ctx->q_new;
  g.c32_cols = sw;
  g.wt = wq_t;
  g.rope = bx.rope;  // queries and keys are rotated as they are written; the fp32 copy
  g.rope_dh = cf.head_dim;  // that feeds the score is not
  g.rope_seq = seq;
  if (mode == DARE_MODE_DENSE || mode == DARE_MODE_O) {
    g.n = 3 * d;  // Q, K, V for every row (App. E.2; Alg. 2 lines 2 and 7)
    g.c[0] = ctx->q_buf;
    g.c[1] = k_cache;
    g.c[2] = v_cache;
    g.rope_cols = 2 * d;
  } else if (mode == DARE_MODE_KV) {
    g.n = d;  // Q for every row (Alg. 1 line 2)
    g.c[0] = ctx->q_buf;
    g.rope_cols = d;
  } else {
    g.rope = nullptr;
    g.n = sw;  // only the scored columns of Q for every row
    // few output tiles, long k: cut k into ranges that the score kernel adds up
    if (cf.dtype == DARE_BF16) {
      const int tiles = ((n_act + 63) / 64) * ((sw + 63) / 64), ksteps = d / 64;
      while (tiles * k_parts * 2 <= 256 && k_parts * 2 <= 8 && ksteps % (k_parts * 2) == 0 &&
             ksteps / (k_parts * 2) >= 4 && (size_t)n_tok * sw * (k_parts * 2) <= ctx->q_new_elems)
        k_parts *= 2;
      g.k_parts = k_parts;
      g.c32_part_stride = (long)n_tok * sw;
    }
  }
  if ((e = gemm(ctx, g, s)) != hipSuccess) return fail_hip(ctx, e, "query projection");

  // 2. Drift score, reuse decision, score-cache update (Alg. 1/2 lines 3-5).  Under the
  //    quantile rule the score kernel's decision is replaced by the one the select
  //    kernel takes; with statistics on, that kernel also (or only) adds up the scores.
  const bool by_rate = ctx->rule == DARE_RULE_QUANTILE;
  float* sc = scores;
  if (!sc && (by_rate || ctx->stats_on)) sc = ctx->scores_buf;
  e = launch_score(ctx->q_new, sw, sw, k_parts, (long)n_tok * sw, q_prev, n_tok, by_rate ? 0.f : threshold,
                   mode == DARE_MODE_DENSE || by_rate, sc, nullptr, reuse_mask, seq, P, s);
  if (e != hipSuccess) return fail_hip(ctx, e, "score");
  if (by_rate || ctx->stats_on) {
    const int rank = by_rate ? (int)ceilf(threshold * (float)(seq - P)) : -1;
    double* sum = ctx->stats_on ? ctx->stat_sum : nullptr;
    e = launch_quantile_mask(sc, batch, seq, P, seq - P, rank, mode == DARE_MODE_DENSE, ctx->tau_dev, reuse_mask,
                             sum, reinterpret_cast<unsigned long long*>(sum ? sum + cf.max_batch : nullptr), s);
    if (e != hipSuccess) return fail_hip(ctx, e, "threshold selection");
  }

  // 3. Index list of the refreshed tokens.  With at most kSelMaxTokens tokens the bf16
  //    refreshed-row projection derives the list itself (and leaves it for the kernels after
  //    it): one launch less.
  const bool fused_sel = sel_kv && cf.dtype == DARE_BF16 && n_tok <= kSelMaxTokens;
  if (!fused_sel && (mode != DARE_MODE_DENSE || sel_idx || sel_count)) {
    e = launch_compact(reuse_mask, batch, seq, ctx->sel_idx, sel_idx, sel_count, nullptr,
                       ctx->sel_off, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "compaction");
  }

  // 4. Projections of the refreshed rows (Alg. 1 lines 6-9), written straight into
  //    the token-indexed caches / query buffer.
  if (sel_kv) {
    GemmArgs r{};
    r.a = hidden;
    r.lda = d;
    r.k = d;
    r.m_max = n_tok;
    if (fused_sel) {
      r.sel_mask = reuse_mask;
      r.sel_batch = batch;
      r.sel_seq = seq;
      r.sel_idx_out = ctx->sel_idx;
      r.sel_idx_out2 = sel_idx;
      r.sel_off_out = ctx->sel_off;
      r.sel_count_out = sel_count;
    } else {
      r.idx = ctx->sel_idx;
      r.m_dev = n_sel;
    }
    r.ldc = d;
    r.seg_n = d;
    r.rope = bx.rope;
    r.rope_dh = cf.head_dim;
    r.rope_seq = seq;
    if (mode == DARE_MODE_KV) {
      r.wt = wkv_t;
      r.n = 2 * d;
      r.c[0] = k_cache;
      r.c[1] = v_cache;
      r.rope_cols = d;
    } else {
      r.wt = wq_t;
      r.n = 3 * d;
      r.c[0] = ctx->q_buf;
      r.c[1] = k_cache;
      r.c[2] = v_cache;
      r.rope_cols = 2 * d;
    }
    if ((e = gemm(ctx, r, s)) != hipSuccess) return fail_hip(ctx, e, "refreshed-row projection");
  }

  // 5. Attention (Alg. 1 line 10 / Alg. 2 line 8).
  AttnArgs a{};
  a.q = ctx->q_buf;
  a.k = k_cache;
  a.v = v_cache;
  a.out = ctx->attn_buf;
  a.batch = batch;
  a.seq = seq;
  a.n_heads = cf.n_heads;
  a.head_dim = cf.head_dim;
  a.idx = sel_o ? ctx->sel_idx : act_idx;
  a.sel_off = sel_o ? ctx->sel_off : (pre ? ctx->act_off : nullptr);
  a.many_rows = !sel_o && pre;
  if ((e = attn(ctx, a, s)) != hipSuccess) return fail_hip(ctx, e, "attention");

  // 6. Output projection (Alg. 1 line 11; Alg. 2 lines 9-11 with the cache after Wo).
  GemmArgs o{};
  o.a = ctx->attn_buf;
  o.lda = d;
  o.wt = ctx->wo_t;
  o.n = d;
  o.k = d;
  o.m_max = n_tok;
  o.ldc = d;
  o.seg_n = d;
  if (sel_o) {
    o.idx = ctx->sel_idx;
    o.m_dev = n_sel;
    o.c[0] = o_cache;
  } else if (pre) {
    o.idx = act_idx;
    o.m_max = n_act;
    o.c[0] = o_cache;
  } else {
    o.c[0] = bx.x_resid ? o_cache : out;
  }
  if ((e = gemm(ctx, o, s)) != hipSuccess) return fail_hip(ctx, e, "output projection");

  // 7. out = x + O for every row from the refreshed and the cached rows of O, or keep
  //    out and o_cache equal when they are different buffers.
  if (bx.x_resid) {
    e = launch_residual_add(cf.dtype, bx.x_resid, o_cache, out, (long)n_tok * d, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "residual sum");
  } else if (out != o_cache) {
    e = (sel_o || pre) ? launch_copy_rows(o_cache, out, n_tok, (int)(d * es), nullptr, nullptr, s)
                       : launch_copy_rows(out, o_cache, n_tok, (int)(d * es), nullptr, nullptr, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "output copy");
  }
  return DARE_OK;
}

}  // namespace

dare_status dare_layer_step(dare_ctx* ctx, int mode, float threshold, int batch, int seq,
                            const void* hidden, float* q_prev, void* k_cache, void* v_cache,
                            void* o_cache, void* out, uint8_t* reuse_mask, int32_t* sel_idx,
                            int32_t* sel_count, float* scores, void* hip_stream) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  dare_status st = check_step_args(ctx, mode, threshold, batch, seq, hidden, q_prev, k_cache, v_cache,
                                   o_cache, out, reuse_mask);
  if (st != DARE_OK) return st;
  return step_impl(ctx, mode, threshold, batch, seq, hidden, q_prev, k_cache, v_cache, o_cache, out,
                   reuse_mask, sel_idx, sel_count, scores, BlockExtras{nullptr, nullptr}, hip_stream);
}

// ---------------------------------------------------------------------------
// The layer step for callers that cannot allocate: no context, scratch in a file-scope
// device array.
// ---------------------------------------------------------------------------
namespace {

// Layout of the static scratch (bytes): queries | attention rows | fp32 scored query (up to
// 8 k-range slabs) | refreshed-row list | per-sequence offsets.
constexpr size_t kStaticRowBytes = DARE_STATIC_MAX_ROW_BYTES;          // batch * seq * hidden * sizeof(dtype)
constexpr size_t kStaticScoreElems = DARE_STATIC_MAX_SCORE_ELEMS;     // fp32 elements of the scored query, slabs included
constexpr size_t kStaticMaxTokens = kStaticRowBytes / (64 * 2);        // hidden >= 64, two bytes per element
constexpr size_t kStaticOffQ = 0;
constexpr size_t kStaticOffAttn = kStaticOffQ + kStaticRowBytes;
constexpr size_t kStaticOffScore = kStaticOffAttn + kStaticRowBytes;
constexpr size_t kStaticOffIdx = kStaticOffScore + kStaticScoreElems * sizeof(float);
constexpr size_t kStaticOffOff = kStaticOffIdx + kStaticMaxTokens * sizeof(int32_t);
constexpr size_t kStaticBytes = kStaticOffOff + (kStaticMaxTokens + 64) * sizeof(int32_t);
static_assert(kStaticOffAttn % 256 == 0 && kStaticOffScore % 256 == 0 && kStaticOffIdx % 256 == 0 &&
                  kStaticOffOff % 256 == 0, "scratch regions must stay aligned");

}  // namespace

// Every GPU the library runs on holds its own copy of this array until the process ends.  In
// host code the name is only a handle: the memory is reached through the per-device address
// that hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_lock;
unsigned char* g_static_ptr[kMaxDevices];  // device address of `scratch` on each device, once looked up

// The address of this device's copy of the scratch array (the device must be current).
dare_status static_scratch(int device, unsigned char** out) {
  if (device < 0 || device >= kMaxDevices) return fail(nullptr, DARE_ERR_INVALID_ARG, "device ordinal out of range");
  std::lock_guard<std::mutex> lock(g_static_lock);
  if (!g_static_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(nullptr, e, "hipGetSymbolAddress(scratch)");
    if (!p) return fail(nullptr, DARE_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
    g_static_ptr[device] = static_cast<unsigned char*>(p);
  }
  *out = g_static_ptr[device];
  return DARE_OK;
}

}  // namespace

extern "C" {

dare_status dare_static_init(int device) {
  DeviceGuard guard;
  hipError_t e = guard.enter(device);
  if (e != hipSuccess) return fail_hip(nullptr, e, "hipSetDevice");
  unsigned char* p = nullptr;
  return static_scratch(device, &p);
}

dare_status dare_layer_step_static(const dare_config* cfg, const void* wqkv_t, const void* wo_t, int mode,
                                   float threshold, int batch, int seq, const void* hidden, float* q_prev,
                                   void* k_cache, void* v_cache, void* o_cache, void* out, uint8_t* reuse_mask,
                                   int32_t* sel_idx, int32_t* sel_count, float* scores, void* hip_stream) {
  if (!cfg) return fail(nullptr, DARE_ERR_INVALID_ARG, "null config");
  if (cfg->struct_size != sizeof(dare_config))
    return fail(nullptr, DARE_ERR_INVALID_ARG, "struct_size does not match this library");
  if (!wqkv_t || !wo_t) return fail(nullptr, DARE_ERR_INVALID_ARG, "null weight pointer");
  if (cfg->flags != 0) return fail(nullptr, DARE_ERR_INVALID_ARG, "flags must be 0");
  if (cfg->dtype != DARE_F32 && cfg->dtype != DARE_BF16) return fail(nullptr, DARE_ERR_INVALID_ARG, "unknown dtype");
  if (cfg->hidden < 1 || cfg->n_heads < 1 || cfg->head_dim < 1 || cfg->device < 0)
    return fail(nullptr, DARE_ERR_INVALID_ARG, "non-positive size");
  if ((long)cfg->n_heads * cfg->head_dim != cfg->hidden)
    return fail(nullptr, DARE_ERR_INVALID_ARG, "hidden != n_heads * head_dim");
  if (cfg->score_head != 0 && cfg->score_head != -1)
    return fail(nullptr, DARE_ERR_UNSUPPORTED, "score_head must be 0 or -1");
  if (cfg->head_dim != 64 && cfg->head_dim != 128)
    return fail(nullptr, DARE_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
  if (cfg->hidden % 64 != 0) return fail(nullptr, DARE_ERR_UNSUPPORTED, "hidden must be a multiple of 64");
  if (batch < 1 || seq < 1) return fail(nullptr, DARE_ERR_INVALID_ARG, "batch and seq must be >= 1");
  const size_t esize = cfg->dtype == DARE_BF16 ? 2 : 4;
  const int score_width = cfg->score_head < 0 ? cfg->hidden : cfg->head_dim;
  const size_t n_tok = (size_t)batch * (size_t)seq;
  if (n_tok * (size_t)cfg->hidden * esize > kStaticRowBytes)
    return fail(nullptr, DARE_ERR_UNSUPPORTED,
                "batch * seq * hidden * sizeof(dtype) exceeds DARE_STATIC_MAX_ROW_BYTES, the static scratch");
  if (n_tok * (size_t)score_width > kStaticScoreElems)
    return fail(nullptr, DARE_ERR_UNSUPPORTED,
                "batch * seq * scored width exceeds DARE_STATIC_MAX_SCORE_ELEMS, the static scratch");

  DeviceGuard guard;
  hipError_t e = guard.enter(cfg->device);
  if (e != hipSuccess) return fail_hip(nullptr, e, "hipSetDevice");
  unsigned char* base = nullptr;
  dare_status st = static_scratch(cfg->device, &base);
  if (st != DARE_OK) return st;

  // a context on the stack: the caller's packed weights, scratch inside the static array
  dare_ctx c{};
  c.cfg = *cfg;
  c.cfg.max_batch = batch;
  c.cfg.max_seq = seq;
  c.esize = esize;
  c.score_width = score_width;
  c.wqkv_t = const_cast<void*>(wqkv_t);
  c.wo_t = const_cast<void*>(wo_t);
  c.q_buf = base + kStaticOffQ;
  c.attn_buf = base + kStaticOffAttn;
  c.q_new = reinterpret_cast<float*>(base + kStaticOffScore);
  c.q_new_elems = kStaticScoreElems;
  c.sel_idx = reinterpret_cast<int32_t*>(base + kStaticOffIdx);
  c.sel_off = reinterpret_cast<int32_t*>(base + kStaticOffOff);
  c.rule = DARE_RULE_SCORE;
  st = check_step_args(&c, mode, threshold, batch, seq, hidden, q_prev, k_cache, v_cache, o_cache, out, reuse_mask);
  if (st == DARE_OK)
    st = step_impl(&c, mode, threshold, batch, seq, hidden, q_prev, k_cache, v_cache, o_cache, out, reuse_mask,
                   sel_idx, sel_count, scores, BlockExtras{nullptr, nullptr}, hip_stream);
  if (st != DARE_OK) g_create_err = c.err;
  return st;
}

}  // extern "C"

namespace {
// (cos, sin) of pos * base^(-2 i / head_dim) in double precision, rounded to fp32
void fill_rope_table(float* t, int n_pos, int head_dim, double base) {
  const int half = head_dim / 2;
  for (int p = 0; p < n_pos; ++p)
    for (int i = 0; i < half; ++i) {
      const double ang = (double)p * std::pow(base, -2.0 * (double)i / (double)head_dim);
      t[((size_t)p * half + i) * 2 + 0] = (float)std::cos(ang);
      t[((size_t)p * half + i) * 2 + 1] = (float)std::sin(ang);
    }
}
}  // namespace

dare_status dare_block_attach(dare_ctx* ctx, const dare_block_config* cfg, const void* gain,
                              const void* bias, void* hip_stream) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  if (!cfg || cfg->struct_size != sizeof(dare_block_config))
    return fail(ctx, DARE_ERR_INVALID_ARG, "null block config or struct_size mismatch");
  if (cfg->norm != DARE_NORM_NONE && cfg->norm != DARE_NORM_LAYER && cfg->norm != DARE_NORM_RMS)
    return fail(ctx, DARE_ERR_INVALID_ARG, "unknown norm kind");
  if (cfg->norm != DARE_NORM_NONE && !gain) return fail(ctx, DARE_ERR_INVALID_ARG, "norm needs a gain vector");
  if (cfg->norm != DARE_NORM_NONE && !(cfg->eps >= 0.f)) return fail(ctx, DARE_ERR_INVALID_ARG, "eps must be >= 0");
  if (cfg->norm != DARE_NORM_LAYER && bias) return fail(ctx, DARE_ERR_INVALID_ARG, "bias is for LayerNorm only");
  if (!(cfg->rope_base >= 0.f) || std::isinf(cfg->rope_base))
    return fail(ctx, DARE_ERR_INVALID_ARG, "rope_base must be 0 (off) or a positive number");
  if (cfg->residual != 0 && cfg->residual != 1) return fail(ctx, DARE_ERR_INVALID_ARG, "residual must be 0 or 1");
  if (ctx->cfg.hidden % 8 != 0) return fail(ctx, DARE_ERR_UNSUPPORTED, "hidden must be a multiple of 8");

  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->cfg.device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // work on the stream may still read the vectors of an earlier attach
  if ((e = hipStreamSynchronize(s)) != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
  ctx->has_block = false;
  const size_t vec_bytes = (size_t)ctx->cfg.hidden * ctx->esize;
  const size_t max_tok = (size_t)ctx->cfg.max_batch * ctx->cfg.max_seq;
  auto ensure = [&](void** p, size_t bytes) -> hipError_t {
    if (*p) return hipSuccess;
    hipError_t r = hipMalloc(p, bytes);
    if (r != hipSuccess) *p = nullptr;
    return r;
  };
  if (cfg->norm != DARE_NORM_NONE) {
    if ((e = ensure(&ctx->gain, vec_bytes)) != hipSuccess) return fail_hip(ctx, e, "hipMalloc");
    if ((e = ensure(&ctx->h_buf, max_tok * vec_bytes)) != hipSuccess) return fail_hip(ctx, e, "hipMalloc");
    if ((e = hipMemcpyAsync(ctx->gain, gain, vec_bytes, hipMemcpyDeviceToDevice, s)) != hipSuccess)
      return fail_hip(ctx, e, "gain copy");
    if (bias) {
      if ((e = ensure(&ctx->bias, vec_bytes)) != hipSuccess) return fail_hip(ctx, e, "hipMalloc");
      if ((e = hipMemcpyAsync(ctx->bias, bias, vec_bytes, hipMemcpyDeviceToDevice, s)) != hipSuccess)
        return fail_hip(ctx, e, "bias copy");
    }
  }
  if (cfg->rope_base > 0.f) {
    const size_t elems = (size_t)ctx->cfg.max_seq * ctx->cfg.head_dim;  // (cos, sin) x head_dim / 2
    if ((e = ensure((void**)&ctx->rope_table, elems * sizeof(float))) != hipSuccess)
      return fail_hip(ctx, e, "hipMalloc");
    dare_status st = dare_k_rope_table(ctx->rope_table, ctx->cfg.max_seq, ctx->cfg.head_dim,
                                       (double)cfg->rope_base);
    if (st != DARE_OK) return fail(ctx, st, "rotary table");
  }
  if ((e = hipStreamSynchronize(s)) != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
  ctx->block = *cfg;
  ctx->has_bias = bias != nullptr;
  ctx->has_block = true;
  return DARE_OK;
}

dare_status dare_block_step(dare_ctx* ctx, int mode, float threshold, int batch, int seq, const void* x,
                            float* q_prev, void* k_cache, void* v_cache, void* o_cache, void* out,
                            uint8_t* reuse_mask, int32_t* sel_idx, int32_t* sel_count, float* scores,
                            void* hip_stream) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  if (!ctx->has_block) return fail(ctx, DARE_ERR_INVALID_ARG, "no block attached");
  dare_status st = check_step_args(ctx, mode, threshold, batch, seq, x, q_prev, k_cache, v_cache, o_cache,
                                   out, reuse_mask);
  if (st != DARE_OK) return st;
  const dare_block_config& bc = ctx->block;
  if (bc.residual && out == o_cache)
    return fail(ctx, DARE_ERR_INVALID_ARG, "with the residual sum, out must not be o_cache");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const void* hidden = x;
  if (bc.norm != DARE_NORM_NONE) {  // Alg. 1/2 line 1
    const int P = ctx->prefix;  // frozen rows are not normalised: nothing reads them
    hipError_t e = launch_norm(ctx->cfg.dtype, bc.norm, x, ctx->gain, ctx->has_bias ? ctx->bias : nullptr,
                               bc.eps, batch * (seq - P), ctx->cfg.hidden, ctx->h_buf, P > 0 ? seq : 0, P, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "normalisation");
    hidden = ctx->h_buf;
  }
  BlockExtras bx{bc.rope_base > 0.f ? ctx->rope_table : nullptr, bc.residual ? x : nullptr};
  return step_impl(ctx, mode, threshold, batch, seq, hidden, q_prev, k_cache, v_cache, o_cache, out,
                   reuse_mask, sel_idx, sel_count, scores, bx, hip_stream);
}

}  // extern "C"

namespace dare {
dare_status block_core(dare_ctx* ctx, int mode, float threshold, int batch, int seq, const void* h, float* q_prev,
                       void* k_cache, void* v_cache, void* o_cache, uint8_t* reuse_mask, int32_t* sel_count,
                       void* hip_stream) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  if (!ctx->has_block) return fail(ctx, DARE_ERR_INVALID_ARG, "no block attached");
  dare_status st = check_step_args(ctx, mode, threshold, batch, seq, h, q_prev, k_cache, v_cache, o_cache,
                                   o_cache, reuse_mask);
  if (st != DARE_OK) return st;
  BlockExtras bx{ctx->block.rope_base > 0.f ? ctx->rope_table : nullptr, nullptr};
  return step_impl(ctx, mode, threshold, batch, seq, h, q_prev, k_cache, v_cache, o_cache, o_cache, reuse_mask,
                   nullptr, sel_count, nullptr, bx, hip_stream);
}
}  // namespace dare

extern "C" {

// ---------------------------------------------------------------------------
// kernel-level entry points
// ---------------------------------------------------------------------------
dare_status dare_k_pack_weight(int dtype, const void* w, int rows_k, int cols_n, void* wt, int ldwt,
                               void* hip_stream) {
  if (!w || !wt || rows_k < 1 || cols_n < 1 || ldwt < rows_k) return DARE_ERR_INVALID_ARG;
  if (dtype != DARE_F32 && dtype != DARE_BF16) return DARE_ERR_INVALID_ARG;
  hipError_t e = launch_pack_weight(dtype, w, rows_k, cols_n, wt, ldwt, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_gemm(int dtype, const void* a, int lda, const void* wt, int n, int k, int m_max,
                        const int32_t* idx, const int32_t* m_dev, void* const* c, int ldc, int seg_n,
                        float* c32, int c32_cols, int k_parts, long c32_part_stride, void* hip_stream) {
  if (!a || !wt || !c || n < 1 || k < 1 || m_max < 0 || lda < k) return DARE_ERR_INVALID_ARG;
  if (dtype != DARE_F32 && dtype != DARE_BF16) return DARE_ERR_INVALID_ARG;
  if (seg_n < 1 || n % seg_n != 0 || n / seg_n > 3) return DARE_ERR_INVALID_ARG;
  if (c32 && (c32_cols < 1 || c32_cols > n || c32_cols % 4 != 0)) return DARE_ERR_INVALID_ARG;
  if (k % 64 != 0 || n % (dtype == DARE_BF16 ? 64 : 16) != 0 || seg_n % 4 != 0) return DARE_ERR_UNSUPPORTED;
  if (k_parts < 1) return DARE_ERR_INVALID_ARG;
  if (k_parts > 1) {
    if (!c32 || c32_cols != n || c[0] || idx || m_dev || c32_part_stride < (long)m_max * c32_cols)
      return DARE_ERR_INVALID_ARG;
    if (dtype != DARE_BF16 || (k / 64) % k_parts != 0) return DARE_ERR_UNSUPPORTED;
  }
  GemmArgs g{};
  g.a = a;
  g.lda = lda;
  g.wt = wt;
  g.n = n;
  g.k = k;
  g.m_max = m_max;
  g.idx = idx;
  g.m_dev = m_dev;
  for (int i = 0; i < n / seg_n; ++i) g.c[i] = c[i];
  g.ldc = ldc;
  g.seg_n = seg_n;
  g.c32 = c32;
  g.c32_cols = c32 ? c32_cols : 0;
  g.k_parts = k_parts;
  g.c32_part_stride = c32_part_stride;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = dtype == DARE_BF16 ? launch_gemm_bf16(g, s) : launch_gemm_f32(g, s);
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

namespace {
// scratch of the threshold rule and the statistics, allocated on first use
dare_status ensure_threshold_buffers(dare_ctx* ctx) {
  const size_t max_tok = (size_t)ctx->cfg.max_batch * ctx->cfg.max_seq;
  struct { void** p; size_t bytes; } need[] = {
      {(void**)&ctx->tau_dev, (size_t)ctx->cfg.max_batch * sizeof(float)},
      {(void**)&ctx->scores_buf, max_tok * sizeof(float)},
      {(void**)&ctx->stat_sum, 2 * (size_t)ctx->cfg.max_batch * sizeof(double)},
  };
  for (auto& n : need) {
    if (*n.p) continue;
    hipError_t e = hipMalloc(n.p, n.bytes);
    if (e != hipSuccess) {
      *n.p = nullptr;
      return fail_hip(ctx, e, "hipMalloc");
    }
    if ((e = hipMemset(*n.p, 0, n.bytes)) != hipSuccess) return fail_hip(ctx, e, "hipMemset");
  }
  return DARE_OK;
}
}  // namespace

dare_status dare_set_threshold_rule(dare_ctx* ctx, int rule) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  if (rule != DARE_RULE_SCORE && rule != DARE_RULE_QUANTILE) return fail(ctx, DARE_ERR_INVALID_ARG, "unknown rule");
  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->cfg.device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  dare_status st = ensure_threshold_buffers(ctx);
  if (st != DARE_OK) return st;
  ctx->rule = rule;
  return DARE_OK;
}

dare_status dare_set_prefix(dare_ctx* ctx, int prefix_len) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  if (prefix_len < 0 || prefix_len >= ctx->cfg.max_seq)
    return fail(ctx, DARE_ERR_INVALID_ARG, "prefix_len must lie in [0, max_seq)");
  if (prefix_len > 0 && !ctx->act_idx) {
    DeviceGuard guard;
    hipError_t e = guard.enter(ctx->cfg.device);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
    const size_t max_tok = (size_t)ctx->cfg.max_batch * ctx->cfg.max_seq;
    if ((e = hipMalloc((void**)&ctx->act_idx, max_tok * sizeof(int32_t))) != hipSuccess) {
      ctx->act_idx = nullptr;
      return fail_hip(ctx, e, "hipMalloc");
    }
    if ((e = hipMalloc((void**)&ctx->act_off, ((size_t)ctx->cfg.max_batch + 1) * sizeof(int32_t))) != hipSuccess) {
      ctx->act_off = nullptr;
      (void)hipFree(ctx->act_idx);
      ctx->act_idx = nullptr;
      return fail_hip(ctx, e, "hipMalloc");
    }
  }
  ctx->prefix = prefix_len;
  return DARE_OK;
}

dare_status dare_get_thresholds(dare_ctx* ctx, float* dst, int batch, void* hip_stream) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  if (!dst || batch < 1 || batch > ctx->cfg.max_batch) return fail(ctx, DARE_ERR_INVALID_ARG, "bad dst or batch");
  if (!ctx->tau_dev) return fail(ctx, DARE_ERR_INVALID_ARG, "no threshold rule was set on this context");
  hipError_t e = hipMemcpyAsync(dst, ctx->tau_dev, (size_t)batch * sizeof(float), hipMemcpyDeviceToDevice,
                                static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? DARE_OK : fail_hip(ctx, e, "hipMemcpyAsync");
}

dare_status dare_drift_stats_enable(dare_ctx* ctx, int on, void* hip_stream) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  if (on != 0 && on != 1) return fail(ctx, DARE_ERR_INVALID_ARG, "on must be 0 or 1");
  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->cfg.device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  if (on) {
    dare_status st = ensure_threshold_buffers(ctx);
    if (st != DARE_OK) return st;
    // ordered on the stream after the steps already enqueued
    e = launch_zero_words(ctx->stat_sum, 2 * ctx->cfg.max_batch, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(ctx, e, "statistics reset");
  }
  ctx->stats_on = on != 0;
  return DARE_OK;
}

dare_status dare_drift_stats_read(dare_ctx* ctx, double* mean, int64_t* count, void* hip_stream) {
  if (!ctx) return DARE_ERR_INVALID_ARG;
  if (!mean || !count) return fail(ctx, DARE_ERR_INVALID_ARG, "null output pointer");
  if (!ctx->stat_sum) return fail(ctx, DARE_ERR_INVALID_ARG, "statistics were never enabled");
  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->cfg.device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int nb = ctx->cfg.max_batch;
  std::vector<double> host(2 * (size_t)nb);
  if ((e = hipMemcpyAsync(host.data(), ctx->stat_sum, host.size() * sizeof(double), hipMemcpyDeviceToHost, s)) !=
      hipSuccess)
    return fail_hip(ctx, e, "hipMemcpyAsync");
  if ((e = hipStreamSynchronize(s)) != hipSuccess) return fail_hip(ctx, e, "hipStreamSynchronize");
  double sum = 0.0;
  uint64_t n = 0;
  for (int b = 0; b < nb; ++b) {  // per-sequence slots, added in sequence order
    uint64_t nb_b;
    std::memcpy(&nb_b, &host[(size_t)nb + b], sizeof(nb_b));
    sum += host[b];
    n += nb_b;
  }
  *count = (int64_t)n;
  *mean = n ? sum / (double)n : 0.0;
  return DARE_OK;
}

dare_status dare_allocate_quantiles(int n_layers, const double* s, double phi_bar, double eps,
                                    double* phi_out) {
  if (n_layers < 1 || !s || !phi_out || !(eps > 0.0) || !(phi_bar >= 0.0 && phi_bar <= 1.0))
    return DARE_ERR_INVALID_ARG;
  double zmax = -INFINITY;
  for (int l = 0; l < n_layers; ++l) {
    if (std::isnan(s[l])) return DARE_ERR_INVALID_ARG;
    const double z = -s[l] / eps;
    if (z > zmax) zmax = z;
  }
  double den = 0.0;
  for (int l = 0; l < n_layers; ++l) den += std::exp(-s[l] / eps - zmax);
  for (int l = 0; l < n_layers; ++l) {
    const double phi = (double)n_layers * phi_bar * std::exp(-s[l] / eps - zmax) / den;
    phi_out[l] = phi < 1.0 ? phi : 1.0;
  }
  return DARE_OK;
}

int dare_policy_mode(int mode, int layer, int step, int skip_layers, int refresh_interval) {
  if (layer < skip_layers) return DARE_MODE_DENSE;
  if (refresh_interval > 0 && step % refresh_interval == 0) return DARE_MODE_DENSE;
  return mode;
}

dare_status dare_k_quantile_mask(const float* scores, int batch, int seq, float phi, int force_refresh,
                                 float* tau_out, uint8_t* mask, double* stat_sum, uint64_t* stat_count,
                                 void* hip_stream) {
  if (!scores || batch < 1 || seq < 1 || std::isnan(phi) || phi > 1.f) return DARE_ERR_INVALID_ARG;
  if ((stat_sum == nullptr) != (stat_count == nullptr)) return DARE_ERR_INVALID_ARG;
  if (phi >= 0.f && !mask) return DARE_ERR_INVALID_ARG;
  if (phi < 0.f && !stat_sum) return DARE_ERR_INVALID_ARG;
  const int rank = phi >= 0.f ? (int)ceilf(phi * (float)seq) : -1;
  hipError_t e = launch_quantile_mask(scores, batch, seq, 0, seq, rank, force_refresh, tau_out, mask, stat_sum,
                                      reinterpret_cast<unsigned long long*>(stat_count),
                                      static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_gemm_rope(int dtype, const void* a, int lda, const void* wt, int n, int k, int m_max,
                             const int32_t* idx, const int32_t* m_dev, void* const* c, int ldc, int seg_n,
                             float* c32, int c32_cols, const float* rope_table, int rope_cols,
                             int head_dim, int seq, void* hip_stream) {
  if (!a || !wt || !c || n < 1 || k < 1 || m_max < 0 || lda < k) return DARE_ERR_INVALID_ARG;
  if (dtype != DARE_F32 && dtype != DARE_BF16) return DARE_ERR_INVALID_ARG;
  if (seg_n < 1 || n % seg_n != 0 || n / seg_n > 3) return DARE_ERR_INVALID_ARG;
  if (c32 && (c32_cols < 1 || c32_cols > n || c32_cols % 4 != 0)) return DARE_ERR_INVALID_ARG;
  if (k % 64 != 0 || n % (dtype == DARE_BF16 ? 64 : 16) != 0 || seg_n % 4 != 0) return DARE_ERR_UNSUPPORTED;
  if (!rope_table || seq < 1 || head_dim < 4 || head_dim % 4 != 0 || rope_cols < 0 || rope_cols > n ||
      rope_cols % head_dim != 0 || seg_n % head_dim != 0)
    return DARE_ERR_INVALID_ARG;
  GemmArgs g{};
  g.a = a;
  g.lda = lda;
  g.wt = wt;
  g.n = n;
  g.k = k;
  g.m_max = m_max;
  g.idx = idx;
  g.m_dev = m_dev;
  for (int i = 0; i < n / seg_n; ++i) g.c[i] = c[i];
  g.ldc = ldc;
  g.seg_n = seg_n;
  g.c32 = c32;
  g.c32_cols = c32 ? c32_cols : 0;
  g.k_parts = 1;
  g.rope = rope_table;
  g.rope_cols = rope_cols;
  g.rope_dh = head_dim;
  g.rope_seq = seq;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = dtype == DARE_BF16 ? launch_gemm_bf16(g, s) : launch_gemm_f32(g, s);
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_rope_table(float* table, int n_pos, int head_dim, double base) {
  if (!table || n_pos < 1 || head_dim < 2 || head_dim % 2 != 0 || !(base > 0.0)) return DARE_ERR_INVALID_ARG;
  const size_t elems = (size_t)n_pos * head_dim;
  float* host = new (std::nothrow) float[elems];
  if (!host) return DARE_ERR_OOM;
  fill_rope_table(host, n_pos, head_dim, base);
  hipError_t e = hipMemcpy(table, host, elems * sizeof(float), hipMemcpyHostToDevice);
  delete[] host;
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_norm(int dtype, int kind, const void* x, const void* gain, const void* bias, float eps,
                        int n_rows, int d, void* out, void* hip_stream) {
  if (!x || !gain || !out || n_rows < 0 || d < 8 || d % 8 != 0 || !(eps >= 0.f)) return DARE_ERR_INVALID_ARG;
  if (dtype != DARE_F32 && dtype != DARE_BF16) return DARE_ERR_INVALID_ARG;
  if (kind != DARE_NORM_LAYER && kind != DARE_NORM_RMS) return DARE_ERR_INVALID_ARG;
  if (kind == DARE_NORM_RMS && bias) return DARE_ERR_INVALID_ARG;
  hipError_t e = launch_norm(dtype, kind, x, gain, bias, eps, n_rows, d, out, 0, 0, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_residual_add(int dtype, const void* x, const void* o, void* out, long n_elems,
                                void* hip_stream) {
  if (!x || !o || !out || n_elems < 0 || n_elems % 8 != 0) return DARE_ERR_INVALID_ARG;
  if (dtype != DARE_F32 && dtype != DARE_BF16) return DARE_ERR_INVALID_ARG;
  hipError_t e = launch_residual_add(dtype, x, o, out, n_elems, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_score(const float* q_new, int ld_new, int width, int n_parts, long part_stride,
                         float* q_prev, int n_tokens, float threshold, int force_refresh,
                         float* scores, uint8_t* mask, void* hip_stream) {
  if (!q_new || !q_prev || !mask || width < 1 || ld_new < width || n_tokens < 0 || std::isnan(threshold))
    return DARE_ERR_INVALID_ARG;
  if (n_parts < 1 || (n_parts > 1 && part_stride < (long)n_tokens * ld_new)) return DARE_ERR_INVALID_ARG;
  hipError_t e = launch_score(q_new, ld_new, width, n_parts, part_stride, q_prev, n_tokens, threshold,
                              force_refresh, scores,
                              nullptr, mask, 1, 0, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_compact(const uint8_t* mask, int batch, int seq, int32_t* sel_idx, int32_t* sel_count,
                           int32_t* sel_off, void* hip_stream) {
  if (!mask || batch < 1 || seq < 1 || batch > 65535) return DARE_ERR_INVALID_ARG;
  hipError_t e = launch_compact(mask, batch, seq, sel_idx, nullptr, sel_count, nullptr, sel_off,
                                static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_attention(int dtype, const void* q, const void* k, const void* v, void* out, int batch,
                             int seq, int n_heads, int head_dim, const int32_t* idx,
                             const int32_t* sel_off, void* hip_stream) {
  if (!q || !k || !v || !out || batch < 1 || seq < 1 || n_heads < 1) return DARE_ERR_INVALID_ARG;
  if (dtype != DARE_F32 && dtype != DARE_BF16) return DARE_ERR_INVALID_ARG;
  if ((idx == nullptr) != (sel_off == nullptr)) return DARE_ERR_INVALID_ARG;
  if (head_dim != 64 && head_dim != 128) return DARE_ERR_UNSUPPORTED;
  if (batch > 65535 || n_heads > 65535) return DARE_ERR_UNSUPPORTED;
  AttnArgs a{};
  a.q = q;
  a.k = k;
  a.v = v;
  a.out = out;
  a.batch = batch;
  a.seq = seq;
  a.n_heads = n_heads;
  a.head_dim = head_dim;
  a.idx = idx;
  a.sel_off = sel_off;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = dtype == DARE_BF16 ? launch_attn_bf16(a, s) : launch_attn_f32(a, s);
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

dare_status dare_k_copy_rows(const void* src, void* dst, int n_rows, int row_bytes, const int32_t* idx,
                             const int32_t* m_dev, void* hip_stream) {
  if (!src || !dst || n_rows < 0 || row_bytes < 16 || row_bytes % 16 != 0) return DARE_ERR_INVALID_ARG;
  hipError_t e = launch_copy_rows(src, dst, n_rows, row_bytes, idx, m_dev, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? DARE_OK : DARE_ERR_HIP;
}

}  // extern "C"
