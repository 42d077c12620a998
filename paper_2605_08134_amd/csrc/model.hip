// A masked-diffusion language model made of DARE layers: host-side runtime (buffers,
// per-layer contexts, the launch sequence of one denoising step) plus the two small
// kernels the model adds to the layer's: row gather (token embedding, rows for the
// output embedding) and the SwiGLU gate of the fp32 path (the bf16 path applies it in the
// epilogue of the gate/up projection).  The attention of every layer is the core of
// dare_block_step, with its normalisation and residual sum fused into the model's own
// residual + norm passes; the feed-forward uses the projection kernels of the layer.
#include <cmath>
#include <new>
#include <string>
#include <vector>

#include "dare_common.h"
#include "dare_model.h"

using namespace dare;

namespace dare {
namespace {

// dst[r] = src[ids[r]] (rows of row_vec 16-byte units); ids outside [0, n_src) give zeros.
__global__ void __launch_bounds__(256) gather_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         const int32_t* __restrict__ ids, int n_rows, int n_src,
                                                         int row_vec) {
  for (int r = blockIdx.x; r < n_rows; r += gridDim.x) {
    const int id = ids[r];
    const bool ok = id >= 0 && id < n_src;
    const uint4* s = src + (long)(ok ? id : 0) * row_vec;
    uint4* d = dst + (long)r * row_vec;
    for (int c = threadIdx.x; c < row_vec; c += 256) {
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (ok) v = s[c];
      d[c] = v;
    }
  }
}

// gate[t, :] <- silu(gate[t, :]) * up[t, :] for the listed (or all) rows, 8 elements per
// thread and step, fp32 arithmetic.
template <typename T>
__global__ void __launch_bounds__(256) swiglu_kernel(T* __restrict__ gate, const T* __restrict__ up, int n_rows,
                                                     int width, const int32_t* __restrict__ idx) {
  const int groups = width >> 3;
  for (int r = blockIdx.x; r < n_rows; r += gridDim.x) {
    const long tok = idx ? (long)idx[r] : (long)r;
    T* g = gate + tok * width;
    const T* u = up + tok * width;
    for (int c = threadIdx.x; c < groups; c += 256) {
      float a[8], b[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        a[e] = (float)g[c * 8 + e];
        b[e] = (float)u[c * 8 + e];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = a[e] / (1.0f + expf(-a[e])) * b[e];
#pragma unroll
      for (int e = 0; e < 8; ++e) g[c * 8 + e] = (T)a[e];
    }
  }
}

}  // namespace

hipError_t launch_gather_rows(const void* src, void* dst, const int32_t* ids, int n_rows, int n_src,
                              int row_bytes, hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(n_rows < 8192 ? n_rows : 8192), dim3(256), 0, s,
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), ids, n_rows, n_src, row_bytes / 16);
  return hipGetLastError();
}

hipError_t launch_swiglu(int dtype, void* gate, const void* up, int n_rows, int width, const int32_t* idx,
                         hipStream_t s) {
  if (n_rows == 0) return hipSuccess;
  const int grid = n_rows < 8192 ? n_rows : 8192;
  if (dtype == DARE_BF16)
    hipLaunchKernelGGL(swiglu_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, static_cast<bf16_t*>(gate),
                       static_cast<const bf16_t*>(up), n_rows, width, idx);
  else
    hipLaunchKernelGGL(swiglu_kernel<float>, dim3(grid), dim3(256), 0, s, static_cast<float*>(gate),
                       static_cast<const float*>(up), n_rows, width, idx);
  return hipGetLastError();
}

}  // namespace dare

struct dare_model {
  dare_model_config cfg;
  size_t esize;
  std::vector<dare_ctx*> layers;
  struct LayerMem {
    void* attn_gain;  // gains of the two normalisations (the fused residual + norm kernels read them)
    void* ffn_gain;
    void* w_gu_t;     // [2 ffn, hidden] packed gate | up
    void* w_down_t;   // [hidden, ffn] packed
    float* q_prev;
    void* k_cache;
    void* v_cache;
    void* o_cache;
  };
  std::vector<LayerMem> mem;
  void* embed;        // [vocab, hidden]
  void* final_gain;
  void* head_t;       // [vocab, hidden] packed output embedding, or nullptr
  void* x;            // [max tokens, hidden] residual stream
  void* h1;           // normalised rows feeding the attention block
  void* h2;           // normalised rows feeding the feed-forward
  void* gate;         // [max tokens, ffn]
  void* up;
  void* f;            // [max tokens, hidden] feed-forward output
  void* rows_buf;     // [max tokens, hidden] gathered rows for the output embedding
  uint8_t* mask;      // [max tokens] reuse mask of the layer being run
  int32_t* act_idx;   // frozen prefix: rows that are not frozen
  int32_t* act_off;
  int rule, prefix;
  std::vector<void*> owned;
  std::string err;
};

namespace {

thread_local std::string g_model_create_err;

dare_status mfail(dare_model* m, dare_status st, const std::string& what) {
  if (m) m->err = what; else g_model_create_err = what;
  return st;
}
dare_status mfail_hip(dare_model* m, hipError_t e, const char* where) {
  return mfail(m, e == hipErrorOutOfMemory ? DARE_ERR_OOM : DARE_ERR_HIP, std::string(where) + ": " + hipGetErrorString(e));
}

struct Dev {
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
  ~Dev() {
    if (changed) (void)hipSetDevice(prev);
  }
};

hipError_t alloc(dare_model* m, void** p, size_t bytes, bool zero) {
  *p = nullptr;
  hipError_t e = hipMalloc(p, bytes ? bytes : 16);
  if (e != hipSuccess) {
    *p = nullptr;
    return e;
  }
  m->owned.push_back(*p);
  return zero ? hipMemset(*p, 0, bytes) : hipSuccess;
}

void free_model(dare_model* m) {
  if (!m) return;
  for (dare_ctx* c : m->layers)
    if (c) dare_destroy(c);
  for (void* p : m->owned) (void)hipFree(p);
  delete m;
}

}  // namespace

extern "C" {

const char* dare_model_last_error(const dare_model* m) { return m ? m->err.c_str() : g_model_create_err.c_str(); }

dare_status dare_model_create(const dare_model_config* cfg, void* hip_stream, dare_model** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return mfail(nullptr, DARE_ERR_INVALID_ARG, "null config or out");
  if (cfg->struct_size != sizeof(dare_model_config))
    return mfail(nullptr, DARE_ERR_INVALID_ARG, "struct_size does not match this library");
  if (cfg->flags != 0 || (cfg->dtype != DARE_F32 && cfg->dtype != DARE_BF16))
    return mfail(nullptr, DARE_ERR_INVALID_ARG, "bad flags or dtype");
  if (cfg->n_layers < 1 || cfg->hidden < 1 || cfg->n_heads < 1 || cfg->head_dim < 1 || cfg->ffn < 1 ||
      cfg->vocab < 1 || cfg->max_batch < 1 || cfg->max_seq < 1 || cfg->device < 0)
    return mfail(nullptr, DARE_ERR_INVALID_ARG, "non-positive size");
  if ((long)cfg->n_heads * cfg->head_dim != cfg->hidden)
    return mfail(nullptr, DARE_ERR_INVALID_ARG, "hidden != n_heads * head_dim");
  if (cfg->hidden % 64 || cfg->ffn % 64 || cfg->vocab % 64)
    return mfail(nullptr, DARE_ERR_UNSUPPORTED, "hidden, ffn and vocab must be multiples of 64");
  if (cfg->head_dim != 64 && cfg->head_dim != 128)
    return mfail(nullptr, DARE_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
  if (!(cfg->norm_eps >= 0.f) || !(cfg->rope_base >= 0.f) || std::isinf(cfg->rope_base))
    return mfail(nullptr, DARE_ERR_INVALID_ARG, "bad norm_eps or rope_base");
  const long max_tok = (long)cfg->max_batch * cfg->max_seq;
  if (max_tok > (1l << 30) / 2) return mfail(nullptr, DARE_ERR_UNSUPPORTED, "max_batch * max_seq too large");

  Dev guard;
  hipError_t e = guard.enter(cfg->device);
  if (e != hipSuccess) return mfail_hip(nullptr, e, "hipSetDevice");
  dare_model* m = new (std::nothrow) dare_model();
  if (!m) return mfail(nullptr, DARE_ERR_OOM, "host allocation failed");
  m->cfg = *cfg;
  m->esize = cfg->dtype == DARE_BF16 ? 2 : 4;
  m->layers.assign(cfg->n_layers, nullptr);
  m->mem.assign(cfg->n_layers, dare_model::LayerMem{});
  m->embed = m->final_gain = m->head_t = nullptr;
  m->rule = DARE_RULE_SCORE;
  m->prefix = 0;
  const size_t d = cfg->hidden, es = m->esize, tok = (size_t)max_tok;
  struct { void** p; size_t bytes; bool zero; } bufs[] = {
      {&m->x, tok * d * es, false},          {&m->h2, tok * d * es, false},
      {&m->h1, tok * d * es, false},
      {&m->gate, tok * cfg->ffn * es, false}, {&m->up, tok * cfg->ffn * es, false},
      {&m->f, tok * d * es, false},          {&m->rows_buf, tok * d * es, false},
      {(void**)&m->mask, tok, false},        {(void**)&m->act_idx, tok * sizeof(int32_t), false},
      {(void**)&m->act_off, ((size_t)cfg->max_batch + 1) * sizeof(int32_t), false},
      {&m->embed, (size_t)cfg->vocab * d * es, false}, {&m->final_gain, d * es, false},
  };
  for (auto& b : bufs)
    if ((e = alloc(m, b.p, b.bytes, b.zero)) != hipSuccess) {
      dare_status st = mfail_hip(nullptr, e, "hipMalloc");
      free_model(m);
      return st;
    }
  for (int l = 0; l < cfg->n_layers; ++l) {
    dare_model::LayerMem& lm = m->mem[l];
    struct { void** p; size_t bytes; bool zero; } lb[] = {
        {&lm.attn_gain, d * es, false},
        {&lm.ffn_gain, d * es, false},
        {&lm.w_gu_t, 2 * (size_t)cfg->ffn * d * es, false},
        {&lm.w_down_t, (size_t)cfg->ffn * d * es, false},
        {(void**)&lm.q_prev, tok * cfg->head_dim * sizeof(float), true},
        {&lm.k_cache, tok * d * es, true},
        {&lm.v_cache, tok * d * es, true},
        {&lm.o_cache, tok * d * es, true},
    };
    for (auto& b : lb)
      if ((e = alloc(m, b.p, b.bytes, b.zero)) != hipSuccess) {
        dare_status st = mfail_hip(nullptr, e, "hipMalloc");
        free_model(m);
        return st;
      }
  }
  if ((e = hipStreamSynchronize(static_cast<hipStream_t>(hip_stream))) != hipSuccess) {
    dare_status st = mfail_hip(nullptr, e, "hipStreamSynchronize");
    free_model(m);
    return st;
  }
  *out = m;
  return DARE_OK;
}

dare_status dare_model_destroy(dare_model* m) {
  if (!m) return DARE_OK;
  Dev guard;
  (void)guard.enter(m->cfg.device);
  free_model(m);
  return DARE_OK;
}

dare_status dare_model_set_layer(dare_model* m, int layer, const void* attn_gain, const void* wq, const void* wk,
                                 const void* wv, const void* wo, const void* ffn_gain, const void* w_gate,
                                 const void* w_up, const void* w_down, void* hip_stream) {
  if (!m) return DARE_ERR_INVALID_ARG;
  if (layer < 0 || layer >= m->cfg.n_layers) return mfail(m, DARE_ERR_INVALID_ARG, "layer out of range");
  if (!attn_gain || !wq || !wk || !wv || !wo || !ffn_gain || !w_gate || !w_up || !w_down)
    return mfail(m, DARE_ERR_INVALID_ARG, "null weight pointer");
  Dev guard;
  hipError_t e = guard.enter(m->cfg.device);
  if (e != hipSuccess) return mfail_hip(m, e, "hipSetDevice");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const dare_model_config& c = m->cfg;
  dare_model::LayerMem& lm = m->mem[layer];
  if (m->layers[layer]) {
    dare_destroy(m->layers[layer]);
    m->layers[layer] = nullptr;
  }
  dare_config lc{};
  lc.struct_size = sizeof(dare_config);
  lc.hidden = c.hidden;
  lc.n_heads = c.n_heads;
  lc.head_dim = c.head_dim;
  lc.max_batch = c.max_batch;
  lc.max_seq = c.max_seq;
  lc.dtype = c.dtype;
  lc.score_head = 0;
  lc.device = c.device;
  dare_ctx* ctx = nullptr;
  dare_status st = dare_create(&lc, wq, wk, wv, wo, hip_stream, &ctx);
  if (st != DARE_OK) return mfail(m, st, std::string("layer context: ") + dare_last_error(nullptr));
  m->layers[layer] = ctx;
  dare_block_config bc{};
  bc.struct_size = sizeof(dare_block_config);
  bc.norm = DARE_NORM_RMS;
  bc.eps = c.norm_eps;
  bc.rope_base = c.rope_base;
  bc.residual = 1;
  if ((st = dare_block_attach(ctx, &bc, attn_gain, nullptr, hip_stream)) != DARE_OK)
    return mfail(m, st, std::string("block attach: ") + dare_last_error(ctx));
  if ((st = dare_set_threshold_rule(ctx, m->rule)) != DARE_OK || (st = dare_set_prefix(ctx, m->prefix)) != DARE_OK)
    return mfail(m, st, std::string("layer settings: ") + dare_last_error(ctx));
  const size_t es = m->esize, d = c.hidden, ff = c.ffn;
  e = hipMemcpyAsync(lm.ffn_gain, ffn_gain, d * es, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(lm.attn_gain, attn_gain, d * es, hipMemcpyDeviceToDevice, s);
  if (c.dtype == DARE_BF16) {
    // gate and up rows interleaved (gate_0, up_0, gate_1, ...): the projection's epilogue
    // then holds each (gate, up) pair in one lane and applies the SwiGLU gate itself
    if (e == hipSuccess) e = launch_pack_weight(c.dtype, w_gate, c.hidden, c.ffn, lm.w_gu_t, 2 * c.hidden, s);
    if (e == hipSuccess)
      e = launch_pack_weight(c.dtype, w_up, c.hidden, c.ffn, static_cast<char*>(lm.w_gu_t) + d * es, 2 * c.hidden, s);
  } else {
    if (e == hipSuccess) e = launch_pack_weight(c.dtype, w_gate, c.hidden, c.ffn, lm.w_gu_t, c.hidden, s);
    if (e == hipSuccess)
      e = launch_pack_weight(c.dtype, w_up, c.hidden, c.ffn, static_cast<char*>(lm.w_gu_t) + ff * d * es, c.hidden, s);
  }
  if (e == hipSuccess) e = launch_pack_weight(c.dtype, w_down, c.ffn, c.hidden, lm.w_down_t, c.ffn, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return mfail_hip(m, e, "feed-forward weights");
  return DARE_OK;
}

dare_status dare_model_set_io(dare_model* m, const void* embed, const void* final_gain, const void* head,
                              void* hip_stream) {
  if (!m) return DARE_ERR_INVALID_ARG;
  if (!embed || !final_gain) return mfail(m, DARE_ERR_INVALID_ARG, "null embedding or gain");
  Dev guard;
  hipError_t e = guard.enter(m->cfg.device);
  if (e != hipSuccess) return mfail_hip(m, e, "hipSetDevice");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const dare_model_config& c = m->cfg;
  const size_t es = m->esize, d = c.hidden;
  e = hipMemcpyAsync(m->embed, embed, (size_t)c.vocab * d * es, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess) e = hipMemcpyAsync(m->final_gain, final_gain, d * es, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && head) {
    if (!m->head_t) e = alloc(m, &m->head_t, (size_t)c.vocab * d * es, false);
    if (e == hipSuccess) e = launch_pack_weight(c.dtype, head, c.hidden, c.vocab, m->head_t, c.hidden, s);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return mfail_hip(m, e, "embedding / output weights");
  return DARE_OK;
}

dare_status dare_model_set_rule(dare_model* m, int rule) {
  if (!m) return DARE_ERR_INVALID_ARG;
  if (rule != DARE_RULE_SCORE && rule != DARE_RULE_QUANTILE) return mfail(m, DARE_ERR_INVALID_ARG, "unknown rule");
  for (dare_ctx* c : m->layers)
    if (c) {
      dare_status st = dare_set_threshold_rule(c, rule);
      if (st != DARE_OK) return mfail(m, st, dare_last_error(c));
    }
  m->rule = rule;
  return DARE_OK;
}

dare_status dare_model_set_prefix(dare_model* m, int prefix_len) {
  if (!m) return DARE_ERR_INVALID_ARG;
  if (prefix_len < 0 || prefix_len >= m->cfg.max_seq)
    return mfail(m, DARE_ERR_INVALID_ARG, "prefix_len must lie in [0, max_seq)");
  for (dare_ctx* c : m->layers)
    if (c) {
      dare_status st = dare_set_prefix(c, prefix_len);
      if (st != DARE_OK) return mfail(m, st, dare_last_error(c));
    }
  m->prefix = prefix_len;
  return DARE_OK;
}

dare_ctx* dare_model_layer(dare_model* m, int layer) {
  return (m && layer >= 0 && layer < m->cfg.n_layers) ? m->layers[layer] : nullptr;
}

dare_status dare_model_step(dare_model* m, const int32_t* modes, const float* thresholds, int batch, int seq,
                            const int32_t* ids, void* hidden_out, int32_t* refreshed, void* trace,
                            void* hip_stream) {
  if (!m) return DARE_ERR_INVALID_ARG;
  if (!modes || !thresholds || !ids) return mfail(m, DARE_ERR_INVALID_ARG, "null required pointer");
  const dare_model_config& c = m->cfg;
  if (batch < 1 || seq < 1 || batch > c.max_batch || seq > c.max_seq)
    return mfail(m, DARE_ERR_INVALID_ARG, "batch or seq out of range");
  if (m->prefix >= seq) return mfail(m, DARE_ERR_INVALID_ARG, "the frozen prefix covers the whole sequence");
  for (int l = 0; l < c.n_layers; ++l)
    if (!m->layers[l]) return mfail(m, DARE_ERR_INVALID_ARG, "a layer has no weights yet");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int n_tok = batch * seq, d = c.hidden, ff = c.ffn, P = m->prefix;
  const size_t es = m->esize, act_bytes = (size_t)n_tok * d * es;
  const bool pre = P > 0;
  const int n_act = batch * (seq - P);
  hipError_t e;
  if (pre && (e = launch_active_list(batch, seq, P, m->act_idx, m->act_off, s)) != hipSuccess)
    return mfail_hip(m, e, "active-row list");
  const int32_t* act = pre ? m->act_idx : nullptr;
  char* tr = static_cast<char*>(trace);
  auto snapshot = [&](int slot) -> hipError_t {
    return tr ? hipMemcpyAsync(tr + (size_t)slot * act_bytes, m->x, act_bytes, hipMemcpyDeviceToDevice, s) : hipSuccess;
  };

  if ((e = launch_gather_rows(m->embed, m->x, ids, n_tok, c.vocab, (int)(d * es), s)) != hipSuccess)
    return mfail_hip(m, e, "embedding");
  // Every residual sum is fused with the normalisation that follows it (one pass over the
  // stream instead of two): x <- x + O, n = rmsnorm(x) before the feed-forward; x <- x + F,
  // h = rmsnorm(x) before the next layer's attention.  Only the first normalisation and the
  // last sum stand alone.
  e = launch_norm(c.dtype, DARE_NORM_RMS, m->x, m->mem[0].attn_gain, nullptr, c.norm_eps, n_act, d, m->h1,
                  pre ? seq : 0, P, s);
  if (e != hipSuccess) return mfail_hip(m, e, "first norm");
  for (int l = 0; l < c.n_layers; ++l) {
    dare_model::LayerMem& lm = m->mem[l];
    if ((e = snapshot(2 * l)) != hipSuccess) return mfail_hip(m, e, "trace");
    // attention block on the normalised rows; its output O goes to the layer's output cache
    dare_status st = block_core(m->layers[l], modes[l], thresholds[l], batch, seq, m->h1, lm.q_prev, lm.k_cache,
                                lm.v_cache, lm.o_cache, m->mask, refreshed ? refreshed + (size_t)l * batch : nullptr,
                                hip_stream);
    if (st != DARE_OK) return mfail(m, st, "layer " + std::to_string(l) + ": " + dare_last_error(m->layers[l]));
    // x <- x + O for every row (frozen rows add their cached O), n = rmsnorm(x)
    e = launch_residual_norm(c.dtype, m->x, lm.o_cache, lm.ffn_gain, c.norm_eps, n_tok, d, m->h2, 0, 0, s);
    if (e != hipSuccess) return mfail_hip(m, e, "attention residual + feed-forward norm");
    if ((e = snapshot(2 * l + 1)) != hipSuccess) return mfail_hip(m, e, "trace");
    // feed-forward on the rows that are not frozen: F = (silu(n Wg) * (n Wu)) Wd
    GemmArgs g{};
    g.a = m->h2;
    g.lda = d;
    g.wt = lm.w_gu_t;
    g.n = 2 * ff;
    g.k = d;
    g.m_max = n_act;
    g.idx = act;
    g.c[0] = m->gate;
    g.ldc = ff;
    g.k_parts = 1;
    if (c.dtype == DARE_BF16) {
      g.seg_n = 2 * ff;
      g.swiglu_pairs = 1;  // silu(gate) * up leaves the epilogue; gate and up are never stored
      e = launch_gemm_bf16(g, s);
    } else {
      g.c[1] = m->up;
      g.seg_n = ff;
      e = launch_gemm_f32(g, s);
      if (e == hipSuccess) e = launch_swiglu(c.dtype, m->gate, m->up, n_act, ff, act, s);
    }
    if (e != hipSuccess) return mfail_hip(m, e, "gate / up projection");
    GemmArgs h{};
    h.a = m->gate;
    h.lda = ff;
    h.wt = lm.w_down_t;
    h.n = d;
    h.k = ff;
    h.m_max = n_act;
    h.idx = act;
    h.c[0] = m->f;
    h.ldc = d;
    h.seg_n = d;
    h.k_parts = 1;
    e = c.dtype == DARE_BF16 ? launch_gemm_bf16(h, s) : launch_gemm_f32(h, s);
    if (e != hipSuccess) return mfail_hip(m, e, "down projection");
    if (l + 1 < c.n_layers) {
      // x <- x + F on the rows that are not frozen, h = rmsnorm(x) for the next layer
      e = launch_residual_norm(c.dtype, m->x, m->f, m->mem[l + 1].attn_gain, c.norm_eps, n_act, d, m->h1,
                               pre ? seq : 0, P, s);
    } else if (pre) {
      e = launch_residual_rows(c.dtype, m->x, m->f, n_act, d, act, s);
    } else {
      e = launch_residual_add(c.dtype, m->x, m->f, m->x, (long)n_tok * d, s);
    }
    if (e != hipSuccess) return mfail_hip(m, e, "feed-forward residual");
  }
  if ((e = snapshot(2 * c.n_layers)) != hipSuccess) return mfail_hip(m, e, "trace");
  if (hidden_out) {
    e = launch_norm(c.dtype, DARE_NORM_RMS, m->x, m->final_gain, nullptr, c.norm_eps, n_tok, d, hidden_out, 0, 0, s);
    if (e != hipSuccess) return mfail_hip(m, e, "final norm");
  }
  return DARE_OK;
}

dare_status dare_model_logits(dare_model* m, const void* hidden, const int32_t* rows, int n_rows, void* logits,
                              void* hip_stream) {
  if (!m) return DARE_ERR_INVALID_ARG;
  if (!hidden || !rows || !logits || n_rows < 0) return mfail(m, DARE_ERR_INVALID_ARG, "null pointer or negative count");
  if (!m->head_t) return mfail(m, DARE_ERR_INVALID_ARG, "the model has no output embedding");
  const dare_model_config& c = m->cfg;
  const long max_tok = (long)c.max_batch * c.max_seq;
  if (n_rows > max_tok) return mfail(m, DARE_ERR_INVALID_ARG, "more rows than max_batch * max_seq");
  if (n_rows == 0) return DARE_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = launch_gather_rows(hidden, m->rows_buf, rows, n_rows, (int)max_tok, (int)(c.hidden * m->esize), s);
  if (e != hipSuccess) return mfail_hip(m, e, "row gather");
  GemmArgs g{};
  g.a = m->rows_buf;
  g.lda = c.hidden;
  g.wt = m->head_t;
  g.n = c.vocab;
  g.k = c.hidden;
  g.m_max = n_rows;
  g.c[0] = logits;
  g.ldc = c.vocab;
  g.seg_n = c.vocab;
  g.k_parts = 1;
  e = c.dtype == DARE_BF16 ? launch_gemm_bf16(g, s) : launch_gemm_f32(g, s);
  if (e != hipSuccess) return mfail_hip(m, e, "output embedding");
  return DARE_OK;
}

}  // extern "C"
