"""ctypes binding of libdare.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU (torch provides device memory and streams);
every computation happens in the library's HIP kernels.  There is no fallback:
if libdare.so is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libdare.so")

DARE_OK, DARE_ERR_INVALID_ARG, DARE_ERR_UNSUPPORTED, DARE_ERR_OOM, DARE_ERR_HIP = range(5)
DARE_F32, DARE_BF16 = 0, 1
MODE_DENSE, MODE_KV, MODE_O, MODE_KVO = 0, 1, 2, 3
MODE_NAMES = {MODE_DENSE: "dense", MODE_KV: "kv", MODE_O: "o", MODE_KVO: "kvo"}

EXPORTS = (
    "dare_create", "dare_layer_step", "dare_destroy", "dare_last_error", "dare_version",
    "dare_static_init", "dare_layer_step_static",
    "dare_k_pack_weight", "dare_k_gemm", "dare_k_score", "dare_k_compact",
    "dare_k_attention", "dare_k_copy_rows",
    "dare_block_attach", "dare_block_step", "dare_k_gemm_rope", "dare_k_rope_table",
    "dare_k_norm", "dare_k_residual_add",
    "dare_set_threshold_rule", "dare_get_thresholds", "dare_drift_stats_enable", "dare_drift_stats_read",
    "dare_allocate_quantiles", "dare_policy_mode", "dare_k_quantile_mask", "dare_set_prefix",
    "dare_model_create", "dare_model_set_layer", "dare_model_set_io", "dare_model_set_rule",
    "dare_model_set_prefix", "dare_model_step", "dare_model_logits", "dare_model_layer",
    "dare_model_destroy", "dare_model_last_error",
)
RULE_SCORE, RULE_QUANTILE = 0, 1
NORM_NONE, NORM_LAYER, NORM_RMS = 0, 1, 2
NORM_KINDS = {None: NORM_NONE, "layer": NORM_LAYER, "rms": NORM_RMS}


class DareConfig(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("hidden", ctypes.c_int32),
        ("n_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("max_batch", ctypes.c_int32),
        ("max_seq", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("score_head", ctypes.c_int32),
        ("device", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
    ]


class DareBlockConfig(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("norm", ctypes.c_int32),
        ("eps", ctypes.c_float),
        ("rope_base", ctypes.c_float),
        ("residual", ctypes.c_int32),
    ]


class DareModelConfig(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("n_layers", ctypes.c_int32), ("hidden", ctypes.c_int32), ("n_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("ffn", ctypes.c_int32), ("vocab", ctypes.c_int32),
        ("max_batch", ctypes.c_int32), ("max_seq", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("norm_eps", ctypes.c_float),
        ("rope_base", ctypes.c_float),
        ("device", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
    ]


class DareError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("libdare status %d: %s" % (status, text))
        self.status = status


_lib = None


def lib():
    """The loaded library (loaded on first use; raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libdare.so is not built: run `python -m paper_2605_08134_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, f32, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_uint64
    L.dare_create.argtypes = [ctypes.POINTER(DareConfig), vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
    L.dare_create.restype = i32
    L.dare_layer_step.argtypes = [vp, i32, f32, i32, i32] + [vp] * 11
    L.dare_layer_step.restype = i32
    L.dare_static_init.argtypes = [i32]
    L.dare_static_init.restype = i32
    L.dare_layer_step_static.argtypes = [ctypes.POINTER(DareConfig), vp, vp, i32, f32, i32, i32] + [vp] * 11
    L.dare_layer_step_static.restype = i32
    L.dare_destroy.argtypes = [vp]
    L.dare_destroy.restype = i32
    L.dare_last_error.argtypes = [vp]
    L.dare_last_error.restype = ctypes.c_char_p
    L.dare_version.argtypes = []
    L.dare_version.restype = ctypes.c_char_p
    L.dare_k_pack_weight.argtypes = [i32, vp, i32, i32, vp, i32, vp]
    L.dare_k_pack_weight.restype = i32
    L.dare_k_gemm.argtypes = [i32, vp, i32, vp, i32, i32, i32, vp, vp, ctypes.POINTER(vp), i32, i32,
                              vp, i32, i32, ctypes.c_long, vp]
    L.dare_k_gemm.restype = i32
    L.dare_k_score.argtypes = [vp, i32, i32, i32, ctypes.c_long, vp, i32, f32, i32, vp, vp, vp]
    L.dare_k_score.restype = i32
    L.dare_k_compact.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    L.dare_k_compact.restype = i32
    L.dare_k_attention.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
    L.dare_k_attention.restype = i32
    L.dare_k_copy_rows.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    L.dare_k_copy_rows.restype = i32
    L.dare_block_attach.argtypes = [vp, ctypes.POINTER(DareBlockConfig), vp, vp, vp]
    L.dare_block_attach.restype = i32
    L.dare_block_step.argtypes = [vp, i32, f32, i32, i32] + [vp] * 11
    L.dare_block_step.restype = i32
    L.dare_k_gemm_rope.argtypes = [i32, vp, i32, vp, i32, i32, i32, vp, vp, ctypes.POINTER(vp), i32, i32,
                                   vp, i32, vp, i32, i32, i32, vp]
    L.dare_k_gemm_rope.restype = i32
    L.dare_k_rope_table.argtypes = [vp, i32, i32, ctypes.c_double]
    L.dare_k_rope_table.restype = i32
    L.dare_k_norm.argtypes = [i32, i32, vp, vp, vp, f32, i32, i32, vp, vp]
    L.dare_k_norm.restype = i32
    L.dare_k_residual_add.argtypes = [i32, vp, vp, vp, ctypes.c_long, vp]
    L.dare_k_residual_add.restype = i32
    dbl_p = ctypes.POINTER(ctypes.c_double)
    L.dare_set_threshold_rule.argtypes = [vp, i32]
    L.dare_set_threshold_rule.restype = i32
    L.dare_get_thresholds.argtypes = [vp, vp, i32, vp]
    L.dare_get_thresholds.restype = i32
    L.dare_drift_stats_enable.argtypes = [vp, i32, vp]
    L.dare_drift_stats_enable.restype = i32
    L.dare_drift_stats_read.argtypes = [vp, dbl_p, ctypes.POINTER(ctypes.c_int64), vp]
    L.dare_drift_stats_read.restype = i32
    L.dare_allocate_quantiles.argtypes = [i32, dbl_p, ctypes.c_double, ctypes.c_double, dbl_p]
    L.dare_allocate_quantiles.restype = i32
    L.dare_policy_mode.argtypes = [i32] * 5
    L.dare_policy_mode.restype = i32
    L.dare_model_create.argtypes = [ctypes.POINTER(DareModelConfig), vp, ctypes.POINTER(vp)]
    L.dare_model_create.restype = i32
    L.dare_model_set_layer.argtypes = [vp, i32] + [vp] * 10
    L.dare_model_set_layer.restype = i32
    L.dare_model_set_io.argtypes = [vp, vp, vp, vp, vp]
    L.dare_model_set_io.restype = i32
    L.dare_model_set_rule.argtypes = [vp, i32]
    L.dare_model_set_rule.restype = i32
    L.dare_model_set_prefix.argtypes = [vp, i32]
    L.dare_model_set_prefix.restype = i32
    L.dare_model_step.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float), i32, i32,
                                  vp, vp, vp, vp, vp]
    L.dare_model_step.restype = i32
    L.dare_model_logits.argtypes = [vp, vp, vp, i32, vp, vp]
    L.dare_model_logits.restype = i32
    L.dare_model_layer.argtypes = [vp, i32]
    L.dare_model_layer.restype = vp
    L.dare_model_destroy.argtypes = [vp]
    L.dare_model_destroy.restype = i32
    L.dare_model_last_error.argtypes = [vp]
    L.dare_model_last_error.restype = ctypes.c_char_p
    L.dare_set_prefix.argtypes = [vp, i32]
    L.dare_set_prefix.restype = i32
    L.dare_k_quantile_mask.argtypes = [vp, i32, i32, f32, i32, vp, vp, vp, vp, vp]
    L.dare_k_quantile_mask.restype = i32
    _lib = L
    return L


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensor must be contiguous"
    return t.data_ptr()


def _stream(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _torch_dtype(dtype):
    import torch
    return torch.bfloat16 if dtype == DARE_BF16 else torch.float32


def _check(st, ctx=None):
    if st != DARE_OK:
        msg = lib().dare_last_error(ctx)
        raise DareError(st, msg.decode() if msg else "")


def dare_version():
    return lib().dare_version().decode()


STATIC_MAX_ROW_BYTES = 8 << 20      # DARE_STATIC_MAX_ROW_BYTES
STATIC_MAX_SCORE_ELEMS = 1 << 20    # DARE_STATIC_MAX_SCORE_ELEMS


def dare_static_init(device=0):
    _check(lib().dare_static_init(device), None)


def dare_layer_step_static(wqkv_t, wo_t, n_heads, mode, threshold, hidden, q_prev, k_cache, v_cache, o_cache, out,
                           reuse_mask, sel_idx=None, sel_count=None, scores=None, score_head=0, stream=None):
    """dare_layer_step_static: the layer step without a context and without any allocation.
    wqkv_t [3d, d] and wo_t [d, d] are the packed weights (dare_k_pack_weight)."""
    import torch
    batch, seq, d = hidden.shape
    dtype = DARE_BF16 if hidden.dtype == torch.bfloat16 else DARE_F32
    cfg = DareConfig(ctypes.sizeof(DareConfig), d, n_heads, d // n_heads, batch, seq, dtype, score_head,
                     hidden.device.index or 0, 0)
    st = lib().dare_layer_step_static(ctypes.byref(cfg), _ptr(wqkv_t), _ptr(wo_t), mode, threshold, batch, seq,
                                      _ptr(hidden), _ptr(q_prev), _ptr(k_cache), _ptr(v_cache), _ptr(o_cache),
                                      _ptr(out), _ptr(reuse_mask), _ptr(sel_idx), _ptr(sel_count), _ptr(scores),
                                      _stream(stream))
    _check(st, None)


class DareLayer:
    """dare_create / dare_layer_step / dare_destroy for one layer's weights."""

    @classmethod
    def view(cls, ctx_ptr, device):
        """A non-owning handle on a context that something else owns (a model's layer)."""
        self = cls.__new__(cls)
        self._ctx = ctypes.c_void_p(ctx_ptr)
        self.device = device
        self._borrowed = True
        return self

    def __init__(self, wq, wk, wv, wo, n_heads, max_batch, max_seq, score_head=0, stream=None):
        import torch
        d = wq.shape[0]
        dtype = DARE_BF16 if wq.dtype == torch.bfloat16 else DARE_F32
        for w in (wq, wk, wv, wo):
            assert w.is_cuda and w.shape == (d, d) and w.dtype == wq.dtype
        self.cfg = DareConfig(ctypes.sizeof(DareConfig), d, n_heads, d // n_heads, max_batch, max_seq,
                              dtype, score_head, wq.device.index or 0, 0)
        self.dtype = dtype
        self.hidden, self.n_heads, self.head_dim = d, n_heads, d // n_heads
        self.score_width = d if score_head < 0 else self.head_dim
        self.device = wq.device
        self._ctx = ctypes.c_void_p()
        st = lib().dare_create(ctypes.byref(self.cfg), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo),
                               _stream(stream), ctypes.byref(self._ctx))
        _check(st, None)

    def new_state(self, batch, seq):
        """Zeroed caches for dare_layer_step (a DENSE step fills them)."""
        import torch
        td = _torch_dtype(self.dtype)
        z = lambda *s, dt=td: torch.zeros(*s, dtype=dt, device=self.device)
        return {
            "q_prev": z(batch, seq, self.score_width, dt=torch.float32),
            "k_cache": z(batch, seq, self.hidden),
            "v_cache": z(batch, seq, self.hidden),
            "o_cache": z(batch, seq, self.hidden),
        }

    def layer_step(self, mode, threshold, hidden, q_prev, k_cache, v_cache, o_cache, out,
                   reuse_mask, sel_idx=None, sel_count=None, scores=None, stream=None):
        batch, seq, _ = hidden.shape
        st = lib().dare_layer_step(self._ctx, mode, threshold, batch, seq, _ptr(hidden), _ptr(q_prev),
                                   _ptr(k_cache), _ptr(v_cache), _ptr(o_cache), _ptr(out),
                                   _ptr(reuse_mask), _ptr(sel_idx), _ptr(sel_count), _ptr(scores),
                                   _stream(stream))
        _check(st, self._ctx)

    def block_attach(self, norm=None, gain=None, bias=None, eps=1e-5, rope_base=0.0, residual=True,
                     stream=None):
        """dare_block_attach: norm is None, "layer" or "rms"."""
        cfg = DareBlockConfig(ctypes.sizeof(DareBlockConfig), NORM_KINDS[norm], eps, rope_base,
                              int(bool(residual)))
        st = lib().dare_block_attach(self._ctx, ctypes.byref(cfg), _ptr(gain), _ptr(bias), _stream(stream))
        _check(st, self._ctx)

    def block_step(self, mode, threshold, x, q_prev, k_cache, v_cache, o_cache, out,
                   reuse_mask, sel_idx=None, sel_count=None, scores=None, stream=None):
        batch, seq, _ = x.shape
        st = lib().dare_block_step(self._ctx, mode, threshold, batch, seq, _ptr(x), _ptr(q_prev),
                                   _ptr(k_cache), _ptr(v_cache), _ptr(o_cache), _ptr(out),
                                   _ptr(reuse_mask), _ptr(sel_idx), _ptr(sel_count), _ptr(scores),
                                   _stream(stream))
        _check(st, self._ctx)

    def set_prefix(self, prefix_len):
        _check(lib().dare_set_prefix(self._ctx, prefix_len), self._ctx)

    def set_threshold_rule(self, rule):
        _check(lib().dare_set_threshold_rule(self._ctx, rule), self._ctx)

    def thresholds(self, batch, stream=None):
        """The per-sequence thresholds of the last quantile step (float32 tensor [batch])."""
        import torch
        out = torch.empty(batch, dtype=torch.float32, device=self.device)
        _check(lib().dare_get_thresholds(self._ctx, _ptr(out), batch, _stream(stream)), self._ctx)
        return out

    def drift_stats_enable(self, on=True, stream=None):
        _check(lib().dare_drift_stats_enable(self._ctx, int(bool(on)), _stream(stream)), self._ctx)

    def drift_stats_read(self, stream=None):
        mean, count = ctypes.c_double(0.0), ctypes.c_int64(0)
        _check(lib().dare_drift_stats_read(self._ctx, ctypes.byref(mean), ctypes.byref(count),
                                           _stream(stream)), self._ctx)
        return mean.value, count.value

    def destroy(self):
        if self._ctx and not getattr(self, "_borrowed", False):
            lib().dare_destroy(self._ctx)
        self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class DareModel:
    """dare_model_*: a masked-diffusion model of DARE layers.  Weights are torch tensors on
    the GPU; they are copied at the set_* calls."""

    def __init__(self, n_layers, hidden, n_heads, ffn, vocab, max_batch, max_seq, dtype, norm_eps=1e-5,
                 rope_base=10000.0, device=None, stream=None):
        import torch
        self.device = device or torch.device("cuda", torch.cuda.current_device())
        self.dtype = dtype
        self.cfg = DareModelConfig(ctypes.sizeof(DareModelConfig), n_layers, hidden, n_heads, hidden // n_heads,
                                   ffn, vocab, max_batch, max_seq, dtype, norm_eps, rope_base,
                                   self.device.index or 0, 0)
        self._m = ctypes.c_void_p()
        st = lib().dare_model_create(ctypes.byref(self.cfg), _stream(stream), ctypes.byref(self._m))
        self._check(st, created=False)

    def _check(self, st, created=True):
        if st != DARE_OK:
            msg = lib().dare_model_last_error(self._m if created else None)
            raise DareError(st, msg.decode() if msg else "")

    def set_layer(self, layer, attn_gain, wq, wk, wv, wo, ffn_gain, w_gate, w_up, w_down, stream=None):
        self._check(lib().dare_model_set_layer(self._m, layer, _ptr(attn_gain), _ptr(wq), _ptr(wk), _ptr(wv),
                                               _ptr(wo), _ptr(ffn_gain), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                               _stream(stream)))

    def set_io(self, embed, final_gain, head=None, stream=None):
        self._check(lib().dare_model_set_io(self._m, _ptr(embed), _ptr(final_gain), _ptr(head), _stream(stream)))

    def set_rule(self, rule):
        self._check(lib().dare_model_set_rule(self._m, rule))

    def set_prefix(self, prefix_len):
        self._check(lib().dare_model_set_prefix(self._m, prefix_len))

    def step(self, modes, thresholds, ids, hidden_out=None, refreshed=None, trace=None, stream=None):
        L = self.cfg.n_layers
        batch, seq = ids.shape
        if isinstance(modes, int):
            modes = [modes] * L
        if isinstance(thresholds, (int, float)):
            thresholds = [float(thresholds)] * L
        assert len(modes) == L and len(thresholds) == L
        ma = (ctypes.c_int32 * L)(*modes)
        ta = (ctypes.c_float * L)(*thresholds)
        self._check(lib().dare_model_step(self._m, ma, ta, batch, seq, _ptr(ids), _ptr(hidden_out),
                                          _ptr(refreshed), _ptr(trace), _stream(stream)))

    def logits(self, hidden, rows, stream=None):
        import torch
        out = torch.empty((rows.numel(), self.cfg.vocab), dtype=_torch_dtype(self.dtype), device=self.device)
        self._check(lib().dare_model_logits(self._m, _ptr(hidden), _ptr(rows), rows.numel(), _ptr(out),
                                            _stream(stream)))
        return out

    def layer(self, index):
        ptr = lib().dare_model_layer(self._m, index)
        if not ptr:
            raise IndexError("no such layer, or its weights are not set")
        return DareLayer.view(ptr, self.device)

    def destroy(self):
        if self._m:
            lib().dare_model_destroy(self._m)
            self._m = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def dare_allocate_quantiles(s_layers, phi_bar, eps):
    n = len(s_layers)
    src = (ctypes.c_double * n)(*[float(v) for v in s_layers])
    out = (ctypes.c_double * n)()
    _check(lib().dare_allocate_quantiles(n, src, float(phi_bar), float(eps), out))
    return list(out)


def dare_policy_mode(mode, layer, step, skip_layers=0, refresh_interval=0):
    return lib().dare_policy_mode(mode, layer, step, skip_layers, refresh_interval)


# ---- kernel-level entry points ---------------------------------------------------------

def dare_k_pack_weight(w, stream=None):
    import torch
    k, n = w.shape
    wt = torch.empty((n, k), dtype=w.dtype, device=w.device)
    dtype = DARE_BF16 if w.dtype == torch.bfloat16 else DARE_F32
    _check(lib().dare_k_pack_weight(dtype, _ptr(w), k, n, _ptr(wt), k, _stream(stream)))
    return wt


def dare_k_gemm(a, wt, outs, seg_n, idx=None, m_dev=None, m_max=None, c32=None, k_parts=1, stream=None):
    import torch
    n, k = wt.shape
    dtype = DARE_BF16 if a.dtype == torch.bfloat16 else DARE_F32
    arr = (ctypes.c_void_p * 3)(*[_ptr(o) for o in list(outs) + [None] * (3 - len(outs))])
    ldc = next(o for o in outs if o is not None).shape[-1] if any(o is not None for o in outs) else seg_n
    if m_max is None:
        m_max = a.shape[0] if idx is None else idx.shape[0]
    _check(lib().dare_k_gemm(dtype, _ptr(a), a.shape[-1], _ptr(wt), n, k, m_max, _ptr(idx), _ptr(m_dev),
                             arr, ldc, seg_n, _ptr(c32), 0 if c32 is None else c32.shape[-1],
                             k_parts, 0 if c32 is None else m_max * c32.shape[-1], _stream(stream)))


def dare_k_quantile_mask(scores, phi, mask, tau_out=None, force_refresh=False, stat_sum=None,
                         stat_count=None, stream=None):
    batch, seq = scores.shape
    _check(lib().dare_k_quantile_mask(_ptr(scores), batch, seq, phi, int(force_refresh), _ptr(tau_out),
                                      _ptr(mask), _ptr(stat_sum), _ptr(stat_count), _stream(stream)))


def dare_k_gemm_rope(a, wt, outs, seg_n, rope_table, rope_cols, head_dim, seq, idx=None, m_dev=None,
                     m_max=None, c32=None, stream=None):
    import torch
    n, k = wt.shape
    dtype = DARE_BF16 if a.dtype == torch.bfloat16 else DARE_F32
    arr = (ctypes.c_void_p * 3)(*[_ptr(o) for o in list(outs) + [None] * (3 - len(outs))])
    ldc = next(o for o in outs if o is not None).shape[-1]
    if m_max is None:
        m_max = a.shape[0] if idx is None else idx.shape[0]
    _check(lib().dare_k_gemm_rope(dtype, _ptr(a), a.shape[-1], _ptr(wt), n, k, m_max, _ptr(idx),
                                  _ptr(m_dev), arr, ldc, seg_n, _ptr(c32),
                                  0 if c32 is None else c32.shape[-1], _ptr(rope_table), rope_cols,
                                  head_dim, seq, _stream(stream)))


def dare_k_rope_table(n_pos, head_dim, base, device="cuda"):
    import torch
    table = torch.empty((n_pos, head_dim // 2, 2), dtype=torch.float32, device=device)
    _check(lib().dare_k_rope_table(_ptr(table), n_pos, head_dim, float(base)))
    return table


def dare_k_norm(kind, x, gain, bias, eps, out, stream=None):
    import torch
    dtype = DARE_BF16 if x.dtype == torch.bfloat16 else DARE_F32
    d = x.shape[-1]
    _check(lib().dare_k_norm(dtype, NORM_KINDS[kind], _ptr(x), _ptr(gain), _ptr(bias), eps,
                             x.numel() // d, d, _ptr(out), _stream(stream)))


def dare_k_residual_add(x, o, out, stream=None):
    import torch
    dtype = DARE_BF16 if x.dtype == torch.bfloat16 else DARE_F32
    _check(lib().dare_k_residual_add(dtype, _ptr(x), _ptr(o), _ptr(out), x.numel(), _stream(stream)))


def dare_k_score(q_new, q_prev, threshold, force_refresh, scores, mask, n_parts=1, stream=None):
    n_tokens, width = q_prev.shape[0], q_prev.shape[-1]
    _check(lib().dare_k_score(_ptr(q_new), q_new.shape[-1], width, n_parts, n_tokens * q_new.shape[-1],
                              _ptr(q_prev), n_tokens, threshold,
                              int(force_refresh), _ptr(scores), _ptr(mask), _stream(stream)))


def dare_k_compact(mask, batch, seq, sel_idx, sel_count, sel_off, stream=None):
    _check(lib().dare_k_compact(_ptr(mask), batch, seq, _ptr(sel_idx), _ptr(sel_count), _ptr(sel_off),
                                _stream(stream)))


def dare_k_attention(q, k, v, out, batch, seq, n_heads, head_dim, idx=None, sel_off=None, stream=None):
    import torch
    dtype = DARE_BF16 if q.dtype == torch.bfloat16 else DARE_F32
    _check(lib().dare_k_attention(dtype, _ptr(q), _ptr(k), _ptr(v), _ptr(out), batch, seq, n_heads,
                                  head_dim, _ptr(idx), _ptr(sel_off), _stream(stream)))


def dare_k_copy_rows(src, dst, idx=None, m_dev=None, stream=None):
    n_rows = src.shape[0]
    row_bytes = src.shape[-1] * src.element_size()
    _check(lib().dare_k_copy_rows(_ptr(src), _ptr(dst), n_rows, row_bytes, _ptr(idx), _ptr(m_dev),
                                  _stream(stream)))


# ---- benchmark aids (libdare_bench.so, include/dare_bench.h) ------------------------------

BENCH_LIB_PATH = os.path.join(PKG_DIR, "libdare_bench.so")
BENCH_EXPORTS = ("dare_bench_mfma_loop", "dare_bench_stream")
_bench_lib = None


def bench_lib():
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(BENCH_LIB_PATH):
            raise RuntimeError("libdare_bench.so is not built: run `python -m paper_2605_08134_amd.build`")
        L = ctypes.CDLL(BENCH_LIB_PATH)
        L.dare_bench_mfma_loop.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p, ctypes.POINTER(ctypes.c_double),
                                                                ctypes.c_void_p]
        L.dare_bench_mfma_loop.restype = ctypes.c_int
        L.dare_bench_stream.argtypes = [ctypes.c_int, ctypes.c_ulonglong, ctypes.c_int, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p]
        L.dare_bench_stream.restype = ctypes.c_int
        _bench_lib = L
    return _bench_lib


def dare_bench_stream(n_blocks, bytes_per_block, depth, src, stream=None):
    """Enqueue the one-workgroup-per-CU stream over src (a device tensor of at least
    n_blocks * bytes_per_block bytes)."""
    if src.numel() * src.element_size() < n_blocks * bytes_per_block:
        raise ValueError("source buffer too small")
    st = bench_lib().dare_bench_stream(n_blocks, bytes_per_block, depth, _ptr(src), None, _stream(stream))
    if st != 0:
        raise DareError(st, "dare_bench_stream failed")


def dare_bench_mfma_loop(n_blocks, n_iter, pattern, stream=None):
    """Enqueue the register-resident MFMA loop; returns the flop count of the launch."""
    flops = ctypes.c_double(0.0)
    st = bench_lib().dare_bench_mfma_loop(n_blocks, n_iter, pattern, None, ctypes.byref(flops), _stream(stream))
    if st != 0:
        raise DareError(st, "dare_bench_mfma_loop failed")
    return flops.value
