"""CPU oracle for one DARE attention-layer step.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain reference that the parity tests, the smoke test
and the benchmark's ``cpu_baseline`` leg compare the HIP library against.  The
product path never imports it, and it imports nothing from the product.

Everything is numpy in float64.  Inputs may arrive in any float dtype and are
widened exactly.  Nothing here is blocked, fused or reordered: each function
is the paper's definition or the paper's algorithm written out step by step.

What the layer computes (paper Sec. 3, Alg. 1 "DARE-KV", Alg. 2 "DARE-O",
App. E.1/E.2):

  dense       Q = X Wq, K = X Wk, V = X Wv, per head softmax(Q K^T / sqrt(Dh)) V,
              concatenated heads times Wo                          (App. E.2)
  drift score s_i = 1 - <q_i, p_i> / (|q_i| |p_i|), q_i = head 0 of the query of
              token i at this step, p_i = the same at the previous step
                                                    (Sec. 3.1 eq. 1, Sec. 3.2)
  reuse set   R = {i : s_i <= tau}, refreshed set = complement   (Sec. 3.2 eq. 2)
  DARE-KV     K, V rows of the refreshed set are recomputed, rows of R keep the
              cached values; attention and Wo over all rows             (Alg. 1)
  DARE-O      K, V dense; attention (and, since the cache holds the layer
              output, Wo) only for the refreshed rows, rows of R return the
              cached output                        (Alg. 2, App. E.1 second form)
  both        hybrid K/V cache and refreshed-row-only attention at once.

Readings taken where the paper is silent or has two forms:
  * weights are [d_in, d_out], Y = X W                   (Sec. 3.2 eq. 3, App. E.1)
  * softmax scale is 1/sqrt(head_dim) per head (App. E writes the one-head form)
  * the score uses the cosine form of Sec. 3.1 on head 0 = output columns
    [0, head_dim) of Wq; score_head = -1 scores the whole query vector
  * the previous query is the previous *step's* query: it is replaced for
    every token at every step, whatever the mode
  * the output cache holds rows *after* Wo (App. E.1); ``step_o_prewo`` below is
    the literal Alg. 2 (cache before Wo) and is used only to test that both
    readings are the same function
  * the threshold test is taken on the score rounded to float32 against the
    float32 threshold (the precision the kernels decide in); NaN scores refresh
  * a zero-norm query gives cosine 0 (denominator floored at 1e-30)
  * a dense or DARE-O step writes the dense K, V into the K/V caches, so a later
    DARE-KV step starts from valid rows
  * index lists are ascending flat token ids b*T + i.
  * the block around the layer (``block_step``).  Alg. 1/2 line 1 normalises the
    hidden state before the projections: ``layer_norm`` is that line; ``rms_norm`` is
    the variant LLaDA-class models use in its place.  The paper says nothing about
    position encoding or the residual connection; for a model that has them the
    reading is: rotary embedding (pairs of neighbouring channels (2i, 2i+1) of each
    head, angle = position * base^(-2i/head_dim)) on the queries and on the keys as
    they are projected, so the K cache holds rotated keys and a reused row keeps the
    rotation of its own position; the drift score is taken on the query BEFORE the
    rotation (the rotation of a token is the same at both steps, so the cosine is
    the same up to rounding); the output cache holds the attention block's output
    before the residual sum, and ``out = x + O`` is formed for every row from the
    current hidden state.
  * thresholds from reuse rates (Sec. 3.1, "Reuse rate allocation").  The threshold of a
    layer is "the drift score corresponding to the phi-quantile": read as the order
    statistic s_(k), k = ceil(phi * T), of the T scores of one sequence at the current
    step (per sequence, so sequences stay independent; "reuse rates are computed
    dynamically at runtime", Sec. 5).  With the rule s <= tau this reuses the k tokens
    of smallest drift (and whatever ties with the k-th).  phi = 0 gives tau = -inf
    (nothing reused).  NaN scores sort last and are never reused: a NaN order
    statistic is replaced by +inf.  k = ceil(phi * T) with the product formed in
    float32 (phi and T as float32 numbers, one rounding), so that a rate such as 0.3,
    which is not a binary fraction, times 40 tokens gives 12 and not 13.  ``allocate_quantiles`` is the layer-wise formula
    phi_l = L phi_bar softmax(-s_l / eps) with s_l the mean drift of layer l over tokens
    and steps (Sec. 3.1 eq. 2 of that paragraph); values above 1 are cut to 1 (a
    quantile cannot exceed 1; the paper does not say).  ``policy_mode`` is the
    host-side schedule of Sec. 5 (Fast-dLLM-v2 setting): the first layers are not
    reused at all and every r-th step recomputes everything.
  * frozen prefix (``prefix=P``).  The paper composes DARE with prefix caching (Sec. 1,
    Sec. 5 "P+C") without defining it; the reading taken is the usual one for
    diffusion LLMs: the first P tokens of every sequence (the prompt) are frozen: they
    are never projected, scored or queried, their K, V and output rows stay what the
    caches hold, and the other tokens attend to them through the K/V caches.  In the
    terms of this file a frozen token is a token that is always reused, in every mode,
    DENSE included (there "all rows" means all rows that are not frozen); its score is
    reported as 0, its mask bit as 1, and its score-cache row is left as it was.  A
    quantile threshold ranks the scores of the tokens that are not frozen only.
  * precision.  The paper runs in BF16 (Sec. 5, App. A): the tensors its
    algorithms name -- Q, K, V, the attention rows before Wo, the layer output --
    are bf16 tensors, with wide accumulation inside each product.  ``storage=None``
    (default) keeps everything in float64: that is the mathematical definition and
    what the fp32 path is checked against.  ``storage="bf16"`` rounds Q, K, V and
    the attention rows to bf16 (one rounding from float64, ties to even) at the
    point the algorithm produces them; all arithmetic stays float64.  The drift
    score is always taken from the unrounded query.  In that mode the returned
    "out", "k_cache", "v_cache" are what the next step reads (rounded), and
    "exact" holds the same tensors before their final rounding, which is what a
    bf16 result is compared with (it may differ by half a bf16 ulp plus the
    propagated error; comparing rounded with rounded would turn a harmless
    last-bit flip into a whole ulp).

Parity pinning: every function here is pinned by tests/test_oracle_pins.py
(brute force in Python loops, closed forms, invariants).  The paper prints no
worked numeric example, so there is no golden fixture from the paper.
"""
from __future__ import annotations

import numpy as np

MODE_DENSE = 0
MODE_KV = 1
MODE_O = 2
MODE_KVO = 3

_DENOM_FLOOR = 1e-30


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def round_storage(a, storage):
    """Round float64 values to the storage format: None = keep, "bf16" = nearest
    bfloat16 (8 significant bits, ties to even), in one rounding."""
    a = _f64(a)
    if storage is None:
        return a
    if storage != "bf16":
        raise ValueError("storage must be None or 'bf16'")
    u = np.ascontiguousarray(a).view(np.uint64)
    drop = np.uint64(45)                      # 52 - 7 explicit significand bits
    half = (np.uint64(1) << np.uint64(44)) - np.uint64(1)
    odd = (u >> drop) & np.uint64(1)
    r = ((u + half + odd) >> drop) << drop
    return r.view(np.float64).reshape(a.shape)


def drift_scores(q, p):
    """Sec. 3.1 eq. 1: s = 1 - cos(q, p), row by row.  q, p: [..., n]."""
    q = _f64(q)
    p = _f64(p)
    dot = np.sum(q * p, axis=-1)
    nq = np.sum(q * q, axis=-1)
    npp = np.sum(p * p, axis=-1)
    den = np.maximum(np.sqrt(nq * npp), _DENOM_FLOOR)
    return 1.0 - dot / den


def reuse_decision(scores, tau):
    """Sec. 3.2 eq. 2: reuse iff s <= tau, decided in float32.  NaN -> refresh."""
    s32 = np.asarray(scores, dtype=np.float64).astype(np.float32)
    t32 = np.float32(tau)
    with np.errstate(invalid="ignore"):
        return s32 <= t32


def quantile_threshold(scores, phi):
    """Sec. 3.1: per sequence, the drift score at the phi-quantile = the k-th smallest
    of the T scores, k = ceil(phi * T).  scores [B, T] (pass only the columns that take
    part in the ranking); returns float32 tau [B] (-inf when k = 0; +inf when the k-th
    smallest is NaN)."""
    s32 = np.asarray(scores, dtype=np.float64).astype(np.float32)
    B, T = s32.shape
    k = int(np.ceil(np.float32(phi) * np.float32(T)))
    if not 0 <= k <= T:
        raise ValueError("phi must lie in [0, 1]")
    tau = np.full(B, -np.inf, dtype=np.float32)
    if k > 0:
        srt = np.sort(s32, axis=1)              # NaN sorts last
        tau = srt[:, k - 1].copy()
        tau[np.isnan(tau)] = np.inf
    return tau


def allocate_quantiles(s_layers, phi_bar, eps):
    """Sec. 3.1: phi_l = (L phi_bar) softmax(-s_l / eps) over the L layers, cut to [0, 1]."""
    s = _f64(s_layers)
    z = -s / float(eps)
    w = np.exp(z - np.max(z))
    phi = len(s) * float(phi_bar) * w / np.sum(w)
    return np.minimum(phi, 1.0)


def policy_mode(mode, layer, step, skip_layers=0, refresh_interval=0):
    """Sec. 5 (Fast-dLLM-v2 setting): layers [0, skip_layers) always recompute, and
    with a refresh interval r > 0 every step whose index is a multiple of r recomputes
    everything; otherwise the requested mode stands."""
    if layer < skip_layers:
        return MODE_DENSE
    if refresh_interval > 0 and step % refresh_interval == 0:
        return MODE_DENSE
    return mode


def selection(reuse):
    """Ascending flat ids of refreshed tokens, per-sequence counts and offsets.

    reuse: bool [B, T].  Returns (sel_idx int32 [n], sel_count int32 [B],
    sel_off int32 [B+1])."""
    reuse = np.asarray(reuse, dtype=bool)
    B, T = reuse.shape
    sel_idx = np.flatnonzero(~reuse.reshape(-1)).astype(np.int32)
    sel_count = (~reuse).sum(axis=1).astype(np.int32)
    sel_off = np.zeros(B + 1, dtype=np.int32)
    sel_off[1:] = np.cumsum(sel_count)
    return sel_idx, sel_count, sel_off


def attention_rows(q, k, v, n_heads):
    """App. E.2: bidirectional softmax attention of query rows q [n, d] against
    all keys/values k, v [T, d] of one sequence, head by head."""
    q = _f64(q)
    k = _f64(k)
    v = _f64(v)
    n, d = q.shape
    dh = d // n_heads
    out = np.empty((n, d), dtype=np.float64)
    for h in range(n_heads):
        c = slice(h * dh, (h + 1) * dh)
        z = (q[:, c] @ k[:, c].T) / np.sqrt(float(dh))
        m = np.max(z, axis=1, keepdims=True)
        w = np.exp(z - m)
        out[:, c] = (w @ v[:, c]) / np.sum(w, axis=1, keepdims=True)
    return out


def dense_layer(x, wq, wk, wv, wo, n_heads):
    """App. E.2 for a batch: x [B, T, d] -> (out, Q, K, V), all [B, T, d]."""
    x = _f64(x)
    wq, wk, wv, wo = _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    Q = x @ wq
    K = x @ wk
    V = x @ wv
    out = np.empty_like(Q)
    for b in range(x.shape[0]):
        out[b] = attention_rows(Q[b], K[b], V[b], n_heads) @ wo
    return out, Q, K, V


def layer_norm(x, gain, bias=None, eps=1e-5):
    """Alg. 1/2 line 1: per token, (x - mean) / sqrt(var + eps) * gain + bias over the
    channel axis (biased variance)."""
    x = _f64(x)
    mu = np.mean(x, axis=-1, keepdims=True)
    var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
    y = (x - mu) / np.sqrt(var + eps) * _f64(gain)
    return y if bias is None else y + _f64(bias)


def rms_norm(x, gain, eps=1e-5):
    """The root-mean-square variant of line 1: x / sqrt(mean(x^2) + eps) * gain."""
    x = _f64(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _f64(gain)


def rope(x, positions, n_heads, base=10000.0):
    """Rotary position embedding of x [..., T, d] with per-token positions [T]: in
    every head, the channel pair (2i, 2i+1) is rotated by positions * base^(-2i/Dh)."""
    x = _f64(x)
    d = x.shape[-1]
    dh = d // n_heads
    i = np.arange(dh // 2, dtype=np.float64)
    theta = base ** (-2.0 * i / dh)                              # [Dh/2]
    ang = _f64(positions)[:, None] * theta[None, :]              # [T, Dh/2]
    c = np.tile(np.cos(ang), (1, n_heads))                       # [T, d/2], head after head
    s = np.tile(np.sin(ang), (1, n_heads))
    xe, xo = x[..., 0::2], x[..., 1::2]
    y = np.empty_like(x)
    y[..., 0::2] = xe * c - xo * s
    y[..., 1::2] = xe * s + xo * c
    return y


def layer_step(mode, tau, x, wq, wk, wv, wo, q_prev, k_cache, v_cache, o_cache,
               n_heads, score_head=0, storage=None, rope_base=None, quantile=False, prefix=0):
    """One step of the layer in mode DENSE / KV (Alg. 1) / O (Alg. 2) / KVO.

    x [B,T,d]; w* [d,d]; q_prev [B,T,Dh] (or [B,T,d] when score_head = -1);
    k_cache, v_cache, o_cache [B,T,d] hold the previous step's state.
    rope_base: None, or the base of the rotary embedding applied to Q and to the K rows
    projected at this step (see the header).
    quantile: tau is a reuse rate phi in [0, 1]; each sequence's threshold is
    quantile_threshold of its scores (returned as "tau", float32 [B]).
    prefix: the first `prefix` tokens of every sequence are frozen (see the header).
    Returns a dict with out, k_cache, v_cache, o_cache, q_prev (all updated,
    float64), scores [B,T] float64, reuse_mask uint8 [B,T] (1 = reused),
    sel_idx, sel_count, sel_off, and exact = {out, k_cache, v_cache} before the
    final storage rounding (identical to the former when storage is None).
    """
    if mode not in (MODE_DENSE, MODE_KV, MODE_O, MODE_KVO):
        raise ValueError("unknown mode")
    x = _f64(x)
    wq, wk, wv, wo = _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    B, T, d = x.shape
    dh = d // n_heads

    # Alg. 1/2 line 2: the query of every token.
    Q = x @ wq

    # Alg. 1/2 line 3: drift of head 0 against the previous step's head 0.
    q_sc = Q if score_head < 0 else Q[:, :, score_head * dh:(score_head + 1) * dh]
    scores = drift_scores(q_sc, _f64(q_prev))

    # Alg. 1/2 lines 4-5.
    if not 0 <= prefix < T:
        raise ValueError("prefix must lie in [0, seq)")
    frozen = np.zeros((B, T), dtype=bool)
    frozen[:, :prefix] = True
    scores[frozen] = 0.0
    if quantile:
        tau_b = quantile_threshold(scores[:, prefix:], tau)
    else:
        tau_b = np.full(B, np.float32(tau), dtype=np.float32)
    if mode == MODE_DENSE:
        reuse = np.zeros((B, T), dtype=bool)
    else:
        reuse = np.stack([reuse_decision(scores[b], tau_b[b]) for b in range(B)])
    reuse |= frozen
    sel_idx, sel_count, sel_off = selection(reuse)
    # rows the "all rows" steps of a mode run over: every token that is not frozen
    active = ~frozen
    # rotary embedding of queries and of the keys projected at this step (position =
    # index in the sequence); the score above used the unrotated query
    pos = np.arange(T, dtype=np.float64)
    rot = (lambda a, rows=None: a) if rope_base is None else (
        lambda a, rows=None: rope(a, pos if rows is None else pos[rows], n_heads, rope_base))
    Qs = round_storage(rot(Q), storage)

    # Keys and values.
    if mode in (MODE_KV, MODE_KVO):
        # Alg. 1 lines 6-9: refresh the selected rows, keep the cached ones.
        K_exact = _f64(k_cache).copy()
        V_exact = _f64(v_cache).copy()
        for b in range(B):
            rows = np.flatnonzero(~reuse[b])
            K_exact[b, rows] = rot(x[b, rows] @ wk, rows)
            V_exact[b, rows] = x[b, rows] @ wv
    elif prefix == 0:
        # Alg. 2 line 7 / App. E.2.
        K_exact = rot(x @ wk)
        V_exact = x @ wv
    else:
        # the same for the rows that are not frozen; frozen rows keep the cache
        K_exact = _f64(k_cache).copy()
        V_exact = _f64(v_cache).copy()
        rows = np.arange(prefix, T)
        K_exact[:, rows] = rot(x[:, rows] @ wk, rows)
        V_exact[:, rows] = x[:, rows] @ wv
    K = round_storage(K_exact, storage)
    V = round_storage(V_exact, storage)

    # Attention and output projection.
    if mode in (MODE_O, MODE_KVO):
        # Alg. 2 lines 6, 8-11 with the cache holding rows after Wo.
        out_exact = _f64(o_cache).copy()
        for b in range(B):
            rows = np.flatnonzero(~reuse[b])
            attn = round_storage(attention_rows(Qs[b, rows], K[b], V[b], n_heads), storage)
            out_exact[b, rows] = attn @ wo
    else:
        # Alg. 1 lines 10-11 (frozen rows return the cached output).
        out_exact = _f64(o_cache).copy()
        for b in range(B):
            rows = np.flatnonzero(active[b])
            attn = round_storage(attention_rows(Qs[b, rows], K[b], V[b], n_heads), storage)
            out_exact[b, rows] = attn @ wo
    out = round_storage(out_exact, storage)

    return {
        "out": out,
        "k_cache": K,
        "v_cache": V,
        "o_cache": out.copy(),
        "exact": {"out": out_exact, "k_cache": K_exact, "v_cache": V_exact},
        "q_prev": np.where(frozen[:, :, None], _f64(q_prev), q_sc),
        "scores": scores,
        "tau": tau_b,
        "reuse_mask": reuse.astype(np.uint8),
        "sel_idx": sel_idx,
        "sel_count": sel_count,
        "sel_off": sel_off,
    }


def block_step(mode, tau, x, norm, gain, bias, eps, wq, wk, wv, wo, q_prev, k_cache,
               v_cache, o_cache, n_heads, score_head=0, storage=None, rope_base=None,
               residual=True, quantile=False, prefix=0):
    """The attention block around ``layer_step``: h = norm(x) (Alg. 1/2 line 1; norm is
    "layer", "rms" or None), the layer step on h, then out = x + O when residual.

    o_cache holds O, the block output before the residual sum.  Returns layer_step's
    dict (its "out" and "o_cache" are O) plus "h" and "block_out"; exact["block_out"]
    is x + exact O."""
    x = _f64(x)
    if norm == "layer":
        h = layer_norm(x, gain, bias, eps)
    elif norm == "rms":
        h = rms_norm(x, gain, eps)
    elif norm is None:
        h = x
    else:
        raise ValueError("norm must be 'layer', 'rms' or None")
    h = round_storage(h, storage)          # the normalised hidden state is a stored tensor
    r = layer_step(mode, tau, h, wq, wk, wv, wo, q_prev, k_cache, v_cache, o_cache,
                   n_heads, score_head=score_head, storage=storage, rope_base=rope_base,
                   quantile=quantile, prefix=prefix)
    r["h"] = h
    exact_block = x + r["out"] if residual else r["out"].copy()
    r["exact"]["block_out"] = exact_block
    r["block_out"] = round_storage(exact_block, storage)
    return r


def step_o_prewo(tau, x, wq, wk, wv, wo, q_prev, attn_cache, n_heads,
                 score_head=0):
    """Alg. 2 exactly as listed: the cache holds attention rows *before* Wo and
    Wo multiplies every row.  Returns (out, new attn cache, reuse mask)."""
    x = _f64(x)
    wq, wk, wv, wo = _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    B, T, d = x.shape
    dh = d // n_heads
    Q = x @ wq
    q_sc = Q if score_head < 0 else Q[:, :, score_head * dh:(score_head + 1) * dh]
    reuse = reuse_decision(drift_scores(q_sc, _f64(q_prev)), tau)
    K = x @ wk
    V = x @ wv
    attn = _f64(attn_cache).copy()
    for b in range(B):
        rows = np.flatnonzero(~reuse[b])
        attn[b, rows] = attention_rows(Q[b, rows], K[b], V[b], n_heads)
    return attn @ wo, attn, reuse.astype(np.uint8)
