"""CPU oracle for a masked-diffusion language model built from DARE layers.
TEST INFRASTRUCTURE ONLY: tests, the smoke test and the benchmark's CPU leg use it; the
product never imports it.

The paper applies DARE to the self-attention of every layer of LLaDA / Dream (Sec. 5);
the model around the attention is the standard pre-norm transformer those models use
and is not the paper's subject.  What this file fixes, so that the HIP model runtime has
something to be checked against:

  x_0      = E[ids]                                         token embedding
  layer l: x' = x + O_l(norm(x))                            attention block = dare_oracle.block_step
           x''= x' + (silu(n W_g) * (n W_u)) W_d,  n = norm'(x')     SwiGLU feed-forward
  final:   y = norm_f(x_L);  logits = y W_head (only for the rows asked for)

with RMS normalisation (gain only), rotary embedding on Q and K, no biases, weights
[d_in, d_out].  silu(z) = z / (1 + exp(-z)).  Numpy float64 throughout; with
storage="bf16" every tensor that is stored (the normalised rows, the gated product
silu(n W_g) * (n W_u), the feed-forward output, each residual sum, y) is rounded to
bfloat16 where it is produced, as in dare_oracle; the gate and up projections themselves
are not stored tensors (they are consumed where they are produced) and are not rounded.

The decoding schedule (``blockwise_schedule``) is the block-wise one the paper uses
(block size 32, Sec. 5 / App. A): the generated region is filled block by block, left
to right; at every denoising step the listed number of still-masked positions of the
current block is replaced by a token.  Which position and which token come from the
caller's seeded generator (a trained model would pick them from its logits); the
schedule only fixes the order of blocks and that a position is written once.
"""
from __future__ import annotations

import numpy as np

from . import dare_oracle as orc


def silu(z):
    z = np.asarray(z, dtype=np.float64)
    return z / (1.0 + np.exp(-z))


def embed(ids, table):
    """x_0[b, t] = table[ids[b, t]]."""
    return np.asarray(table, dtype=np.float64)[np.asarray(ids)]


def ffn_block(x, gain, eps, w_gate, w_up, w_down, storage=None, rows=None):
    """x + (silu(n W_g) * (n W_u)) W_d with n = rms_norm(x).  rows: optional boolean
    [B, T]; where False the row is returned unchanged (a frozen prefix)."""
    x = np.asarray(x, dtype=np.float64)
    rs = orc.round_storage
    n = rs(orc.rms_norm(x, gain, eps), storage)
    g = n @ np.asarray(w_gate, dtype=np.float64)
    u = n @ np.asarray(w_up, dtype=np.float64)
    a = rs(silu(g) * u, storage)
    f = rs(a @ np.asarray(w_down, dtype=np.float64), storage)
    exact = x + f
    if rows is not None:
        exact = np.where(np.asarray(rows, dtype=bool)[:, :, None], exact, x)
    return rs(exact, storage), exact


def model_step(modes, taus, ids, params, caches, n_heads, eps, rope_base, storage=None,
               quantile=False, prefix=0, x0=None):
    """One denoising step of the whole model.

    modes, taus: per-layer lists.  params: dict with "embed" [V, d], "final_gain" [d],
    optional "head" [d, V], and "layers": list of dicts attn_gain, wq, wk, wv, wo, ffn_gain,
    w_gate, w_up, w_down.  caches: list of per-layer dicts q_prev, k_cache, v_cache,
    o_cache (not modified).  Returns dict: hidden (after the final norm), x_last, layers =
    list of per-layer results (the dare_oracle.block_step dict plus "x_in", "x_mid",
    "x_out"), new_caches."""
    x = embed(ids, params["embed"]) if x0 is None else np.asarray(x0, dtype=np.float64)
    x = orc.round_storage(x, storage)
    B, T, _ = x.shape
    active = np.ones((B, T), dtype=bool)
    active[:, :prefix] = False
    per_layer, new_caches = [], []
    for l, lp in enumerate(params["layers"]):
        c = caches[l]
        r = orc.block_step(modes[l], taus[l], x, "rms", lp["attn_gain"], None, eps, lp["wq"], lp["wk"],
                           lp["wv"], lp["wo"], c["q_prev"], c["k_cache"], c["v_cache"], c["o_cache"],
                           n_heads, storage=storage, rope_base=rope_base, residual=True,
                           quantile=quantile, prefix=prefix)
        x_mid = r["block_out"]
        x_out, _ = ffn_block(x_mid, lp["ffn_gain"], eps, lp["w_gate"], lp["w_up"], lp["w_down"], storage,
                             rows=active if prefix else None)
        r.update(x_in=x, x_mid=x_mid, x_out=x_out)
        per_layer.append(r)
        new_caches.append({k: r[k] for k in ("q_prev", "k_cache", "v_cache", "o_cache")})
        x = x_out
    hidden = orc.round_storage(orc.rms_norm(x, params["final_gain"], eps), storage)
    return {"hidden": hidden, "x_last": x, "layers": per_layer, "new_caches": new_caches}


def logits(hidden_rows, head):
    """hidden_rows [n, d] (after the final norm) times the output embedding [d, V]."""
    return np.asarray(hidden_rows, dtype=np.float64) @ np.asarray(head, dtype=np.float64)


def blockwise_schedule(prompt_len, gen_len, block, per_step, rng):
    """Positions written at each denoising step: the generated region [prompt_len,
    prompt_len + gen_len) is filled block by block; each step takes `per_step` of the
    still-masked positions of the current block, in the order of a seeded permutation.
    Returns a list (one entry per step) of int arrays."""
    steps = []
    for b0 in range(prompt_len, prompt_len + gen_len, block):
        order = b0 + rng.permutation(min(block, prompt_len + gen_len - b0))
        for i in range(0, len(order), per_step):
            steps.append(np.sort(order[i:i + per_step]))
    return steps
