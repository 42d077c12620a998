"""Seeded synthetic inputs for one attention layer at two consecutive denoising steps.

This module only draws random numbers and rounds them to the storage dtype.  It
holds none of the layer's arithmetic, and both the HIP path's tests/benchmark
and the CPU checker feed on the arrays it returns.

Recipe (stands in for the activations of a trained diffusion LLM, which are not
available): weights ~ N(0, 0.02^2); hidden states of the previous step ~ N(0, 1);
this step = previous step + sigma_i * N(0, 1) with sigma_i = 0.5 on a seeded
random subset of tokens (the "perturbed fraction") and 0.01 on the rest.  The
head-0 query drift then has two well separated modes (about 5e-5 for the stable
tokens, about 0.1 for the perturbed ones), the shape the paper describes for its
per-token drift histograms (Sec. 5, Fig. 3).
"""
from __future__ import annotations

import numpy as np

SIGMA_PERTURBED = 0.5
SIGMA_STABLE = 0.01
WEIGHT_STD = 0.02
# Any threshold between the two drift modes reuses exactly the stable tokens.
TAU_SEPARATING = 5e-3


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even); the result is
    float32 holding bf16-representable values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a):
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def _store(a, dtype):
    if dtype == "bf16":
        return round_to_bf16(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError("dtype must be 'bf16' or 'f32'")


def make_weights(seed, hidden, dtype):
    """Wq, Wk, Wv, Wo as float32 [hidden, hidden] arrays, row-major [d_in, d_out]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name in ("wq", "wk", "wv", "wo"):
        w = rng.standard_normal((hidden, hidden), dtype=np.float32) * np.float32(WEIGHT_STD)
        out[name] = _store(w, dtype)
    return out


def make_hidden_pair(seed, batch, seq, hidden, fraction, dtype):
    """Hidden states of steps t-1 and t.

    fraction: a float (the same perturbed fraction for every sequence) or a pair
    (lo, hi): each sequence draws its own fraction uniformly in [lo, hi].
    Returns dict x_prev, x_cur float32 [B,T,d] and perturbed bool [B,T]."""
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    x_prev = rng.standard_normal((batch, seq, hidden), dtype=np.float32)
    perturbed = np.zeros((batch, seq), dtype=bool)
    for b in range(batch):
        if isinstance(fraction, (tuple, list)):
            f = float(rng.uniform(fraction[0], fraction[1]))
        else:
            f = float(fraction)
        n = int(round(f * seq))
        perturbed[b, rng.permutation(seq)[:n]] = True
    sigma = np.where(perturbed, np.float32(SIGMA_PERTURBED), np.float32(SIGMA_STABLE))
    noise = rng.standard_normal((batch, seq, hidden), dtype=np.float32)
    x_cur = x_prev + sigma[:, :, None].astype(np.float32) * noise
    return {"x_prev": _store(x_prev, dtype), "x_cur": _store(x_cur, dtype),
            "perturbed": perturbed}


def make_norm_params(seed, hidden, dtype):
    """Gain ~ 1 + 0.1 N(0,1) and bias ~ 0.05 N(0,1) of the normalisation in front of the
    projections, float32 [hidden] each."""
    rng = np.random.Generator(np.random.PCG64(seed + 104729))
    gain = np.float32(1.0) + np.float32(0.1) * rng.standard_normal(hidden, dtype=np.float32)
    bias = np.float32(0.05) * rng.standard_normal(hidden, dtype=np.float32)
    return {"gain": _store(gain, dtype), "bias": _store(bias, dtype)}


def make_model_params(seed, n_layers, hidden, ffn, vocab, dtype, with_head=True):
    """Random-init weights of a masked-diffusion model: projection matrices ~ N(0, 0.02^2),
    normalisation gains ~ 1 + 0.1 N(0,1), token embedding ~ N(0,1).  float32 arrays holding
    values representable in `dtype`."""
    rng = np.random.Generator(np.random.PCG64(seed + 15485863))
    nrm = lambda *shape, std=WEIGHT_STD: _store(rng.standard_normal(shape, dtype=np.float32) * np.float32(std), dtype)
    gain = lambda: _store(np.float32(1.0) + np.float32(0.1) * rng.standard_normal(hidden, dtype=np.float32), dtype)
    layers = []
    for _ in range(n_layers):
        layers.append(dict(attn_gain=gain(), wq=nrm(hidden, hidden), wk=nrm(hidden, hidden), wv=nrm(hidden, hidden),
                           wo=nrm(hidden, hidden), ffn_gain=gain(), w_gate=nrm(hidden, ffn), w_up=nrm(hidden, ffn),
                           w_down=nrm(ffn, hidden)))
    params = dict(embed=nrm(vocab, hidden, std=1.0), final_gain=gain(), layers=layers)
    if with_head:
        params["head"] = nrm(hidden, vocab)
    return params


def make_ids(seed, batch, seq, vocab, prompt_len, mask_id):
    """A prompt of uniform random ids followed by mask ids, int32 [batch, seq]."""
    rng = np.random.Generator(np.random.PCG64(seed + 32452843))
    ids = np.full((batch, seq), mask_id, dtype=np.int32)
    ids[:, :prompt_len] = rng.integers(0, vocab - 1, (batch, prompt_len))
    return ids


# Layer shapes of the workloads.  "tiny" is the small fp32 case; "llada8b" is one
# LLaDA-8B-shaped layer at 512 prompt + 512 generated tokens; "llada8b_b8" is the
# same layer at 2048 tokens and 8 sequences with per-sequence perturbed fractions.
CONFIGS = {
    "tiny": dict(batch=1, seq=128, hidden=256, n_heads=4, head_dim=64, dtype="f32",
                 fraction=0.20),
    "llada8b": dict(batch=1, seq=1024, hidden=4096, n_heads=32, head_dim=128,
                    dtype="bf16", fraction=0.20),
    "llada8b_b8": dict(batch=8, seq=2048, hidden=4096, n_heads=32, head_dim=128,
                       dtype="bf16", fraction=(0.05, 0.30)),
}


def make_case(name, seed=1234, fraction=None, **override):
    """Weights plus a hidden-state pair for a named config (fields can be overridden)."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    if fraction is not None:
        cfg["fraction"] = fraction
    w = make_weights(seed, cfg["hidden"], cfg["dtype"])
    h = make_hidden_pair(seed, cfg["batch"], cfg["seq"], cfg["hidden"], cfg["fraction"],
                         cfg["dtype"])
    case = dict(cfg)
    case.update(w)
    case.update(h)
    case.update(make_norm_params(seed, cfg["hidden"], cfg["dtype"]))
    return case
