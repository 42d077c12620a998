"""Pins for the model-level oracle: SwiGLU feed-forward against torch's routines and scalar
loops, embedding, the layer composition against a model written a second time with torch
modules' functional forms, and the block-wise schedule against its statement."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import dare_oracle as orc
from oracle import dllm_oracle as dl


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _params(r, L, d, ffn, V, with_head=True):
    layers = []
    for _ in range(L):
        layers.append(dict(attn_gain=1 + 0.1 * r.standard_normal(d), ffn_gain=1 + 0.1 * r.standard_normal(d),
                           wq=r.standard_normal((d, d)) * 0.2, wk=r.standard_normal((d, d)) * 0.2,
                           wv=r.standard_normal((d, d)) * 0.2, wo=r.standard_normal((d, d)) * 0.2,
                           w_gate=r.standard_normal((d, ffn)) * 0.2, w_up=r.standard_normal((d, ffn)) * 0.2,
                           w_down=r.standard_normal((ffn, d)) * 0.2))
    p = dict(embed=r.standard_normal((V, d)), final_gain=1 + 0.1 * r.standard_normal(d), layers=layers)
    if with_head:
        p["head"] = r.standard_normal((d, V)) * 0.2
    return p


def _zero_caches(L, B, T, d, dh):
    z = np.zeros((B, T, d))
    return [dict(q_prev=np.ones((B, T, dh)), k_cache=z, v_cache=z, o_cache=z) for _ in range(L)]


def test_silu_matches_library_and_limits():
    z = np.linspace(-30, 30, 241)
    assert np.allclose(dl.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=0, atol=1e-14)
    assert dl.silu(0.0) == 0.0 and abs(dl.silu(40.0) - 40.0) < 1e-12 and abs(dl.silu(-40.0)) < 1e-12


def test_ffn_block_against_library_routines_and_scalar_loop():
    r = _rng(1)
    x = r.standard_normal((2, 3, 8)) * 2
    g = 1 + 0.1 * r.standard_normal(8)
    wg, wu, wd = r.standard_normal((8, 12)), r.standard_normal((8, 12)), r.standard_normal((12, 8))
    got, exact = dl.ffn_block(x, g, 1e-5, wg, wu, wd)
    assert np.array_equal(got, exact)
    xt = torch.from_numpy(x)
    n = F.rms_norm(xt, (8,), torch.from_numpy(g), eps=1e-5)
    want = xt + (F.silu(n @ torch.from_numpy(wg)) * (n @ torch.from_numpy(wu))) @ torch.from_numpy(wd)
    assert np.allclose(got, want.numpy(), rtol=0, atol=1e-12)
    # one element by scalar loops
    row = x[1, 2]
    nrm = row / np.sqrt(np.mean(row ** 2) + 1e-5) * g
    acc = 0.0
    for j in range(12):
        gj = sum(nrm[c] * wg[c, j] for c in range(8))
        uj = sum(nrm[c] * wu[c, j] for c in range(8))
        acc += gj / (1 + np.exp(-gj)) * uj * wd[j, 5]
    assert abs(got[1, 2, 5] - (row[5] + acc)) < 1e-12


def test_ffn_block_row_mask_and_storage_rounding():
    r = _rng(2)
    x = orc.round_storage(r.standard_normal((1, 4, 8)), "bf16")
    g = np.ones(8)
    w = [r.standard_normal((8, 16)) * 0.3, r.standard_normal((8, 16)) * 0.3, r.standard_normal((16, 8)) * 0.3]
    rows = np.array([[False, True, True, False]])
    got, exact = dl.ffn_block(x, g, 1e-5, *w, storage="bf16", rows=rows)
    assert np.array_equal(got[0, [0, 3]], x[0, [0, 3]])
    assert np.array_equal(got, orc.round_storage(exact, "bf16"))
    full, _ = dl.ffn_block(x, g, 1e-5, *w, storage="bf16")
    assert np.array_equal(got[0, 1:3], full[0, 1:3])


def test_embed_is_a_row_lookup():
    t = _rng(3).standard_normal((11, 4))
    ids = np.array([[3, 3, 10], [0, 7, 1]])
    e = dl.embed(ids, t)
    assert e.shape == (2, 3, 4) and np.array_equal(e[1, 1], t[7]) and np.array_equal(e[0, 0], e[0, 1])


def test_dense_model_step_against_a_second_formulation():
    """All layers in DENSE mode = a plain pre-norm transformer, written again with torch's
    functional routines (scaled_dot_product_attention, rms_norm, silu) and an explicit
    rotary embedding in complex form."""
    r = _rng(4)
    L, B, T, d, H, ffn, V = 3, 2, 9, 16, 2, 24, 13
    dh = d // H
    p = _params(r, L, d, ffn, V)
    ids = r.integers(0, V, (B, T))
    res = dl.model_step([orc.MODE_DENSE] * L, [0.0] * L, ids, p, _zero_caches(L, B, T, d, dh), H, 1e-5, 10000.0)

    def rot(t):  # [B, T, d] -> rotary, pairs (2i, 2i+1) of each head as complex numbers
        tt = t.reshape(B, T, H, dh // 2, 2)
        z = torch.view_as_complex(tt.contiguous())
        ang = torch.arange(T, dtype=torch.float64)[:, None] * 10000.0 ** (-2.0 * torch.arange(dh // 2, dtype=torch.float64) / dh)
        z = z * torch.polar(torch.ones_like(ang), ang)[None, :, None, :]
        return torch.view_as_real(z).reshape(B, T, d)

    x = torch.from_numpy(p["embed"])[torch.from_numpy(ids)]
    for lp in p["layers"]:
        tw = {k: torch.from_numpy(v) for k, v in lp.items()}
        n = F.rms_norm(x, (d,), tw["attn_gain"], eps=1e-5)
        q, k, v = rot(n @ tw["wq"]), rot(n @ tw["wk"]), n @ tw["wv"]
        sp = lambda t: t.reshape(B, T, H, dh).transpose(1, 2)
        a = F.scaled_dot_product_attention(sp(q), sp(k), sp(v)).transpose(1, 2).reshape(B, T, d)
        x = x + a @ tw["wo"]
        n = F.rms_norm(x, (d,), tw["ffn_gain"], eps=1e-5)
        x = x + (F.silu(n @ tw["w_gate"]) * (n @ tw["w_up"])) @ tw["w_down"]
    y = F.rms_norm(x, (d,), torch.from_numpy(p["final_gain"]), eps=1e-5)
    assert np.allclose(res["hidden"], y.numpy(), rtol=0, atol=1e-9)
    assert np.allclose(dl.logits(res["hidden"][0], p["head"]), (y[0] @ torch.from_numpy(p["head"])).numpy(), atol=1e-9)


def test_second_step_on_unchanged_ids_reuses_everything_and_changes_nothing():
    r = _rng(5)
    L, B, T, d, H, ffn, V = 2, 1, 8, 16, 2, 24, 9
    p = _params(r, L, d, ffn, V, with_head=False)
    ids = r.integers(0, V, (B, T))
    first = dl.model_step([orc.MODE_DENSE] * L, [0.0] * L, ids, p, _zero_caches(L, B, T, d, d // H), H, 1e-5, 10000.0)
    again = dl.model_step([orc.MODE_KVO] * L, [0.0] * L, ids, p, first["new_caches"], H, 1e-5, 10000.0)
    assert all(lay["reuse_mask"].all() for lay in again["layers"])
    assert np.array_equal(again["hidden"], first["hidden"])
    # one token changed: layer 0 refreshes exactly that token (its score is the only non-zero one)
    ids2 = ids.copy()
    ids2[0, 3] = (ids[0, 3] + 1) % V
    third = dl.model_step([orc.MODE_KVO] * L, [0.0] * L, ids2, p, first["new_caches"], H, 1e-5, 10000.0)
    assert third["layers"][0]["reuse_mask"][0].tolist() == [1, 1, 1, 0, 1, 1, 1, 1]


def test_blockwise_schedule_statement():
    r = _rng(6)
    steps = dl.blockwise_schedule(5, 70, 32, 1, r)
    pos = np.concatenate(steps)
    assert len(steps) == 70 and sorted(pos.tolist()) == list(range(5, 75))      # every position once
    blocks = [(int(s[0]) - 5) // 32 for s in steps]
    assert blocks == sorted(blocks)                                             # block after block
    four = dl.blockwise_schedule(8, 64, 32, 4, _rng(6))
    assert len(four) == 16 and all(len(s) == 4 for s in four)
    assert all(len({(int(q) - 8) // 32 for q in s}) == 1 for s in four)          # a step stays inside one block
