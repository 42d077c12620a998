"""Pins for the oracle's block functions (normalisation of Alg. 1/2 line 1, rotary
embedding, residual sum), against things other than the oracle itself: torch's library
routines, scalar loops, hand-computed rotations and the invariants of a rotation."""
import math

import numpy as np
import pytest
import torch

from oracle import dare_oracle as orc


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---- normalisation -----------------------------------------------------------------------

def test_layer_norm_matches_library_routine():
    r = _rng(1)
    x = r.standard_normal((3, 5, 16)) * 3 + 1.5
    g, b = r.standard_normal(16), r.standard_normal(16)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x), (16,), torch.from_numpy(g),
                                          torch.from_numpy(b), eps=1e-5).numpy()
    assert np.allclose(orc.layer_norm(x, g, b, 1e-5), want, rtol=0, atol=1e-12)


def test_layer_norm_moments_and_invariances():
    r = _rng(2)
    x = r.standard_normal((7, 32)) * 4 - 2
    y = orc.layer_norm(x, np.ones(32), None, 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-12)
    assert np.allclose((y * y).mean(-1), 1, atol=1e-12)
    # shift and positive scale of a token do not change its normalised value
    assert np.allclose(orc.layer_norm(3.0 * x + 11.0, np.ones(32), None, 0.0), y, atol=1e-10)
    # a sign flip does (a dropped mean subtraction or a squared-only formula would not notice)
    assert np.allclose(orc.layer_norm(-x, np.ones(32), None, 0.0), -y, atol=1e-12)


def test_rms_norm_matches_library_routine_and_scalar_loop():
    r = _rng(3)
    x = r.standard_normal((4, 24)) * 2 + 0.7
    g = r.standard_normal(24)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(g), eps=1e-6).numpy()
    got = orc.rms_norm(x, g, 1e-6)
    assert np.allclose(got, want, rtol=0, atol=1e-12)
    for t in range(4):
        ms = sum(float(v) ** 2 for v in x[t]) / 24
        for c in range(24):
            assert abs(got[t, c] - x[t, c] / math.sqrt(ms + 1e-6) * g[c]) < 1e-12


def test_rms_norm_keeps_the_mean_layer_norm_removes_it():
    x = np.full((1, 8), 5.0)
    assert np.allclose(orc.rms_norm(x, np.ones(8), 0.0), 1.0)
    assert np.allclose(orc.layer_norm(x, np.ones(8), None, 1e-5), 0.0)


# ---- rotary embedding --------------------------------------------------------------------

def test_rope_hand_values_one_head_two_pairs():
    # head_dim 4: pair 0 turns by pos * 1, pair 1 by pos * base^(-1/2)
    x = np.array([[1.0, 0.0, 0.0, 2.0]])
    pos = np.array([0.5])
    y = orc.rope(x, pos, 1, base=100.0)
    a0, a1 = 0.5, 0.5 * 100.0 ** -0.5
    want = [math.cos(a0), math.sin(a0), -2.0 * math.sin(a1), 2.0 * math.cos(a1)]
    assert np.allclose(y[0], want, atol=1e-15)


def test_rope_position_zero_is_identity_and_every_head_gets_the_same_angles():
    r = _rng(4)
    x = r.standard_normal((3, 16))
    assert np.array_equal(orc.rope(x, np.zeros(3), 2), x)
    one = r.standard_normal((3, 8))
    both = np.concatenate([one, one], axis=1)
    y = orc.rope(both, np.array([1.0, 5.0, 9.0]), 2)
    assert np.allclose(y[:, :8], y[:, 8:])
    assert np.allclose(y[:, :8], orc.rope(one, np.array([1.0, 5.0, 9.0]), 1))


def test_rope_is_a_rotation_composes_and_depends_on_relative_position_only():
    r = _rng(5)
    T, H, d = 6, 2, 16
    q, k = r.standard_normal((T, d)), r.standard_normal((T, d))
    pos = np.arange(T, dtype=np.float64)
    rq = orc.rope(q, pos, H)
    # pairwise norms kept
    assert np.allclose(rq[:, 0::2] ** 2 + rq[:, 1::2] ** 2, q[:, 0::2] ** 2 + q[:, 1::2] ** 2)
    # rotation by a then b = rotation by a + b
    assert np.allclose(orc.rope(orc.rope(q, pos, H), 2 * pos + 1, H), orc.rope(q, 3 * pos + 1, H))
    # per-head logits depend on the position difference only
    def logits(shift):
        a, b = orc.rope(q, pos + shift, H), orc.rope(k, pos + shift, H)
        return np.stack([a[:, h * 8:(h + 1) * 8] @ b[:, h * 8:(h + 1) * 8].T for h in range(H)])
    assert np.allclose(logits(0.0), logits(37.0), atol=1e-10)
    # and they do depend on it (an identity "rotation" would pass the line above)
    assert not np.allclose(logits(0.0)[0], q[:, :8] @ k[:, :8].T)


def test_rope_scalar_loop():
    r = _rng(6)
    T, H, d = 3, 2, 12
    dh = d // H
    x = r.standard_normal((T, d))
    pos = np.array([2.0, 7.0, 11.0])
    y = orc.rope(x, pos, H, base=500.0)
    for t in range(T):
        for h in range(H):
            for i in range(dh // 2):
                ang = pos[t] * 500.0 ** (-2.0 * i / dh)
                a, b = x[t, h * dh + 2 * i], x[t, h * dh + 2 * i + 1]
                assert abs(y[t, h * dh + 2 * i] - (a * math.cos(ang) - b * math.sin(ang))) < 1e-12
                assert abs(y[t, h * dh + 2 * i + 1] - (a * math.sin(ang) + b * math.cos(ang))) < 1e-12


# ---- the layer step with rotary embedding, and the block ----------------------------------

def _weights(r, d, std=0.4):
    return {k: r.standard_normal((d, d)) * std for k in ("wq", "wk", "wv", "wo")}


def _dense_with_rope(x, w, H, base):
    """Dense attention with rotated Q and K, written with the oracle's dense pieces only."""
    B, T, d = x.shape
    pos = np.arange(T, dtype=np.float64)
    out = np.empty_like(x)
    Ks, Vs, Qs = [], [], []
    for b in range(B):
        Q = x[b] @ w["wq"]
        K = orc.rope(x[b] @ w["wk"], pos, H, base)
        V = x[b] @ w["wv"]
        out[b] = orc.attention_rows(orc.rope(Q, pos, H, base), K, V, H) @ w["wo"]
        Qs.append(Q), Ks.append(K), Vs.append(V)
    return out, np.stack(Qs), np.stack(Ks), np.stack(Vs)


def test_step_with_rope_dense_and_score_is_taken_before_the_rotation():
    r = _rng(7)
    B, T, d, H = 2, 5, 8, 2
    w = _weights(r, d)
    x = r.standard_normal((B, T, d))
    want, Q, K, V = _dense_with_rope(x, w, H, 10000.0)
    z = np.zeros((B, T, d))
    q_prev = r.standard_normal((B, T, d // H))
    res = orc.layer_step(orc.MODE_DENSE, 0.0, x, w["wq"], w["wk"], w["wv"], w["wo"], q_prev, z, z, z,
                         H, rope_base=10000.0)
    assert np.allclose(res["out"], want, atol=1e-12)
    assert np.allclose(res["k_cache"], K, atol=1e-12)
    # score and score cache use the unrotated head-0 query
    assert np.allclose(res["q_prev"], Q[:, :, :d // H], atol=1e-12)
    assert np.allclose(res["scores"], orc.drift_scores(Q[:, :, :d // H], q_prev), atol=1e-12)


def test_kv_step_with_rope_keeps_cached_keys_and_rotates_fresh_ones_by_their_position():
    r = _rng(8)
    B, T, d, H = 1, 6, 8, 2
    w = _weights(r, d)
    x0 = r.standard_normal((B, T, d))
    x1 = x0.copy()
    x1[0, [1, 4]] += r.standard_normal((2, d))           # tokens 1 and 4 change
    _, Q0, K0, V0 = _dense_with_rope(x0, w, H, 10000.0)
    _, Q1, K1, V1 = _dense_with_rope(x1, w, H, 10000.0)
    res = orc.layer_step(orc.MODE_KV, 1e-9, x1, w["wq"], w["wk"], w["wv"], w["wo"], Q0[:, :, :d // H],
                         K0, V0, np.zeros_like(x0), H, rope_base=10000.0)
    assert res["sel_idx"].tolist() == [1, 4]
    # unchanged tokens have identical rows in K0 and K1; the changed ones must be K1's,
    # i.e. rotated by positions 1 and 4 (a rotation by the row's index in the list, 0 and
    # 1, would differ)
    assert np.allclose(res["k_cache"], K1, atol=1e-12)
    assert np.allclose(res["v_cache"], V1, atol=1e-12)


@pytest.mark.parametrize("norm", ["layer", "rms", None])
def test_block_is_norm_then_layer_then_residual(norm):
    r = _rng(9)
    B, T, d, H = 1, 5, 8, 2
    w = _weights(r, d)
    x = r.standard_normal((B, T, d)) * 2 + 0.5
    g, bias = r.standard_normal(d), r.standard_normal(d)
    z = np.zeros((B, T, d))
    q_prev = np.zeros((B, T, d // H))
    res = orc.block_step(orc.MODE_DENSE, 0.0, x, norm, g, bias, 1e-5, w["wq"], w["wk"], w["wv"], w["wo"],
                         q_prev, z, z, z, H, rope_base=10000.0)
    h = {"layer": lambda: orc.layer_norm(x, g, bias, 1e-5), "rms": lambda: orc.rms_norm(x, g, 1e-5),
         None: lambda: x}[norm]()
    o, _, _, _ = _dense_with_rope(h, w, H, 10000.0)
    assert np.allclose(res["out"], o, atol=1e-12)               # the cached quantity: before the sum
    assert np.allclose(res["block_out"], x + o, atol=1e-12)


def test_block_residual_closed_forms():
    r = _rng(10)
    B, T, d, H = 1, 4, 8, 2
    w = _weights(r, d)
    x = r.standard_normal((B, T, d))
    z = np.zeros((B, T, d))
    qp = np.zeros((B, T, d // H))
    # Wo = 0: the block returns its input
    res = orc.block_step(orc.MODE_DENSE, 0.0, x, "rms", np.ones(d), None, 1e-5, w["wq"], w["wk"], w["wv"],
                         np.zeros((d, d)), qp, z, z, z, H)
    assert np.array_equal(res["block_out"], x)
    # reuse everything in O mode: current hidden state plus the cached block output
    cache = r.standard_normal((B, T, d))
    res = orc.block_step(orc.MODE_O, 2.5, x, "rms", np.ones(d), None, 1e-5, w["wq"], w["wk"], w["wv"],
                         w["wo"], r.standard_normal((B, T, d // H)), z, z, cache, H, rope_base=10000.0)
    assert res["reuse_mask"].all()
    assert np.array_equal(res["block_out"], x + cache)
    # without the residual sum the block output is the layer output
    res2 = orc.block_step(orc.MODE_O, 2.5, x, "rms", np.ones(d), None, 1e-5, w["wq"], w["wk"], w["wv"],
                          w["wo"], r.standard_normal((B, T, d // H)), z, z, cache, H, residual=False)
    assert np.array_equal(res2["block_out"], cache)


def test_block_storage_model_rounds_the_normalised_state():
    r = _rng(11)
    B, T, d, H = 1, 4, 8, 2
    w = _weights(r, d)
    x = r.standard_normal((B, T, d))
    z = np.zeros((B, T, d))
    res = orc.block_step(orc.MODE_DENSE, 0.0, x, "rms", np.ones(d), None, 1e-5, w["wq"], w["wk"], w["wv"],
                         w["wo"], np.zeros((B, T, d // H)), z, z, z, H, storage="bf16")
    h = res["h"]
    assert np.array_equal(h, orc.round_storage(h, "bf16"))
    assert not np.array_equal(h, orc.rms_norm(x, np.ones(d), 1e-5))
    assert np.array_equal(res["block_out"], orc.round_storage(res["exact"]["block_out"], "bf16"))
