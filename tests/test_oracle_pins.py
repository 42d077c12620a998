"""Pins for the CPU oracle: it is checked against things other than itself.

The paper prints no worked numeric example for the layer (no score, mask or
activation value appears anywhere), so the pins are: a brute-force version in
Python scalar loops, closed forms, hand-computed values, and the invariants the
paper states (Sec. 3.2 eq. 2; Sec. 4: threshold that reuses nothing leaves no
reuse error; Alg. 1 lines 8-9 and Alg. 2 lines 9-10: reused rows are the cached
rows)."""
import math

import numpy as np
import pytest

from oracle import dare_oracle as orc


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _case(seed, B=1, T=6, d=8, H=2, wstd=0.5):
    r = _rng(seed)
    w = {k: r.standard_normal((d, d)) * wstd for k in ("wq", "wk", "wv", "wo")}
    x0 = r.standard_normal((B, T, d))
    x1 = x0 + r.standard_normal((B, T, d)) * np.where(r.random((B, T, 1)) < 0.4, 0.7, 0.01)
    return w, x0, x1, H


def _fill(w, x0, H):
    """State after a dense step on x0."""
    out, Q, K, V = orc.dense_layer(x0, w["wq"], w["wk"], w["wv"], w["wo"], H)
    dh = x0.shape[2] // H
    return dict(q_prev=Q[:, :, :dh].copy(), k_cache=K, v_cache=V, o_cache=out)


def _step(mode, tau, w, x, st, H, **kw):
    return orc.layer_step(mode, tau, x, w["wq"], w["wk"], w["wv"], w["wo"],
                          st["q_prev"], st["k_cache"], st["v_cache"], st["o_cache"], H, **kw)


# ----------------------------------------------------------------------------
# dense attention against an independent scalar-loop version (App. E.2)
# ----------------------------------------------------------------------------
def _brute_dense(x, wq, wk, wv, wo, H):
    T, d = len(x), len(x[0])
    dh = d // H

    def matvec(row, w):
        return [sum(row[k] * w[k][j] for k in range(d)) for j in range(d)]

    Q = [matvec(r, wq) for r in x]
    K = [matvec(r, wk) for r in x]
    V = [matvec(r, wv) for r in x]
    out = []
    for i in range(T):
        cat = [0.0] * d
        for h in range(H):
            lo = h * dh
            logits = [sum(Q[i][lo + c] * K[j][lo + c] for c in range(dh)) / math.sqrt(dh)
                      for j in range(T)]
            big = max(logits)
            e = [math.exp(z - big) for z in logits]
            tot = sum(e)
            for c in range(dh):
                cat[lo + c] = sum(e[j] / tot * V[j][lo + c] for j in range(T))
        out.append(matvec(cat, wo))
    return out


@pytest.mark.parametrize("T,d,H", [(5, 6, 1), (7, 8, 2), (4, 12, 3)])
def test_dense_matches_scalar_loops(T, d, H):
    r = _rng(11 + T)
    x = r.standard_normal((1, T, d))
    ws = [r.standard_normal((d, d)) * 0.6 for _ in range(4)]
    ref = np.array(_brute_dense(x[0].tolist(), *[w.tolist() for w in ws], H))
    got, _, _, _ = orc.dense_layer(x, *ws, H)
    assert np.max(np.abs(got[0] - ref)) < 1e-12


def test_dense_hand_value_two_tokens():
    # d = Dh = 2, one head, identity Wq/Wk/Wv/Wo.  Token 0 = (1,0), token 1 = (0,1).
    # Query 0: logits (1/sqrt2, 0) -> weights (a, 1-a), a = 1/(1+exp(-1/sqrt2)).
    I = np.eye(2)
    x = np.array([[[1.0, 0.0], [0.0, 1.0]]])
    out, _, _, _ = orc.dense_layer(x, I, I, I, I, 1)
    a = 1.0 / (1.0 + math.exp(-1.0 / math.sqrt(2.0)))
    assert np.allclose(out[0, 0], [a, 1 - a], atol=1e-15)
    assert np.allclose(out[0, 1], [1 - a, a], atol=1e-15)


def test_dense_scale_uses_head_dim_not_hidden():
    # Same tokens placed in head 1 of a 2-head layer (d = 4, Dh = 2): the weights
    # must still be those of scale 1/sqrt(2), not 1/sqrt(4).
    I = np.eye(4)
    x = np.array([[[0, 0, 1.0, 0.0], [0, 0, 0.0, 1.0]]])
    out, _, _, _ = orc.dense_layer(x, I, I, I, I, 2)
    a = 1.0 / (1.0 + math.exp(-1.0 / math.sqrt(2.0)))
    assert np.allclose(out[0, 0, 2:], [a, 1 - a], atol=1e-15)
    # head 0 has all-zero queries and keys: uniform weights over zero values
    assert np.allclose(out[0, :, :2], 0.0)


def test_dense_closed_forms():
    r = _rng(3)
    d, H = 8, 2
    wq, wk, wv, wo = (r.standard_normal((d, d)) for _ in range(4))
    # one token: softmax over a single key is 1
    x = r.standard_normal((1, 1, d))
    out, _, _, _ = orc.dense_layer(x, wq, wk, wv, wo, H)
    assert np.allclose(out[0, 0], x[0, 0] @ wv @ wo, rtol=1e-12, atol=1e-12)
    # Wq = 0: uniform attention -> mean of the value rows
    x = r.standard_normal((1, 5, d))
    out, _, _, _ = orc.dense_layer(x, np.zeros((d, d)), wk, wv, wo, H)
    want = (x[0] @ wv).mean(axis=0) @ wo
    assert np.allclose(out[0], np.tile(want, (5, 1)), rtol=1e-12, atol=1e-12)
    # all value rows equal: output is that row times Wo whatever Q and K are
    q = r.standard_normal((4, d))
    k = r.standard_normal((6, d))
    v = np.tile(r.standard_normal((1, d)), (6, 1))
    assert np.allclose(orc.attention_rows(q, k, v, H), np.tile(v[0], (4, 1)), atol=1e-13)


def test_attention_is_bidirectional_and_per_head():
    r = _rng(5)
    d, H, T = 8, 2, 6
    q, k, v = (r.standard_normal((T, d)) for _ in range(3))
    base = orc.attention_rows(q, k, v, H)
    # a change in the LAST key/value moves the FIRST query's output: no causal mask
    k2, v2 = k.copy(), v.copy()
    k2[-1] += 1.0
    v2[-1] += 1.0
    assert np.max(np.abs(orc.attention_rows(q, k2, v2, H)[0] - base[0])) > 1e-3
    # a change confined to head 1's columns leaves head 0's output untouched
    k3 = k.copy()
    k3[2, d // H:] += 1.0
    got = orc.attention_rows(q, k3, v, H)
    assert np.array_equal(got[:, :d // H], base[:, :d // H])
    assert np.max(np.abs(got[:, d // H:] - base[:, d // H:])) > 1e-3
    # large logits do not overflow
    big = orc.attention_rows(q * 1e3, k * 1e3, v, H)
    assert np.all(np.isfinite(big))


# ----------------------------------------------------------------------------
# drift score (Sec. 3.1 eq. 1)
# ----------------------------------------------------------------------------
def test_score_hand_values():
    s = orc.drift_scores
    assert s([1.0, 0.0], [1.0, 1.0]) == pytest.approx(1 - 1 / math.sqrt(2), abs=1e-15)
    assert s([3.0, 4.0], [4.0, 3.0]) == pytest.approx(1 - 24.0 / 25.0, abs=1e-15)
    assert s([1.0, 2.0, 2.0], [2.0, 4.0, 4.0]) == pytest.approx(0.0, abs=1e-15)
    assert s([1.0, 2.0, 2.0], [-1.0, -2.0, -2.0]) == pytest.approx(2.0, abs=1e-15)
    assert s([1.0, 0.0], [0.0, 5.0]) == pytest.approx(1.0, abs=1e-15)
    # zero-norm query: cosine taken as 0
    assert s([0.0, 0.0], [1.0, 2.0]) == 1.0


def test_score_invariants():
    r = _rng(7)
    q = r.standard_normal((50, 16))
    p = r.standard_normal((50, 16))
    s = orc.drift_scores(q, p)
    assert s.shape == (50,)
    assert np.all(s >= -1e-15) and np.all(s <= 2 + 1e-15)
    assert np.allclose(orc.drift_scores(p, q), s, atol=1e-15)            # symmetric
    assert np.allclose(orc.drift_scores(3.7 * q, 0.01 * p), s, atol=1e-14)  # scale free
    assert np.allclose(orc.drift_scores(-q, p), 2.0 - s, atol=1e-14)
    assert np.all(orc.drift_scores(q, q) == 0.0)                          # exact zero
    # row-wise: against a scalar loop
    for i in (0, 17, 49):
        dot = sum(a * b for a, b in zip(q[i], p[i]))
        ref = 1 - dot / math.sqrt(sum(a * a for a in q[i]) * sum(b * b for b in p[i]))
        assert s[i] == pytest.approx(ref, abs=1e-14)


def test_score_uses_head0_of_query_only():
    w, x0, x1, H = _case(21, T=9, d=12, H=3)
    st = _fill(w, x0, H)
    dh = 12 // H
    base = _step(orc.MODE_KV, 0.1, w, x1, st, H)
    # definition on head 0, from separately computed queries
    q1 = (x1 @ w["wq"])[:, :, :dh]
    q0 = (x0 @ w["wq"])[:, :, :dh]
    assert np.allclose(base["scores"], orc.drift_scores(q1, q0), atol=1e-14)
    # columns of Wq outside head 0 do not matter to the scores
    w2 = dict(w)
    w2["wq"] = w["wq"].copy()
    w2["wq"][:, dh:] *= -3.0
    st2 = dict(st)
    assert np.array_equal(_step(orc.MODE_KV, 0.1, w2, x1, st2, H)["scores"], base["scores"])
    # columns inside head 0 do
    w3 = dict(w)
    w3["wq"] = w["wq"].copy()
    w3["wq"][:, 0] += 1.0
    assert not np.allclose(_step(orc.MODE_KV, 0.1, w3, x1, st, H)["scores"], base["scores"])
    # the stored previous query becomes this step's head 0, for every token
    assert np.allclose(base["q_prev"], q1, atol=1e-14)
    # whole-vector scoring variant
    st_full = dict(st)
    st_full["q_prev"] = x0 @ w["wq"]
    full = _step(orc.MODE_KV, 0.1, w, x1, st_full, H, score_head=-1)
    assert np.allclose(full["scores"], orc.drift_scores(x1 @ w["wq"], x0 @ w["wq"]), atol=1e-14)


# ----------------------------------------------------------------------------
# reuse set, mask, index list (Sec. 3.2 eq. 2; Alg. 1/2 lines 4-5)
# ----------------------------------------------------------------------------
def test_threshold_rule_and_lists():
    s = np.array([[0.0, 0.25, 0.5, 0.75], [1.0, 0.5, np.nan, 0.1]])
    reuse = orc.reuse_decision(s, 0.5)
    assert reuse.tolist() == [[True, True, True, False], [False, True, False, True]]
    idx, cnt, off = orc.selection(reuse)
    assert idx.tolist() == [3, 4, 6] and idx.dtype == np.int32
    assert cnt.tolist() == [1, 2] and off.tolist() == [0, 1, 3]
    # decision happens in float32: a score above tau by less than half an ulp(f32) ties
    tau = np.float32(0.3)
    assert orc.reuse_decision(np.array([float(tau) + 1e-12]), tau)[0]
    assert not orc.reuse_decision(np.array([float(tau) + 1e-6]), tau)[0]


@pytest.mark.parametrize("mode", [orc.MODE_KV, orc.MODE_O, orc.MODE_KVO])
def test_mask_counts_and_monotone(mode):
    w, x0, x1, H = _case(31, B=3, T=17, d=8, H=2)
    st = _fill(w, x0, H)
    prev = None
    s_all = None
    for tau in (-1.0, 0.0, 1e-4, 1e-2, 0.3, 2.5):
        o = _step(mode, tau, w, x1, st, H)
        s_all = o["scores"]
        mask = o["reuse_mask"]
        assert mask.dtype == np.uint8 and mask.shape == (3, 17)
        assert int(mask.sum()) == int(np.sum(s_all.astype(np.float32) <= np.float32(tau)))
        comp = sorted(b * 17 + i for b in range(3) for i in range(17) if not mask[b, i])
        assert o["sel_idx"].tolist() == comp
        assert np.array_equal(o["sel_count"] + mask.sum(axis=1), np.full(3, 17))
        assert o["sel_off"].tolist() == [0] + np.cumsum(o["sel_count"]).tolist()
        if prev is not None:
            assert np.all(mask >= prev)        # R(tau1) subset of R(tau2)
        prev = mask
    assert prev.all()                           # tau = 2.5 reuses everything


def test_dense_mode_mask_is_zero_and_scores_still_reported():
    w, x0, x1, H = _case(33)
    st = _fill(w, x0, H)
    o = _step(orc.MODE_DENSE, 2.5, w, x1, st, H)
    assert not o["reuse_mask"].any()
    assert o["sel_idx"].tolist() == list(range(6))
    assert np.all(o["scores"] > 0)


# ----------------------------------------------------------------------------
# reuse nothing == dense; reuse everything == cached state
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("mode", [orc.MODE_KV, orc.MODE_O, orc.MODE_KVO])
def test_reuse_nothing_equals_dense(mode):
    w, x0, x1, H = _case(41, B=2, T=9)
    st = _fill(w, x0, H)
    # poison the caches: nothing of them may leak into the result
    st = {k: (v + 100.0 if k != "q_prev" else v) for k, v in st.items()}
    o = _step(mode, -1.0, w, x1, st, H)
    ref, Q, K, V = orc.dense_layer(x1, w["wq"], w["wk"], w["wv"], w["wo"], H)
    assert not o["reuse_mask"].any()
    for got, want in ((o["out"], ref), (o["o_cache"], ref), (o["k_cache"], K), (o["v_cache"], V)):
        assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    d = _step(orc.MODE_DENSE, 0.7, w, x1, st, H)
    assert np.allclose(d["out"], ref, rtol=1e-12, atol=1e-12)
    assert np.allclose(d["k_cache"], K, rtol=1e-12, atol=1e-12)


def test_reuse_everything():
    w, x0, x1, H = _case(43, B=2, T=9)
    st = _fill(w, x0, H)
    # make the caches recognisable (not equal to anything recomputable)
    r = _rng(99)
    st = dict(st, k_cache=r.standard_normal(st["k_cache"].shape),
              v_cache=r.standard_normal(st["v_cache"].shape),
              o_cache=r.standard_normal(st["o_cache"].shape))
    for mode in (orc.MODE_O, orc.MODE_KVO):
        o = _step(mode, 2.5, w, x1, st, H)
        assert o["reuse_mask"].all() and o["sel_idx"].size == 0
        assert np.array_equal(o["out"], st["o_cache"])            # bit for bit
        assert np.array_equal(o["o_cache"], st["o_cache"])
    o = _step(orc.MODE_KVO, 2.5, w, x1, st, H)
    assert np.array_equal(o["k_cache"], st["k_cache"]) and np.array_equal(o["v_cache"], st["v_cache"])
    # O mode alone recomputes K, V densely
    o = _step(orc.MODE_O, 2.5, w, x1, st, H)
    assert np.allclose(o["k_cache"], x1 @ w["wk"], atol=1e-12)
    # KV mode with everything reused: fresh queries against the cached K, V
    o = _step(orc.MODE_KV, 2.5, w, x1, st, H)
    assert np.array_equal(o["k_cache"], st["k_cache"])
    Q = x1 @ w["wq"]
    for b in range(2):
        want = orc.attention_rows(Q[b], st["k_cache"][b], st["v_cache"][b], H) @ w["wo"]
        assert np.allclose(o["out"][b], want, rtol=1e-12, atol=1e-12)
    # the score cache is replaced even when every token is reused
    assert np.allclose(o["q_prev"], Q[:, :, :8 // H], atol=1e-14)


# ----------------------------------------------------------------------------
# general threshold: each mode composed from the dense definition only
# ----------------------------------------------------------------------------
def _mid_tau(scores):
    s = np.sort(scores.reshape(-1))
    return 0.5 * (s[len(s) // 2 - 1] + s[len(s) // 2])


def test_kv_mode_is_dense_attention_on_mixed_inputs():
    w, x0, x1, H = _case(51, B=2, T=10)
    st = _fill(w, x0, H)
    tau = _mid_tau(_step(orc.MODE_KV, 0.0, w, x1, st, H)["scores"])
    o = _step(orc.MODE_KV, tau, w, x1, st, H)
    mask = o["reuse_mask"].astype(bool)
    assert 0 < mask.sum() < mask.size
    # K, V rows come from x1 where refreshed and from x0 where reused
    x_mix = np.where(mask[:, :, None], x0, x1)
    assert np.allclose(o["k_cache"], x_mix @ w["wk"], atol=1e-12)
    assert np.allclose(o["v_cache"], x_mix @ w["wv"], atol=1e-12)
    assert np.array_equal(o["k_cache"][mask], st["k_cache"][mask])    # cached rows bit for bit
    Q = x1 @ w["wq"]
    for b in range(2):
        want = orc.attention_rows(Q[b], x_mix[b] @ w["wk"], x_mix[b] @ w["wv"], H) @ w["wo"]
        assert np.allclose(o["out"][b], want, rtol=1e-11, atol=1e-12)


def test_o_mode_rows():
    w, x0, x1, H = _case(53, B=2, T=10)
    st = _fill(w, x0, H)
    tau = _mid_tau(_step(orc.MODE_O, 0.0, w, x1, st, H)["scores"])
    o = _step(orc.MODE_O, tau, w, x1, st, H)
    mask = o["reuse_mask"].astype(bool)
    assert 0 < mask.sum() < mask.size
    dense, _, K, V = orc.dense_layer(x1, w["wq"], w["wk"], w["wv"], w["wo"], H)
    assert np.allclose(o["out"][~mask], dense[~mask], rtol=1e-11, atol=1e-12)
    assert np.array_equal(o["out"][mask], st["o_cache"][mask])
    assert np.allclose(o["k_cache"], K, atol=1e-12) and np.allclose(o["v_cache"], V, atol=1e-12)


def test_kvo_mode_rows():
    w, x0, x1, H = _case(55, B=2, T=10)
    st = _fill(w, x0, H)
    tau = _mid_tau(_step(orc.MODE_KVO, 0.0, w, x1, st, H)["scores"])
    kvo = _step(orc.MODE_KVO, tau, w, x1, st, H)
    kv = _step(orc.MODE_KV, tau, w, x1, st, H)
    mask = kvo["reuse_mask"].astype(bool)
    assert np.array_equal(kvo["reuse_mask"], kv["reuse_mask"])
    assert np.allclose(kvo["out"][~mask], kv["out"][~mask], rtol=1e-11, atol=1e-12)
    assert np.array_equal(kvo["out"][mask], st["o_cache"][mask])
    assert np.allclose(kvo["k_cache"], kv["k_cache"], atol=1e-13)


def test_prewo_and_postwo_output_caches_agree():
    # Alg. 2 as listed caches attention rows before Wo; App. E.1 caches after Wo.
    w, x0, x1, H = _case(57, B=1, T=12)
    st = _fill(w, x0, H)
    _, Q0, K0, V0 = orc.dense_layer(x0, w["wq"], w["wk"], w["wv"], w["wo"], H)
    attn0 = orc.attention_rows(Q0[0], K0[0], V0[0], H)[None]
    assert np.allclose(attn0 @ w["wo"], st["o_cache"], atol=1e-12)
    tau = _mid_tau(_step(orc.MODE_O, 0.0, w, x1, st, H)["scores"])
    post = _step(orc.MODE_O, tau, w, x1, st, H)
    pre_out, _, pre_mask = orc.step_o_prewo(tau, x1, w["wq"], w["wk"], w["wv"], w["wo"],
                                            st["q_prev"], attn0, H)
    assert np.array_equal(pre_mask, post["reuse_mask"])
    assert np.allclose(pre_out, post["out"], rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("mode", [orc.MODE_DENSE, orc.MODE_KV, orc.MODE_O, orc.MODE_KVO])
def test_token_permutation_equivariance(mode):
    # no positional term in the layer: permuting tokens permutes everything
    w, x0, x1, H = _case(61, B=1, T=11)
    st = _fill(w, x0, H)
    tau = _mid_tau(_step(orc.MODE_KV, 0.0, w, x1, st, H)["scores"])
    a = _step(mode, tau, w, x1, st, H)
    perm = _rng(5).permutation(11)
    stp = {k: v[:, perm] for k, v in st.items()}
    b = _step(mode, tau, w, x1[:, perm], stp, H)
    assert np.array_equal(a["reuse_mask"][:, perm], b["reuse_mask"])
    for key in ("out", "k_cache", "v_cache", "q_prev", "scores"):
        assert np.allclose(a[key][:, perm], b[key], rtol=1e-11, atol=1e-12), key
    assert sorted(perm[i] for i in b["sel_idx"]) == a["sel_idx"].tolist()


def test_sequences_are_independent():
    w, x0, x1, H = _case(63, B=3, T=7)
    st = _fill(w, x0, H)
    tau = _mid_tau(_step(orc.MODE_KVO, 0.0, w, x1, st, H)["scores"])
    full = _step(orc.MODE_KVO, tau, w, x1, st, H)
    for b in range(3):
        one = _step(orc.MODE_KVO, tau, w, x1[b:b + 1], {k: v[b:b + 1] for k, v in st.items()}, H)
        assert np.allclose(one["out"][0], full["out"][b], rtol=1e-11, atol=1e-12)
        assert np.array_equal(one["reuse_mask"][0], full["reuse_mask"][b])


def test_staleness_rows_survive_two_steps():
    # Sec. 4: a reused row is the one computed at the last step that refreshed it.
    w, x0, x1, H = _case(65, B=1, T=10)
    st0 = _fill(w, x0, H)
    s1 = _step(orc.MODE_KV, 0.0, w, x1, st0, H)["scores"]
    tau = _mid_tau(s1)
    o1 = _step(orc.MODE_KV, tau, w, x1, st0, H)
    st1 = {k: o1[k] for k in ("q_prev", "k_cache", "v_cache", "o_cache")}
    o2 = _step(orc.MODE_KV, 2.5, w, x1 * 1.0, st1, H)      # same input again: all reused
    assert np.all(o2["scores"] == 0.0) and o2["reuse_mask"].all()
    m1 = o1["reuse_mask"].astype(bool)
    assert np.array_equal(o2["k_cache"][m1], st0["k_cache"][m1])      # two steps stale


def test_reused_tokens_obey_input_drift_bound():
    # App. E.4 (bound on the input change of a reused token): with whole-vector
    # scoring, one head and rows of norm sqrt(d), a reused token satisfies
    # |x_t - x_{t-1}|^2 <= 4 d tau kappa^2 / (2 + tau (kappa^2 - 1)).
    r = _rng(71)
    d, T = 6, 200
    wq = r.standard_normal((d, d)) + 2.0 * np.eye(d)
    kappa = np.linalg.cond(wq)
    x0 = r.standard_normal((1, T, d))
    x1 = x0 + 0.15 * r.standard_normal((1, T, d))
    x0 *= math.sqrt(d) / np.linalg.norm(x0, axis=2, keepdims=True)
    x1 *= math.sqrt(d) / np.linalg.norm(x1, axis=2, keepdims=True)
    tau = 0.01
    s = orc.drift_scores(x1 @ wq, x0 @ wq)
    reuse = orc.reuse_decision(s, tau)
    assert 0 < reuse.sum() < T
    bound = 4 * d * tau * kappa ** 2 / (2 + tau * (kappa ** 2 - 1))
    diff2 = np.sum((x1 - x0) ** 2, axis=2)
    assert np.all(diff2[reuse] <= bound * (1 + 1e-9))


# ----------------------------------------------------------------------------
# bf16 storage model (the paper's runs are BF16: Sec. 5, App. A)
# ----------------------------------------------------------------------------
def test_round_storage_matches_bfloat16():
    import torch
    r = _rng(81)
    a32 = (r.standard_normal(50000) * 10.0 ** r.integers(-5, 5, 50000)).astype(np.float32)
    a32[:3] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8)]     # ties go to even
    want = torch.from_numpy(a32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.round_storage(a32.astype(np.float64), "bf16"), want)
    # one rounding from float64: 1 + 2^-8 + 2^-30 is above the tie and rounds up,
    # whereas going through float32 first would land on the tie and round down
    assert orc.round_storage(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]), "bf16")[0] == 1.0 + 2.0 ** -7
    assert orc.round_storage(np.array([0.0, -0.0, 3.0, 256.0]), "bf16").tolist() == [0.0, -0.0, 3.0, 256.0]
    x = r.standard_normal(10)
    assert orc.round_storage(x, None) is not None and np.array_equal(orc.round_storage(x, None), x)
    # idempotent
    y = orc.round_storage(x, "bf16")
    assert np.array_equal(orc.round_storage(y, "bf16"), y)
    assert np.max(np.abs(y - x) / np.abs(x)) <= 2.0 ** -8


def test_storage_model_rounds_exactly_the_named_tensors():
    w, x0, x1, H = _case(83, B=2, T=9)
    st = _fill(w, x0, H)
    st = {k: (orc.round_storage(v, "bf16") if k != "q_prev" else v) for k, v in st.items()}
    tau = _mid_tau(_step(orc.MODE_KVO, 0.0, w, x1, st, H)["scores"])
    rb = lambda a: orc.round_storage(a, "bf16")
    for mode in (orc.MODE_DENSE, orc.MODE_KV, orc.MODE_O, orc.MODE_KVO):
        o = _step(mode, tau, w, x1, st, H, storage="bf16")
        ref = _step(mode, tau, w, x1, st, H)
        assert np.array_equal(o["scores"], ref["scores"])          # score from the unrounded query
        assert np.array_equal(o["reuse_mask"], ref["reuse_mask"])
        mask = o["reuse_mask"].astype(bool)
        Q = rb(x1 @ w["wq"])
        if mode in (orc.MODE_KV, orc.MODE_KVO):
            Kx = np.where(mask[:, :, None], st["k_cache"], x1 @ w["wk"])
            Vx = np.where(mask[:, :, None], st["v_cache"], x1 @ w["wv"])
        else:
            Kx, Vx = x1 @ w["wk"], x1 @ w["wv"]
        assert np.allclose(o["exact"]["k_cache"], Kx, atol=1e-13)
        assert np.array_equal(o["k_cache"], rb(o["exact"]["k_cache"]))
        assert np.array_equal(o["v_cache"], rb(o["exact"]["v_cache"]))
        assert np.array_equal(o["out"], rb(o["exact"]["out"]))
        for b in range(2):
            attn = rb(orc.attention_rows(Q[b], rb(Kx[b]), rb(Vx[b]), H))
            want = attn @ w["wo"]
            rows = ~mask[b] if mode in (orc.MODE_O, orc.MODE_KVO) else np.ones(9, bool)
            assert np.allclose(o["exact"]["out"][b][rows], want[rows], rtol=1e-11, atol=1e-12)
            if mode in (orc.MODE_O, orc.MODE_KVO):
                assert np.array_equal(o["out"][b][~rows], st["o_cache"][b][~rows])
        # the rounded model stays close to the unrounded definition
        rms = np.sqrt(np.mean(ref["out"] ** 2))
        assert np.max(np.abs(o["out"] - ref["out"])) / rms < 6e-2
        assert np.max(np.abs(o["out"] - ref["out"])) > 0


def test_storage_model_is_exact_on_representable_data():
    # small integers: every intermediate that gets rounded is already a bf16 value
    # when attention is uniform (Wq = 0), so both models agree bit for bit
    r = _rng(85)
    d, T, H = 4, 4, 1
    wk = r.integers(-2, 3, (d, d)).astype(float)
    wv = r.integers(-2, 3, (d, d)).astype(float)
    wo = np.eye(d)
    x = r.integers(-2, 3, (1, T, d)).astype(float) * 4.0      # sums of 4 values stay multiples of 1
    z = np.zeros((1, T, d))
    st = dict(q_prev=np.ones((1, T, d)), k_cache=z, v_cache=z, o_cache=z)
    a = orc.layer_step(orc.MODE_DENSE, 0.0, x, np.zeros((d, d)), wk, wv, wo, **st, n_heads=H)
    b = orc.layer_step(orc.MODE_DENSE, 0.0, x, np.zeros((d, d)), wk, wv, wo, **st, n_heads=H, storage="bf16")
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["k_cache"], b["k_cache"])
