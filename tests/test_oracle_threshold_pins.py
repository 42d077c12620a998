"""Pins for the oracle's threshold machinery (Sec. 3.1 "Reuse rate allocation", the
schedule of Sec. 5): the quantile threshold against numpy's order-statistic quantile and
a counting definition, the layer-wise allocation against scipy's softmax and the
properties the formula has, the schedule against its statement."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import dare_oracle as orc


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


@pytest.mark.parametrize("phi", [0.01, 0.2, 0.3, 0.5, 0.87, 1.0])
def test_quantile_threshold_is_numpys_inverted_cdf_quantile(phi):
    s = _rng(1).random((3, 257)).astype(np.float32)
    want = np.quantile(s.astype(np.float64), float(np.float32(phi)), axis=1, method="inverted_cdf")
    assert np.array_equal(orc.quantile_threshold(s, phi), want.astype(np.float32))


@pytest.mark.parametrize("T,phi", [(1, 0.3), (1, 1.0), (7, 0.5), (128, 0.3), (100, 0.25), (64, 0.999)])
def test_quantile_threshold_counting_definition(T, phi):
    # tau is the smallest score with at least ceil(phi T) scores <= it
    s = _rng(T).standard_normal((4, T)).astype(np.float32)
    tau = orc.quantile_threshold(s, phi)
    k = int(np.ceil(np.float32(phi) * np.float32(T)))
    for b in range(4):
        assert (s[b] <= tau[b]).sum() >= k
        assert (s[b] < tau[b]).sum() < k
        assert tau[b] in s[b]
        assert orc.reuse_decision(s[b], tau[b]).sum() == k        # distinct scores: exactly k reused


@pytest.mark.parametrize("phi,T,k", [(0.3, 40, 12), (0.25, 100, 25), (0.7, 10, 7), (0.1, 1000, 100),
                                     (0.301, 1000, 301), (0.3001, 40, 13), (1.0, 33, 33)])
def test_quantile_rank_of_decimal_rates(phi, T, k):
    # the rank is the count a person expects from the decimal rate
    s = np.arange(T, dtype=np.float32)[None, ::-1].copy()
    assert orc.quantile_threshold(s, phi)[0] == np.float32(k - 1)


def test_quantile_threshold_edge_cases():
    s = np.array([[0.3, 0.1, 0.1, 0.2]], dtype=np.float32)
    assert orc.quantile_threshold(s, 0.0)[0] == -np.inf
    assert not orc.reuse_decision(s[0], -np.inf).any()            # phi = 0 reuses nothing
    assert orc.quantile_threshold(s, 0.25)[0] == np.float32(0.1)
    assert orc.reuse_decision(s[0], np.float32(0.1)).sum() == 2   # a tie at the threshold is reused too
    assert orc.quantile_threshold(s, 1.0)[0] == np.float32(0.3)
    with pytest.raises(ValueError):
        orc.quantile_threshold(s, 1.5)
    # NaN sorts last, is never reused, and never becomes the threshold
    n = np.array([[0.2, np.nan, 0.1, np.nan]], dtype=np.float32)
    assert orc.quantile_threshold(n, 0.5)[0] == np.float32(0.2)
    assert orc.quantile_threshold(n, 1.0)[0] == np.inf
    assert orc.reuse_decision(n[0], np.inf).tolist() == [True, False, True, False]
    # negative scores (cosine a rounding above 1) order below the positive ones
    m = np.array([[1e-8, -2e-8, 0.0, 0.5]], dtype=np.float32)
    assert orc.quantile_threshold(m, 0.25)[0] == np.float32(-2e-8)


def test_quantile_threshold_is_per_sequence_and_monotone_in_phi():
    s = _rng(5).random((2, 50)).astype(np.float32)
    both = orc.quantile_threshold(s, 0.4)
    assert both[0] == orc.quantile_threshold(s[:1], 0.4)[0]
    assert both[1] == orc.quantile_threshold(s[1:], 0.4)[0]
    taus = [orc.quantile_threshold(s, p)[0] for p in (0.1, 0.3, 0.3001, 0.9)]
    assert taus == sorted(taus)


def test_layer_step_with_a_quantile_reuses_that_fraction():
    r = _rng(9)
    B, T, d, H = 2, 40, 16, 2
    x = r.standard_normal((B, T, d))
    w = [r.standard_normal((d, d)) * 0.3 for _ in range(4)]
    z = np.zeros((B, T, d))
    qp = r.standard_normal((B, T, d // H))
    res = orc.layer_step(orc.MODE_KVO, 0.3, x, *w, qp, z, z, z, H, quantile=True)
    assert res["reuse_mask"].sum(axis=1).tolist() == [12, 12]
    fixed = orc.layer_step(orc.MODE_KVO, float(res["tau"][0]), x[:1], *w, qp[:1], z[:1], z[:1], z[:1], H)
    assert np.array_equal(fixed["reuse_mask"], res["reuse_mask"][:1])
    assert np.allclose(fixed["out"], res["out"][:1], rtol=0, atol=1e-12)


def test_allocate_quantiles_matches_library_softmax_and_budget():
    s = _rng(2).random(32) * 0.2
    phi = orc.allocate_quantiles(s, 0.3, 0.05)
    assert np.allclose(phi, 32 * 0.3 * softmax(-s / 0.05), rtol=1e-12)
    assert abs(phi.sum() - 32 * 0.3) < 1e-9                      # the budget L * phi_bar is spent exactly
    order = np.argsort(s)
    assert np.all(np.diff(phi[order]) <= 0)                      # less drift, larger share


def test_allocate_quantiles_limits():
    s = np.array([0.01, 0.2, 0.05, 0.11])
    assert np.allclose(orc.allocate_quantiles(np.full(5, 0.07), 0.4, 0.01), 0.4)   # equal drift: uniform
    assert np.allclose(orc.allocate_quantiles(s, 0.25, 1e9), 0.25, atol=1e-9)        # high temperature: uniform
    cold = orc.allocate_quantiles(s, 0.2, 1e-4)                                      # low temperature: winner takes all,
    assert np.allclose(cold, [0.8, 0, 0, 0], atol=1e-12)                             # L * phi_bar = 0.8 on the calmest layer
    assert np.all(orc.allocate_quantiles(s, 0.9, 1e-4) <= 1.0)                       # cut at 1
    assert orc.allocate_quantiles(s, 0.9, 1e-4)[0] == 1.0
    a = orc.allocate_quantiles(s, 0.3, 0.05)
    assert np.allclose(orc.allocate_quantiles(s + 3.0, 0.3, 0.05), a)                # a common shift cancels in the softmax


def test_policy_mode_schedule():
    M = orc.MODE_KVO
    assert [orc.policy_mode(M, l, 3, skip_layers=10) for l in (0, 9, 10, 31)] == [0, 0, M, M]
    assert [orc.policy_mode(M, 12, t, refresh_interval=2) for t in range(5)] == [0, M, 0, M, 0]
    assert [orc.policy_mode(M, 12, t) for t in range(3)] == [M, M, M]
    assert orc.policy_mode(orc.MODE_O, 3, 1, skip_layers=10, refresh_interval=2) == orc.MODE_DENSE


# ---- frozen prefix (prefix caching) ---------------------------------------------------------

def _prefix_case(seed=11, B=2, T=24, d=16, H=2, P=9):
    r = _rng(seed)
    w = [r.standard_normal((d, d)) * 0.3 for _ in range(4)]
    x_prev = r.standard_normal((B, T, d))
    x = x_prev + 0.4 * r.standard_normal((B, T, d))
    out, Q, K, V = orc.dense_layer(x_prev, *w, H)
    state = (Q[:, :, :d // H].copy(), K, V, out)
    return w, x, state, H, P


def _loops_attention_row(q, K, V, H):
    """One query row against all keys, scalar loops (second formulation of App. E.2)."""
    d = len(q)
    dh = d // H
    o = np.zeros(d)
    for h in range(H):
        z = [sum(q[h * dh + c] * K[j][h * dh + c] for c in range(dh)) / np.sqrt(dh) for j in range(len(K))]
        m = max(z)
        wgt = [np.exp(v - m) for v in z]
        for c in range(dh):
            o[h * dh + c] = sum(wgt[j] * V[j][h * dh + c] for j in range(len(K))) / sum(wgt)
    return o


@pytest.mark.parametrize("mode", [orc.MODE_DENSE, orc.MODE_KV, orc.MODE_O, orc.MODE_KVO])
def test_frozen_prefix_rows_are_untouched_and_never_scored(mode):
    w, x, (qp, K, V, O), H, P = _prefix_case()
    r = orc.layer_step(mode, 0.05, x, *w, qp, K, V, O, H, prefix=P)
    assert r["reuse_mask"][:, :P].all() and (r["scores"][:, :P] == 0).all()
    assert np.array_equal(r["q_prev"][:, :P], qp[:, :P])
    assert np.array_equal(r["k_cache"][:, :P], K[:, :P]) and np.array_equal(r["v_cache"][:, :P], V[:, :P])
    assert np.array_equal(r["out"][:, :P], O[:, :P])
    assert (r["sel_idx"] % x.shape[1] >= P).all()
    if mode == orc.MODE_DENSE:
        assert (r["reuse_mask"][:, P:] == 0).all()
        assert r["sel_count"].tolist() == [x.shape[1] - P] * x.shape[0]


@pytest.mark.parametrize("mode", [orc.MODE_DENSE, orc.MODE_KV, orc.MODE_O, orc.MODE_KVO])
def test_frozen_prefix_active_rows_by_scalar_loops(mode):
    # the rows that are not frozen, recomputed with scalar loops from the K/V the step must see
    w, x, (qp, K, V, O), H, P = _prefix_case(B=1, T=10, d=8, P=4)
    wq, wk, wv, wo = w
    tau = 0.05
    r = orc.layer_step(mode, tau, x, *w, qp, K, V, O, H, prefix=P)
    T = x.shape[1]
    refreshed = [i for i in range(P, T) if mode == orc.MODE_DENSE or r["scores"][0, i] > np.float32(tau)]
    kv_rows = refreshed if mode in (orc.MODE_KV, orc.MODE_KVO) else list(range(P, T))
    Kx, Vx = K[0].copy(), V[0].copy()
    for i in kv_rows:
        Kx[i], Vx[i] = x[0, i] @ wk, x[0, i] @ wv
    assert np.allclose(r["k_cache"][0], Kx, atol=1e-12) and np.allclose(r["v_cache"][0], Vx, atol=1e-12)
    q_rows = refreshed if mode in (orc.MODE_O, orc.MODE_KVO) else list(range(P, T))
    for i in range(T):
        want = _loops_attention_row(x[0, i] @ wq, Kx, Vx, H) @ wo if i in q_rows else O[0, i]
        assert np.allclose(r["out"][0, i], want, atol=1e-10), i


def test_frozen_prefix_equals_forcing_a_zero_score():
    # without the prefix argument: give the frozen tokens a previous query equal to the current
    # one, so that they score exactly 0 and tau = 0 reuses them; the refreshed rows must agree
    w, x, (qp, K, V, O), H, P = _prefix_case()
    q_now = (x @ w[0])[:, :, :qp.shape[2]]
    qp2 = qp.copy()
    qp2[:, :P] = q_now[:, :P]
    a = orc.layer_step(orc.MODE_KVO, 0.0, x, *w, qp2, K, V, O, H)
    b = orc.layer_step(orc.MODE_KVO, 0.0, x, *w, qp, K, V, O, H, prefix=P)
    assert np.array_equal(a["reuse_mask"], b["reuse_mask"]) and np.array_equal(a["sel_idx"], b["sel_idx"])
    for k in ("out", "k_cache", "v_cache"):
        assert np.allclose(a[k], b[k], atol=1e-12), k


def test_frozen_prefix_quantile_ranks_only_the_other_tokens():
    w, x, (qp, K, V, O), H, P = _prefix_case(T=29, P=9)
    r = orc.layer_step(orc.MODE_KVO, 0.5, x, *w, qp, K, V, O, H, quantile=True, prefix=P)
    assert (r["reuse_mask"][:, P:].sum(axis=1) == 10).all()           # ceil(0.5 * 20) of the 20 others
    assert np.array_equal(r["tau"], np.sort(r["scores"][:, P:].astype(np.float32), axis=1)[:, 9])


def test_frozen_prefix_of_zero_is_the_plain_step_and_bad_values_raise():
    w, x, (qp, K, V, O), H, P = _prefix_case()
    a = orc.layer_step(orc.MODE_KV, 0.05, x, *w, qp, K, V, O, H)
    b = orc.layer_step(orc.MODE_KV, 0.05, x, *w, qp, K, V, O, H, prefix=0)
    assert all(np.array_equal(a[k], b[k]) for k in ("out", "k_cache", "reuse_mask", "q_prev"))
    with pytest.raises(ValueError):
        orc.layer_step(orc.MODE_KV, 0.05, x, *w, qp, K, V, O, H, prefix=x.shape[1])
