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
