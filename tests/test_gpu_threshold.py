"""GPU parity of the threshold machinery (Sec. 3.1 "Reuse rate allocation"): the radix
select against the oracle's order statistic (bit-exact on the same scores), the step
under the quantile rule, and the running drift statistics.

The quantile threshold equals one of the scores, so the token that supplies it always
lies inside the 1e-6 band in which the two sides' scores may differ.  The step tests
therefore check (i) tau and the mask bit for bit against the oracle's rule applied to the
GPU's own scores, (ii) tau against the oracle's tau within the band, and (iii) the
outputs against an oracle step run with a fixed threshold placed in the gap above the
k-th smallest score, which takes the same decisions on both sides."""
import numpy as np
import pytest
import torch

from oracle import dare_oracle as orc
from paper_2605_08134_amd import synth
import parity_util as pu
from parity_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2605_08134_amd import binding
    binding.lib()
    return binding


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _select(B, s, phi, force=False, stats=False):
    sd = dev(s)
    mask = torch.full(s.shape, 7, dtype=torch.uint8, device="cuda")
    tau = torch.full((s.shape[0],), 123.0, dtype=torch.float32, device="cuda")
    ssum = torch.zeros(s.shape[0], dtype=torch.float64, device="cuda") if stats else None   # one slot per sequence
    scnt = torch.zeros(s.shape[0], dtype=torch.int64, device="cuda") if stats else None
    B.dare_k_quantile_mask(sd, phi, mask, tau, force, ssum, scnt)
    torch.cuda.synchronize()
    return host(tau), host(mask), (None if not stats else (host(ssum), host(scnt)))


@pytest.mark.parametrize("batch,seq", [(1, 1), (3, 7), (2, 1024), (5, 1000), (2, 5000), (8, 2048)])
@pytest.mark.parametrize("phi", [0.0, 0.001, 0.3, 0.5, 0.87, 1.0])
def test_radix_select_matches_order_statistic(B, batch, seq, phi):
    r = _rng(batch * seq)
    # drift-like values: a cluster near 0 (with exact ties and a few tiny negatives), a spread mode
    s = np.where(r.random((batch, seq)) < 0.7, r.random((batch, seq)) * 1e-4, 0.05 + r.random((batch, seq)) * 0.2)
    s = s.astype(np.float32)
    s[r.random((batch, seq)) < 0.05] = 0.0
    s[r.random((batch, seq)) < 0.02] *= -1e-3
    tau, mask, _ = _select(B, s, phi)
    want = orc.quantile_threshold(s, phi)
    assert np.array_equal(tau, want)
    for b in range(batch):
        assert np.array_equal(mask[b].astype(bool), orc.reuse_decision(s[b], want[b]))


def test_radix_select_special_values(B):
    s = np.array([[0.2, np.nan, -0.0, 0.0, -np.nan, 1e-38, -1e-38, np.inf, 2.0, -1.0]], dtype=np.float32)
    for phi in (0.1, 0.3, 0.5, 0.8, 0.9, 1.0):
        tau, mask, _ = _select(B, s, phi)
        want = orc.quantile_threshold(s, phi)
        assert np.array_equal(tau, want), (phi, tau, want)
        assert np.array_equal(mask[0].astype(bool), orc.reuse_decision(s[0], want[0]))
    tau, mask, _ = _select(B, s, 1.0)
    assert tau[0] == np.inf and mask[0].tolist() == [1, 0, 1, 1, 0, 1, 1, 1, 1, 1]


def test_radix_select_force_refresh_and_statistics(B):
    r = _rng(3)
    s = r.random((4, 777)).astype(np.float32)
    s[1, 5] = np.nan
    tau, mask, st = _select(B, s, 0.5, force=True, stats=True)
    assert not mask.any()
    assert np.array_equal(tau, orc.quantile_threshold(s, 0.5))
    ok = ~np.isnan(s)
    assert np.array_equal(st[1], ok.sum(axis=1))                   # per-sequence slots
    want_sum = np.where(ok, s, 0.0).astype(np.float64).sum(axis=1)
    assert np.all(np.abs(st[0] - want_sum) <= 1e-9 * st[1])
    # statistics only: mask and tau untouched; a second call adds to the same slots, and the
    # sums are the same bits from run to run (no atomics)
    sd = dev(s)
    mask2 = torch.full(s.shape, 7, dtype=torch.uint8, device="cuda")
    ssum = torch.zeros(4, dtype=torch.float64, device="cuda")
    scnt = torch.zeros(4, dtype=torch.int64, device="cuda")
    B.dare_k_quantile_mask(sd, -1.0, mask2, None, False, ssum, scnt)
    torch.cuda.synchronize()
    assert np.array_equal(host(ssum), st[0])
    B.dare_k_quantile_mask(sd, -1.0, mask2, None, False, ssum, scnt)
    torch.cuda.synchronize()
    assert (host(mask2) == 7).all() and np.array_equal(host(scnt), 2 * ok.sum(axis=1))
    assert np.array_equal(host(ssum), 2 * st[0])


# ------------------------------------------------------------------ the step under the quantile rule
def _gap_above_rank(s_row, k):
    srt = np.sort(s_row.astype(np.float64))
    if k == 0:
        return -1.0
    if k == len(srt):
        return 2.5
    assert srt[k] - srt[k - 1] > 8e-6, "test input has no gap above the k-th smallest score"
    return float(np.float32(0.5 * (srt[k] + srt[k - 1])))


@pytest.mark.parametrize("name,shape,phi_kind", [
    ("tiny", {}, "stable"), ("tiny", dict(batch=2, seq=75), "zero"), ("tiny", {}, "one"),
    ("llada8b", dict(batch=3, seq=100, hidden=256, n_heads=4, head_dim=64, fraction=0.25), "stable"),
])
@pytest.mark.parametrize("mode", [orc.MODE_KV, orc.MODE_O, orc.MODE_KVO, orc.MODE_DENSE])
def test_step_under_quantile_rule(name, shape, phi_kind, mode):
    case = synth.make_case(name, seed=21, **shape)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    gl.layer.set_threshold_rule(gl.B.RULE_QUANTILE)
    T = case["seq"]
    # every sequence has the same perturbed count by construction of `fraction` as a float
    n_stable = int((~case["perturbed"][0]).sum())
    phi = {"stable": n_stable / T, "zero": 0.0, "one": 1.0}[phi_kind]
    k = int(np.ceil(np.float32(phi) * np.float32(T)))
    got = gl.step(mode, phi, case["x_cur"], state)
    tau_gpu = host(gl.layer.thresholds(case["batch"]))
    # (i) the rule applied to the GPU's own scores
    assert np.array_equal(tau_gpu, orc.quantile_threshold(got["scores"], phi))
    if mode != orc.MODE_DENSE:
        for b in range(case["batch"]):
            assert np.array_equal(got["reuse_mask"][b].astype(bool), orc.reuse_decision(got["scores"][b], tau_gpu[b]))
        assert (got["reuse_mask"].sum(axis=1) >= k).all()
    # (ii) against the oracle's own threshold
    want_q = pu.oracle_step(case, state, mode, phi, quantile=True)
    fin = np.isfinite(want_q["tau"])
    assert np.array_equal(np.isfinite(tau_gpu), fin)
    assert np.all(np.abs(tau_gpu[fin] - want_q["tau"][fin]) < pu.TIE_BAND)
    # (iii) outputs: fixed threshold in the gap above the k-th smallest score, one sequence at a time
    for b in range(case["batch"]):
        one = dict(case, batch=1, x_cur=case["x_cur"][b:b + 1])
        st_b = {key: v[b:b + 1] for key, v in state.items()}
        tau_fixed = _gap_above_rank(want_q["scores"][b], k)
        want = pu.oracle_step(one, st_b, mode, tau_fixed)
        sub = {key: (v[b:b + 1] if isinstance(v, np.ndarray) and v.ndim >= 2 else v) for key, v in got.items()}
        n_before = int(got["sel_count"][:b].sum())
        n_b = int(got["sel_count"][b])
        sub["sel_idx"] = np.concatenate([got["sel_idx"][n_before:n_before + n_b] - b * T,
                                         np.full(T - n_b, -1, dtype=np.int32)])
        sub["sel_count"] = got["sel_count"][b:b + 1]
        pu.check_step(sub, want, st_b, mode, tau_fixed, case["dtype"])
    gl.layer.destroy()


def test_quantile_rule_argument_errors_and_switching_back():
    case = synth.make_case("tiny", seed=2)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    Bm = gl.B
    with pytest.raises(Bm.DareError):
        gl.layer.thresholds(1)                     # no rule set yet
    gl.layer.set_threshold_rule(Bm.RULE_QUANTILE)
    for bad in (-0.1, 1.5):
        with pytest.raises(Bm.DareError) as ei:
            gl.step(orc.MODE_KVO, bad, case["x_cur"], state)
        assert ei.value.status == Bm.DARE_ERR_INVALID_ARG
    with pytest.raises(Bm.DareError):
        gl.layer.set_threshold_rule(5)
    gl.layer.set_threshold_rule(Bm.RULE_SCORE)     # back to thresholds that are scores
    tau = synth.TAU_SEPARATING
    want = pu.oracle_step(case, state, orc.MODE_KVO, tau)
    got = gl.step(orc.MODE_KVO, tau, case["x_cur"], state)
    pu.check_step(got, want, state, orc.MODE_KVO, tau, "f32")
    gl.layer.destroy()


def test_running_drift_statistics_over_steps():
    """s_l = mean drift over tokens and steps: two steps, both rules, scores not requested."""
    case = synth.make_case("tiny", seed=8, batch=2, seq=96)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    gl.layer.drift_stats_enable(True)
    a = gl.step(orc.MODE_KVO, synth.TAU_SEPARATING, case["x_cur"], state, want_scores=False)
    st2 = {k: a[k] for k in ("q_prev", "k_cache", "v_cache", "o_cache")}
    gl.layer.set_threshold_rule(gl.B.RULE_QUANTILE)
    b = gl.step(orc.MODE_O, 0.5, case["x_prev"], st2)
    mean, count = gl.layer.drift_stats_read()
    w1 = pu.oracle_step(case, state, orc.MODE_KVO, synth.TAU_SEPARATING)
    w2 = pu.oracle_step(case, st2, orc.MODE_O, 0.5, x=case["x_prev"], quantile=True)
    want = np.concatenate([w1["scores"].ravel(), w2["scores"].ravel()])
    assert count == want.size
    assert abs(mean - want.mean()) < 1e-6
    assert a["reuse_mask"].sum() == (~case["perturbed"]).sum()    # the first step's decisions are unaffected
    gl.layer.drift_stats_enable(True)                             # enabling again starts from zero
    mean, count = gl.layer.drift_stats_read()
    assert count == 0 and mean == 0.0
    gl.layer.drift_stats_enable(False)
    gl.step(orc.MODE_O, 0.5, case["x_cur"], st2)
    assert gl.layer.drift_stats_read()[1] == 0
    gl.layer.destroy()
