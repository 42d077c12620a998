"""Helpers of the GPU parity tests: moving seeded inputs to the device, filling the
caches with the oracle's dense step, and the comparison rules.

Comparison rules (stated once here, used by every parity test):
  * reuse masks, index lists, counts: bit-exact, after setting aside tokens whose
    ORACLE score lies within 1e-6 of the threshold ("ties": the two sides sum in
    different orders); ties are counted and must stay under 1 % of the tokens.
  * outputs and updated caches, fp32 path: max |gpu - oracle| / rms(oracle) <= 1e-4
    against the plain float64 oracle.
  * outputs and updated caches, bf16 storage: the oracle runs its bf16 storage model
    (Q, K, V and the attention rows rounded where the algorithm produces them) and
    each GPU tensor is compared with the oracle's tensor BEFORE its final rounding.
    A bf16 value cannot be closer to a real number than half a bf16 ulp (2^-8
    relative at worst), and the layer output has elements of 7-8 times its rms, for
    which that half ulp alone is 1.7-2.4 % of the rms: no bf16 tensor can meet
    "max error <= 2e-2 rms" against an unrounded reference.  The 2e-2 bound is
    therefore applied to the error IN EXCESS of the final storage rounding,
        excess = max(0, |gpu - exact| - half_ulp_bf16(exact)),   max excess / rms <= 2e-2,
    and the plain max |gpu - exact| / rms is reported next to it.
  * bf16 storage, second gate, independent of where the kernels round: every GPU tensor is
    also compared with the PLAIN float64 oracle (no storage rounding anywhere: the
    definition).  Two figures are bounded: the rms error rms(gpu - definition) /
    rms(definition), which the few many-sigma elements do not dominate, and the plain
    max |gpu - definition| / rms(definition).  The bounds (DEF_RMS_TOL, DEF_MAX_TOL) sit just
    above what five bf16 roundings (Q, K, V, attention rows, output) give on these inputs.
  * rows the step must not touch (reused K/V/O rows) equal the input bit for bit.
"""
import numpy as np
import torch

from oracle import dare_oracle as orc
from paper_2605_08134_amd import synth

TOL = {"bf16": 2e-2, "f32": 1e-4}
TIE_BAND = 1e-6
# bf16 path against the unrounded float64 definition (see the header).  Measured on the
# LLaDA-8B-shaped layer, all modes, 1 to 1024 refreshed rows of 1024 tokens and 8 x 2048 tokens:
# rms error 0.37-0.53 % of the output's rms (K, V: 0.17 %); max error 1.5-4.1 % (1024 tokens),
# up to 4.6 % (8 x 2048: the maximum is taken over 8 times as many elements; K, V: 1.2 %).
DEF_RMS_TOL = 7e-3
DEF_MAX_TOL = 5.5e-2


def orc_mode_name(mode):
    return {orc.MODE_DENSE: "dense", orc.MODE_KV: "kv", orc.MODE_O: "o", orc.MODE_KVO: "kvo"}[mode]


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def store(a, dtype):
    """Round a float64/float32 array to the storage dtype; float32 array back."""
    a32 = np.asarray(a, dtype=np.float32)
    return synth.round_to_bf16(a32) if dtype == "bf16" else a32


def dev(a, dtype=None):
    """numpy -> cuda tensor (values must already be representable in dtype)."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(tdtype(dtype))
    return t.cuda()


def host(t):
    return t.detach().to(torch.float32).cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    rms = float(np.sqrt(np.mean(want ** 2))) if want.size else 1.0
    if want.size == 0:
        return 0.0
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - want))) / max(rms, 1e-30)


def rms_err(got, want):
    """rms(got - want) / rms(want)."""
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(want ** 2)))
    diff = np.asarray(got, dtype=np.float64) - want
    return float(np.sqrt(np.mean(diff ** 2))) / max(rms, 1e-30)


def check_against_definition(got, plain, mode):
    """The bf16 path against the oracle's plain float64 step (storage=None) on the same
    inputs: rms and max error of out, k_cache and v_cache relative to the rms of the
    definition's tensor, over the rows this step computed (a reused row is a copy of a
    cache row and is compared bit for bit elsewhere).  Returns the measured figures."""
    info = {}
    fresh = np.asarray(plain["reuse_mask"]) == 0
    assert np.array_equal(np.asarray(got["reuse_mask"]) == 0, fresh)
    every = np.ones_like(fresh)
    rows_of = {"out": fresh if mode in (orc.MODE_O, orc.MODE_KVO) else every,
               "k_cache": fresh if mode in (orc.MODE_KV, orc.MODE_KVO) else every,
               "v_cache": fresh if mode in (orc.MODE_KV, orc.MODE_KVO) else every}
    for key, rows in rows_of.items():
        g = np.asarray(got[key], dtype=np.float64)[rows]
        w = np.asarray(plain[key], dtype=np.float64)[rows]
        if w.size == 0:
            continue
        info[key + "_rms"] = rms_err(g, w)
        info[key + "_max"] = rel_err(g, w)
        assert info[key + "_rms"] <= DEF_RMS_TOL, "%s: rms error %g of rms" % (key, info[key + "_rms"])
        assert info[key + "_max"] <= DEF_MAX_TOL, "%s: max error %g of rms" % (key, info[key + "_max"])
    return info


def half_ulp_bf16(x):
    """Half the spacing of bfloat16 numbers at |x| (8 significant bits)."""
    ax = np.abs(np.asarray(x, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(ax, 2.0 ** -126)))
    return 2.0 ** (e - 8)


def excess_err(got, exact):
    """max over elements of (|got - exact| - half_ulp_bf16(exact))+ / rms(exact)."""
    exact = np.asarray(exact, dtype=np.float64)
    if exact.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(exact ** 2)))
    ex = np.abs(np.asarray(got, dtype=np.float64) - exact) - half_ulp_bf16(exact)
    return float(max(np.max(ex), 0.0)) / max(rms, 1e-30)


def assert_close(got, want, dtype, slack=1.0):
    """Per-element check of a single kernel's output: within the rounding of the
    storage dtype (half an ulp of bf16 is at most 2^-8 relative; fp32 path 2^-20) plus an
    absolute term of slack * 2e-3 (bf16) / 2e-6 (fp32) of the output's rms for the
    error carried in from rounded intermediates and the fp32 summation order."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = float(np.sqrt(np.mean(want ** 2))) if want.size else 0.0
    rel, ab = (2.0 ** -8, 2e-3) if dtype == "bf16" else (2.0 ** -20, 2e-6)
    bad = np.abs(got - want) > rel * np.abs(want) + slack * ab * rms
    assert not bad.any(), "%d of %d elements off, worst %g (rms %g)" % (
        int(bad.sum()), bad.size, float(np.max(np.abs(got - want))), rms)


def oracle_fill(case):
    """Caches after a dense step on x_prev, rounded to the storage dtype."""
    dt = case["dtype"]
    out, Q, K, V = orc.dense_layer(case["x_prev"], case["wq"], case["wk"], case["wv"], case["wo"],
                                   case["n_heads"])
    dh = case["head_dim"]
    return {
        "q_prev": np.asarray(Q[:, :, :dh], dtype=np.float32),
        "k_cache": store(K, dt),
        "v_cache": store(V, dt),
        "o_cache": store(out, dt),
    }


def oracle_step(case, state, mode, tau, x=None, storage="auto", quantile=False):
    x = case["x_cur"] if x is None else x
    if storage == "auto":
        storage = "bf16" if case["dtype"] == "bf16" else None
    return orc.layer_step(mode, tau, x, case["wq"], case["wk"], case["wv"], case["wo"],
                          state["q_prev"], state["k_cache"], state["v_cache"], state["o_cache"],
                          case["n_heads"], storage=storage, quantile=quantile)


def gap_threshold(scores, quantile=0.5, min_gap=8e-6):
    """A threshold near the given quantile of the scores that sits in the middle of
    a gap between two neighbouring scores (so no score ties with it)."""
    s = np.sort(np.asarray(scores, dtype=np.float64).reshape(-1))
    mid = int(round(quantile * (len(s) - 1)))
    for step in range(len(s)):
        for i in (mid - step, mid + step):
            if 0 <= i < len(s) - 1 and s[i + 1] - s[i] >= min_gap:
                return float(np.float32(0.5 * (s[i] + s[i + 1])))
    raise AssertionError("no gap between scores")


class GpuLayer:
    """A DareLayer plus device copies of one case's inputs and caches."""

    def __init__(self, case, max_batch=None, max_seq=None):
        from paper_2605_08134_amd import binding as B
        self.B = B
        self.case = case
        dt = case["dtype"]
        self.dt = dt
        w = [dev(case[k], dt) for k in ("wq", "wk", "wv", "wo")]
        self.layer = B.DareLayer(*w, n_heads=case["n_heads"],
                                 max_batch=max_batch or case["batch"], max_seq=max_seq or case["seq"])
        torch.cuda.synchronize()

    def step(self, mode, tau, x, state, alias_out=True, want_lists=True, want_scores=True):
        """Run dare_layer_step on device copies of `state`; returns numpy results."""
        c = self.case
        Bn, T = x.shape[0], x.shape[1]
        xd = dev(x, self.dt)
        st = {k: dev(v, None if k == "q_prev" else self.dt) for k, v in state.items()}
        out = st["o_cache"] if alias_out else torch.full_like(st["o_cache"], float("nan"))
        mask = torch.full((Bn, T), 7, dtype=torch.uint8, device="cuda")
        sel_idx = torch.full((Bn * T,), -1, dtype=torch.int32, device="cuda") if want_lists else None
        sel_count = torch.full((Bn,), -1, dtype=torch.int32, device="cuda") if want_lists else None
        scores = torch.full((Bn, T), float("nan"), dtype=torch.float32, device="cuda") if want_scores else None
        self.layer.layer_step(mode, float(tau), xd, st["q_prev"], st["k_cache"], st["v_cache"],
                              st["o_cache"], out, mask, sel_idx, sel_count, scores)
        torch.cuda.synchronize()
        res = {k: host(v) for k, v in st.items()}
        res["out"] = host(out)
        res["reuse_mask"] = host(mask)
        if want_scores:
            res["scores"] = host(scores)
        if want_lists:
            res["sel_idx"] = host(sel_idx)
            res["sel_count"] = host(sel_count)
        return res


def check_step(got, want, state_in, mode, tau, dtype, expect_no_ties=True, tie_band=TIE_BAND, q_prev_tol=1e-4):
    """Compare one GPU step with the oracle's.  Returns a dict of measured errors.
    tie_band: how far a GPU score may lie from the oracle's, and the width of the band around
    the threshold inside which a decision may fall either way.  q_prev_tol: bound on the
    fp32 score cache (max error / rms)."""
    tol = TOL[dtype]
    s_or = want["scores"]
    ties = np.abs(s_or - float(np.float32(tau))) < tie_band if mode != orc.MODE_DENSE else np.zeros_like(s_or, bool)
    n_ties = int(ties.sum())
    assert n_ties <= max(0.01 * ties.size, 0 if expect_no_ties else 16), "too many ties: %d" % n_ties
    if expect_no_ties:
        assert n_ties == 0, "threshold ties with %d scores" % n_ties
    info = {"ties": n_ties}

    info["score_err"] = float(np.max(np.abs(got["scores"].astype(np.float64) - s_or)))
    assert info["score_err"] < tie_band

    # masks and lists, bit-exact outside the ties
    gm, wm = got["reuse_mask"], want["reuse_mask"]
    assert set(np.unique(gm).tolist()) <= {0, 1}
    assert np.array_equal(gm[~ties], wm[~ties])
    if "sel_idx" in got:
        n = int((gm == 0).sum())
        assert np.array_equal(got["sel_idx"][:n], np.flatnonzero(gm.reshape(-1) == 0))
        assert np.all(got["sel_idx"][n:] == -1)                 # rest untouched
        assert np.array_equal(got["sel_count"], (gm == 0).sum(axis=1))
        if n_ties == 0:
            assert np.array_equal(got["sel_idx"][:n], want["sel_idx"])
            assert np.array_equal(got["sel_count"], want["sel_count"])
    if n_ties and not np.array_equal(gm, wm):
        return info  # a tie fell differently: the remaining outputs legitimately differ

    reused = wm.astype(bool)
    exact = want["exact"]
    for key, ref in (("out", exact["out"]), ("o_cache", exact["out"]), ("k_cache", exact["k_cache"]),
                     ("v_cache", exact["v_cache"]), ("q_prev", want["q_prev"])):
        if key == "q_prev" or dtype == "f32":
            t = q_prev_tol if key == "q_prev" else 1e-4
            info[key] = rel_err(got[key], ref)
        else:
            t = tol
            info[key] = excess_err(got[key], ref)
            info[key + "_plain"] = rel_err(got[key], ref)
        assert info[key] <= t, "%s: %g > %g" % (key, info[key], t)
    # rows that must be bit-copies of the input caches
    if mode in (orc.MODE_KV, orc.MODE_KVO):
        assert np.array_equal(got["k_cache"][reused], state_in["k_cache"][reused])
        assert np.array_equal(got["v_cache"][reused], state_in["v_cache"][reused])
    if mode in (orc.MODE_O, orc.MODE_KVO):
        assert np.array_equal(got["out"][reused], state_in["o_cache"][reused])
        assert np.array_equal(got["o_cache"][reused], state_in["o_cache"][reused])
    assert np.array_equal(got["out"], got["o_cache"])
    return info
