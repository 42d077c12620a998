"""GPU parity of dare_layer_step against the oracle: every mode, the thresholds
that reuse nothing / about half / everything, small ragged shapes, and the
LLaDA-8B-shaped layer at full size."""
import numpy as np
import pytest
import torch

from oracle import dare_oracle as orc
from paper_2605_08134_amd import synth
import parity_util as pu

pytestmark = pytest.mark.gpu

MODES = [orc.MODE_DENSE, orc.MODE_KV, orc.MODE_O, orc.MODE_KVO]


def _run(case, gl, state, mode, tau, **kw):
    want = pu.oracle_step(case, state, mode, tau)
    got = gl.step(mode, tau, case["x_cur"], state, **kw)
    return pu.check_step(got, want, state, mode, tau, case["dtype"]), got, want


# ------------------------------------------------------------------ tiny fp32 layer
@pytest.fixture(scope="module")
def tiny():
    case = synth.make_case("tiny", seed=1234)
    state = pu.oracle_fill(case)
    return case, state, pu.GpuLayer(case)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("which", ["zero", "median", "above_max", "nothing", "everything"])
def test_tiny_fp32_all_modes_and_thresholds(tiny, mode, which):
    case, state, gl = tiny
    s = pu.oracle_step(case, state, orc.MODE_KV, 0.0)["scores"]
    srt = np.sort(s.reshape(-1))
    median = float(np.float32(0.5 * (srt[len(srt) // 2 - 1] + srt[len(srt) // 2])))
    tau = {"zero": 0.0, "median": median, "above_max": float(s.max()) + 4e-6,
           "nothing": -1.0, "everything": 2.5}[which]
    if which == "median":
        # the stable tokens' scores lie closer together than the tie band, so the
        # median threshold has ties by construction: they are counted, not forbidden
        want = pu.oracle_step(case, state, mode, tau)
        got = gl.step(mode, tau, case["x_cur"], state)
        info = pu.check_step(got, want, state, mode, tau, "f32", expect_no_ties=False)
        print("median threshold: %d ties" % info["ties"])
    else:
        info, got, want = _run(case, gl, state, mode, tau)
    n_reused = int(got["reuse_mask"].sum())
    if mode == orc.MODE_DENSE or which in ("zero", "nothing"):
        assert n_reused == 0          # every token of this input is perturbed: scores > 0
    elif which in ("above_max", "everything"):
        assert n_reused == case["seq"]
    else:
        assert 0.4 * case["seq"] <= n_reused <= 0.6 * case["seq"]


def test_tiny_threshold_exactly_at_max_score_ties(tiny):
    # tau equal to the largest score: that token is a tie by construction; the
    # masks must agree everywhere else and the tie is counted.
    case, state, gl = tiny
    s = pu.oracle_step(case, state, orc.MODE_KV, 0.0)["scores"]
    tau = float(np.float32(s.max()))
    want = pu.oracle_step(case, state, orc.MODE_O, tau)
    got = gl.step(orc.MODE_O, tau, case["x_cur"], state)
    info = pu.check_step(got, want, state, orc.MODE_O, tau, "f32", expect_no_ties=False)
    assert info["ties"] >= 1
    assert int(got["reuse_mask"].sum()) >= case["seq"] - 1


def test_tiny_separate_out_buffer_and_no_lists(tiny):
    case, state, gl = tiny
    tau = synth.TAU_SEPARATING
    for mode in MODES:
        want = pu.oracle_step(case, state, mode, tau)
        got = gl.step(mode, tau, case["x_cur"], state, alias_out=False, want_lists=False)
        pu.check_step(got, want, state, mode, tau, "f32")


def test_tiny_two_steps_unchanged_input_scores_zero(tiny):
    # second step on the same hidden states: every score is exactly 0 and tau = 0 reuses all
    case, state, gl = tiny
    first = gl.step(orc.MODE_KVO, -1.0, case["x_cur"], state)
    st2 = {k: first[k] for k in ("q_prev", "k_cache", "v_cache", "o_cache")}
    second = gl.step(orc.MODE_KVO, 0.0, case["x_cur"], st2)
    assert np.all(second["scores"] == 0.0)
    assert second["reuse_mask"].all()
    assert np.array_equal(second["out"], first["out"])
    assert np.array_equal(second["k_cache"], first["k_cache"])


def test_tiny_is_deterministic(tiny):
    case, state, gl = tiny
    tau = synth.TAU_SEPARATING
    a = gl.step(orc.MODE_KVO, tau, case["x_cur"], state)
    b = gl.step(orc.MODE_KVO, tau, case["x_cur"], state)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_step_argument_errors_leave_buffers_untouched(tiny):
    case, state, gl = tiny
    B = gl.B
    x = pu.dev(case["x_cur"], "f32")
    st = {k: pu.dev(v) for k, v in state.items()}
    before = {k: v.clone() for k, v in st.items()}
    mask = torch.zeros((1, 128), dtype=torch.uint8, device="cuda")

    def call(mode=1, tau=0.1, hidden=x, batch_hidden=None):
        gl.layer.layer_step(mode, tau, hidden, st["q_prev"], st["k_cache"], st["v_cache"],
                            st["o_cache"], st["o_cache"], mask)

    for kw in (dict(mode=9), dict(tau=float("nan"))):
        with pytest.raises(B.DareError) as ei:
            call(**kw)
        assert ei.value.status == B.DARE_ERR_INVALID_ARG
    big = torch.zeros((2, 128, 256), dtype=torch.float32, device="cuda")
    with pytest.raises(B.DareError):
        call(hidden=big)                      # batch 2 > max_batch 1
    torch.cuda.synchronize()
    for k in st:
        assert torch.equal(st[k], before[k])


# ------------------------------------------------------------------ small bf16 layers, ragged
@pytest.mark.parametrize("shape", [
    dict(batch=2, seq=320, hidden=512, n_heads=4, head_dim=128, fraction=0.2),
    dict(batch=3, seq=100, hidden=256, n_heads=4, head_dim=64, fraction=(0.05, 0.5)),
    dict(batch=1, seq=1, hidden=128, n_heads=1, head_dim=128, fraction=1.0),
])
@pytest.mark.parametrize("mode", MODES)
def test_small_bf16(shape, mode):
    case = synth.make_case("llada8b", seed=77, **shape)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case, max_batch=case["batch"] + 1, max_seq=case["seq"] + 37)
    s = pu.oracle_step(case, state, orc.MODE_KV, 0.0)["scores"]
    taus = [-1.0, 2.5] + ([pu.gap_threshold(s, 0.6)] if s.size > 4 else [])
    for tau in taus:
        _run(case, gl, state, mode, tau)
    gl.layer.destroy()


def test_small_fp32_head128_ragged():
    case = synth.make_case("tiny", seed=5, batch=2, seq=75, hidden=256, n_heads=2, head_dim=128)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    for mode in MODES:
        _run(case, gl, state, mode, synth.TAU_SEPARATING)


def test_more_sequences_than_threads_in_the_fused_row_list():
    """600 sequences of 3 tokens: the refreshed-row projection derives the row list itself
    (at most 2048 tokens) and writes one offset and one count per sequence, more of them
    than its workgroup has threads."""
    case = synth.make_case("llada8b", seed=91, batch=600, seq=3, hidden=128, n_heads=1, head_dim=128,
                           fraction=(0.0, 1.0))
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    for mode in (orc.MODE_KVO, orc.MODE_KV):
        info, got, want = _run(case, gl, state, mode, synth.TAU_SEPARATING)
        assert np.array_equal(got["sel_count"], case["perturbed"].sum(axis=1))
        assert 0 < int(got["sel_count"].sum()) < 1800 and got["sel_count"][511:].sum() > 0
    gl.layer.destroy()


def test_refreshed_rows_beyond_one_pass_of_the_grid():
    """2 x 1024 tokens, all of them refreshed, hidden 2048: the refreshed-row projection of the KV
    mode (2048 rows x 4096 columns in 128 x 128 tiles = 512 tiles) takes two passes of its 256
    workgroups and derives its row list from the mask again in front of the second."""
    case = synth.make_case("llada8b", seed=93, batch=2, seq=1024, hidden=2048, n_heads=16, head_dim=128,
                           fraction=1.0)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    for mode in (orc.MODE_KV, orc.MODE_KVO):
        info, got, want = _run(case, gl, state, mode, synth.TAU_SEPARATING)
        assert int(got["sel_count"].sum()) == 2048
    # and with a third of the rows kept: rows gathered through the list in both passes
    case = dict(case, **synth.make_hidden_pair(94, 2, 1024, 2048, 0.66, "bf16"))     # same weights, other rows
    state = pu.oracle_fill(case)
    info, got, want = _run(case, gl, state, orc.MODE_KV, synth.TAU_SEPARATING)
    assert int(got["sel_count"].sum()) == 2 * 676
    gl.layer.destroy()


# ------------------------------------------------------------------ LLaDA-8B-shaped layer, full size
class _Llada:
    """One GPU layer with the LLaDA-8B-shaped weights of seed 1234 and, per perturbed fraction,
    the hidden-state pair and the oracle's caches of the dense step on x_prev."""

    def __init__(self):
        self.base = synth.make_case("llada8b", seed=1234, fraction=0.20)
        self.gl = pu.GpuLayer(self.base)
        self.cases = {}

    def at(self, fraction):
        if fraction not in self.cases:
            c = self.base
            h = synth.make_hidden_pair(1234, c["batch"], c["seq"], c["hidden"], fraction, c["dtype"])
            case = dict(c, fraction=fraction, **h)
            self.cases = {fraction: (case, pu.oracle_fill(case))}      # one at a time: 0.3 GB each
        return self.cases[fraction]


@pytest.fixture(scope="module")
def llada():
    return _Llada()


# Perturbed fractions of the workload definition (5, 13, 25, 50, 100 %), the 20 % point the
# target is stated at, and row counts that put every tile shape of the device-side choice in
# the refreshed-row projection under a whole-layer check at k = 4096:
#   1, 24 rows  register-fed stream for Wo (one and two row blocks), 64 x 64 tiles for Q/K/V
#   51 rows     64 x 64 tiles, one per workgroup
#   100 rows    128 x 48 (Q/K/V)             133, 205, 256 rows   128 x 96 (Q/K/V), 128 x 64 (K/V alone)
#   400, 512    128 x 192 (Q/K/V), 128 x 64 (Wo)
#   600 rows    128 x 128                    1024 rows            256 x 192 (Q/K/V), 128 x 128 (Wo)
ROWS = [1, 24, 51, 100, 133, 205, 256, 400, 512, 600, 1024]


@pytest.mark.parametrize("n_rows", ROWS)
def test_llada8b_layer_full_size(llada, n_rows):
    """Every mode at every reuse ratio of the sweep (and the row counts between them), whole
    layer, full size: against the oracle's bf16 storage model under the excess rule, and
    against the plain float64 definition by rms and max error."""
    case, state = llada.at(n_rows / 1024.0)
    assert int(case["perturbed"].sum()) == n_rows
    tau = synth.TAU_SEPARATING
    for mode in MODES:
        info, got, want = _run(case, llada.gl, state, mode, tau)
        if mode != orc.MODE_DENSE:
            assert np.array_equal(got["reuse_mask"].astype(bool), ~case["perturbed"])
            assert int(got["sel_count"][0]) == n_rows
        plain = pu.oracle_step(case, state, mode, tau, storage=None)
        dinfo = pu.check_against_definition(got, plain, mode)
        print("llada8b %4d rows mode %s: ties %d, excess out %.4f k %.4f v %.4f | plain out %.4f | "
              "vs definition: out rms %.4f max %.4f, k rms %.4f max %.4f" % (
                  n_rows, pu.orc_mode_name(mode), info["ties"], info["out"], info["k_cache"], info["v_cache"],
                  info["out_plain"], dinfo["out_rms"], dinfo["out_max"], dinfo["k_cache_rms"], dinfo["k_cache_max"]))


# ------------------------------------------------------------------ batch 8 x 2048, per-sequence fractions
@pytest.fixture(scope="module")
def llada_b8():
    case = synth.make_case("llada8b_b8", seed=4321)
    # sequences are independent: the oracle runs one sequence at a time
    states = []
    for b in range(case["batch"]):
        one = dict(case, batch=1, x_prev=case["x_prev"][b:b + 1], x_cur=case["x_cur"][b:b + 1])
        states.append((one, pu.oracle_fill(one)))
    state = {k: np.concatenate([s[k] for _, s in states], axis=0) for k in states[0][1]}
    return case, states, state, pu.GpuLayer(case)


@pytest.mark.parametrize("mode", [orc.MODE_KVO, orc.MODE_KV, orc.MODE_O])
def test_llada8b_batch8_variable_rows(llada_b8, mode):
    """8 sequences of 2048 tokens, 5-30 % of each perturbed: masks, lists and counts of all
    sequences; outputs and caches of the first and the last sequence against the oracle."""
    case, states, state, gl = llada_b8
    tau = synth.TAU_SEPARATING
    got = gl.step(mode, tau, case["x_cur"], state)
    assert np.array_equal(got["reuse_mask"].astype(bool), ~case["perturbed"])
    assert np.array_equal(got["sel_count"], case["perturbed"].sum(axis=1))
    assert len(set(got["sel_count"].tolist())) > 1
    n_all = int(got["sel_count"].sum())
    assert np.array_equal(got["sel_idx"][:n_all], np.flatnonzero(case["perturbed"].reshape(-1)))
    for b in (0, case["batch"] - 1):
        one, st = states[b]
        want = pu.oracle_step(one, st, mode, tau)
        sub = {k: (v[b:b + 1] if v.ndim >= 2 and v.shape[0] == case["batch"] else v) for k, v in got.items()}
        n_before = int(got["sel_count"][:b].sum())
        n_b = int(got["sel_count"][b])
        sub["sel_idx"] = np.concatenate([got["sel_idx"][n_before:n_before + n_b] - b * case["seq"],
                                         np.full(case["seq"] - n_b, -1, dtype=np.int32)])
        sub["sel_count"] = got["sel_count"][b:b + 1]
        info = pu.check_step(sub, want, st, mode, tau, "bf16")
        dinfo = pu.check_against_definition(sub, pu.oracle_step(one, st, mode, tau, storage=None), mode)
        print("8 x 2048 mode %s sequence %d (%d rows): excess out %.4f plain %.4f | vs definition: out rms %.4f "
              "max %.4f" % (pu.orc_mode_name(mode), b, n_b, info["out"], info["out_plain"], dinfo["out_rms"],
                            dinfo["out_max"]))


# ------------------------------------------------------------------ whole-query scoring (score_head = -1)
@pytest.mark.parametrize("name,shape", [("tiny", {}), ("llada8b", dict(batch=2, seq=150, hidden=256, n_heads=2, head_dim=128))])
@pytest.mark.parametrize("mode", MODES)
def test_score_over_the_whole_query(name, shape, mode):
    """Sec. 3.1 defines the drift on the whole query; Sec. 3.2 takes head 0.  score_head = -1 selects
    the former: the score cache is [B, T, hidden] and the scored columns are all of Q."""
    from paper_2605_08134_amd import binding as B
    case = synth.make_case(name, seed=31, **shape)
    dt = case["dtype"]
    out, Q, K, V = orc.dense_layer(case["x_prev"], case["wq"], case["wk"], case["wv"], case["wo"], case["n_heads"])
    state = {"q_prev": np.asarray(Q, dtype=np.float32), "k_cache": pu.store(K, dt), "v_cache": pu.store(V, dt),
             "o_cache": pu.store(out, dt)}
    gl = pu.GpuLayer.__new__(pu.GpuLayer)
    gl.B, gl.case, gl.dt = B, case, dt
    gl.layer = B.DareLayer(*[pu.dev(case[k], dt) for k in ("wq", "wk", "wv", "wo")], n_heads=case["n_heads"],
                           max_batch=case["batch"], max_seq=case["seq"], score_head=-1)
    storage = "bf16" if dt == "bf16" else None
    run = lambda tau: orc.layer_step(mode, tau, case["x_cur"], case["wq"], case["wk"], case["wv"], case["wo"],
                                     state["q_prev"], state["k_cache"], state["v_cache"], state["o_cache"],
                                     case["n_heads"], score_head=-1, storage=storage)
    s = run(0.0)["scores"]
    for tau in (-1.0, pu.gap_threshold(s, 0.7), 2.5):
        got = gl.step(mode, tau, case["x_cur"], state)
        pu.check_step(got, run(tau), state, mode, tau, dt)
        assert got["q_prev"].shape[-1] == case["hidden"]
    gl.layer.destroy()
