"""GPU parity of the frozen prefix (prefix caching composed with the reuse modes): every
mode, score and quantile thresholds, the fp32 and bf16 paths, the block with rotary
embedding, and the LLaDA-8B-shaped layer with half the sequence frozen."""
import numpy as np
import pytest
import torch

from oracle import dare_oracle as orc
from paper_2605_08134_amd import synth
import parity_util as pu

pytestmark = pytest.mark.gpu

MODES = [orc.MODE_DENSE, orc.MODE_KV, orc.MODE_O, orc.MODE_KVO]


def _oracle(case, state, mode, tau, P, **kw):
    storage = "bf16" if case["dtype"] == "bf16" else None
    return orc.layer_step(mode, tau, case["x_cur"], case["wq"], case["wk"], case["wv"], case["wo"],
                          state["q_prev"], state["k_cache"], state["v_cache"], state["o_cache"],
                          case["n_heads"], storage=storage, prefix=P, **kw)


def _frozen_rows_untouched(got, state, P):
    for key in ("k_cache", "v_cache", "o_cache", "q_prev"):
        assert np.array_equal(got[key][:, :P], state[key][:, :P]), key
    assert np.array_equal(got["out"][:, :P], state["o_cache"][:, :P])
    assert (got["reuse_mask"][:, :P] == 1).all() and (got["scores"][:, :P] == 0).all()


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("P", [1, 37, 127])
def test_prefix_tiny_fp32(mode, P):
    case = synth.make_case("tiny", seed=1234)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    gl.layer.set_prefix(P)
    for tau in (-1.0, synth.TAU_SEPARATING, 2.5):
        want = _oracle(case, state, mode, tau, P)
        got = gl.step(mode, tau, case["x_cur"], state, alias_out=(tau != 2.5))
        pu.check_step(got, want, state, mode, tau, "f32")
        _frozen_rows_untouched(got, state, P)
        if mode == orc.MODE_DENSE:
            assert got["sel_count"].tolist() == [case["seq"] - P]
    gl.layer.set_prefix(0)                           # off again: the plain step
    want = pu.oracle_step(case, state, mode, synth.TAU_SEPARATING)
    got = gl.step(mode, synth.TAU_SEPARATING, case["x_cur"], state)
    pu.check_step(got, want, state, mode, synth.TAU_SEPARATING, "f32")
    gl.layer.destroy()


@pytest.mark.parametrize("shape,P", [
    (dict(batch=2, seq=320, hidden=512, n_heads=4, head_dim=128, fraction=0.2), 130),
    (dict(batch=3, seq=100, hidden=256, n_heads=4, head_dim=64, fraction=(0.05, 0.5)), 33),
])
@pytest.mark.parametrize("mode", MODES)
def test_prefix_small_bf16(shape, P, mode):
    case = synth.make_case("llada8b", seed=79, **shape)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case, max_batch=case["batch"] + 1, max_seq=case["seq"] + 5)
    gl.layer.set_prefix(P)
    s = _oracle(case, state, orc.MODE_KV, 0.0, P)["scores"][:, P:]
    for tau in (-1.0, pu.gap_threshold(s, 0.6), 2.5):
        want = _oracle(case, state, mode, tau, P)
        got = gl.step(mode, tau, case["x_cur"], state)
        pu.check_step(got, want, state, mode, tau, "bf16")
        _frozen_rows_untouched(got, state, P)
    gl.layer.destroy()


def test_prefix_with_quantile_rule_ranks_the_other_tokens():
    case = synth.make_case("tiny", seed=5, batch=2, seq=96)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    P = 32
    gl.layer.set_prefix(P)
    gl.layer.set_threshold_rule(gl.B.RULE_QUANTILE)
    got = gl.step(orc.MODE_KVO, 0.5, case["x_cur"], state)
    tau = pu.host(gl.layer.thresholds(2))
    assert np.array_equal(tau, orc.quantile_threshold(got["scores"][:, P:], 0.5))
    assert (got["reuse_mask"][:, P:].sum(axis=1) >= 32).all()       # ceil(0.5 * 64) of the 64 others
    for b in range(2):
        assert np.array_equal(got["reuse_mask"][b, P:].astype(bool), orc.reuse_decision(got["scores"][b, P:], tau[b]))
    _frozen_rows_untouched(got, state, P)
    want = _oracle(case, state, orc.MODE_KVO, 0.5, P, quantile=True)
    assert np.all(np.abs(tau - want["tau"]) < pu.TIE_BAND)
    gl.layer.destroy()


def test_prefix_argument_errors():
    case = synth.make_case("tiny", seed=5)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    for bad in (-1, 128, 4096):
        with pytest.raises(gl.B.DareError):
            gl.layer.set_prefix(bad)
    gl2 = pu.GpuLayer(case, max_seq=256)
    gl2.layer.set_prefix(128)                         # fine for the context, too long for this step
    with pytest.raises(gl.B.DareError) as ei:
        gl2.step(orc.MODE_KVO, 0.1, case["x_cur"], state)
    assert ei.value.status == gl.B.DARE_ERR_INVALID_ARG
    gl.layer.destroy()
    gl2.layer.destroy()


@pytest.mark.parametrize("mode", MODES)
def test_prefix_block_with_rope_fp32(mode):
    """The block (RMS norm, rotary embedding, residual) with a frozen prefix, end to end in fp32."""
    from test_gpu_block import GpuBlock, ROPE_BASE
    case = synth.make_case("tiny", seed=1234, batch=2, seq=75)
    P = 30
    gb = GpuBlock(case, "rms", ROPE_BASE, True)
    args = (case["wq"], case["wk"], case["wv"], case["wo"])
    z = np.zeros((2, 75, case["hidden"]))
    fill = orc.block_step(orc.MODE_DENSE, 0.0, case["x_prev"], "rms", case["gain"], None, 1e-5, *args,
                          np.ones((2, 75, case["head_dim"])), z, z, z, case["n_heads"], rope_base=ROPE_BASE)
    state = {"q_prev": np.asarray(fill["q_prev"], dtype=np.float32), "k_cache": pu.store(fill["k_cache"], "f32"),
             "v_cache": pu.store(fill["v_cache"], "f32"), "o_cache": pu.store(fill["out"], "f32")}
    gb.layer.set_prefix(P)
    tau = synth.TAU_SEPARATING
    want = orc.block_step(mode, tau, case["x_cur"], "rms", case["gain"], None, 1e-5, *args, state["q_prev"],
                          state["k_cache"], state["v_cache"], state["o_cache"], case["n_heads"],
                          rope_base=ROPE_BASE, residual=True, prefix=P)
    got = gb.block_step(mode, tau, case["x_cur"], state)
    pu.check_step(dict(got, out=got["o_cache"]), want, state, mode, tau, "f32")
    assert pu.rel_err(got["block_out"], want["exact"]["block_out"]) <= 1e-4
    assert np.array_equal(got["o_cache"][:, :P], state["o_cache"][:, :P])
    gb.layer.destroy()


@pytest.mark.parametrize("mode", [orc.MODE_DENSE, orc.MODE_KVO])
def test_prefix_llada8b_full_size(mode):
    """512 prompt tokens frozen, 512 generated tokens active, 20 % of all tokens perturbed."""
    case = synth.make_case("llada8b", seed=1234, fraction=0.20)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    P = 512
    gl.layer.set_prefix(P)
    tau = synth.TAU_SEPARATING
    want = _oracle(case, state, mode, tau, P)
    got = gl.step(mode, tau, case["x_cur"], state)
    info = pu.check_step(got, want, state, mode, tau, "bf16")
    _frozen_rows_untouched(got, state, P)
    if mode == orc.MODE_KVO:
        assert np.array_equal(got["reuse_mask"][:, P:].astype(bool), ~case["perturbed"][:, P:])
    print("llada8b prefix 512 mode %d errors: %s" % (mode, info))
    gl.layer.destroy()
