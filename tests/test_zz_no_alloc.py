"""The layer step that allocates nothing (dare_layer_step_static) against dare_layer_step.

Both entry points run the same kernels; the static one keeps its scratch in a device array
inside the library instead of a context.  Two calls in a row, the second on a smaller input
(the array keeps the first call's contents), every output compared bit for bit; the GPU's free
memory does not move across the calls; sizes beyond the array are refused with a message."""
import numpy as np
import pytest
import torch

from oracle import dare_oracle as orc
from paper_2605_08134_amd import synth
import parity_util as pu

pytestmark = pytest.mark.gpu

KEYS = ("q_prev", "k_cache", "v_cache", "o_cache", "out", "reuse_mask", "sel_idx", "sel_count", "scores")


def _static_step(B, case, packed, mode, tau, state):
    dt = case["dtype"]
    x = pu.dev(case["x_cur"], dt)
    Bn, T = x.shape[0], x.shape[1]
    st = {k: pu.dev(v, None if k == "q_prev" else dt) for k, v in state.items()}
    mask = torch.full((Bn, T), 7, dtype=torch.uint8, device="cuda")
    sel_idx = torch.full((Bn * T,), -1, dtype=torch.int32, device="cuda")
    sel_count = torch.full((Bn,), -1, dtype=torch.int32, device="cuda")
    scores = torch.full((Bn, T), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    B.dare_layer_step_static(packed[0], packed[1], case["n_heads"], mode, float(tau), x, st["q_prev"], st["k_cache"],
                             st["v_cache"], st["o_cache"], st["o_cache"], mask, sel_idx, sel_count, scores)
    torch.cuda.synchronize()
    free1 = torch.cuda.mem_get_info()[0]
    res = {k: pu.host(v) for k, v in st.items()}
    res.update(out=res["o_cache"], reuse_mask=pu.host(mask), sel_idx=pu.host(sel_idx), sel_count=pu.host(sel_count),
               scores=pu.host(scores))
    return res, free0 - free1


def _packed(B, case):
    dt = case["dtype"]
    w = [B.dare_k_pack_weight(pu.dev(case[k], dt)) for k in ("wq", "wk", "wv", "wo")]
    return torch.cat(w[:3], dim=0).contiguous(), w[3]


def test_static_step_equals_layer_step_on_two_calls_in_a_row():
    from paper_2605_08134_amd import binding as B
    B.dare_static_init(0)
    tau = synth.TAU_SEPARATING
    big = synth.make_case("llada8b", seed=55, batch=2, seq=320, hidden=512, n_heads=4, head_dim=128, fraction=0.3)
    small = synth.make_case("llada8b", seed=56, batch=1, seq=100, hidden=256, n_heads=4, head_dim=64, fraction=0.5)
    calls = [(big, orc.MODE_KVO), (small, orc.MODE_KVO), (big, orc.MODE_KV), (small, orc.MODE_O),
             (small, orc.MODE_DENSE)]
    ctx = {}
    for case in (big, small):
        ctx[id(case)] = (pu.oracle_fill(case), pu.GpuLayer(case), _packed(B, case))
    # one untimed call first: the first launch of a kernel loads its code object
    _static_step(B, big, ctx[id(big)][2], orc.MODE_KVO, tau, ctx[id(big)][0])
    for case, mode in calls:
        state, gl, packed = ctx[id(case)]
        want = gl.step(mode, tau, case["x_cur"], state)
        got, grew = _static_step(B, case, packed, mode, tau, state)
        for k in KEYS:
            assert np.array_equal(got[k], want[k], equal_nan=True), (case["seq"], mode, k)
        assert grew == 0, "device memory in use changed by %d bytes across the call" % grew
        # and the result stands on its own against the oracle, like dare_layer_step's
        pu.check_step(got, pu.oracle_step(case, state, mode, tau), state, mode, tau, case["dtype"])
    for _, gl, _ in ctx.values():
        gl.layer.destroy()


def test_static_step_fp32():
    from paper_2605_08134_amd import binding as B
    case = synth.make_case("tiny", seed=57, batch=2, seq=75)
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case)
    packed = _packed(B, case)
    for mode in (orc.MODE_KVO, orc.MODE_O):
        want = gl.step(mode, synth.TAU_SEPARATING, case["x_cur"], state)
        got, _ = _static_step(B, case, packed, mode, synth.TAU_SEPARATING, state)
        for k in KEYS:
            assert np.array_equal(got[k], want[k], equal_nan=True), (mode, k)
    gl.layer.destroy()


def test_static_step_refuses_what_does_not_fit():
    from paper_2605_08134_amd import binding as B
    d, H = 4096, 32
    w3 = torch.zeros((3 * d, d), dtype=torch.bfloat16, device="cuda")
    wo = torch.zeros((d, d), dtype=torch.bfloat16, device="cuda")
    for batch, seq in ((1, 1025), (2, 1024)):       # 1024 tokens of hidden 4096 in bf16 are the limit
        x = torch.zeros((batch, seq, d), dtype=torch.bfloat16, device="cuda")
        qp = torch.zeros((batch, seq, d // H), dtype=torch.float32, device="cuda")
        kc, vc, oc = (torch.ones_like(x) for _ in range(3))
        mask = torch.full((batch, seq), 7, dtype=torch.uint8, device="cuda")
        with pytest.raises(B.DareError) as ei:
            B.dare_layer_step_static(w3, wo, H, orc.MODE_KVO, 0.1, x, qp, kc, vc, oc, oc, mask)
        assert ei.value.status == B.DARE_ERR_UNSUPPORTED
        assert "DARE_STATIC_MAX_ROW_BYTES" in str(ei.value)
        torch.cuda.synchronize()
        assert bool((mask == 7).all()) and bool((oc == 1).all())      # nothing was enqueued
    # the whole query scored: the fp32 scored query is the tighter limit
    x = torch.zeros((1, 512, d), dtype=torch.bfloat16, device="cuda")
    qp = torch.zeros((1, 512, d), dtype=torch.float32, device="cuda")
    mask = torch.zeros((1, 512), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.DareError) as ei:
        B.dare_layer_step_static(w3, wo, H, orc.MODE_KVO, 0.1, x, qp, x, x, x, x, mask, score_head=-1)
    assert ei.value.status == B.DARE_ERR_UNSUPPORTED and "DARE_STATIC_MAX_SCORE_ELEMS" in str(ei.value)
