"""The step calls only enqueue kernels on the caller's stream (no allocation, no memset, no
host synchronisation), so they can be captured into a HIP graph.  A captured KV+O step is
replayed several times, with eager work of the same program and synchronisations between
the replays, and every replay is compared bit for bit with the eager step on the same
inputs."""
import numpy as np
import pytest
import torch

from oracle import dare_oracle as orc
from paper_2605_08134_amd import synth
import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,shape", [("tiny", {}), ("llada8b", dict(batch=2, seq=300, hidden=512, n_heads=4, head_dim=128))])
@pytest.mark.parametrize("block", [False, True])
def test_captured_step_replays_like_the_eager_step(name, shape, block):
    case = synth.make_case(name, seed=11, **shape)
    dt = case["dtype"]
    gl = pu.GpuLayer(case)
    if block:
        gl.layer.block_attach("rms", pu.dev(case["gain"], dt), None, 1e-5, 10000.0, True)
    state0 = pu.oracle_fill(case)
    Bn, T = case["batch"], case["seq"]
    tau = synth.TAU_SEPARATING
    xs = [pu.dev(case["x_cur"], dt), pu.dev(case["x_prev"], dt)]

    def fresh():
        st = {k: pu.dev(v, None if k == "q_prev" else dt) for k, v in state0.items()}
        st["mask"] = torch.full((Bn, T), 7, dtype=torch.uint8, device="cuda")
        st["out"] = torch.zeros_like(st["o_cache"])
        st["cnt"] = torch.zeros((Bn,), dtype=torch.int32, device="cuda")
        return st

    def step(st, x, stream=None):
        fn = gl.layer.block_step if block else gl.layer.layer_step
        fn(orc.MODE_KVO, tau, x, st["q_prev"], st["k_cache"], st["v_cache"], st["o_cache"], st["out"], st["mask"],
           None, st["cnt"], None, stream=stream)

    # eager trajectory: x_cur, x_prev, x_cur, ...
    eager = fresh()
    want = []
    for i in range(6):
        step(eager, xs[i % 2])
        torch.cuda.synchronize()
        want.append({k: v.clone() for k, v in eager.items()})

    # the same trajectory from a graph of two steps, replayed three times
    cap = fresh()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):              # warm-up on the capture stream, then restore the state
        step(cap, xs[0])
    torch.cuda.synchronize()
    for k, v in fresh().items():
        cap[k].copy_(v)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step(cap, xs[0])
        step(cap, xs[1])
    torch.cuda.synchronize()
    for k, v in fresh().items():               # capture does not run anything, but start from a known state
        cap[k].copy_(v)
    scratch = fresh()
    for rep in range(3):
        g.replay()
        torch.cuda.synchronize()
        for k in ("q_prev", "k_cache", "v_cache", "o_cache", "out", "mask", "cnt"):
            assert torch.equal(cap[k], want[2 * rep + 1][k]), (rep, k)
        step(scratch, xs[rep % 2])             # eager work of the same library between the replays
        torch.cuda.synchronize()
    assert int(cap["cnt"].sum()) > 0 and int(cap["mask"].sum()) > 0
    gl.layer.destroy()
