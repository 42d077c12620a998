"""Seeded sweep of odd shapes through dare_layer_step against the oracle: head counts that
are not powers of two, sequence lengths that straddle every tile size, sequences of one
batch with nothing / everything / a few tokens to refresh, frozen prefixes, both dtypes."""
import numpy as np
import pytest

from oracle import dare_oracle as orc
from paper_2605_08134_amd import synth
import parity_util as pu

pytestmark = pytest.mark.gpu


def _case(seed):
    r = np.random.Generator(np.random.PCG64(1000 + seed))
    dh = int(r.choice([64, 128]))
    heads = int(r.choice([1, 2, 3, 5]))
    batch = int(r.integers(1, 5))
    seq = int(r.choice([1, 2, 31, 33, 63, 64, 65, 127, 129, 200, 257, 300]))
    dtype = "bf16" if seed % 2 else "f32"
    case = synth.make_case("tiny", seed=seed, batch=batch, seq=seq, hidden=heads * dh, n_heads=heads,
                           head_dim=dh, dtype=dtype, fraction=(0.0, 0.6))
    # sequence 0 does not move at all; the last sequence moves everywhere
    case["x_cur"][0] = case["x_prev"][0]
    if batch > 1:
        case["x_cur"][-1] = pu.store(case["x_prev"][-1] + 0.5 * r.standard_normal(case["x_prev"][-1].shape), dtype)
    mode = int(r.integers(0, 4))
    prefix = int(r.integers(0, seq)) if seed % 3 == 0 else 0
    return case, mode, prefix, r


@pytest.mark.parametrize("seed", range(24))
def test_random_shape(seed):
    case, mode, prefix, r = _case(seed)
    dt = case["dtype"]
    state = pu.oracle_fill(case)
    gl = pu.GpuLayer(case, max_batch=case["batch"] + int(r.integers(0, 2)), max_seq=case["seq"] + int(r.integers(0, 70)))
    gl.layer.set_prefix(prefix)
    storage = "bf16" if dt == "bf16" else None
    run = lambda tau: orc.layer_step(mode, tau, case["x_cur"], case["wq"], case["wk"], case["wv"], case["wo"],
                                     state["q_prev"], state["k_cache"], state["v_cache"], state["o_cache"],
                                     case["n_heads"], storage=storage, prefix=prefix)
    s = run(0.0)["scores"][:, prefix:]
    taus = [-1.0, 2.5]
    pos = s[s > 0]
    if pos.size > 2 and float(pos.max()) - float(pos.min()) > 1e-4:
        taus.append(pu.gap_threshold(pos, float(r.uniform(0.2, 0.8))))
    for tau in taus:
        want = run(tau)
        got = gl.step(mode, tau, case["x_cur"], state, alias_out=bool(r.integers(0, 2)))
        pu.check_step(got, want, state, mode, tau, dt, expect_no_ties=False)
    # tau = 0 on caches the GPU wrote itself: a sequence that does not move then scores exactly 0
    # and is reused whole (its tokens are all "ties" for check_step, so the masks are compared here)
    first = gl.step(mode if mode != orc.MODE_DENSE else orc.MODE_KVO, -1.0, case["x_cur"], state)
    st2 = {k: first[k] for k in ("q_prev", "k_cache", "v_cache", "o_cache")}
    x2 = case["x_cur"].copy()
    if case["batch"] > 1:
        x2[1:] = case["x_prev"][1:]
    got = gl.step(mode, 0.0, x2, st2)
    want = orc.layer_step(mode, 0.0, x2, case["wq"], case["wk"], case["wv"], case["wo"], st2["q_prev"],
                          st2["k_cache"], st2["v_cache"], st2["o_cache"], case["n_heads"], storage=storage,
                          prefix=prefix)
    sure = np.abs(want["scores"]) > pu.TIE_BAND
    assert np.array_equal(got["reuse_mask"][sure], want["reuse_mask"][sure])
    if mode != orc.MODE_DENSE:
        assert got["reuse_mask"][0].all() and (got["scores"][0] == 0).all()
        if mode in (orc.MODE_O, orc.MODE_KVO):
            assert np.array_equal(got["out"][0], st2["o_cache"][0])
        if mode in (orc.MODE_KV, orc.MODE_KVO):
            assert np.array_equal(got["k_cache"][0], st2["k_cache"][0])
    gl.layer.destroy()
