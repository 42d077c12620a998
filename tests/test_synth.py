"""The seeded input generator: storage rounding and the drift it produces."""
import numpy as np
import torch

from oracle import dare_oracle as orc
from paper_2605_08134_amd import synth


def test_bf16_rounding_matches_torch():
    r = np.random.Generator(np.random.PCG64(1))
    a = (r.standard_normal(20000) * 10.0 ** r.integers(-6, 6, 20000)).astype(np.float32)
    a[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]      # ties: to even
    got = synth.round_to_bf16(a)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    bits = synth.bf16_bits(got)
    back = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(back, got)


def test_case_is_seeded_and_shaped():
    a = synth.make_case("tiny", seed=5)
    b = synth.make_case("tiny", seed=5)
    c = synth.make_case("tiny", seed=6)
    assert a["x_cur"].shape == (1, 128, 256) and a["wq"].shape == (256, 256)
    assert np.array_equal(a["x_cur"], b["x_cur"]) and np.array_equal(a["wo"], b["wo"])
    assert not np.array_equal(a["x_cur"], c["x_cur"])
    assert int(a["perturbed"].sum()) == round(0.2 * 128)
    assert abs(float(a["wq"].std()) - 0.02) < 2e-3


def test_drift_is_bimodal_and_tau_separates():
    c = synth.make_case("tiny", seed=1234)
    q1 = (c["x_cur"].astype(np.float64) @ c["wq"])[:, :, :64]
    q0 = (c["x_prev"].astype(np.float64) @ c["wq"])[:, :, :64]
    s = orc.drift_scores(q1, q0)
    assert s[c["perturbed"]].min() > 10 * synth.TAU_SEPARATING / 5
    assert s[~c["perturbed"]].max() < synth.TAU_SEPARATING / 5
    reuse = orc.reuse_decision(s, synth.TAU_SEPARATING)
    assert np.array_equal(reuse, ~c["perturbed"])


def test_per_sequence_fractions():
    h = synth.make_hidden_pair(3, 8, 200, 16, (0.05, 0.30), "bf16")
    n = h["perturbed"].sum(axis=1)
    assert n.min() >= 10 and n.max() <= 60 and len(set(n.tolist())) > 3
    x = h["x_cur"]
    assert np.array_equal(synth.round_to_bf16(x), x)


def test_half_ulp_helper_of_the_parity_rule():
    import sys, os
    sys.path.insert(0, os.path.dirname(__file__))
    import parity_util as pu
    x = np.array([1.0, 1.99, 2.0, 0.75, -3.0, 1e-3])
    spacing = np.array([2.0 ** -7, 2.0 ** -7, 2.0 ** -6, 2.0 ** -8, 2.0 ** -6, 2.0 ** -17])
    assert np.array_equal(pu.half_ulp_bf16(x), spacing / 2)
    r = np.random.Generator(np.random.PCG64(2)).standard_normal(10000) * 3
    # rounding a value to bf16 never moves it by more than the helper says
    assert np.all(np.abs(synth.round_to_bf16(r.astype(np.float32)).astype(np.float64) - r.astype(np.float32)) <= pu.half_ulp_bf16(r.astype(np.float32)))
    assert pu.excess_err(synth.round_to_bf16(r.astype(np.float32)), r.astype(np.float32)) == 0.0
