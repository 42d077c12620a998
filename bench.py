"""Benchmark of the DARE layer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--quick]

One "step" is one dare_layer_step call (every stage of the hot path) on a
LLaDA-8B-shaped layer (hidden 4096, 32 heads x 128, 1024 tokens, batch 1, bf16),
with synthetic seeded inputs already resident in HBM.  The headline value is
tokens/s of the combined KV+O reuse mode at 80 % reuse; the dense path of the same
library, the other modes and the other reuse ratios are reported in "sweep".
Two consecutive steps alternate between the two hidden-state tensors of the input
pair, so every timed step sees the same reuse mask (the drift score is symmetric)
while the caches really change.  Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--quick", action="store_true", help="headline point and dense only")
    ap.add_argument("--model-steps", type=int, default=512,
                    help="denoising steps of the 32-layer model leg: 512 is the whole block-wise schedule of "
                         "the workload definition (0 skips the leg)")
    ap.add_argument("--only-model", action="store_true",
                    help="run only the 32-layer model leg (for profiler passes)")
    ap.add_argument("--only-dominant", action="store_true",
                    help="run only the dominant-kernel loop (for profiler passes)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_08134_amd import binding as B
    from paper_2605_08134_amd import synth

    B.lib()  # fails loudly when the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.only_model:
        print(json.dumps({"model": model_leg(torch, B, np, dev, max(1, args.model_steps))}))
        return

    cfg = dict(synth.CONFIGS["llada8b"])
    Bn, T, d, H, Dh = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["n_heads"], cfg["head_dim"]
    tau = synth.TAU_SEPARATING
    seed = 1234

    weights = synth.make_weights(seed, d, "bf16")
    wdev = [torch.from_numpy(weights[k]).to(torch.bfloat16).to(dev) for k in ("wq", "wk", "wv", "wo")]
    layer = B.DareLayer(*wdev, n_heads=H, max_batch=Bn, max_seq=T)
    torch.cuda.synchronize()

    def to_dev(a):
        return torch.from_numpy(a).to(torch.bfloat16).to(dev)

    mask = torch.zeros((Bn, T), dtype=torch.uint8, device=dev)
    sel_count = torch.zeros((Bn,), dtype=torch.int32, device=dev)

    def fill(state, x_prev):
        layer.layer_step(B.MODE_DENSE, 0.0, x_prev, state["q_prev"], state["k_cache"], state["v_cache"],
                         state["o_cache"], state["o_cache"], mask)

    def run_steps(mode, xa, xb, state, n):
        # the per-sequence counts are asked for in the reuse modes only: in the dense mode they
        # would cost the dense step a compaction launch it has no use for
        cnt = None if mode == B.MODE_DENSE else sel_count
        for i in range(n):
            x = xb if i % 2 == 0 else xa
            layer.layer_step(mode, tau, x, state["q_prev"], state["k_cache"], state["v_cache"],
                             state["o_cache"], state["o_cache"], mask, None, cnt, None)

    host_ms = {}

    def time_mode(mode, xa, xb, steps, warmup):
        state = layer.new_state(Bn, T)
        fill(state, xa)
        # set-up: 100 steps that bring clocks and caches to their running state (the first tens of
        # steps after an idle gap run 10-15 % slow, the dense leg's more than the reuse leg's), then
        # the W warm-up steps proper; an even count, so that the next step sees xb again
        run_steps(mode, xa, xb, state, 100 + warmup + (warmup % 2))
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        run_steps(mode, xa, xb, state, steps)
        e1.record()
        host_ms[mode] = (time.perf_counter() - t0) * 1e3 / steps   # enqueue only, no wait
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        ms = e0.elapsed_time(e1) / steps
        reuse = float(mask.float().mean().item())
        return ms, wall_ms / steps, reuse, (0 if mode == B.MODE_DENSE else int(sel_count.sum().item()))

    def latency_distribution(mode, xa, xb, steps):
        """Per-step latency (an event after every step, outside the headline timing)."""
        state = layer.new_state(Bn, T)
        fill(state, xa)
        run_steps(mode, xa, xb, state, 20)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        ev[0].record()
        for i in range(steps):
            x = xb if i % 2 == 0 else xa
            layer.layer_step(mode, tau, x, state["q_prev"], state["k_cache"], state["v_cache"],
                             state["o_cache"], state["o_cache"], mask, None,
                             None if mode == B.MODE_DENSE else sel_count, None)
            ev[i + 1].record()
        torch.cuda.synchronize()
        us = np.sort(np.array([ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(steps)]))
        return {"median": float(us[steps // 2]), "p10": float(us[steps // 10]),
                "p90": float(us[(9 * steps) // 10])}

    pairs = {}

    def pair(fraction):
        if fraction not in pairs:
            h = synth.make_hidden_pair(seed, Bn, T, d, fraction, "bf16")
            pairs[fraction] = (to_dev(h["x_prev"]), to_dev(h["x_cur"]))
        return pairs[fraction]

    # ---- dominant kernel: the refreshed-row Q/K/V projection at 80 % reuse ----------------
    n_sel = int(round(0.20 * T)) * Bn
    wqkv_t = torch.cat([B.dare_k_pack_weight(w) for w in wdev[:3]], dim=0).contiguous()
    xa, xb = pair(0.20)
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = np.sort(rng.permutation(Bn * T)[:n_sel]).astype(np.int32)
    idx = torch.from_numpy(rows).to(dev)
    m_dev = torch.tensor([n_sel], dtype=torch.int32, device=dev)
    qkv_out = [torch.empty((Bn * T, d), dtype=torch.bfloat16, device=dev) for _ in range(3)]

    def dominant(n):
        for _ in range(n):
            B.dare_k_gemm(xb.view(Bn * T, d), wqkv_t, qkv_out, d, idx=idx, m_dev=m_dev, m_max=Bn * T)

    dominant(300)          # clocks at their running state (the first hundreds of launches run 10 % slow)
    torch.cuda.synchronize()
    n_dom = 200
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    dominant(n_dom)
    e1.record()
    torch.cuda.synchronize()
    dom_ms = e0.elapsed_time(e1) / n_dom
    # algorithmic bytes of one launch: the three weight matrices once, the selected
    # rows of X once, the selected rows of Q, K, V once
    dom_bytes = 3 * d * d * 2 + n_sel * d * 2 + 3 * n_sel * d * 2
    dom_flops = 2.0 * n_sel * d * 3 * d
    roofline = {
        "kernel": "gemm_bf16_rows_wide_kernel (refreshed-row Q/K/V projection, %d rows x %d x %d)" % (n_sel, 3 * d, d),
        "bound": "hbm",
        "achieved": dom_bytes / (dom_ms * 1e-3) / 1e9,
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": dom_bytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "traffic": stored_traffic(),
        "traffic_source": "profiles/gemm_rows_qkv_llada8b_pmc.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                          "`bench.py --only-dominant`, scaled by the copy kernel of the same runs; not measured "
                          "in this run",
        "us_per_launch": dom_ms * 1e3,
        "tflops": dom_flops / (dom_ms * 1e-3) / 1e12,
    }
    if args.only_dominant:
        # profiler passes: the same launches plus a plain copy of known size, whose
        # counter readings calibrate FETCH_SIZE / WRITE_SIZE (64 MiB read, 64 MiB written)
        src = torch.ones((8192, d), dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(20):
            B.dare_k_copy_rows(src, dst)
        torch.cuda.synchronize()
        print(json.dumps({"roofline": roofline}))
        return

    # ---- the timed headline: K steps of KV+O reuse at 80 % reuse ------------------------------
    ms_kvo, wall_kvo, reuse, n_ref = time_mode(B.MODE_KVO, xa, xb, args.steps, args.warmup)
    host_kvo = host_ms[B.MODE_KVO]
    ms_dense, _, _, _ = time_mode(B.MODE_DENSE, xa, xb, args.steps, args.warmup)   # same protocol as the headline

    graph = None
    if not args.quick:
        graph = graph_replay(torch, layer, B, xa, xb, Bn, T, tau, mask, fill)

    # per-step latency (an event after every step, 20 warm-up steps, both legs alike): the medians
    # give the ratio that is reported as the headline ratio
    latency = {"kvo_us": latency_distribution(B.MODE_KVO, xa, xb, 200),
               "dense_us": latency_distribution(B.MODE_DENSE, xa, xb, 200)}

    sweep = [{"mode": "kvo", "perturbed": 0.20, "reuse": reuse, "us": ms_kvo * 1e3,
              "tokens_per_s": Bn * T / (ms_kvo * 1e-3), "vs_dense": ms_kvo / ms_dense},
             {"mode": "dense", "perturbed": None, "reuse": 0.0, "us": ms_dense * 1e3,
              "tokens_per_s": Bn * T / (ms_dense * 1e-3), "vs_dense": 1.0}]
    if not args.quick:
        for fraction in (0.05, 0.13, 0.20, 0.25, 0.50, 1.00):
            a, b = pair(fraction)
            for mode in (B.MODE_KV, B.MODE_O, B.MODE_KVO):
                if mode == B.MODE_KVO and fraction == 0.20:
                    continue
                ms, _, r, _ = time_mode(mode, a, b, max(20, args.steps // 4), 10)
                sweep.append({"mode": B.MODE_NAMES[mode], "perturbed": fraction, "reuse": r,
                              "us": ms * 1e3, "tokens_per_s": Bn * T / (ms * 1e-3),
                              "vs_dense": ms / ms_dense})

    # dense-path MFMA evidence: the all-row Q/K/V projection
    def dense_gemm(n):
        for _ in range(n):
            B.dare_k_gemm(xb.view(Bn * T, d), wqkv_t, qkv_out, d)
    dense_gemm(5)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    dense_gemm(50)
    e1.record()
    torch.cuda.synchronize()
    dg_ms = e0.elapsed_time(e1) / 50
    dg_tflops = 2.0 * Bn * T * d * 3 * d / (dg_ms * 1e-3) / 1e12
    roofline_other = [{
        "kernel": "gemm_bf16_kernel (all-row Q/K/V projection, %d x %d x %d)" % (Bn * T, 3 * d, d),
        "bound": "mfma", "achieved": dg_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": dg_tflops / MFMA_BF16_PEAK_TFLOPS, "us_per_launch": dg_ms * 1e3}]

    cold = peaks = None
    if not args.quick:
        cold = cold_weights(torch, B, layer, wdev, xa, xb, Bn, T, d, H, tau)
        peaks = measured_peaks(torch, B, dev, d)
        roofline_other += other_kernels_at_c2(torch, B, np, dev, d, H, Dh)

    # ---- the rows beyond the layer step: block, quantile rule, frozen prefix, whole model ----
    features = model = None
    if not args.quick:
        features = feature_legs(torch, B, synth, wdev, weights, seed, xa, xb, Bn, T, d, H, Dh, tau, ms_dense)
        features["layer_step_8x2048"] = step_at_c2(torch, B, synth, wdev, seed, tau)
        if args.model_steps > 0:
            model = model_leg(torch, B, np, dev, args.model_steps)
            model["prefix_parallel"] = model_leg_prefix_parallel(torch, B, np, dev, max(4, min(32, args.model_steps // 8)))

    # ---- CPU oracle on the host cores (reported baseline, not a target) ----------------------
    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(weights, seed, cfg, tau)

    out = {
        "metric": "layer-step throughput, KV+O reuse at 80% reuse (tokens/s); per-layer latency in sweep",
        "value": Bn * T / (ms_kvo * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_kvo,
        "wall_ms_per_step": wall_kvo,
        "host_enqueue_ms_per_step": host_kvo,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "llada8b layer: hidden 4096, 32 heads x 128, seq 1024, batch 1, "
                               "20% of tokens perturbed, threshold 5e-3, mode KV+O",
                   "reuse": reuse, "refreshed_rows": n_ref, "dense_us": ms_dense * 1e3,
                   # ratio of the per-step medians (200 steps each after 20 warm-up steps); the ratio of
                   # the means of the K timed steps and the ratio with 8 layers' weights in rotation
                   # (nothing stays in the last-level cache) beside it
                   "latency_vs_dense": latency["kvo_us"]["median"] / latency["dense_us"]["median"],
                   "latency_vs_dense_mean_of_timed_steps": ms_kvo / ms_dense,
                   "latency_vs_dense_cold_weights": cold["latency_vs_dense"] if cold else None,
                   "targets_not_met": "dominant kernel and the matrix-core kernels are below the 60 % HBM / "
                                      "50 % MFMA marks: see roofline and roofline_other"},
        "roofline": roofline,
        "roofline_other": roofline_other,
        "measured_peaks": peaks,
        "latency": latency,
        "graph_replay": graph,
        "cold_weights": cold,
        "features": features,
        "model": model,
        "cpu_baseline": cpu,
        "sweep": sweep,
    }
    print(json.dumps(out))


def graph_replay(torch, layer, B, xa, xb, Bn, T, tau, mask, fill):
    """The same steps captured once into a HIP graph (8 steps per graph) and replayed: what the
    launches cost when the host is out of the loop."""
    res = {}
    for name, mode in (("kvo_us", B.MODE_KVO), ("dense_us", B.MODE_DENSE)):
        st = layer.new_state(Bn, T)
        fill(st, xa)
        side = torch.cuda.Stream()
        call = lambda x: layer.layer_step(mode, tau, x, st["q_prev"], st["k_cache"], st["v_cache"], st["o_cache"],
                                          st["o_cache"], mask)
        with torch.cuda.stream(side):
            call(xb)
            call(xa)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for _ in range(4):
                call(xb)
                call(xa)
        torch.cuda.synchronize()
        res[name] = _time_us(torch, lambda n: [g.replay() for _ in range(n)], 25, warm=3) / 8
    res["latency_vs_dense"] = res["kvo_us"] / res["dense_us"]
    return res


def _time_graph_us(torch, call, reps=20, iters=20):
    """Per-launch time of a short kernel: `reps` launches captured into one HIP graph and the
    graph replayed, so that the figure is the kernel's and not the host's enqueue rate
    (a ctypes call costs about 8 us, more than these kernels take).  call(stream) enqueues one
    launch on the given stream."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        call(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for _ in range(reps):
            call(side)
    torch.cuda.synchronize()
    return _time_us(torch, lambda n: [g.replay() for _ in range(n)], iters, warm=2) / reps


def _time_us(torch, fn, iters, warm=3):
    fn(warm)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn(iters)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3


def feature_legs(torch, B, synth, wdev, weights, seed, xa, xb, Bn, T, d, H, Dh, tau, ms_dense):
    """The same layer with what the next rows add, each timed like the headline (KV+O at 80 %
    reuse unless stated): the block (RMS norm, rotary embedding, residual sum), the quantile
    rule (reuse rate 0.8), and a frozen prefix of half the sequence."""
    dev = xa.device
    layer = B.DareLayer(*wdev, n_heads=H, max_batch=Bn, max_seq=T)
    gain = torch.from_numpy(synth.make_norm_params(seed, d, "bf16")["gain"]).to(torch.bfloat16).to(dev)
    mask = torch.zeros((Bn, T), dtype=torch.uint8, device=dev)
    out = torch.empty((Bn, T, d), dtype=torch.bfloat16, device=dev)
    cnt = torch.zeros((Bn,), dtype=torch.int32, device=dev)

    def timed(call, steps=100):
        st = layer.new_state(Bn, T)
        call(B.MODE_DENSE, 0.0, xa, st)
        def run(n):
            for i in range(n):
                call(run.mode, run.tau, xb if i % 2 == 0 else xa, st)
        def go(mode, t):
            run.mode, run.tau = mode, t
            us = _time_us(torch, run, steps, warm=10)
            return us, float(mask.float().mean().item())
        return go

    res = {}
    plain = timed(lambda mode, t, x, st: layer.layer_step(mode, t, x, st["q_prev"], st["k_cache"], st["v_cache"],
                                                          st["o_cache"], st["o_cache"], mask, None, cnt, None))
    layer.block_attach("rms", gain, None, 1e-5, 10000.0, True)
    block = timed(lambda mode, t, x, st: layer.block_step(mode, t, x, st["q_prev"], st["k_cache"], st["v_cache"],
                                                          st["o_cache"], out, mask, None, cnt, None))
    us_d, _ = block(B.MODE_DENSE, 0.0)
    us_k, r = block(B.MODE_KVO, tau)
    res["block_rms_rope_residual"] = {"kvo_us": us_k, "dense_us": us_d, "reuse": r, "vs_dense": us_k / us_d}
    layer.set_threshold_rule(B.RULE_QUANTILE)
    us_q, r = plain(B.MODE_KVO, 0.8)
    res["quantile_rule_phi_0.8"] = {"kvo_us": us_q, "reuse": r, "vs_dense": us_q / (ms_dense * 1e3)}
    layer.set_threshold_rule(B.RULE_SCORE)
    layer.set_prefix(T // 2)
    us_pd, _ = plain(B.MODE_DENSE, 0.0)
    us_pk, r = plain(B.MODE_KVO, tau)
    res["frozen_prefix_%d" % (T // 2)] = {"kvo_us": us_pk, "dense_us": us_pd, "reuse_incl_frozen": r,
                                          "vs_dense_with_prefix": us_pk / us_pd,
                                          "dense_with_prefix_vs_dense": us_pd / (ms_dense * 1e3)}
    layer.destroy()
    return res


def step_at_c2(torch, B, synth, wdev, seed, tau):
    """The whole layer step at 8 sequences of 2048 tokens, per-sequence perturbed fraction
    drawn in [5 %, 30 %] (the variable-row-count workload), KV+O against dense."""
    c = synth.CONFIGS["llada8b_b8"]
    Bn, T, d, H = c["batch"], c["seq"], c["hidden"], c["n_heads"]
    dev = wdev[0].device
    h = synth.make_hidden_pair(seed + 2, Bn, T, d, c["fraction"], "bf16")
    xa = torch.from_numpy(h["x_prev"]).to(torch.bfloat16).to(dev)
    xb = torch.from_numpy(h["x_cur"]).to(torch.bfloat16).to(dev)
    layer = B.DareLayer(*wdev, n_heads=H, max_batch=Bn, max_seq=T)
    mask = torch.zeros((Bn, T), dtype=torch.uint8, device=dev)
    st = layer.new_state(Bn, T)
    call = lambda mode, x: layer.layer_step(mode, tau, x, st["q_prev"], st["k_cache"], st["v_cache"],
                                            st["o_cache"], st["o_cache"], mask)
    call(B.MODE_DENSE, xa)
    res = {}
    for name, mode in (("kvo", B.MODE_KVO), ("dense", B.MODE_DENSE)):
        res[name + "_us"] = _time_us(torch, lambda n, mode=mode: [call(mode, xb if i % 2 == 0 else xa)
                                                                  for i in range(n)], 20, warm=4)
        if mode == B.MODE_KVO:
            res["reuse"] = float(mask.float().mean().item())
    res["latency_vs_dense"] = res["kvo_us"] / res["dense_us"]
    res["tokens_per_s_kvo"] = Bn * T / (res["kvo_us"] * 1e-6)
    layer.destroy()
    return res


def model_leg_prefix_parallel(torch, B, np, dev, n_steps):
    """The model leg with prefix caching and parallel unmasking: 4 sequences of 4096 tokens
    (2048 prompt + 2048 mask ids), the prompt frozen after the first step, 4 positions of the
    current block unmasked per step.  Three runs of the same schedule: all layers dense without
    the frozen prefix, dense with it, KV+O reuse with it."""
    L, d, H, ffn, V, Bn, T, P = 32, 4096, 32, 12288, 126464, 4, 4096, 2048
    gen = torch.Generator(device=dev)
    gen.manual_seed(20260509)
    rn = lambda *shape, std=0.02: (torch.randn(shape, device=dev, generator=gen) * std).to(torch.bfloat16)
    gain = lambda: (1.0 + 0.1 * torch.randn((d,), device=dev, generator=gen)).to(torch.bfloat16)
    m = B.DareModel(L, d, H, ffn, V, Bn, T, B.DARE_BF16, 1e-5, 10000.0)
    for l in range(L):
        m.set_layer(l, gain(), rn(d, d), rn(d, d), rn(d, d), rn(d, d), gain(), rn(d, ffn), rn(d, ffn), rn(ffn, d))
    m.set_io(rn(V, d, std=1.0), gain(), None)
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.PCG64(20260509))
    mask_id = V - 1
    ids0 = np.full((Bn, T), mask_id, dtype=np.int32)
    ids0[:, :P] = rng.integers(0, mask_id, (Bn, P))
    order = np.stack([np.concatenate([b0 + rng.permutation(32) for b0 in range(P, T, 32)]) for _ in range(Bn)])
    refreshed = torch.zeros((L, Bn), dtype=torch.int32, device=dev)
    out = {}
    for name, mode, thr, prefix in (("dense_no_prefix", B.MODE_DENSE, 0.0, 0), ("dense_prefix", B.MODE_DENSE, 0.0, P),
                                    ("kvo_prefix", B.MODE_KVO, 1e-3, P)):
        ids = torch.from_numpy(ids0.copy()).to(dev)
        m.set_prefix(0)
        m.step(B.MODE_DENSE, 0.0, ids)               # fills every layer's caches, prompt included
        m.set_prefix(prefix)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        counts = []
        e0.record()
        for t in range(n_steps):
            for b in range(Bn):
                ids[b, torch.from_numpy(order[b, 4 * t:4 * t + 4]).to(dev)] = int(rng.integers(0, mask_id))
            m.step(mode, thr, ids, None, refreshed)
            counts.append(refreshed.clone())
        e1.record()
        torch.cuda.synchronize()
        ref = torch.stack(counts).float().cpu().numpy()                   # [steps, layers, batch]
        out[name] = {"step_us_mean": e0.elapsed_time(e1) * 1e3 / n_steps,
                     "layer_us_mean": e0.elapsed_time(e1) * 1e3 / n_steps / L,
                     "refreshed_per_sequence_mean": float(ref.mean()),
                     "reuse_of_unfrozen_mean": float(1.0 - ref.mean() / (T - prefix))}
    out["prefix_vs_no_prefix"] = out["dense_prefix"]["layer_us_mean"] / out["dense_no_prefix"]["layer_us_mean"]
    out["reuse_and_prefix_vs_prefix"] = out["kvo_prefix"]["layer_us_mean"] / out["dense_prefix"]["layer_us_mean"]
    out["config"] = {"layers": L, "batch": Bn, "seq": T, "prompt_frozen": P, "unmasked_per_step": 4, "block": 32,
                     "steps_timed": n_steps, "threshold": 1e-3}
    m.destroy()
    return out


def model_leg(torch, B, np, dev, n_steps):
    """A random-init LLaDA-8B-shaped masked-diffusion model: 32 layers, hidden 4096, 32 x 128
    heads, SwiGLU feed-forward 12288, RMS norm, rotary embedding, vocabulary 126464, bf16.
    512 prompt ids followed by 512 mask ids; block-wise schedule with blocks of 32; every
    denoising step replaces one seeded random mask position of the current block by a random
    id.  Weights come from torch's seeded generator (timing and reuse statistics only; the
    parity tests use the numpy generator).  DARE (KV+O, threshold 1e-3) runs in every layer;
    the same schedule is run again with every layer dense.  Reuse here is not injected: it is
    what one changed token does to the other tokens' queries in a random network."""
    L, d, H, ffn, V, T, P = 32, 4096, 32, 12288, 126464, 1024, 512
    gen = torch.Generator(device=dev)
    gen.manual_seed(20260508)
    rn = lambda *shape, std=0.02: (torch.randn(shape, device=dev, generator=gen) * std).to(torch.bfloat16)
    gain = lambda: (1.0 + 0.1 * torch.randn((d,), device=dev, generator=gen)).to(torch.bfloat16)
    m = B.DareModel(L, d, H, ffn, V, 1, T, B.DARE_BF16, 1e-5, 10000.0)
    for l in range(L):
        m.set_layer(l, gain(), rn(d, d), rn(d, d), rn(d, d), rn(d, d), gain(), rn(d, ffn), rn(d, ffn), rn(ffn, d))
    m.set_io(rn(V, d, std=1.0), gain(), None)
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.PCG64(20260508))
    mask_id = V - 1
    ids0 = np.full((1, T), mask_id, dtype=np.int32)
    ids0[0, :P] = rng.integers(0, mask_id, P)
    order = []
    for b0 in range(P, T, 32):
        order += list(b0 + rng.permutation(32))
    new_ids = rng.integers(0, mask_id, len(order))
    refreshed = torch.zeros((L, 1), dtype=torch.int32, device=dev)
    out = {}
    for name, mode, thr in (("kvo", B.MODE_KVO, 1e-3), ("dense", B.MODE_DENSE, 0.0)):
        ids = torch.from_numpy(ids0.copy()).to(dev)
        m.step(B.MODE_DENSE, 0.0, ids)               # fills every layer's caches
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_steps + 1)]
        counts = []
        ev[0].record()
        for t in range(n_steps):
            ids[0, order[t]] = int(new_ids[t])
            m.step(mode, thr, ids, None, refreshed)
            ev[t + 1].record()
            counts.append(refreshed.clone())
        torch.cuda.synchronize()
        us = np.array([ev[t].elapsed_time(ev[t + 1]) * 1e3 for t in range(n_steps)])
        ref = torch.stack(counts).float().cpu().numpy()[:, :, 0]          # [steps, layers]
        out[name] = {"step_us_median": float(np.median(us)), "layer_us_mean": float(np.mean(us) / L),
                     "reuse_mean": float(1.0 - ref.mean() / T),
                     "reuse_by_layer_first_mid_last": [float(1.0 - ref[:, l].mean() / T) for l in (0, L // 2, L - 1)]}
    out["layer_latency_vs_dense"] = out["kvo"]["layer_us_mean"] / out["dense"]["layer_us_mean"]

    # Layer-wise reuse rates as the paper sets them (Sec. 3.1): mean drift per layer over a few
    # calibration steps, phi_l = L phi_bar softmax(-s_l / eps) with the paper's phi_bar = 0.3, then
    # the quantile rule with each layer's own rate.
    ids = torch.from_numpy(ids0.copy()).to(dev)
    m.step(B.MODE_DENSE, 0.0, ids)
    for l in range(L):
        m.layer(l).drift_stats_enable(True)
    n_cal = min(8, n_steps)
    for t in range(n_cal):
        ids[0, order[t]] = int(new_ids[t])
        m.step(B.MODE_DENSE, 0.0, ids)
    s_layers = [m.layer(l).drift_stats_read()[0] for l in range(L)]
    for l in range(L):
        m.layer(l).drift_stats_enable(False)
    eps = max(float(np.std(s_layers)), 1e-9)
    phis = B.dare_allocate_quantiles(s_layers, 0.3, eps)
    m.set_rule(B.RULE_QUANTILE)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    counts = []
    n_q = max(4, n_steps // 4)
    ev[0].record()
    for t in range(n_cal, n_cal + n_q):
        ids[0, order[t]] = int(new_ids[t])
        m.step(B.MODE_KVO, phis, ids, None, refreshed)
        counts.append(refreshed.clone())
    ev[1].record()
    torch.cuda.synchronize()
    m.set_rule(B.RULE_SCORE)
    ref = torch.stack(counts).float().cpu().numpy()[:, :, 0]
    out["quantile_allocation"] = {
        "phi_bar": 0.3, "eps": eps, "mean_drift_first_mid_last": [s_layers[0], s_layers[L // 2], s_layers[-1]],
        "phi_min_max": [float(min(phis)), float(max(phis))], "phi_mean": float(np.mean(phis)),
        "reuse_mean": float(1.0 - ref.mean() / T), "layer_us_mean": ev[0].elapsed_time(ev[1]) * 1e3 / n_q / L,
        "vs_dense": ev[0].elapsed_time(ev[1]) * 1e3 / n_q / L / out["dense"]["layer_us_mean"]}
    out["config"] = {"layers": L, "hidden": d, "heads": H, "ffn": ffn, "vocab": V, "seq": T, "prompt": P,
                     "block": 32, "steps_timed": n_steps, "threshold": 1e-3,
                     "note": "per-layer latency includes the layer's feed-forward, which DARE does not touch"}
    m.destroy()
    return out


def cold_weights(torch, B, layer0, wdev, xa, xb, Bn, T, d, H, tau, n_layers=8):
    """The same step with weights that cannot stay in the 256 MB last-level cache:
    round-robin over 8 layers with distinct weights (1 GiB of packed weights), each with
    its own caches.  Weight values come from torch's seeded generator (timing only)."""
    gen = torch.Generator(device=xa.device)
    gen.manual_seed(4321)
    layers, states = [layer0], []
    for _ in range(n_layers - 1):
        ws = [(torch.randn((d, d), device=xa.device, generator=gen) * 0.02).to(torch.bfloat16)
              for _ in range(4)]
        layers.append(B.DareLayer(*ws, n_heads=H, max_batch=Bn, max_seq=T))
        del ws
    mask = torch.zeros((Bn, T), dtype=torch.uint8, device=xa.device)
    for ly in layers:
        st = ly.new_state(Bn, T)
        ly.layer_step(B.MODE_DENSE, 0.0, xa, st["q_prev"], st["k_cache"], st["v_cache"],
                      st["o_cache"], st["o_cache"], mask)
        states.append(st)
    out = {}
    for name, mode in (("kvo", B.MODE_KVO), ("dense", B.MODE_DENSE)):
        def run(n, mode=mode):
            # layer l sees x_cur, x_prev, x_cur, ... on its own consecutive steps
            for i in range(n * n_layers):
                ly, st = layers[i % n_layers], states[i % n_layers]
                x = xb if (i // n_layers) % 2 == 0 else xa
                ly.layer_step(mode, tau, x, st["q_prev"], st["k_cache"], st["v_cache"],
                              st["o_cache"], st["o_cache"], mask)
        out[name + "_us"] = _time_us(torch, run, 12, warm=2) / n_layers
        out[name + "_reuse_last"] = float(mask.float().mean().item())
    out["latency_vs_dense"] = out["kvo_us"] / out["dense_us"]
    out["layers"] = n_layers
    for ly in layers[1:]:
        ly.destroy()
    return out


def measured_peaks(torch, B, dev, d):
    """What this GPU sustains on a plain copy (1 GiB read + 1 GiB written) and on a
    register-resident MFMA loop, next to the datasheet peaks the fractions use."""
    src = torch.ones((1 << 17, d), dtype=torch.bfloat16, device=dev)   # 1 GiB
    dst = torch.empty_like(src)
    us = _time_us(torch, lambda n: [B.dare_k_copy_rows(src, dst) for _ in range(n)], 10)
    copy_gbs = 2.0 * src.numel() * 2 / (us * 1e-6) / 1e9
    del src, dst
    res = {"hbm_copy_GBs": copy_gbs, "hbm_datasheet_GBs": HBM_PEAK_GBS,
           "mfma_bf16_datasheet_TFLOPs": MFMA_BF16_PEAK_TFLOPS}
    for pattern, key in ((0, "mfma_bf16_loop_zero_operands_TFLOPs"), (1, "mfma_bf16_loop_varied_operands_TFLOPs")):
        flops = [0.0]

        def run(n, pattern=pattern):
            for _ in range(n):
                flops[0] = B.dare_bench_mfma_loop(2048, 4096, pattern)
        us = _time_us(torch, run, 5, warm=2)
        res[key] = flops[0] / (us * 1e-6) / 1e12
    # what one CU pulls from memory into LDS when 8 .. 256 CUs pull at once (every workgroup
    # walks 12 MiB of its own, 3 GiB in all at 256: nothing is re-read)
    per_block = 12 << 20
    big = torch.ones(((256 * per_block) // 4,), dtype=torch.int32, device=dev)
    res["stream_to_lds_GBs_per_cu"] = {}
    for n_blocks in (8, 32, 64, 128, 256):
        us = _time_us(torch, lambda n, nb=n_blocks: [B.dare_bench_stream(nb, per_block, 2, big) for _ in range(n)],
                      3, warm=1)
        res["stream_to_lds_GBs_per_cu"][str(n_blocks)] = per_block / (us * 1e-6) / 1e9
    del big
    return res


def other_kernels_at_c2(torch, B, np, dev, d, H, Dh):
    """Kernel-level evidence at the large configuration (8 x 2048 tokens): the stages that
    move too few bytes at 1024 tokens to say anything about bandwidth, and the
    MFMA-bound stages at a size that fills the chip."""
    Bn, T = 8, 2048
    n_tok = Bn * T
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    rnd = lambda *shape: torch.randn(shape, device=dev, generator=gen)
    out = []
    # drift score + decision + score-cache update
    q_new = rnd(n_tok, Dh)
    q_prev = rnd(n_tok, Dh)
    scores = torch.empty(n_tok, dtype=torch.float32, device=dev)
    mask = torch.empty(n_tok, dtype=torch.uint8, device=dev)
    us = _time_graph_us(torch, lambda st: B.dare_k_score(q_new, q_prev, 5e-3, False, scores, mask, stream=st))
    nbytes = n_tok * (3 * Dh * 4 + 5)
    out.append({"kernel": "score_kernel (%d tokens)" % n_tok, "bound": "hbm",
                "achieved": nbytes / (us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "us_per_launch": us})
    # compaction
    mask.copy_((torch.rand(n_tok, device=dev, generator=gen) < 0.8).to(torch.uint8))
    sel_idx = torch.empty(n_tok, dtype=torch.int32, device=dev)
    sel_count = torch.empty(Bn, dtype=torch.int32, device=dev)
    sel_off = torch.empty(Bn + 1, dtype=torch.int32, device=dev)
    us = _time_graph_us(torch, lambda st: B.dare_k_compact(mask, Bn, T, sel_idx, sel_count, sel_off, stream=st))
    n_sel = int(sel_off[-1].item())
    nbytes = n_tok + 4 * n_sel
    out.append({"kernel": "compact_kernel (%d tokens, %d refreshed)" % (n_tok, n_sel), "bound": "hbm",
                "achieved": nbytes / (us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "us_per_launch": us,
                "note": "latency bound: one pass over %d KiB" % (nbytes >> 10)})
    # row copy of the refreshed rows (cache merge when out and o_cache differ)
    src = rnd(n_tok, d).to(torch.bfloat16)
    dst = torch.empty_like(src)
    m_dev = sel_off[-1:].clone()
    us = _time_graph_us(torch, lambda st: B.dare_k_copy_rows(src, dst, idx=sel_idx, m_dev=m_dev, stream=st))
    nbytes = 2 * n_sel * d * 2
    out.append({"kernel": "copy_rows_kernel (%d rows of 8 KiB)" % n_sel, "bound": "hbm",
                "achieved": nbytes / (us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "us_per_launch": us})
    # refreshed-row Q/K/V projection at this size: MFMA bound (n well above the crossover)
    wt = (rnd(3 * d, d) * 0.02).to(torch.bfloat16)
    outs = [torch.empty((n_tok, d), dtype=torch.bfloat16, device=dev) for _ in range(3)]
    us = _time_us(torch, lambda n: [B.dare_k_gemm(src, wt, outs, d, idx=sel_idx, m_dev=m_dev, m_max=n_tok)
                                    for _ in range(n)], 10)
    tf = 2.0 * n_sel * d * 3 * d / (us * 1e-6) / 1e12
    out.append({"kernel": "gemm_bf16_rows_wide_kernel (%d refreshed rows x %d x %d)" % (n_sel, 3 * d, d),
                "bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "us_per_launch": us})
    us = _time_us(torch, lambda n: [B.dare_k_gemm(src, wt, outs, d) for _ in range(n)], 5)
    tf = 2.0 * n_tok * d * 3 * d / (us * 1e-6) / 1e12
    out.append({"kernel": "gemm_bf16_kernel (all-row Q/K/V projection, %d x %d x %d)" % (n_tok, 3 * d, d),
                "bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "us_per_launch": us})
    # attention, all rows and refreshed rows
    q, k, v = outs
    att = torch.empty_like(q)
    us = _time_us(torch, lambda n: [B.dare_k_attention(q, k, v, att, Bn, T, H, Dh) for _ in range(n)], 5)
    tf = 4.0 * n_tok * T * d / (us * 1e-6) / 1e12
    out.append({"kernel": "attn_bf16_kernel (all rows, %d x %d tokens)" % (Bn, T), "bound": "mfma",
                "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "us_per_launch": us})
    us = _time_us(torch, lambda n: [B.dare_k_attention(q, k, v, att, Bn, T, H, Dh, idx=sel_idx, sel_off=sel_off)
                                    for _ in range(n)], 10)
    tf = 4.0 * n_sel * T * d / (us * 1e-6) / 1e12
    out.append({"kernel": "attn_bf16_kernel (%d refreshed rows of %d x %d tokens)" % (n_sel, Bn, T),
                "bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "us_per_launch": us})
    return out


def stored_traffic():
    """HBM bytes per launch of the dominant kernel, from the committed counter summary
    (two rocprofv3 --pmc passes over `bench.py --only-dominant`, scaled by the copy
    kernel of the same run); None when the summary is absent."""
    path = os.path.join(ROOT, "profiles", "gemm_rows_qkv_llada8b_pmc.txt")
    try:
        for line in open(path):
            if line.strip().startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(weights, seed, cfg, tau):
    """Time the CPU oracle (as it stands) on the same workload: one dense step to fill
    the caches (untimed), then KV+O steps for a bounded time."""
    import numpy as np
    from oracle import dare_oracle as orc
    from paper_2605_08134_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    Bn, T, d, H, Dh = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["n_heads"], cfg["head_dim"]
    h = synth.make_hidden_pair(seed, Bn, T, d, 0.20, "bf16")
    w = weights
    out, Q, K, V = orc.dense_layer(h["x_prev"], w["wq"], w["wk"], w["wv"], w["wo"], H)
    st = dict(q_prev=Q[:, :, :Dh], k_cache=K, v_cache=V, o_cache=out)
    xs = (h["x_cur"], h["x_prev"])
    t0 = time.perf_counter()
    n = 0
    while n < 2 or (time.perf_counter() - t0 < 12.0 and n < 400):
        r = orc.layer_step(orc.MODE_KVO, tau, xs[n % 2], w["wq"], w["wk"], w["wv"], w["wo"],
                           st["q_prev"], st["k_cache"], st["v_cache"], st["o_cache"], H)
        st = {k: r[k] for k in st}
        n += 1
    dt = (time.perf_counter() - t0) / n
    return {"value": Bn * T / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d KV+O steps of the full workload (1024 tokens, 80%% reuse); the oracle is numpy "
                      "float64 whose matrix products run in the threaded BLAS numpy links (not plain loops), "
                      "%.2f s per step" % (n, dt)}


if __name__ == "__main__":
    main()
