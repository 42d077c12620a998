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
        for i in range(n):
            x = xb if i % 2 == 0 else xa
            layer.layer_step(mode, tau, x, state["q_prev"], state["k_cache"], state["v_cache"],
                             state["o_cache"], state["o_cache"], mask, None, sel_count, None)

    def time_mode(mode, xa, xb, steps, warmup):
        state = layer.new_state(Bn, T)
        fill(state, xa)
        run_steps(mode, xa, xb, state, warmup + (warmup % 2))   # even: next step sees xb again
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        run_steps(mode, xa, xb, state, steps)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        ms = e0.elapsed_time(e1) / steps
        reuse = float(mask.float().mean().item())
        return ms, wall_ms / steps, reuse, int(sel_count.sum().item())

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

    dominant(10)
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
        "kernel": "gemm_bf16_kernel (refreshed-row Q/K/V projection, %d rows x %d x %d)" % (n_sel, 3 * d, d),
        "bound": "hbm",
        "achieved": dom_bytes / (dom_ms * 1e-3) / 1e9,
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": dom_bytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "traffic": stored_traffic(),
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
    ms_dense, _, _, _ = time_mode(B.MODE_DENSE, xa, xb, max(20, args.steps // 4), args.warmup)

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
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "llada8b layer: hidden 4096, 32 heads x 128, seq 1024, batch 1, "
                               "20% of tokens perturbed, threshold 5e-3, mode KV+O",
                   "reuse": reuse, "refreshed_rows": n_ref, "dense_us": ms_dense * 1e3,
                   "latency_vs_dense": ms_kvo / ms_dense},
        "roofline": roofline,
        "roofline_other": roofline_other,
        "cpu_baseline": cpu,
        "sweep": sweep,
    }
    print(json.dumps(out))


def stored_traffic():
    """HBM bytes per launch of the dominant kernel, from the committed counter summary
    (two rocprofv3 --pmc passes over `bench.py --only-dominant`, scaled by the copy
    kernel of the same run); None when the summary is absent."""
    path = os.path.join(ROOT, "profiles", "gemm_rows_qkv_llada8b_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
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
    while n < 2 or (time.perf_counter() - t0 < 10.0 and n < 50):
        r = orc.layer_step(orc.MODE_KVO, tau, xs[n % 2], w["wq"], w["wk"], w["wv"], w["wo"],
                           st["q_prev"], st["k_cache"], st["v_cache"], st["o_cache"], H)
        st = {k: r[k] for k in st}
        n += 1
    dt = (time.perf_counter() - t0) / n
    return {"value": Bn * T / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d KV+O steps of the full workload (1024 tokens, 80%% reuse), numpy float64, "
                      "%.2f s per step" % (n, dt)}


if __name__ == "__main__":
    main()
