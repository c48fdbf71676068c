#!/usr/bin/env python3
"""Benchmark of the PowerGossip hot path on one MI355X.

A "step" is one gossip round over the whole synthetic parameter set (every worker, every
layer): power_steps x (P-sweep, orthonormalise, Q-sweep, combine) and the rank-r update.
The timed region runs `--steps` rounds through pg_run (consecutive rounds, the update of one
round sharing its pass with the first sweep of the next) with all inputs resident in HBM.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published

# Bytes that crossed the L2 -> fabric boundary per launch of a kernel kind, from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this script, each scaled by the same counter's reading for a plain
# device copy of known size (factors 2.000 and 1.000); see profiles/vgg16_r1_traffic_counters.txt.
MEASURED_TRAFFIC_BYTES = {
    ("vgg16_r1", "update_sweep_p"): 960.2e6 + 943.6e6,
    ("vgg16_r1", "update"): 962.4e6 + 941.8e6,
    ("vgg16_r1", "update_sgd"): 1902.9e6 + 941.8e6,
    ("vgg16_r1", "sweep_p"): 957.5e6 + 1.8e6,
    ("vgg16_r1", "sweep_q"): 945.9e6 + 8.7e6,
}


def cpu_baseline(wl, seconds_budget: float):
    """Time the CPU oracle (as it stands, single-threaded) on the same workload."""
    import numpy as np
    from oracle import pg_oracle as O
    prob = O.Problem(wl.n_workers, wl.edges, wl.edge_w.astype(np.float64), wl.shapes,
                     wl.rank, wl.power_steps)
    X, Q = wl.all_params(), wl.all_q()
    O.build()
    t0 = time.perf_counter()
    rounds = 0
    while True:
        O.gossip_round(prob, X, Q)
        rounds += 1
        dt = time.perf_counter() - t0
        if dt >= seconds_budget or rounds >= 50:
            break
    return {"value": rounds / dt, "unit": "rounds/s", "cores": 1, "kind": "oracle",
            "sample": f"{rounds} full round(s) of the same workload, all layers and workers, "
                      f"{dt:.1f} s on one host core ({os.cpu_count()} visible)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="vgg16_r1",
                    help="tiny | resnet20 | vgg16_r1 | vgg16_r2 | lstm | resnet50")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="CPU time budget of the oracle baseline (0 = skip)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run a plain device copy of this many MiB (known traffic, for scaling "
                         "hardware byte counters in a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all simulated workers share its HBM); "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2008_01425_amd import binding as B
    from paper_2008_01425_amd import workloads as W
    from paper_2008_01425_amd.device import GossipBuffers

    wl = W.get(args.workload)
    gb = GossipBuffers.from_workload(wl)
    K, Wm = args.steps, args.warmup
    stream = torch.cuda.current_stream()

    # ---- timed region: K consecutive rounds, fused pipeline -------------------------------
    if Wm > 0:
        gb.run(Wm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    gb.run(K)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / K

    # ---- the same K rounds as isolated pg_round calls (no cross-round fusion) -------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        gb.round()
    torch.cuda.synchronize()
    dt_unfused = time.perf_counter() - t0

    # ---- per-kernel durations: HIP events on the launch stream, both pipelines ------------
    def profile(fn):
        B.pg_profile_enable(gb.ctx, True)
        fn()
        torch.cuda.synchronize()
        rows = B.pg_profile_collect(gb.ctx)
        B.pg_profile_enable(gb.ctx, False)
        out = {}
        for r in rows:
            gbs = r["bytes"] / (r["ms"] * 1e-3) / 1e9 if r["ms"] > 0 else 0.0
            out[r["name"]] = {"launches": r["launches"], "avg_ms": r["ms"] / max(1, r["launches"]),
                              "total_ms": r["ms"], "algorithmic_bytes_per_launch": r["bytes"] / max(1, r["launches"]),
                              "GBps": gbs, "frac_of_peak": gbs / HBM_PEAK_GBS}
        return out

    Kp = min(K, 50)
    k_fused = profile(lambda: gb.run(Kp))
    k_unfused = profile(lambda: [gb.round() for _ in range(Kp)])

    # ---- Algorithm 1's step: the same round with the gradient term fused into the update ----
    gb.alloc_grads()
    for g in gb.g:
        g.normal_(0.0, 1e-3)
    gb.round_sgd(0.1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(Kp):
        gb.round_sgd(0.1)
    torch.cuda.synchronize()
    dt_sgd = time.perf_counter() - t0
    k_sgd = profile(lambda: [gb.round_sgd(0.1) for _ in range(Kp)])

    # ---- Algorithm 2 one iteration per call (the paper's "1 iteration" setting), with gradient
    gb.alloc_pstate()
    gb.iterate(0, 1, 0.1)
    gb.iterate(1, 1, 0.1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(2, 2 + 2 * Kp):
        gb.iterate(k, 1, 0.1)
    torch.cuda.synchronize()
    dt_it = time.perf_counter() - t0

    # the dominant kernel of the timed (fused) pipeline
    dom = max(k_fused.items(), key=lambda kv: kv[1]["total_ms"])
    roofline = {"bound": "hbm", "kernel": dom[0], "achieved": dom[1]["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": dom[1]["GBps"] / HBM_PEAK_GBS,
                "traffic": MEASURED_TRAFFIC_BYTES.get((wl.name, dom[0])),
                "algorithmic_bytes_per_launch": dom[1]["algorithmic_bytes_per_launch"],
                "avg_launch_ms": dom[1]["avg_ms"]}

    bytes_fused = B.pg_round_bytes(gb.ctx, True)
    bytes_unfused = B.pg_round_bytes(gb.ctx, False)
    result = {
        "metric": "gossip rounds/sec + achieved HBM GB/s (% of peak), fp32, 1 MI355X",
        "value": K / dt,
        "unit": "rounds/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "n_workers": wl.n_workers, "n_edges": wl.n_edges,
                   "layers": len(wl.shapes), "params_per_worker": wl.params_per_worker,
                   "rank": wl.rank, "power_steps": wl.power_steps,
                   "storage": "f32", "accumulate": "f64", "pipeline": "pg_run (fused update + next sweep)"},
        "round_GBps": bytes_fused / (ms_per_step * 1e-3) / 1e9,
        "round_frac_of_peak": bytes_fused / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "bytes_per_param_per_round": bytes_fused / (wl.n_workers * wl.params_per_worker),
        "pg_round_unfused": {"rounds_per_s": K / dt_unfused, "ms_per_step": dt_unfused * 1e3 / K,
                             "GBps": bytes_unfused / (dt_unfused / K) / 1e9,
                             "bytes_per_param_per_round": bytes_unfused / (wl.n_workers * wl.params_per_worker)},
        "pg_round_sgd": {"rounds_per_s": Kp / dt_sgd, "ms_per_step": dt_sgd * 1e3 / Kp,
                         "bytes_per_param_per_round": (bytes_unfused / (wl.n_workers * wl.params_per_worker)) + 4,
                         "update_sgd_kernel": k_sgd.get("update_sgd")},
        "pg_iterate_1_sgd": {"iterations_per_s": 2 * Kp / dt_it, "ms_per_iteration": dt_it * 1e3 / (2 * Kp),
                             "bytes_per_param_per_iteration": 16.0,
                             "GBps": 16.0 * wl.n_workers * wl.params_per_worker / (dt_it / (2 * Kp)) / 1e9},
        "roofline": roofline,
        "kernels_fused": k_fused,
        "kernels_unfused": k_unfused,
    }
    gb.close()
    del gb
    torch.cuda.empty_cache()
    # ---- practical ceiling: a plain device-to-device copy of 1 GiB (read + write counted) ----
    n_copy = (1 << 30) // 4
    src = torch.ones(n_copy, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        dst.copy_(src)
    torch.cuda.synchronize()
    dt_copy = (time.perf_counter() - t0) / 20
    result["copy_ceiling"] = {"GBps": 8.0 * n_copy / dt_copy / 1e9, "frac_of_peak": 8.0 * n_copy / dt_copy / 1e9 / HBM_PEAK_GBS,
                              "what": "torch device-to-device copy of 1 GiB, bytes read + bytes written per second"}
    del src, dst
    torch.cuda.empty_cache()
    if args.copy_calibration > 0:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["copy_calibration"] = {"MiB": args.copy_calibration, "bytes_read": 4 * n, "bytes_written": 4 * n}
        del src, dst
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(wl, args.cpu_seconds)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
