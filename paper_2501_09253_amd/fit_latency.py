"""Fit the scheduler's latency model on this machine: measure pserve_block_forward on a set of mixed-resolution batch
compositions (seeded, synthetic weights), fit per-step latency = w0 + w1 * patches + w2 * resolutions
+ w3 * 1e-6 * sum tokens^2 by pserve_latency_fit on 80 % of them and report the error on the rest.

    python -m paper_2501_09253_amd.fit_latency [--samples 40] [--C 640]

Stands in for the 200 measured resolution combinations behind the paper's latency predictor ("Mixed-Resolution
Throughput Analyzer"); prints one JSON line with the model and its errors.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--samples", type=int, default=40)
    ap.add_argument("--C", type=int, default=640)
    ap.add_argument("--patch", type=int, default=16)
    args = ap.parse_args()
    import numpy as np
    import torch
    import paper_2501_09253_amd as ps
    import workloads as wl
    from harness import GpuRun

    rng = np.random.default_rng(2501)
    sizes = (32, 48, 64, 96)
    stages = (wl.LSATTN, wl.LXATTN, wl.LFFN)
    X, y = [], []
    for k in range(args.samples):
        n = int(rng.integers(1, 9))
        res = [(int(s), int(s)) for s in rng.choice(sizes, n)]
        cfg = wl.custom_config(res, (args.patch, args.patch), C=args.C, G=32, heads=args.C // 64, stages=stages,
                               dtype="bf16", ctx_len=77, ctx_dim=2048, seed=7)
        run = GpuRun(wl.make_workload(cfg))
        yb = torch.empty_like(run.x)
        for _ in range(3):
            run.cache.forward(run.x, run.ctx, None, y=yb)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            run.cache.forward(run.x, run.ctx, None, y=yb)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        X.append([float(run.plan.P), float(len(set(res))), 1e-6 * sum(float(h * w) ** 2 for h, w in res)])
        y.append(ms)
        del run
    X, y = np.array(X), np.array(y)
    n_fit = max(4, int(0.8 * len(y)))
    w = ps.latency_fit(X[:n_fit], y[:n_fit])
    pred = w[0] + X @ np.array(w[1:])
    err = np.abs(pred - y) / y
    print(json.dumps({"model": w, "samples": len(y), "fit_on": n_fit, "max_rel_err_fit": float(err[:n_fit].max()),
                      "max_rel_err_held_out": float(err[n_fit:].max()) if n_fit < len(y) else None,
                      "mean_rel_err": float(err.mean()), "latency_ms_range": [float(y.min()), float(y.max())],
                      "block": "LSATTN+LXATTN+LFFN", "C": args.C, "patch": args.patch}))


if __name__ == "__main__":
    main()
