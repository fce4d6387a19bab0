#!/usr/bin/env python3
"""Benchmark of the DGS hot path on one MI355X.

A step = one pass of the whole hot path on the ResNet-50-shaped workload
(25,557,032 fp32 parameters in 161 tensors, density 1e-3, one worker):
dgs_worker_step -> dgs_server_push -> dgs_server_pull.  Inputs are seeded and
synthetic (per-tensor log-uniform scale, Gaussian values, a pool of 8 gradient
sets cycled), resident in HBM before the timed region starts.

Prints ONE JSON line: params/s over the timed steps, the roofline of the
dominant kernel (the fused accumulate + candidate streaming pass, timed with HIP
events on its own stream), and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
POOL = 8
DENSITY = 1e-3
LR, MOMENTUM = 1.0, 0.9
SEED = 2

# HBM traffic per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs (see profiles/); None until measured for this workload.
MEASURED_TRAFFIC_BYTES = None


def make_workload():
    from paper_1910_10929_amd import synth
    off = synth.layout_resnet50()
    scales = synth.tensor_scales(len(off) - 1, SEED)
    rng = np.random.default_rng(SEED)
    grads = [synth.gaussian_grads(off, scales, rng) for _ in range(POOL)]
    return off, grads


def cpu_baseline(off, grads, steps=2):
    """The oracle as it stands, single thread, on the first `steps` steps of the
    same workload."""
    from oracle import dgs_oracle as oracle
    n = int(off[-1])
    state = np.zeros(n, np.float32)
    model = np.zeros(n, np.float32)
    diff = np.zeros((1, n), np.float32)
    oracle.lib()
    t0 = time.perf_counter()
    for t in range(steps):
        i, v = oracle.worker_step(grads[t % POOL], state, off, LR, np.float32(MOMENTUM), DENSITY)
        oracle.server_push(model, diff, i, v)
        oracle.server_pull(diff, 0, off, DENSITY)
    dt = time.perf_counter() - t0
    return {"value": n * steps / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": f"first {steps} steps of the same workload (worker_step + push + pull), {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--force-exact", action="store_true", help="time the non-predicted two-pass path")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1910_10929_amd import dgs

    dgs.lib()                       # no fallback: fails if libdgs.so is missing
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    dev = "cuda:0"
    off, grads = make_workload()
    n = int(off[-1])
    J = len(off) - 1

    ctx = dgs.Context(off, W=1, device=dev)
    if args.force_exact:
        ctx.set_option(dgs.OPT_FORCE_EXACT, 1)
    K = ctx.nnz(DENSITY)
    g_dev = [torch.from_numpy(g).to(dev) for g in grads]
    state = torch.zeros(n, dtype=torch.float32, device=dev)
    model = torch.zeros(n, dtype=torch.float32, device=dev)
    diff = torch.zeros((1, n), dtype=torch.float32, device=dev)
    ctx.server_attach(diff)
    idx = torch.zeros(K, dtype=torch.int32, device=dev)
    val = torch.zeros(K, dtype=torch.float32, device=dev)
    pidx = torch.zeros(K, dtype=torch.int32, device=dev)
    pval = torch.zeros(K, dtype=torch.float32, device=dev)

    def step(t):
        ctx.worker_step(g_dev[t % POOL], state, LR, MOMENTUM, DENSITY, idx, val)
        ctx.server_push(model, 0, idx, val, K)
        ctx.server_pull(0, DENSITY, pidx, pval)

    t = 0
    for _ in range(args.warmup):
        step(t)
        t += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(t)
        t += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # per-kernel durations, HIP events on the context's stream, same workload continuing
    ctx.set_option(dgs.OPT_PROFILE, 1)
    prof_steps = min(args.steps, 200)
    for _ in range(prof_steps):
        step(t)
        t += 1
    torch.cuda.synchronize()
    kinds = {"worker_stream": dgs.PROF_WORKER_STREAM, "worker_select": dgs.PROF_WORKER_SELECT,
             "pull_stream": dgs.PROF_PULL_STREAM, "pull_select": dgs.PROF_PULL_SELECT,
             "push": dgs.PROF_PUSH, "exact_extra": dgs.PROF_EXACT_EXTRA}
    kernel_us = {}
    for name, kind in kinds.items():
        cnt, ms = ctx.profile_read(kind)
        kernel_us[name] = (ms / cnt * 1e3) if cnt else None
    ctx.set_option(dgs.OPT_PROFILE, 0)
    st = ctx.stats()

    # roofline of the dominant kernel: 12 B per parameter (read grad, read state, write state)
    alg_bytes = 12.0 * n
    ws_us = kernel_us["worker_stream"]
    achieved = alg_bytes / (ws_us * 1e-6) / 1e9 if ws_us else None
    roofline = {"bound": "hbm", "kernel": "k_stream<fma,collect> (dgs_worker_step streaming pass)",
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                "traffic": MEASURED_TRAFFIC_BYTES, "algorithmic_bytes": alg_bytes,
                "avg_launch_us": ws_us}

    out = {
        "metric": "params/sec and HBM GB/s (% of peak) for dgs_worker_step + server push/pull",
        "value": n * args.steps / dt,
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "resnet50-shaped 25,557,032 fp32 params in 161 tensors, density 1e-3, "
                               "1 worker: worker_step + server_push + server_pull per step",
                   "n": n, "tensors": J, "density": DENSITY, "K": K, "workers": 1,
                   "momentum": MOMENTUM, "path": "exact" if args.force_exact else "predicted"},
        "roofline": roofline,
        "kernel_us": kernel_us,
        "step_algorithmic_GBs": (12.0 * n + 12.0 * K + 8.0 * K + 16.0 * K + 4.0 * n + 12.0 * K) / (dt / args.steps) / 1e9,
        "stats": {"exact_calls": st.exact_calls, "fallback_tensors": st.fallback_tensors,
                  "internal_errors": st.internal_errors},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(off, grads)
    else:
        out["cpu_baseline"] = None
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
