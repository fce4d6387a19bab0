#!/usr/bin/env python3
"""Benchmark of the DGS hot path on one MI355X.

Default workload (`--workload c2`): a step = one pass of the whole hot path on
the ResNet-50-shaped parameter set (25,557,032 fp32 parameters in 161 tensors,
density 1e-3, one worker): dgs_worker_step -> dgs_server_push ->
dgs_server_pull.  Inputs are seeded and synthetic (per-tensor log-uniform scale,
Gaussian values, a pool of gradient sets cycled), resident in HBM before the
timed region starts.

Other workloads, for the design notes (not the default bench line):
  c1  one flat tensor of 2^20 parameters, density 0.01 (latency-bound)
  c3  server stress: 32 workers' difference rows, step = push + pull of a seeded worker
  c4  transformer-shaped 108M parameters, heavy-tailed gradients, row-sparse embedding
  c5  1e9 parameters in 64 tensors, `--density` 1e-4 or 1e-2, step as in c2

Prints ONE JSON line: params/s over the timed steps, the roofline of the
dominant kernel (the streaming pass, timed with HIP events on the stream it is
launched on), and the CPU oracle timed on a bounded sample.
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
LR, MOMENTUM = 1.0, 0.9

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs (FETCH_SIZE,
# WRITE_SIZE, scaled by the same counters on a copy kernel of known size); the
# summaries are under profiles/.  None = not measured for that workload.
MEASURED_TRAFFIC_BYTES = {"c1": None, "c2": 308.61e6, "c3": None, "c4": None, "c5": None}


def make_workload(name, density):
    from paper_1910_10929_amd import synth
    if name in ("c2", "c3"):
        off = synth.layout_resnet50()
        seed = 2 if name == "c2" else 3
        scales = synth.tensor_scales(len(off) - 1, seed)
        rng = np.random.default_rng(seed)
        if name == "c2":
            grads = [synth.gaussian_grads(off, scales, rng) for _ in range(8)]
            return dict(off=off, grads=grads, W=1, density=density or 1e-3,
                        desc="resnet50-shaped 25,557,032 fp32 params in 161 tensors, 1 worker: "
                             "worker_step + server_push + server_pull per step")
        rho = density or 1e-3
        sizes = np.diff(off.astype(np.int64))
        counts = np.ceil(rho * sizes.astype(np.float64)).astype(np.int64)
        payloads = [synth.sparse_payload(off, counts, scales, rng) for _ in range(32)]
        order = synth.event_schedule(32, 4096, 3)
        return dict(off=off, payloads=payloads, order=order, W=32, density=rho,
                    desc="server stress: 25,557,032-param model, 32 workers' difference rows, "
                         "step = server_push of a pooled payload + server_pull of a seeded worker")
    if name == "c1":
        off = synth.layout_flat(1 << 20)
        rng = np.random.default_rng(0)
        grads = [synth.gaussian(1 << 20, rng) for _ in range(8)]
        return dict(off=off, grads=grads, W=1, density=density or 0.01,
                    desc="one flat tensor of 1,048,576 fp32 params, N(0,1), 1 worker: worker_step + "
                         "server_push + server_pull per step (latency-bound)")
    if name == "c4":
        off = synth.layout_transformer()
        J = len(off) - 1
        scales = synth.tensor_scales(J, 4)
        rng = np.random.default_rng(4)
        grads = []
        for _ in range(4):
            g = synth.student_t_grads(off, scales, rng)
            synth.zero_rows(g, int(off[J - 1]), 30522, 768, 0.05, rng)
            grads.append(g)
        return dict(off=off, grads=grads, W=1, density=density or 1e-3,
                    desc="transformer-shaped 108,375,552 fp32 params in 49 tensors, Student-t(3) gradients, "
                         "embedding gradient 95 % zero rows, 1 worker: worker_step + server_push + "
                         "server_pull per step")
    if name == "c5":
        off = synth.layout_equal(1_000_000_000, 64)
        scales = synth.tensor_scales(64, 5)
        rng = np.random.default_rng(5)
        grads = [synth.tiled_gaussian_grads(off, scales, rng) for _ in range(2)]
        return dict(off=off, grads=grads, W=1, density=density or 1e-4,
                    desc="1e9 fp32 params in 64 equal tensors, 1 worker: worker_step + "
                         "server_push + server_pull per step")
    raise SystemExit(f"unknown workload {name}")


def cpu_baseline(wl, name, budget_s=20.0):
    """The oracle as it stands, single thread, on the first steps of the same
    workload (as many as fit in about `budget_s` seconds, at least one)."""
    from oracle import dgs_oracle as oracle
    off = wl["off"]
    n = int(off[-1])
    rho = wl["density"]
    oracle.lib()
    model = np.zeros(n, np.float32)
    steps = 0
    t0 = time.perf_counter()
    if name == "c3":
        diff = np.zeros((wl["W"], n), np.float32)
        while True:
            i, v = wl["payloads"][steps % len(wl["payloads"])]
            oracle.server_push(model, diff, i, v)
            oracle.server_pull(diff, int(wl["order"][steps]), off, rho)
            steps += 1
            if time.perf_counter() - t0 > budget_s * 0.5 or steps >= 64:
                break
        what = "events (push + pull)"
    else:
        state = np.zeros(n, np.float32)
        diff = np.zeros((1, n), np.float32)
        while True:
            g = wl["grads"][steps % len(wl["grads"])]
            i, v = oracle.worker_step(g, state, off, LR, np.float32(MOMENTUM), rho)
            oracle.server_push(model, diff, i, v)
            oracle.server_pull(diff, 0, off, rho)
            steps += 1
            if time.perf_counter() - t0 > budget_s * 0.5 or steps >= 16:
                break
        what = "steps (worker_step + push + pull)"
    dt = time.perf_counter() - t0
    return {"value": n * steps / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": f"first {steps} {what} of the same workload, {dt:.1f} s on one host core"}


def overlapped(torch, dgs, off, W, rho, K, g_dev, steps, warmup, n, step_bytes):
    """Worker and server as two contexts on two streams of default priority: the worker's
    step t+1 runs while the server handles push / pull t (the asynchrony of the method; with
    one worker the gradient of step t+1 is taken as given).  Messages are double-buffered and
    ordered with events."""
    dev = "cuda:0"
    sa, sb = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
    wctx = dgs.Context(off, W=0, device=dev, stream=sa)
    sctx = dgs.Context(off, W=W, device=dev, stream=sb)
    model = torch.zeros(n, dtype=torch.float32, device=dev)
    diff = torch.zeros((W, n), dtype=torch.float32, device=dev)
    sctx.server_attach(diff)
    state = torch.zeros(n, dtype=torch.float32, device=dev)
    msg = [(torch.zeros(K, dtype=torch.int32, device=dev), torch.zeros(K, dtype=torch.float32, device=dev))
           for _ in range(2)]
    pidx = torch.zeros(K, dtype=torch.int32, device=dev)
    pval = torch.zeros(K, dtype=torch.float32, device=dev)
    produced = [torch.cuda.Event() for _ in range(2)]
    consumed = [torch.cuda.Event() for _ in range(2)]
    torch.cuda.synchronize()

    def step(t):
        b = t % 2
        if t >= 2:
            sa.wait_event(consumed[b])                     # the server has read message t-2
        wctx.worker_step(g_dev[t % len(g_dev)], state, LR, MOMENTUM, rho, msg[b][0], msg[b][1])
        produced[b].record(sa)
        sb.wait_event(produced[b])
        sctx.server_push(model, 0, msg[b][0], msg[b][1], K)
        consumed[b].record(sb)
        sctx.server_pull(0, rho, pidx, pval)

    t = 0
    for _ in range(warmup):
        step(t)
        t += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(t)
        t += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = (wctx.stats(), sctx.stats())
    wctx.close()
    sctx.close()
    return {"ms_per_step": dt / steps * 1e3, "params_per_s": n * steps / dt,
            "step_algorithmic_GBs": step_bytes / (dt / steps) / 1e9,
            "internal_errors": st[0].internal_errors + st[1].internal_errors,
            "fallback_tensors": st[0].fallback_tensors + st[1].fallback_tensors}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--density", type=float, default=None)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--force-exact", action="store_true", help="time the non-predicted two-pass path")
    ap.add_argument("--server-form", default="diff", choices=["diff", "sent"],
                    help="c3 only: per-worker difference rows (default) or the printed form, "
                         "global model + what each worker has been sent")
    ap.add_argument("--overlap", action="store_true",
                    help="c2/c4/c5: also time worker and server on two streams (worker step t+1 "
                         "overlaps push/pull t); reported as an extra field, never as `value`")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run 20 elementwise copies of one 25,557,032-float tensor and exit "
                         "(known traffic, used to scale the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    name = args.workload
    # c3: the configuration's 1,000 events, after every row has been pulled several times (a row
    # is pulled once per 32 events, and its threshold hint needs a few pulls to settle)
    steps = args.steps if args.steps is not None else {"c5": 20, "c3": 1000}.get(name, 200)
    warmup = args.warmup if args.warmup is not None else {"c5": 12, "c3": 320}.get(name, 40)

    import torch
    from paper_1910_10929_amd import dgs

    dgs.lib()                       # no fallback: fails if libdgs.so is missing
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    dev = "cuda:0"
    if args.calibrate_copy:
        src = torch.randn(25_557_032, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(20):
            torch.mul(src, 1.0, out=dst)      # reads 102,228,128 B, writes 102,228,128 B
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"launches": 20, "read_bytes": src.numel() * 4,
                                             "write_bytes": src.numel() * 4}}))
        return
    wl = make_workload(name, args.density)
    off = wl["off"]
    n = int(off[-1])
    J = len(off) - 1
    W = wl["W"]
    rho = wl["density"]

    ctx = dgs.Context(off, W=W, device=dev)
    if args.force_exact:
        ctx.set_option(dgs.OPT_FORCE_EXACT, 1)
    K = ctx.nnz(rho)
    model = torch.zeros(n, dtype=torch.float32, device=dev)
    diff = torch.zeros((W, n), dtype=torch.float32, device=dev)
    ctx.server_attach(diff)
    pidx = torch.zeros(K, dtype=torch.int32, device=dev)
    pval = torch.zeros(K, dtype=torch.float32, device=dev)

    if name == "c3":
        pay = [(torch.from_numpy(i.view(np.int32)).to(dev), torch.from_numpy(v).to(dev), i.size)
               for i, v in wl["payloads"]]
        order = [int(x) for x in wl["order"]]

        if args.server_form == "sent":
            ctx.server_attach_sent(diff)          # W rows, all equal to the (zero) initial model

            def step(t):
                i, v, nn = pay[t % len(pay)]
                w = order[t % len(order)]
                ctx.server_push_model(model, i, v, nn)
                ctx.server_pull_sent(model, w, rho, pidx, pval)
            dominant, dom_kind, dom_bytes = "k_stream<sub,collect> (dgs_server_pull_sent streaming pass)", dgs.PROF_PULL_STREAM, 8.0 * n
            step_bytes = (8.0 * K + 8.0 * K) + (8.0 * n + 16.0 * K)
        else:
            def step(t):
                i, v, nn = pay[t % len(pay)]
                w = order[t % len(order)]
                ctx.server_push(model, w, i, v, nn)
                ctx.server_pull(w, rho, pidx, pval)
            dominant, dom_kind, dom_bytes = "k_stream<ident,collect> (dgs_server_pull streaming pass)", dgs.PROF_PULL_STREAM, 4.0 * n
            step_bytes = (8.0 * K + 8.0 * (W + 1) * K) + (4.0 * n + 12.0 * K)
    else:
        g_dev = [torch.from_numpy(g).to(dev) for g in wl["grads"]]
        state = torch.zeros(n, dtype=torch.float32, device=dev)
        idx = torch.zeros(K, dtype=torch.int32, device=dev)
        val = torch.zeros(K, dtype=torch.float32, device=dev)

        def step(t):
            ctx.worker_step(g_dev[t % len(g_dev)], state, LR, MOMENTUM, rho, idx, val)
            ctx.server_push(model, 0, idx, val, K)
            ctx.server_pull(0, rho, pidx, pval)
        dominant, dom_kind, dom_bytes = "k_stream<fma,collect> (dgs_worker_step streaming pass)", dgs.PROF_WORKER_STREAM, 12.0 * n
        step_bytes = (12.0 * n + 12.0 * K) + (8.0 * K + 8.0 * (W + 1) * K) + (4.0 * n + 12.0 * K)

    t = 0
    for _ in range(warmup):
        step(t)
        t += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(t)
        t += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3

    # per-kernel durations: HIP events attached to each kernel dispatch (begin to end of the
    # kernel) on the context's stream, same workload continuing
    ctx.set_option(dgs.OPT_PROFILE, 1)
    for _ in range(min(steps, 200)):
        step(t)
        t += 1
    torch.cuda.synchronize()
    kinds = {"worker_stream": dgs.PROF_WORKER_STREAM, "worker_select": dgs.PROF_WORKER_SELECT,
             "pull_stream": dgs.PROF_PULL_STREAM, "pull_select": dgs.PROF_PULL_SELECT,
             "push": dgs.PROF_PUSH, "exact_extra": dgs.PROF_EXACT_EXTRA,
             "worker_segmented": dgs.PROF_WORKER_SEGMENTED, "pull_segmented": dgs.PROF_PULL_SEGMENTED}
    kernel_us, dom_us = {}, None
    for kname, kind in kinds.items():
        cnt, ms = ctx.profile_read(kind)
        kernel_us[kname] = round(ms / cnt * 1e3, 2) if cnt else None
        if kind == dom_kind and cnt:
            dom_us = ms / cnt * 1e3
    # wire form of the last pulled message (outside the timed step: the paper's encode() is the
    # coordinate format the step already produces; this is the byte layout for a network)
    wire = torch.zeros(ctx.wire_bytes(rho), dtype=torch.uint8, device=dev)
    didx, dval = torch.zeros_like(pidx), torch.zeros_like(pval)
    for _ in range(20):
        ctx.encode(rho, pidx, pval, wire)
        ctx.decode(rho, wire, didx, dval)
    torch.cuda.synchronize()
    wire_info = {"bytes": int(wire.numel()), "pair_bytes": 8 * K,
                 "round_trip_ok": bool(torch.equal(didx, pidx) and torch.equal(dval.view(torch.int32),
                                                                              pval.view(torch.int32)))}
    for kname, kind in (("encode_us", dgs.PROF_ENCODE), ("decode_us", dgs.PROF_DECODE)):
        cnt, ms = ctx.profile_read(kind)
        wire_info[kname] = round(ms / cnt * 1e3, 2) if cnt else None
    ctx.set_option(dgs.OPT_PROFILE, 0)
    st = ctx.stats()

    achieved = dom_bytes / (dom_us * 1e-6) / 1e9 if dom_us else None
    roofline = {"bound": "hbm", "kernel": dominant,
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                "traffic": MEASURED_TRAFFIC_BYTES[name], "algorithmic_bytes": dom_bytes,
                "avg_launch_us": dom_us}

    out = {
        "metric": "params/sec and HBM GB/s (% of peak) for dgs_worker_step + server push/pull",
        "value": n * steps / dt,
        "unit": "params/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{name}: {wl['desc']}, density {rho:g}",
                   "n": n, "tensors": J, "density": rho, "K": K, "workers": W,
                   "momentum": MOMENTUM, "path": "exact" if args.force_exact else "predicted",
                   "server_form": args.server_form},
        "roofline": roofline,
        "kernel_us": kernel_us,
        "wire_form": wire_info,
        "step_algorithmic_GBs": step_bytes / (dt / steps) / 1e9,
        "stats": {"exact_calls": st.exact_calls, "fallback_tensors": st.fallback_tensors,
                  "segmented_tensors": st.segmented_tensors, "repaired_tensors": st.repaired_tensors,
                  "internal_errors": st.internal_errors},
    }
    if args.overlap and name != "c3":
        out["overlapped_two_streams"] = overlapped(torch, dgs, off, W, rho, K, g_dev, steps, warmup, n, step_bytes)
    out["cpu_baseline"] = None if args.no_cpu else cpu_baseline(wl, name)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
