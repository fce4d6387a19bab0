#!/usr/bin/env python3
"""Benchmark of the DGS hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
dgs_worker_step -> dgs_server_push -> dgs_server_pull (one worker, one difference row).
Inputs are seeded and synthetic, resident in HBM before the timed region starts.

Default workload (`--workload c5`, the largest single-GPU configuration): 1e9 fp32
parameters in 64 equal tensors, Gaussian gradients with per-tensor log-uniform scale,
density 1e-4.  The same JSON line carries, as extra objects, the 25.6M-parameter
ResNet-50-shaped workload (`also_c2`: its step, kernels, roofline, a cold variant with
rotating buffers), calls without a prediction (`forced_exact`: two passes; `sampled_every_call`: thresholds
from a sample) and the CPU oracle
timed on a bounded sample of the same arrays (`cpu_baseline`), which doubles as a parity
check of the last timed-regime steps.

Other workloads, for the design notes:
  c1  one flat tensor of 2^20 parameters, density 0.01 (latency-bound)
  c2  ResNet-50 shapes, 25,557,032 parameters in 161 tensors, density 1e-3
  c3  server stress: 32 workers, step = push + pull of a seeded worker; `--server-form sent`
      (default: global model + what each worker was sent, as Algorithm 2 prints it) or `diff`
      (per-worker difference rows)
  c4  transformer-shaped 108M parameters, heavy-tailed gradients, row-sparse embedding
  c5  1e9 parameters in 64 tensors, `--density` 1e-4 (default) or 1e-2

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
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

# Bytes that crossed the L2 <-> fabric boundary (HBM or Infinity Cache behind it) per launch of
# the dominant kernel, from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE), each scaled
# by what the same counter reads for a copy kernel of known size.  Offline profile values, not
# measured in this run; every entry names the summary it comes from.
PROFILED_TRAFFIC = {
    "c5": {"bytes": 12068.64e6, "profile": "profiles/k_stream_k_select_fabric_traffic_c5_c2_c3.txt"},
    "c2": {"bytes": 308.62e6, "profile": "profiles/k_stream_k_select_fabric_traffic_c5_c2_c3.txt"},
    "c3": {"bytes": 207.70e6, "profile": "profiles/k_stream_k_select_fabric_traffic_c5_c2_c3.txt"},
}


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
                    desc="server stress: 25,557,032-param model, 32 workers, "
                         "step = server push of a pooled payload + server pull of a seeded worker")
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


def host_cpu():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return model, os.cpu_count()


def traffic_entry(name, rho):
    default_rho = {"c2": 1e-3, "c3": 1e-3, "c5": 1e-4}.get(name)
    return PROFILED_TRAFFIC.get(name) if rho == default_rho else None


def read_kernel_us(dgs, ctx):
    kinds = {"worker_stream": dgs.PROF_WORKER_STREAM, "worker_select": dgs.PROF_WORKER_SELECT,
             "pull_stream": dgs.PROF_PULL_STREAM, "pull_select": dgs.PROF_PULL_SELECT,
             "push": dgs.PROF_PUSH, "exact_extra": dgs.PROF_EXACT_EXTRA,
             "worker_segmented": dgs.PROF_WORKER_SEGMENTED, "pull_segmented": dgs.PROF_PULL_SEGMENTED}
    out = {}
    for kname, kind in kinds.items():
        cnt, ms = ctx.profile_read(kind)
        out[kname] = round(ms / cnt * 1e3, 2) if cnt else None
    return out


def frac(bytes_, us):
    """Algorithmic bytes over a duration, as GB/s and as a fraction of the HBM peak."""
    if not us:
        return None
    gbs = bytes_ / (us * 1e-6) / 1e9
    return {"GBs": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4), "us": round(us, 2)}


class WorkerServer:
    """One worker + one server row on one context: device buffers and the step."""

    def __init__(self, torch, dgs, wl, g_dev, dev, force_exact=False):
        self.torch, self.dgs = torch, dgs
        off = wl["off"]
        self.n = int(off[-1])
        self.rho = wl["density"]
        self.ctx = dgs.Context(off, W=1, device=dev)
        if force_exact:
            self.ctx.set_option(dgs.OPT_FORCE_EXACT, int(force_exact))    # 1 (True): two passes; 2: sampled estimate
        self.K = self.ctx.nnz(self.rho)
        n, K = self.n, self.K
        self.g_dev = g_dev
        self.model = torch.zeros(n, dtype=torch.float32, device=dev)
        self.diff = torch.zeros((1, n), dtype=torch.float32, device=dev)
        self.ctx.server_attach(self.diff)
        self.state = torch.zeros(n, dtype=torch.float32, device=dev)
        self.idx = torch.zeros(K, dtype=torch.int32, device=dev)
        self.val = torch.zeros(K, dtype=torch.float32, device=dev)
        self.pidx = torch.zeros(K, dtype=torch.int32, device=dev)
        self.pval = torch.zeros(K, dtype=torch.float32, device=dev)

    def step(self, t):
        c = self.ctx
        c.worker_step(self.g_dev[t % len(self.g_dev)], self.state, LR, MOMENTUM, self.rho, self.idx, self.val)
        c.server_push(self.model, 0, self.idx, self.val, self.K)
        c.server_pull(0, self.rho, self.pidx, self.pval)

    def close(self):
        self.ctx.close()


def timed(torch, step, t, warmup, steps, after_warmup=None):
    for _ in range(warmup):
        step(t)
        t += 1
    torch.cuda.synchronize()
    if after_warmup is not None:
        after_warmup()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(t)
        t += 1
    torch.cuda.synchronize()
    return time.perf_counter() - t0, t


def oracle_check_and_time(torch, ws, wl, t, sample_tensor, budget_s=20.0, max_steps=4):
    """CPU baseline and post-run parity check in one: continue the same workload for a few more
    steps; before each, copy the sampled tensor's worker state and server row to the host, let
    the oracle (as it stands, one thread) compute that tensor's worker step, push and pull from
    them, and compare with what the GPU produced for the tensor: indices bit-exact, values and
    the state within 1e-6 relative / 1e-7 absolute.  Only the oracle calls are timed."""
    from oracle import dgs_oracle as oracle
    from paper_1910_10929_amd import synth
    oracle.lib()
    off = wl["off"]
    J = len(off) - 1
    rho = wl["density"]
    if sample_tensor is None:
        lo, hi = 0, int(off[-1])
        soff = np.ascontiguousarray(off, dtype=np.uint64)
        what = "all tensors"
    else:
        lo, hi = int(off[sample_tensor]), int(off[sample_tensor + 1])
        soff = synth.layout_flat(hi - lo)
        what = f"tensor {sample_tensor} ({hi - lo:,} elements)"
    kj, _ = oracle.nnz(np.ascontiguousarray(off, dtype=np.uint64), rho)
    o_lo = int(sum(int(x) for x in kj[:sample_tensor])) if sample_tensor is not None else 0
    o_hi = o_lo + (int(kj[sample_tensor]) if sample_tensor is not None else ws.K)
    cpu_s, steps = 0.0, 0
    while steps < max_steps and (steps == 0 or cpu_s < budget_s * 0.6):
        s = ws.state[lo:hi].cpu().numpy()
        d = ws.diff[0, lo:hi].cpu().numpy().reshape(1, -1).copy()
        g = wl["grads"][t % len(wl["grads"])][lo:hi]
        ws.step(t)
        t += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        wi, wv = oracle.worker_step(np.ascontiguousarray(g), s, soff, LR, np.float32(MOMENTUM), rho)
        oracle.server_push(None, d, wi, wv)
        pi, pv = oracle.server_pull(d, 0, soff, rho)
        cpu_s += time.perf_counter() - t0
        steps += 1
        gi = ws.idx[o_lo:o_hi].cpu().numpy().view(np.uint32) - np.uint32(lo)
        gpi = ws.pidx[o_lo:o_hi].cpu().numpy().view(np.uint32) - np.uint32(lo)
        assert np.array_equal(gi, wi), f"post-run check: worker indices differ from the oracle ({what})"
        assert np.array_equal(gpi, pi), f"post-run check: pull indices differ from the oracle ({what})"
        np.testing.assert_allclose(ws.val[o_lo:o_hi].cpu().numpy(), wv, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(ws.pval[o_lo:o_hi].cpu().numpy(), pv, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(ws.state[lo:hi].cpu().numpy(), s, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(ws.diff[0, lo:hi].cpu().numpy(), d[0], rtol=1e-6, atol=1e-7)
    cpu_model, nproc = host_cpu()
    return {"value": (hi - lo) * steps / cpu_s, "unit": "params/s", "cores": 1, "kind": "oracle",
            "cpu_model": cpu_model, "nproc": nproc,
            "sample": f"{steps} further steps (worker_step + push + pull) of the same workload on {what}, "
                      f"from the GPU's own state after the timed steps; {cpu_s:.1f} s on one host core; "
                      f"every message compared with the GPU's",
            "parity_checked_steps": steps}, t


def run_worker_server(torch, dgs, name, wl, steps, warmup, dev, *, cpu=True, exact_steps=0, cold=False,
                      overlap=False):
    """The step = worker_step + push + pull workloads (c1, c2, c4, c5)."""
    off = wl["off"]
    n, J, rho = int(off[-1]), len(off) - 1, wl["density"]
    g_dev = [torch.from_numpy(g).to(dev) for g in wl["grads"]]
    ws = WorkerServer(torch, dgs, wl, g_dev, dev)
    K, W = ws.K, 1
    snap = {}
    dt, t = timed(torch, ws.step, 0, warmup, steps, after_warmup=lambda: snap.update(w=ws.ctx.stats()))
    snap["t"] = ws.ctx.stats()
    # per-kernel durations: HIP events attached to each kernel dispatch on the context's stream
    ws.ctx.set_option(dgs.OPT_PROFILE, 1)
    for _ in range(min(max(steps, 20), 200)):
        ws.step(t)
        t += 1
    torch.cuda.synchronize()
    kernel_us = read_kernel_us(dgs, ws.ctx)
    ws.ctx.set_option(dgs.OPT_PROFILE, 0)

    step_bytes = (12.0 * n + 12.0 * K) + (8.0 * K + 8.0 * (W + 1) * K) + (4.0 * n + 12.0 * K)
    us = lambda k: kernel_us.get(k) or 0.0
    worker_us = us("worker_stream") + us("worker_select") + us("worker_segmented")
    pull_us = us("pull_stream") + us("pull_select") + us("pull_segmented")
    dom_us = kernel_us["worker_stream"]
    achieved = 12.0 * n / (dom_us * 1e-6) / 1e9 if dom_us else None
    traffic = traffic_entry(name, rho)
    roofline = {
        "bound": "hbm", "kernel": "k_stream<fma,collect> (dgs_worker_step streaming pass)",
        "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
        "traffic": traffic["bytes"] if traffic else None,
        "traffic_note": (f"offline rocprofv3 counter value (L2 <-> fabric bytes per launch), {traffic['profile']}"
                         if traffic else "not profiled for this workload"),
        "algorithmic_bytes": 12.0 * n, "avg_launch_us": dom_us,
        # whole calls: every kernel of the call, algorithmic bytes of the call
        "per_call": {
            "worker_step": frac(12.0 * n + 12.0 * K, worker_us),
            "server_pull": frac(4.0 * n + 12.0 * K, pull_us),
            "server_push": frac(8.0 * K + 8.0 * (W + 1) * K, us("push")),
            "step": frac(step_bytes, dt / steps * 1e6),
        },
    }
    # wire form of the last pulled message (outside the timed step)
    wire = torch.zeros(ws.ctx.wire_bytes(rho), dtype=torch.uint8, device=dev)
    didx, dval = torch.zeros_like(ws.pidx), torch.zeros_like(ws.pval)
    ws.ctx.set_option(dgs.OPT_PROFILE, 1)
    for _ in range(20):
        ws.ctx.encode(rho, ws.pidx, ws.pval, wire)
        ws.ctx.decode(rho, wire, didx, dval)
    torch.cuda.synchronize()
    wire_info = {"bytes": int(wire.numel()), "pair_bytes": 8 * K,
                 "round_trip_ok": bool(torch.equal(didx, ws.pidx) and
                                       torch.equal(dval.view(torch.int32), ws.pval.view(torch.int32)))}
    for kname, kind in (("encode_us", dgs.PROF_ENCODE), ("decode_us", dgs.PROF_DECODE)):
        cnt, ms = ws.ctx.profile_read(kind)
        wire_info[kname] = round(ms / cnt * 1e3, 2) if cnt else None
    ws.ctx.set_option(dgs.OPT_WIRE_VALUE_BITS, 16)
    wire_info["bytes_bf16_values"] = int(ws.ctx.wire_bytes(rho))      # the lossy variant: size only
    ws.ctx.set_option(dgs.OPT_WIRE_VALUE_BITS, 32)
    ws.ctx.set_option(dgs.OPT_PROFILE, 0)
    del wire, didx, dval

    out = {
        "value": n * steps / dt, "ms_per_step": dt / steps * 1e3,
        "config": {"workload": f"{name}: {wl['desc']}, density {rho:g}",
                   "n": n, "tensors": J, "density": rho, "K": K, "workers": W,
                   "momentum": MOMENTUM, "path": "predicted", "server_form": "diff"},
        "roofline": roofline, "kernel_us": kernel_us, "wire_form": wire_info,
        "step_algorithmic_GBs": step_bytes / (dt / steps) / 1e9,
    }
    if cpu:
        # c1 / c2: the whole layout; larger ones: one tensor
        sample = None if n <= 30_000_000 else 0
        out["cpu_baseline"], t = oracle_check_and_time(torch, ws, wl, t, sample)
    st = ws.ctx.stats()
    out["stats"] = {"exact_calls": st.exact_calls, "fallback_tensors": st.fallback_tensors,
                    "segmented_tensors": st.segmented_tensors, "repaired_tensors": st.repaired_tensors,
                    "internal_errors": st.internal_errors}
    # the timed steps alone (the counters above include the warm-up, whose first calls have no
    # usable prediction yet)
    out["stats_timed_steps"] = {k: getattr(snap["t"], k) - getattr(snap["w"], k)
                                for k in ("exact_calls", "fallback_tensors", "segmented_tensors",
                                          "repaired_tensors", "internal_errors")}
    assert st.internal_errors == 0, "libdgs reported internal errors"
    ws.close()
    del ws
    gc.collect()
    torch.cuda.empty_cache()

    # calls without a prediction: `forced_exact` takes two passes on every call (full histogram,
    # pick, read-only collecting pass, selection), `sampled_every_call` what a first call or a new
    # density takes by default (histogram of a sixteenth of the data, pick, then the one pass)
    for key, mode in (("forced_exact", 1), ("sampled_every_call", 2)) if exact_steps else ():
        we = WorkerServer(torch, dgs, wl, g_dev, dev, force_exact=mode)
        dte, te = timed(torch, we.step, 0, 2, exact_steps)
        we.ctx.set_option(dgs.OPT_PROFILE, 1)
        for _ in range(exact_steps):
            we.step(te)
            te += 1
        torch.cuda.synchronize()
        ku = read_kernel_us(dgs, we.ctx)
        ste = we.ctx.stats()
        assert ste.internal_errors == 0
        out[key] = {"ms_per_step": dte / exact_steps * 1e3, "steps": exact_steps,
                    "params_per_s": n * exact_steps / dte,
                    "step_algorithmic_frac": step_bytes / (dte / exact_steps) / 1e9 / HBM_PEAK_GBS,
                    "kernel_us": ku, "exact_extra_us": ku["exact_extra"],
                    "repaired_tensors": ste.repaired_tensors}
        we.close()
        del we
        gc.collect()
        torch.cuda.empty_cache()
    if cold:
        # rotating buffers: R independent replicas (context, state, model, row) used in turn, so
        # that no state or row is found in the 256 MB last-level cache from its previous step
        R = 6
        reps = [WorkerServer(torch, dgs, wl, g_dev, dev) for _ in range(R)]
        dtc, _ = timed(torch, lambda tt: reps[tt % R].step(tt // R), 0, R * max(8, warmup // 2), R * steps)
        for r in reps:
            assert r.ctx.stats().internal_errors == 0
            r.close()
        out["cold_rotating_buffers"] = {"replicas": R, "ms_per_step": dtc / (R * steps) * 1e3,
                                        "params_per_s": n * R * steps / dtc,
                                        "step_algorithmic_frac": step_bytes / (dtc / (R * steps)) / 1e9 / HBM_PEAK_GBS}
        del reps
        gc.collect()
        torch.cuda.empty_cache()
    if overlap:
        out["overlapped_two_streams"] = overlapped(torch, dgs, off, W, rho, K, g_dev, steps, warmup, n, step_bytes)
    del g_dev
    gc.collect()
    torch.cuda.empty_cache()
    return out


def run_server_stress(torch, dgs, wl, steps, warmup, dev, form, cpu=True):
    """c3: step = push of a pooled payload + pull of a seeded worker, 32 workers."""
    off = wl["off"]
    n, J, rho, W = int(off[-1]), len(off) - 1, wl["density"], wl["W"]
    ctx = dgs.Context(off, W=W, device=dev)
    K = ctx.nnz(rho)
    model = torch.zeros(n, dtype=torch.float32, device=dev)
    rows = torch.zeros((W, n), dtype=torch.float32, device=dev)
    pidx = torch.zeros(K, dtype=torch.int32, device=dev)
    pval = torch.zeros(K, dtype=torch.float32, device=dev)
    pay = [(torch.from_numpy(i.view(np.int32)).to(dev), torch.from_numpy(v).to(dev), i.size)
           for i, v in wl["payloads"]]
    order = [int(x) for x in wl["order"]]
    if form == "sent":
        ctx.server_attach_sent(rows)          # W rows, all equal to the (zero) initial model

        def step(t):
            i, v, nn = pay[t % len(pay)]
            ctx.server_push_model(model, i, v, nn)
            ctx.server_pull_sent(model, order[t % len(order)], rho, pidx, pval)
        dominant, dom_bytes = "k_stream<sub,collect> (dgs_server_pull_sent streaming pass)", 8.0 * n
        push_bytes, pull_bytes = 8.0 * K + 8.0 * K, 8.0 * n + 16.0 * K
    else:
        ctx.server_attach(rows)

        def step(t):
            i, v, nn = pay[t % len(pay)]
            w = order[t % len(order)]
            ctx.server_push(model, w, i, v, nn)
            ctx.server_pull(w, rho, pidx, pval)
        dominant, dom_bytes = "k_stream<ident,collect> (dgs_server_pull streaming pass)", 4.0 * n
        push_bytes, pull_bytes = 8.0 * K + 8.0 * (W + 1) * K, 4.0 * n + 12.0 * K
    dt, t = timed(torch, step, 0, warmup, steps)
    ctx.set_option(dgs.OPT_PROFILE, 1)
    for _ in range(min(steps, 200)):
        step(t)
        t += 1
    torch.cuda.synchronize()
    kernel_us = read_kernel_us(dgs, ctx)
    us = lambda k: kernel_us.get(k) or 0.0
    dom_us = kernel_us["pull_stream"]
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9 if dom_us else None
    st = ctx.stats()
    assert st.internal_errors == 0
    out = {
        "value": n * steps / dt, "ms_per_step": dt / steps * 1e3,
        "config": {"workload": f"c3: {wl['desc']}, density {rho:g}", "n": n, "tensors": J, "density": rho,
                   "K": K, "workers": W, "path": "predicted", "server_form": form},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                     "traffic": None, "traffic_note": "not profiled for this workload",
                     "algorithmic_bytes": dom_bytes, "avg_launch_us": dom_us,
                     "per_call": {"server_pull": frac(pull_bytes, us("pull_stream") + us("pull_select") + us("pull_segmented")),
                                  "server_push": frac(push_bytes, us("push")),
                                  "step": frac(push_bytes + pull_bytes, dt / steps * 1e6)}},
        "kernel_us": kernel_us,
        "step_algorithmic_GBs": (push_bytes + pull_bytes) / (dt / steps) / 1e9,
        "stats": {"exact_calls": st.exact_calls, "fallback_tensors": st.fallback_tensors,
                  "segmented_tensors": st.segmented_tensors, "repaired_tensors": st.repaired_tensors,
                  "internal_errors": st.internal_errors},
    }
    ctx.close()
    del rows, model, pay
    gc.collect()
    torch.cuda.empty_cache()
    if cpu:
        from oracle import dgs_oracle as oracle
        oracle.lib()
        model_h = np.zeros(n, np.float32)
        rows_h = np.zeros((W, n), np.float32)
        t0 = time.perf_counter()
        ev = 0
        while ev < 16 and (ev == 0 or time.perf_counter() - t0 < 12.0):
            i, v = wl["payloads"][ev % len(wl["payloads"])]
            if form == "sent":
                oracle.server_push_model(model_h, i, v)
                oracle.server_pull_sent(model_h, rows_h, order[ev], off, rho)
            else:
                oracle.server_push(model_h, rows_h, i, v)
                oracle.server_pull(rows_h, order[ev], off, rho)
            ev += 1
        cs = time.perf_counter() - t0
        cpu_model, nproc = host_cpu()
        out["cpu_baseline"] = {"value": n * ev / cs, "unit": "params/s", "cores": 1, "kind": "oracle",
                               "cpu_model": cpu_model, "nproc": nproc,
                               "sample": f"first {ev} events (push + pull) of the same workload, {cs:.1f} s on one host core"}
    return out


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
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--density", type=float, default=None)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg (and its parity check)")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline workload: no forced-exact run, no 25.6M-parameter leg")
    ap.add_argument("--server-form", default="sent", choices=["diff", "sent"],
                    help="c3 only: the printed form, global model + what each worker has been sent "
                         "(default), or per-worker difference rows; the other form is reported beside it")
    ap.add_argument("--overlap", action="store_true",
                    help="also time worker and server on two streams (worker step t+1 overlaps "
                         "push/pull t); reported as an extra field, never as `value`")
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
    extras = not args.no_extras
    if name == "c3":
        res = run_server_stress(torch, dgs, wl, steps, warmup, dev, args.server_form, cpu=not args.no_cpu)
        if extras:
            other = "diff" if args.server_form == "sent" else "sent"
            o = run_server_stress(torch, dgs, wl, steps, warmup, dev, other, cpu=False)
            res["other_server_form"] = {k: o[k] for k in ("value", "ms_per_step", "kernel_us", "roofline",
                                                          "step_algorithmic_GBs", "stats")}
            res["other_server_form"]["server_form"] = other
    else:
        res = run_worker_server(torch, dgs, name, wl, steps, warmup, dev, cpu=not args.no_cpu,
                                exact_steps=(5 if name in ("c4", "c5") else 20) if extras else 0,
                                cold=extras and name in ("c1", "c2"), overlap=args.overlap)
    del wl
    gc.collect()
    if extras and name == "c5" and args.density in (None, 1e-4):
        # the 25.6M-parameter configuration beside the headline
        wl2 = make_workload("c2", None)
        r2 = run_worker_server(torch, dgs, "c2", wl2, 200, 40, dev, cpu=not args.no_cpu, exact_steps=20,
                               cold=True)
        r2["params_per_s"] = r2.pop("value")
        res["also_c2"] = r2

    out = {
        "metric": "params/sec and HBM GB/s (% of peak) for dgs_worker_step + server push/pull",
        "value": res.pop("value"),
        "unit": "params/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": res.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
    }
    out.update(res)
    if "cpu_baseline" not in out:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
