#!/usr/bin/env python3
"""Throughput of the DoubleSqueeze step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic gradients:
ds_worker_compress (n workers) + ds_server_aggregate_compress + ds_apply_update, i.e. one
iteration of Algorithm 1 of the paper without the gradient computation and the two sends.
Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` = gradient elements (n*d) per second of the headline
workload; `roofline` prices the dominant kernel (the worker pass) in algorithmic HBM bytes
against the 8 TB/s peak, timed live with HIP events on the launch stream; `cpu_baseline` is
the CPU oracle timed on this host on a bounded sample of the same workload.
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

# HBM bytes per launch of the worker pass, measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, each scaled by the same counter's reading for a 1 GiB copy); the runs and
# the scale factors are recorded under profiles/.  None = not profiled yet.
MEASURED_WORKER_TRAFFIC = {
    "c5": 5.9728e9 + 4.1221e9,   # k_sign_chunk_worker
    "c4": 3.3116e9 + 1.9177e9,   # k_qsgd_worker
    "c3": 2.6548e9,              # all kernels of the worker call (dense pass 1.6551e9 + 0.8493e9)
    "clip16": 1.6568e9 + 1.2368e9,   # k_clip_worker
    "rsparse60": 1.7116e9 + 1.3278e9 + 0.0299e9 + 0.0068e9,   # k_rs_worker + k_rs_counts + k_rs_scan
    "c2": 1.1027e9,              # k_sign_pass1_worker + k_sign_reduce, deferred error form (plain form: + pass 2)
}


def algorithmic_bytes(wl, S: int) -> dict:
    """HBM bytes the method must move per step at the three-call boundary: read g and
    delta once, write delta once, write/read every message once, read/write x (and m) once."""
    n, d = wl.n, wl.d
    gb = 2 if wl.grad_dtype == "bf16" else 4
    W8 = 8 * ((d + 63) // 64)
    if wl.comp == "sign":
        msg = W8 + 4 * S
    elif wl.comp == "qsgd":
        msg = W8 + 4 * S + (d + 1) // 2
    elif wl.comp == "topk":
        msg = 8 * wl.k
    elif wl.comp == "clip":
        msg = d * (1 if wl.clip_bits >= 24 else 2 if wl.clip_bits >= 16 else 4)
    elif wl.comp == "rsparse":
        msg = W8 + int(4 * d * wl.keep_prob)        # kept-bit plane + the expected number of kept values
    else:
        msg = 4 * d
    worker = n * (d * (gb + 4 + 4) + msg)
    server = n * msg + d * 8 + msg
    if wl.comp == "topk":
        # the server still reads and writes its dense error once; the update touches k entries
        update = msg + 8 * wl.k * (2 if wl.beta is not None else 1)
    else:
        update = msg + d * (16 if wl.beta is not None else 8)
    return {"worker": worker, "server": server, "update": update, "total": worker + server + update}


def make_workload(name: str):
    import ds_workloads as W
    return {"c2": W.c2, "c3": W.c3, "c4": W.c4, "c5": W.c5, "clip16": W.clip16, "rsparse60": W.rsparse60}[name]()


def run_gpu(wl, steps: int, warmup: int, sets: int = 2, calib_copy: bool = False, deferred_error: bool = True,
            separate_update: bool = False, settle_ms: float = 150.0):
    import torch
    import paper_1905_05957_amd as P

    dev = torch.device("cuda:0")
    ctx = P.Context(wl.comp, wl.n, wl.d, grad_dtype=wl.grad_dtype, scale_mode=wl.scale_mode,
                    chunk=wl.chunk, seg_offsets=wl.seg_offsets if wl.scale_mode == "segments" else None,
                    k=wl.k, bucket=wl.bucket, levels=wl.clip_bits if wl.comp == "clip" else wl.levels,
                    seed=wl.seed, keep_prob=wl.keep_prob if wl.comp == "rsparse" else None,
                    flags=P.FLAG_DEFERRED_ERROR if deferred_error else 0)
    grads = [wl.gradients(s, dev) for s in range(sets)]
    delta = wl.initial_delta(dev)
    delta_s = torch.zeros(wl.d, dtype=torch.float32, device=dev)
    x = wl.initial_x(dev)
    m = torch.zeros(wl.d, dtype=torch.float32, device=dev) if wl.beta is not None else None
    pw, ps = ctx.alloc_payload(wl.n, dev), ctx.alloc_payload(1, dev)
    beta = 0.0 if wl.beta is None else wl.beta
    stream = torch.cuda.current_stream()

    def step(t, ev=None, stages=False):
        g = grads[t % sets]
        if ev is not None:
            ev[0].record(stream)
        ctx.worker_compress(t, g, delta, pw)
        if ev is not None:
            ev[1].record(stream)
        if stages or separate_update:
            ctx.server_aggregate_compress(t, pw, delta_s, ps)
            if stages:
                ev[2].record(stream)
            ctx.apply_update(ps, x, m, wl.gamma, beta)
            if stages:
                ev[3].record(stream)
        else:       # the same two blocks of Algorithm 1 through the one-call entry point
            ctx.server_aggregate_compress_update(t, pw, delta_s, ps, x, m, wl.gamma, beta)

    # The first tens of milliseconds of a memory-bound phase run slower on this machine (seen in
    # kernel traces: the 124 M-element worker pass takes 1.9 ms in steps 1-3 and settles at
    # 1.68 ms after about 30 ms, whatever came before), so the clocks get `settle_ms` of the same
    # steps before the W warm-up steps and the K timed steps.
    t_settle = 0
    t_end = time.perf_counter() + settle_ms * 1e-3
    while time.perf_counter() < t_end:
        step(t_settle)
        t_settle += 1
        if t_settle % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    for t in range(warmup):
        step(t_settle + t)
    torch.cuda.synchronize()
    warmup += t_settle      # step numbers below continue after the settle steps
    # An event record costs a bubble of about 6 us between two kernels that otherwise run back
    # to back (seen in the kernel trace), so the timed region carries events only around the
    # worker call of every 3rd step: enough for the average launch duration of the dominant
    # kernel (roofline) at under 1 % of a step.  The per-stage split comes from a second,
    # untimed pass over the same number of steps (always the three separate calls).
    every = 3     # odd: the sampled steps alternate between the gradient sets
    evs = {t: [torch.cuda.Event(enable_timing=True) for _ in range(2)] for t in range(0, steps, every)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        step(warmup + t, evs.get(t))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    worker_ms = sum(ev[0].elapsed_time(ev[1]) for ev in evs.values()) / len(evs)
    evs2 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for t in range(steps):
        step(warmup + steps + t, evs2[t], stages=True)
    torch.cuda.synchronize()
    stage = [0.0, 0.0, 0.0]
    for ev in evs2:
        for s_ in range(3):
            stage[s_] += ev[s_].elapsed_time(ev[s_ + 1])
    stage_ms = [v / steps for v in stage]
    S = ctx.S
    ctx.close()
    # one plain device-to-device copy of known size (1 GiB read + 1 GiB written): the
    # calibration dispatch for HBM byte counters collected with rocprofv3 --pmc
    if calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    return {"ms_per_step": wall * 1e3 / steps, "stage_ms": stage_ms, "S": S, "worker_ms": worker_ms,
            "worker_samples": len(evs)}


def run_oracle_sample(wl, target_elems: int):
    """The CPU oracle, as it stands, on the first d' elements of every row (d' chosen so that
    n*d' is about target_elems, cut at a scale-group / bucket boundary); one full step."""
    import numpy as np
    import torch
    import dataclasses
    import oracle as O

    dq = max(1, min(wl.d, target_elems // wl.n))
    unit = {"sign": wl.chunk if wl.scale_mode == "chunk" else 64, "qsgd": wl.bucket}.get(wl.comp, 64)
    dq = max(unit, (dq // unit) * unit)
    dq = min(dq, wl.d)
    sub = dataclasses.replace(wl, d=dq, k=max(1, wl.k * dq // wl.d) if wl.k else 0)
    if wl.seg_offsets is not None:
        off = wl.seg_offsets[wl.seg_offsets < dq]
        sub.seg_offsets = np.concatenate([off, [dq]]).astype(np.int64)
        sub.seg_sigma = wl.seg_sigma[: len(off)]
    comp = {"identity": O.IDENTITY, "sign": O.SIGN, "topk": O.TOPK, "qsgd": O.QSGD, "clip": O.CLIP,
            "rsparse": O.RSPARSE}[sub.comp]
    cfg = O.Config(comp, n=sub.n, d=dq, grad_bf16=(sub.grad_dtype == "bf16"),
                   group_off=sub.group_offsets() if sub.comp == "sign" else None, k=sub.k,
                   bucket=sub.bucket, levels=sub.levels, seed=sub.seed, sign_rms=sub.sign_rms,
                   clip_bits=sub.clip_bits,
                   keep_prob=float(np.float32(round(sub.keep_prob * (1 << 24))) / np.float32(1 << 24)))
    g = sub.gradients(0, "cpu")
    hg = g.view(torch.int16).numpy().view(np.uint16) if g.dtype == torch.bfloat16 else g.numpy()
    delta = sub.initial_delta("cpu").numpy()
    delta_s = np.zeros(dq, np.float32)
    x = sub.initial_x("cpu").numpy()
    m = np.zeros(dq, np.float32) if sub.beta is not None else None
    O.lib()
    t0 = time.perf_counter()
    pw = O.worker_compress(cfg, 0, hg, delta)
    ps = O.server_aggregate_compress(cfg, 0, pw, delta_s)
    O.apply_update(cfg, ps, x, m, sub.gamma, 0.0 if sub.beta is None else sub.beta)
    dt = time.perf_counter() - t0
    return {"value": sub.n * dq / dt, "unit": "gradient elements/s", "cores": 1, "kind": "oracle",
            "sample": f"one full step on the first {dq} of {wl.d} elements of all {wl.n} rows "
                      f"({dt:.1f} s, single thread)"}


def run_ceiling():
    """Reference points for the roofline fractions, with torch's own kernels (nothing of this
    library): a device-to-device copy, and out = a + b in place at the shape of C3's dense
    worker pass (read 8 B, write 4 B per element: the traffic no top-k worker pass can avoid)."""
    import torch
    dev = torch.device("cuda:0")
    out = {}

    def timed(f, reps=20):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            f()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    ms = timed(lambda: dst.copy_(src))
    out["copy_1GiB"] = {"ms": ms, "GBs": 2 * src.numel() * 4 / ms / 1e6}
    del src, dst
    n, d = 8, 25_557_032
    g = [torch.empty((n, d), dtype=torch.float32, device=dev).normal_() for _ in range(2)]
    delta = torch.zeros((n, d), dtype=torch.float32, device=dev)
    it = [0]

    def axpy():
        it[0] += 1
        torch.add(g[it[0] % 2], delta, out=delta)
    ms = timed(axpy)
    out["add_in_place_8x25557032"] = {"ms": ms, "GBs": 12 * n * d / ms / 1e6}
    print(json.dumps({"hbm_peak_GBs": HBM_PEAK_GBS, "reference": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c5", choices=["c2", "c3", "c4", "c5", "clip16", "rsparse60"])
    ap.add_argument("--others", default="c2,c3,c4", help="further workloads reported in the same line ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (calibration dispatch for rocprofv3 --pmc byte counters)")
    ap.add_argument("--cpu-elems", type=int, default=1_000_000_000)
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="untimed steps run for this long before the warm-up steps, for the clocks to settle")
    ap.add_argument("--ceiling", action="store_true",
                    help="instead of the benchmark: time torch's copy and in-place add kernels as reference points")
    ap.add_argument("--separate-update", action="store_true",
                    help="time ds_server_aggregate_compress and ds_apply_update as two calls (default: the "
                         "one-call form ds_server_aggregate_compress_update, same results)")
    ap.add_argument("--plain-error", action="store_true",
                    help="keep the error buffers in plain form after every call (sign with scale groups that "
                         "span workgroups then takes two looks per call; default: DS_FLAG_DEFERRED_ERROR)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (n workers are rows of one tensor); "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if a.ceiling:
        run_ceiling()
        return

    def measure(name, steps, warmup, calib_copy=False):
        wl = make_workload(name)
        r = run_gpu(wl, steps, warmup, calib_copy=calib_copy, deferred_error=not a.plain_error,
                    separate_update=a.separate_update, settle_ms=a.settle_ms)
        ab = algorithmic_bytes(wl, r["S"])
        ms = r["ms_per_step"]
        wk_ms = r["worker_ms"]
        out = {
            "workload": wl.name, "n": wl.n, "d": wl.d, "ms_per_step": ms,
            "calls": "ds_worker_compress + " + ("ds_server_aggregate_compress + ds_apply_update" if a.separate_update
                                                else "ds_server_aggregate_compress_update"),
            "error_state": "plain" if a.plain_error or not (wl.comp == "sign" and wl.scale_mode != "chunk") else "deferred",
            "value": wl.n * wl.d / (ms * 1e-3),
            "stage_ms": {"worker": r["stage_ms"][0], "server": r["stage_ms"][1], "update": r["stage_ms"][2]},
            "algorithmic_bytes_per_step": ab["total"],
            "step_hbm_GBs": ab["total"] / (ms * 1e-3) / 1e9,
            "step_frac_of_peak": ab["total"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "roofline": {"bound": "hbm", "kernel": "worker pass (ds_worker_compress)",
                         "achieved": ab["worker"] / (wk_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": ab["worker"] / (wk_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "algorithmic_bytes": ab["worker"], "launch_ms": wk_ms,
                         "launch_samples": r["worker_samples"],
                         "traffic": MEASURED_WORKER_TRAFFIC.get(name)},
        }
        return wl, out

    wl, head = measure(a.workload, a.steps, a.warmup, calib_copy=a.calib_copy)
    others = []
    for name in [s for s in a.others.split(",") if s and s != a.workload]:
        try:
            _, o = measure(name, max(5, a.steps // 2), max(2, a.warmup // 2))
            others.append(o)
        except Exception as e:  # a workload whose compressor is not built yet
            others.append({"workload": name, "error": str(e)})
        torch.cuda.empty_cache()

    line = {
        "metric": "DoubleSqueeze step: gradient elements/s (n\u00b7d) and HBM GB/s as % of peak", "value": head["value"],
        "unit": "gradient elements/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "n_workers": wl.n, "d": wl.d,
                   "grad_dtype": wl.grad_dtype, "compressor": wl.comp, "settle_ms": a.settle_ms},
        "stage_ms": head["stage_ms"],
        "algorithmic_bytes_per_step": head["algorithmic_bytes_per_step"],
        "step_hbm_GBs": head["step_hbm_GBs"], "step_frac_of_peak": head["step_frac_of_peak"],
        "hbm_pct_of_peak": 100.0 * head["step_frac_of_peak"],     # the metric's second figure, whole step
        "roofline": head["roofline"],
        "other_workloads": others,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = run_oracle_sample(wl, a.cpu_elems)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
