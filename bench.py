#!/usr/bin/env python3
"""Throughput of the DoubleSqueeze step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic gradients:
ds_worker_compress (n workers) + ds_server_aggregate_compress + ds_apply_update, i.e. one
iteration of Algorithm 1 of the paper without the gradient computation and the two sends.
Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` = gradient elements (n*d) per second of the headline
workload; `roofline` prices the dominant kernel (the worker pass) in algorithmic HBM bytes
against the 8 TB/s peak, timed live with HIP events on the launch stream; `copy_ceiling_GBs` is
the library's plain streaming copy kernel on this machine (the practical ceiling; the
`*_frac_of_copy` figures are fractions of it); `ms_per_step_unsettled` is the same K steps
after the W warm-up steps only, before the settle phase; `other_workloads` carries the other
configurations, each with its own oracle time; `uncompensated_worker_pass` shows the worker
pass of the comparison algorithms (no error buffer traffic); `cpu_baseline` is the CPU oracle
timed on this host, single thread, plus the worker rows on separate threads, with the host's
core count and CPU model.
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
# WRITE_SIZE runs, each scaled by the same counter's reading for a 1 GiB copy): read from
# profiles/traffic.json, which `python -m paper_1905_05957_amd.traffic` writes from the counter
# files of such runs together with the commit they were measured at.
def measured_worker_traffic(name: str):
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            entry = json.load(f).get(name)
        return None if entry is None else entry.get("worker_call_bytes")
    except (OSError, ValueError):
        return None


def algorithmic_bytes(wl, S: int) -> dict:
    """HBM bytes the method must move per step at the three-call boundary: read g and
    delta once, write delta once, write/read every message once, read/write x (and m) once.
    Top-k: the server reads its dense error once and writes it only where it changes (at most
    n k + k positions; the kernels write it densely, which `as_implemented` counts), and the
    update touches the k kept entries."""
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
    as_implemented = None
    if wl.comp == "topk":
        changed = min(d, n * wl.k + wl.k)
        as_implemented = worker + server + msg + 8 * wl.k * (2 if wl.beta is not None else 1)
        server = n * msg + d * 4 + 4 * changed + msg
        update = msg + 8 * wl.k * (2 if wl.beta is not None else 1)
    else:
        update = msg + d * (16 if wl.beta is not None else 8)
    out = {"worker": worker, "server": server, "update": update, "total": worker + server + update,
           "message": msg, "grad_bytes": gb}
    if as_implemented is not None:
        out["as_implemented"] = as_implemented
    return out


def make_workload(name: str):
    import ds_workloads as W
    return {"c2": W.c2, "c3": W.c3, "c4": W.c4, "c5": W.c5, "clip16": W.clip16, "rsparse60": W.rsparse60}[name]()


def _context(wl, deferred_error: bool, extra_flags: int = 0):
    import paper_1905_05957_amd as P
    return P.Context(wl.comp, wl.n, wl.d, grad_dtype=wl.grad_dtype, scale_mode=wl.scale_mode,
                     chunk=wl.chunk, seg_offsets=wl.seg_offsets if wl.scale_mode == "segments" else None,
                     k=wl.k, bucket=wl.bucket, levels=wl.clip_bits if wl.comp == "clip" else wl.levels,
                     seed=wl.seed, keep_prob=wl.keep_prob if wl.comp == "rsparse" else None,
                     flags=(P.FLAG_DEFERRED_ERROR if deferred_error else 0) | extra_flags)


def run_gpu(wl, steps: int, warmup: int, sets: int = 2, calib_copy: bool = False, deferred_error: bool = True,
            separate_update: bool = False, settle_ms: float = 150.0):
    import torch

    dev = torch.device("cuda:0")
    ctx = _context(wl, deferred_error)
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

    def timed(first_step, k, evs=None):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(k):
            step(first_step + t, None if evs is None else evs.get(t))
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / k

    # First the plain reading: W warm-up steps, K timed steps, nothing before them.
    for t in range(warmup):
        step(t)
    ms_unsettled = timed(warmup, steps)
    done = warmup + steps
    # The first tens of milliseconds of a memory-bound phase run slower on this machine (seen in
    # kernel traces: the 124 M-element worker pass takes 1.9 ms in steps 1-3 and settles at
    # 1.68 ms after about 30 ms, whatever came before), so for the headline reading the clocks
    # get `settle_ms` of the same steps before W more warm-up steps and the K timed steps.
    t_end = time.perf_counter() + settle_ms * 1e-3
    while time.perf_counter() < t_end:
        step(done)
        done += 1
        if done % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    for t in range(warmup):
        step(done + t)
    done += warmup
    # An event record costs a bubble of about 6 us between two kernels that otherwise run back
    # to back (seen in the kernel trace), so the timed region carries events only around the
    # worker call of every 3rd step: enough for the average launch duration of the dominant
    # kernel (roofline) at under 1 % of a step.  The per-stage split comes from a second,
    # untimed pass over the same number of steps (always the three separate calls).
    every = 3     # odd: the sampled steps alternate between the gradient sets
    evs = {t: [torch.cuda.Event(enable_timing=True) for _ in range(2)] for t in range(0, steps, every)}
    ms_settled = timed(done, steps, evs)
    done += steps
    worker_ms = sum(ev[0].elapsed_time(ev[1]) for ev in evs.values()) / len(evs)
    evs2 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for t in range(steps):
        step(done + t, evs2[t], stages=True)
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
    return {"ms_per_step": ms_settled, "ms_per_step_unsettled": ms_unsettled, "stage_ms": stage_ms, "S": S,
            "worker_ms": worker_ms, "worker_samples": len(evs)}


def run_uncompensated_worker(wl, steps: int, warmup: int, S: int):
    """The worker pass of the comparison algorithms without compensation (Section 5.1):
    DS_FLAG_NO_ERROR_FEEDBACK, no error buffer traffic, so the pass moves the gradient and the
    message only."""
    import torch
    import paper_1905_05957_amd as P

    dev = torch.device("cuda:0")
    flags = P.FLAG_NO_ERROR_FEEDBACK | (P.FLAG_SERVER_IDENTITY if wl.comp == "topk" else 0)
    ctx = _context(wl, False, flags)
    grads = [wl.gradients(s, dev) for s in range(2)]
    pw = ctx.alloc_payload(wl.n, dev)
    for t in range(warmup + 20):
        ctx.worker_compress(t, grads[t % 2], None, pw)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for t in range(steps):
        ctx.worker_compress(t, grads[t % 2], None, pw)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    ctx.close()
    ab = algorithmic_bytes(wl, S)
    nbytes = wl.n * (wl.d * ab["grad_bytes"] + ab["message"])
    return {"workload": wl.name + " worker pass, DS_FLAG_NO_ERROR_FEEDBACK", "ms": ms, "algorithmic_bytes": nbytes,
            "GBs": nbytes / ms / 1e6, "frac_of_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS}


def run_copy_ceiling():
    """The practical HBM ceiling: the library's plain streaming copy kernel (one 128-bit load and
    store per thread) over 1 GiB, bytes read + written per second."""
    import torch
    import paper_1905_05957_amd as P
    dev = torch.device("cuda:0")
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(5):
        P.ds_probe_copy(src, dst)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    reps = 20
    for _ in range(reps):
        P.ds_probe_copy(src, dst)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    ok = bool(torch.equal(src, dst))
    del src, dst
    torch.cuda.empty_cache()
    if not ok:
        raise RuntimeError("copy probe produced a wrong copy")
    return 2 * (1 << 30) / ms / 1e6


def cpu_info() -> dict:
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"nproc": os.cpu_count(), "cpu_model": model}


def run_oracle(wl, steps: int, target_elems: int, row_parallel: bool = False):
    """The CPU oracle, as it stands, single thread: `steps` full steps (worker, server, update)
    on the first d' elements of every row, d' = d unless n*d exceeds target_elems (then cut at a
    scale-group / bucket boundary).  row_parallel: additionally the worker block of one step with
    the outer loop over workers spread over min(n, cores) threads (one oracle call per row,
    arithmetic per row unchanged; only for compressors that draw no random numbers)."""
    import numpy as np
    import torch
    import dataclasses
    import oracle as O

    dq = max(1, min(wl.d, target_elems // wl.n))
    unit = {"sign": wl.chunk if wl.scale_mode == "chunk" else 64, "qsgd": wl.bucket}.get(wl.comp, 64)
    if dq < wl.d:
        dq = max(unit, (dq // unit) * unit)
    dq = min(dq, wl.d)
    sub = wl if dq == wl.d else dataclasses.replace(wl, d=dq, k=max(1, wl.k * dq // wl.d) if wl.k else 0)
    if dq != wl.d and wl.seg_offsets is not None:
        off = wl.seg_offsets[wl.seg_offsets < dq]
        sub.seg_offsets = np.concatenate([off, [dq]]).astype(np.int64)
        sub.seg_sigma = wl.seg_sigma[: len(off)]
    comp = {"identity": O.IDENTITY, "sign": O.SIGN, "topk": O.TOPK, "qsgd": O.QSGD, "clip": O.CLIP,
            "rsparse": O.RSPARSE}[sub.comp]

    def config(n):
        return O.Config(comp, n=n, d=dq, grad_bf16=(sub.grad_dtype == "bf16"),
                        group_off=sub.group_offsets() if sub.comp == "sign" else None, k=sub.k,
                        bucket=sub.bucket, levels=sub.levels, seed=sub.seed, sign_rms=sub.sign_rms,
                        clip_bits=sub.clip_bits,
                        keep_prob=float(np.float32(round(sub.keep_prob * (1 << 24))) / np.float32(1 << 24)))

    cfg = config(sub.n)
    g = sub.gradients(0, "cpu")
    hg = g.view(torch.int16).numpy().view(np.uint16) if g.dtype == torch.bfloat16 else g.numpy()
    delta = sub.initial_delta("cpu").numpy()
    delta_s = np.zeros(dq, np.float32)
    x = sub.initial_x("cpu").numpy()
    m = np.zeros(dq, np.float32) if sub.beta is not None else None
    O.lib()
    stage = [0.0, 0.0, 0.0]
    for t in range(steps):
        t0 = time.perf_counter()
        pw = O.worker_compress(cfg, t, hg, delta)
        t1 = time.perf_counter()
        ps = O.server_aggregate_compress(cfg, t, pw, delta_s)
        t2 = time.perf_counter()
        O.apply_update(cfg, ps, x, m, sub.gamma, 0.0 if sub.beta is None else sub.beta)
        t3 = time.perf_counter()
        stage = [stage[0] + t1 - t0, stage[1] + t2 - t1, stage[2] + t3 - t2]
    dt = sum(stage)
    what = "all" if dq == wl.d else f"the first {dq} of"
    out = {"value": steps * sub.n * dq / dt, "unit": "gradient elements/s", "cores": 1, "kind": "oracle",
           "seconds": dt, "stage_seconds": {"worker": stage[0], "server": stage[1], "update": stage[2]},
           "sample": f"{steps} full step(s) on {what} {wl.d} elements of all {wl.n} rows ({dt:.1f} s, single thread)"}
    if row_parallel and sub.comp in ("sign", "topk", "clip", "identity"):
        from concurrent.futures import ThreadPoolExecutor
        threads = max(1, min(sub.n, os.cpu_count() or 1))
        one = config(1)
        rows_d = [np.ascontiguousarray(delta[i:i + 1]) for i in range(sub.n)]
        rows_g = [np.ascontiguousarray(hg[i:i + 1]) for i in range(sub.n)]
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=threads) as ex:       # the C routine runs without the interpreter lock
            list(ex.map(lambda i: O.worker_compress(one, steps, rows_g[i], rows_d[i]), range(sub.n)))
        tw = time.perf_counter() - t0
        per_step = tw + (stage[1] + stage[2]) / steps              # server and update have one row: as timed above
        out["row_parallel"] = {"threads": threads, "worker_seconds": tw, "value": sub.n * dq / per_step,
                               "unit": "gradient elements/s",
                               "note": "worker rows on separate threads; server and update single thread"}
    return out


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
    ap.add_argument("--cpu-elems", type=int, default=1_000_000_000,
                    help="the oracle is timed on at most this many gradient elements (n*d') per workload")
    ap.add_argument("--no-modes", action="store_true", help="skip the un-compensated worker pass entries")
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

    copy_gbs = run_copy_ceiling()

    def measure(name, steps, warmup, calib_copy=False):
        wl = make_workload(name)
        r = run_gpu(wl, steps, warmup, calib_copy=calib_copy, deferred_error=not a.plain_error,
                    separate_update=a.separate_update, settle_ms=a.settle_ms)
        ab = algorithmic_bytes(wl, r["S"])
        ms = r["ms_per_step"]
        wk_ms = r["worker_ms"]
        gbs = ab["total"] / (ms * 1e-3) / 1e9
        out = {
            "workload": wl.name, "n": wl.n, "d": wl.d, "ms_per_step": ms,
            "ms_per_step_unsettled": r["ms_per_step_unsettled"],
            "calls": "ds_worker_compress + " + ("ds_server_aggregate_compress + ds_apply_update" if a.separate_update
                                                else "ds_server_aggregate_compress_update"),
            "error_state": "plain" if a.plain_error or not (wl.comp == "sign" and wl.scale_mode != "chunk") else "deferred",
            "value": wl.n * wl.d / (ms * 1e-3),
            "stage_ms": {"worker": r["stage_ms"][0], "server": r["stage_ms"][1], "update": r["stage_ms"][2]},
            "algorithmic_bytes_per_step": ab["total"],
            "step_hbm_GBs": gbs,
            "step_frac_of_peak": gbs / HBM_PEAK_GBS,
            "step_frac_of_copy": gbs / copy_gbs,
            "step_frac_of_peak_unsettled": ab["total"] / (r["ms_per_step_unsettled"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "roofline": {"bound": "hbm", "kernel": "worker pass (ds_worker_compress)",
                         "achieved": ab["worker"] / (wk_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": ab["worker"] / (wk_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "frac_of_copy": ab["worker"] / (wk_ms * 1e-3) / 1e9 / copy_gbs,
                         "algorithmic_bytes": ab["worker"], "launch_ms": wk_ms,
                         "launch_samples": r["worker_samples"],
                         "traffic": measured_worker_traffic(name)},
        }
        if "as_implemented" in ab:
            out["bytes_note"] = ("the server's dense error is counted as read once and written where it changes "
                                 "(n k + k positions); the kernels write it densely: %d bytes per step" % ab["as_implemented"])
        return wl, out, r["S"]

    wl, head, head_S = measure(a.workload, a.steps, a.warmup, calib_copy=a.calib_copy)
    others = []
    modes = []
    # oracle steps per workload: three for the small sign workload, one for the others
    oracle_steps = {"c2": 3}
    for name in [s for s in a.others.split(",") if s and s != a.workload]:
        try:
            owl, o, oS = measure(name, max(5, a.steps // 2), max(2, a.warmup // 2))
            if not a.no_cpu_baseline:
                o["cpu_baseline"] = run_oracle(owl, oracle_steps.get(name, 1), a.cpu_elems)
            if name == "c2" and not a.no_modes:
                modes.append(run_uncompensated_worker(owl, 20, 3, oS))
            others.append(o)
        except Exception as e:  # a workload whose compressor is not built yet
            others.append({"workload": name, "error": str(e)})
        torch.cuda.empty_cache()
    if not a.no_modes and wl.comp not in ("rsparse", "identity"):   # those two have no mode without compensation
        modes.append(run_uncompensated_worker(wl, 20, 3, head_S))

    line = {
        "metric": "DoubleSqueeze step: gradient elements/s (n\u00b7d) and HBM GB/s as % of peak", "value": head["value"],
        "unit": "gradient elements/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "n_workers": wl.n, "d": wl.d,
                   "grad_dtype": wl.grad_dtype, "compressor": wl.comp, "settle_ms": a.settle_ms},
        "ms_per_step_unsettled": head["ms_per_step_unsettled"],
        "stage_ms": head["stage_ms"],
        "algorithmic_bytes_per_step": head["algorithmic_bytes_per_step"],
        "step_hbm_GBs": head["step_hbm_GBs"], "step_frac_of_peak": head["step_frac_of_peak"],
        "step_frac_of_copy": head["step_frac_of_copy"],
        "step_frac_of_peak_unsettled": head["step_frac_of_peak_unsettled"],
        "hbm_pct_of_peak": 100.0 * head["step_frac_of_peak"],     # the metric's second figure, whole step
        "copy_ceiling_GBs": copy_gbs,
        "roofline": head["roofline"],
        "other_workloads": others,
        "uncompensated_worker_pass": modes,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = run_oracle(wl, 1, a.cpu_elems, row_parallel=True)
        line["cpu_baseline"].update(cpu_info())
    print(json.dumps(line))


if __name__ == "__main__":
    main()
