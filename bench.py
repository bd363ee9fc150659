#!/usr/bin/env python3
"""Benchmark of the rTop-k hot path on one MI355X.

One *step* is one pass of the whole hot path over one batch of synthetic
input: the n workers' d-element gradients go through the error-compensated
rTop-k sparsifier (``rtopk_encode_batch``: one call, shared kernel launches,
every worker computed exactly as by ``rtopk_encode``) and the master runs
``rtopk_aggregate`` on the n messages. The headline workload is the
ResNet-50-sized configuration (d = 25,557,032, r = 0.5% d, k = 0.1% d, n = 8
workers) that the metric is quoted on. All gradients are resident in HBM
before any clock starts; everything runs on one stream; every step uses a
step number that was not used before on its residuals.

Order of the run (default flags):
  warm-up      W steps
  steady loop  ``--steady-steps`` further steps (at least 100 ms of device
               time), timed as a whole and with the dominant kernel of every
               ``--trace-every``-th step bracketed by HIP events: the device
               is at its steady clocks afterwards, and the line shows the
               kernel's mean over the first and the last tenth of the loop
  timed region EXACTLY K steps between two synchronisations -> ``value``;
               the dominant kernel of every ``--trace-every``-th of them is
               bracketed in the same way -> ``roofline`` (a bracket holds the
               stream up for ~5 us on either side of the kernel, which is why
               not every step carries one)
  legs         (outside the timed region) the encode / aggregate split of a
               step, one ``rtopk_encode`` call per worker (``per_call``), the
               fused master updates, a bare streaming add over the same
               buffers (what a read-read-write stream reaches on this memory
               system), the other benchmark configurations (``configs``), and
               the CPU oracle on a bounded sample (``cpu_baseline``)

Prints ONE JSON line:
  value      = gradient bytes consumed per second over whole steps
               (n * 4d bytes per step / seconds per step), GB/s
  roofline   = the dominant kernel (fused residual add + candidate append):
               algorithmic bytes per launch (12 d per vector in the launch)
               over its mean duration in the timed region, measured with HIP
               events on the launch stream, against the 8 TB/s HBM peak
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "rTop-k encode gradient GB/s and % of HBM peak at d=25.6M; aggregate GB/s"
TRAFFIC_PROFILE = os.path.join("profiles", "k_fused_cfg3_hbm_traffic.txt")


def traffic_from_profile(d: int, vectors_per_launch: int):
    """HBM bytes per launch of the dominant kernel as the tracked rocprofv3
    counter summary states them (FETCH_SIZE and WRITE_SIZE runs, each scaled by
    a device copy of known size), or None when there is no summary for this
    vector length and launch shape. The summary's last lines are
    ``traffic_bytes_per_launch: N  vectors_per_launch: V  d: D``."""
    try:
        text = open(os.path.join(ROOT, TRAFFIC_PROFILE)).read()
    except OSError:
        return None
    for m in re.finditer(r"traffic_bytes_per_launch:\s*(\d+)\s+vectors_per_launch:\s*(\d+)\s+d:\s*(\d+)",
                         text):
        if int(m.group(2)) == vectors_per_launch and int(m.group(3)) == d:
            return int(m.group(1))
    return None


class HipEvents:
    """Raw hipEvent_t pairs through the HIP runtime that torch already loaded."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so.7")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float),
                                                 ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.events = []

    def new(self) -> int:
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        self.events.append(ev)
        return ev.value

    def pair(self):
        return (self.new(), self.new())

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def close(self):
        for ev in self.events:
            self.hip.hipEventDestroy(ev)
        self.events = []


class Job:
    """Device state of n simulated workers for sizes (d, r, k): residuals,
    message buffers, workspace slices, the dense output; and the step."""

    def __init__(self, rt, torch, dev, d, r, k, n, stream):
        from workloads import philox_seed_for_worker
        self.rt, self.torch, self.stream = rt, torch, stream
        self.d, self.r, self.k, self.n = d, r, k, n
        self.residual = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
        self.idx = torch.empty(n * k, dtype=torch.int32, device=dev)
        self.val = torch.empty(n * k, dtype=torch.float32, device=dev)
        self.out_i = [self.idx[w * k:(w + 1) * k] for w in range(n)]
        self.out_v = [self.val[w * k:(w + 1) * k] for w in range(n)]
        self.seeds = [philox_seed_for_worker(w) for w in range(n)]
        self.out = torch.empty(d, dtype=torch.float32, device=dev)
        self.ws_bytes = rt.encode_workspace_bytes(d, r, k)
        self.ws = torch.empty(n * self.ws_bytes, dtype=torch.uint8, device=dev)
        self.ws_of = [self.ws[w * self.ws_bytes:(w + 1) * self.ws_bytes] for w in range(n)]
        self.next_step = 0                       # step numbers are never reused on these residuals

    def step(self, grads, as_batch=True, trace=None, phase=None):
        """The n workers' encodes (one batched call, or n calls) and the
        master's average. ``trace``: (begin, end) HIP events around the dominant
        kernel (a list of n such pairs or None entries for single calls);
        ``phase``: three torch events recorded before, between and after the calls."""
        rt, stream, n = self.rt, self.stream, self.n
        step_no = self.next_step
        self.next_step += 1
        if phase is not None:
            phase[0].record(stream)
        if as_batch:
            if trace is not None:
                rt.trace_next_encode(rt.STAGES["fused"], *trace)
            rt.encode_batch(grads, self.residual, self.r, self.k, self.seeds, step_no, self.out_i,
                            self.out_v, self.ws, stream)
        else:
            for w in range(n):
                if trace is not None and trace[w] is not None:
                    rt.trace_next_encode(rt.STAGES["fused"], *trace[w])
                rt.encode(grads[w], self.residual[w], self.r, self.k, self.seeds[w], step_no,
                          self.out_i[w], self.out_v[w], self.ws_of[w], stream)
        if phase is not None:
            phase[1].record(stream)
        rt.aggregate(self.idx, self.val, n, self.k, self.out, None, stream)
        if phase is not None:
            phase[2].record(stream)

    def check_stats(self, what):
        last = None
        for w in range(self.n):
            last = self.rt.encode_stats(self.ws_of[w], self.stream)
            if last["error_flags"] != 0:
                raise RuntimeError(f"{what}: encode of worker {w} reported error flags {last}")
        return last


def timed_loop(job, torch, ev, grad_sets, steps, as_batch=True, trace_all=True, trace_every=1):
    """``steps`` steps on job.stream between two events; returns (ms per step,
    list of durations of the dominant kernel in ms, one per bracketed step).
    Every ``trace_every``-th step has its dominant kernel bracketed by HIP
    events: each bracket costs the stream ~5 us on either side of the kernel."""
    n = job.n
    pairs = [ev.pair() if trace_all and s % trace_every == 0 else None for s in range(steps)]
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    t0.record(job.stream)
    for s in range(steps):
        tr = pairs[s]
        if not as_batch and tr is not None:
            # one launch per step is bracketed, a different worker every step
            tr = [pairs[s] if w == s % n else None for w in range(n)]
        job.step(grad_sets[s % len(grad_sets)], as_batch, trace=tr)
    t1.record(job.stream)
    torch.cuda.synchronize()
    fused = [ev.elapsed_ms(*p) for p in pairs if p is not None]
    return t0.elapsed_time(t1) / steps, fused


def split_loop(job, torch, grad_sets, steps, as_batch=True):
    """The same steps with an event after each call: (encode ms per vector,
    aggregate ms per call, ms per step)."""
    phase = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(steps)]
    job.step(grad_sets[0], as_batch)
    for s in range(steps):
        job.step(grad_sets[s % len(grad_sets)], as_batch, phase=phase[s])
    torch.cuda.synchronize()
    enc = sum(p[0].elapsed_time(p[1]) for p in phase) / (steps * job.n)
    agg = sum(p[1].elapsed_time(p[2]) for p in phase) / steps
    whole = phase[0][0].elapsed_time(phase[-1][2]) / steps
    return enc, agg, whole


def mean(xs):
    return sum(xs) / len(xs)


def measure_config(rt, torch, dev, stream, ev, wl, r, k, n, grads, steps, warmup):
    """One benchmark configuration other than the headline one: batched steps
    over ONE resident gradient set (the same n gradients every step, on top of
    the evolving residuals, fresh step numbers)."""
    d = wl.d
    job = Job(rt, torch, dev, d, r, k, n, stream)
    for _ in range(warmup):
        job.step(grads)
    torch.cuda.synchronize()
    ms_step, fused = timed_loop(job, torch, ev, [grads], steps, trace_every=max(1, min(4, steps // 2)))
    enc, agg, _ = split_loop(job, torch, [grads], min(steps, 5))
    st = job.check_stats(f"{wl.config.name} r={r} k={k}")
    # the bare read-read-write stream over the same buffers, for this size's ceiling
    rounds = 3
    for w in range(n):
        rt.diag_stream_add(grads[w], job.residual[w], stream)
    a0, a1 = (torch.cuda.Event(enable_timing=True) for _ in range(2))
    a0.record(stream)
    for _ in range(rounds):
        for w in range(n):
            rt.diag_stream_add(grads[w], job.residual[w], stream)
    a1.record(stream)
    torch.cuda.synchronize()
    add_ms = a0.elapsed_time(a1) / (rounds * n)
    fused_ms = mean(fused)
    res = {"d": d, "r": r, "k": k, "workers": n, "steps": steps,
           "ms_per_step": round(ms_step, 4),
           "value_GBps": round(n * 4.0 * d / (ms_step * 1e-3) / 1e9, 1),
           "encode_us_per_vector": round(enc * 1e3, 2),
           "encode_pct_hbm_peak_at_12d": round(100.0 * 12.0 * d / (enc * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
           "k_fused_ms": round(fused_ms, 5),
           "k_fused_frac": round(n * 12.0 * d / (fused_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
           "stream_add_frac": round(12.0 * d / (add_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
           "aggregate_us": round(agg * 1e3, 2),
           "aggregate_GBps": round(4.0 * d / (agg * 1e-3) / 1e9, 1),
           "path": st["path"], "candidates_per_vector": st["superset_size"]}
    del job
    torch.cuda.empty_cache()
    return res


def other_configs(rt, torch, dev, stream, ev, which, steps, warmup):
    """Configurations 1, 2, 4 and the nine stress points (16 workers each)."""
    from workloads import Workload
    from workloads.gradients import STRESS_K_FRACS, STRESS_R_OVER_K
    out = {}
    for cfg in which:
        wl = Workload(cfg)
        n = wl.n_workers
        grads = [torch.from_numpy(wl.gradient(w, 0)).to(dev) for w in range(n)]
        if cfg != 5:
            out[wl.config.name] = measure_config(rt, torch, dev, stream, ev, wl, wl.r, wl.k, n,
                                                 grads, steps, warmup)
        else:
            points = {}
            for num, den in STRESS_K_FRACS:
                for ratio in STRESS_R_OVER_K:
                    k = (wl.d * num + den - 1) // den
                    points[f"k={100.0 * num / den:g}%d,r={ratio}k"] = measure_config(
                        rt, torch, dev, stream, ev, wl, ratio * k, k, n, grads, steps, warmup)
            out[wl.config.name] = points
        del grads
        torch.cuda.empty_cache()
    return out


def cpu_baseline(wl, n_sample: int):
    """Time the oracle as it stands on a bounded sample: n_sample encodes of
    step 0 and one aggregate of those messages, single thread."""
    import numpy as np
    import oracle
    from workloads import philox_seed_for_worker
    oracle.lib()
    grads = [wl.gradient(w, 0) for w in range(n_sample)]
    zero = np.zeros(wl.d, np.float32)
    t0 = time.perf_counter()
    msgs = [oracle.encode(grads[w], zero, wl.r, wl.k, philox_seed_for_worker(w), 0)
            for w in range(n_sample)]
    t1 = time.perf_counter()
    idx = np.concatenate([m[0] for m in msgs])
    val = np.concatenate([m[1] for m in msgs])
    oracle.aggregate(idx, val, n_sample, wl.d)
    t2 = time.perf_counter()
    total = t2 - t0
    # the same oracle, one thread per simulated worker (the C call releases the
    # interpreter lock), as many workers as the box has cores for, at most n
    from concurrent.futures import ThreadPoolExecutor
    cores = max(1, min(len(os.sched_getaffinity(0)), wl.n_workers))
    more = [wl.gradient(w, 0) for w in range(n_sample, cores)]
    every = grads + more
    t3 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        list(pool.map(lambda w: oracle.encode(every[w], zero, wl.r, wl.k,
                                              philox_seed_for_worker(w), 0), range(cores)))
    t4 = time.perf_counter()
    return {
        "value": round(n_sample * 4 * wl.d / total / 1e9, 4),
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": (f"{n_sample} of {wl.n_workers} workers at step 0: {n_sample} oracle encodes "
                   f"({t1 - t0:.1f} s) + one aggregate of their messages ({t2 - t1:.2f} s), "
                   f"d={wl.d}; host has {len(os.sched_getaffinity(0))} usable cores"),
        "encode_s_per_call": round((t1 - t0) / n_sample, 3),
        "aggregate_s_per_call": round(t2 - t1, 3),
        "all_cores": {"value": round(cores * 4 * wl.d / (t4 - t3) / 1e9, 4), "unit": "GB/s",
                      "cores": cores,
                      "sample": f"{cores} oracle encodes of step 0 side by side, one thread each "
                                f"({t4 - t3:.1f} s wall)"},
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3,
                    help="workload configuration of the timed region (1-5; 6 = the federated update vector)")
    ap.add_argument("--workers", type=int, default=0, help="override the workload's worker count")
    ap.add_argument("--steady-steps", type=int, default=240, metavar="S",
                    help="steps of the steady loop that precedes the timed region (0 = none)")
    ap.add_argument("--trace-every", type=int, default=4, metavar="N",
                    help="bracket the dominant kernel with HIP events on every N-th step of the steady "
                         "loop and the timed region (each bracket costs the stream ~10 us)")
    ap.add_argument("--grad-sets", type=int, default=6, metavar="G",
                    help="distinct gradient sets resident in HBM; step s uses set s mod G")
    ap.add_argument("--sequential", action="store_true",
                    help="the timed steps call rtopk_encode once per worker instead of "
                         "rtopk_encode_batch once per step")
    ap.add_argument("--no-per-call-leg", action="store_true",
                    help="skip the extra pass that times one rtopk_encode call per worker")
    ap.add_argument("--configs", default="1,2,4,5",
                    help="other benchmark configurations to measure after the timed region "
                         "(comma separated; 5 = the nine stress points with 16 workers; "
                         "'none' skips the leg)")
    ap.add_argument("--configs-steps", type=int, default=8)
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="after the timed region, also run N plain device copies of d floats "
                         "(4d bytes read + 4d bytes written each): a kernel of known HBM "
                         "traffic to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters with")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=2, help="oracle encodes to time")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; simulated workers share it and no "
              "collective exists, so --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    import paper_2005_10761_amd as rt
    from workloads import Workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    rt.load_library()
    dev = torch.device("cuda:0")
    wl = Workload(args.config)
    d, r, k = wl.d, wl.r, wl.k
    n = args.workers or wl.n_workers
    K, W = args.steps, args.warmup
    TE = max(1, min(args.trace_every, K))
    batched = not args.sequential

    # ---- inputs: G gradient sets resident in HBM, cycled ------------------
    G = max(1, min(args.grad_sets, K + W + args.steady_steps))
    grad_sets = [[torch.from_numpy(wl.gradient(w, t)).to(dev) for w in range(n)] for t in range(G)]
    stream = torch.cuda.Stream(device=dev)                           # default priority
    job = Job(rt, torch, dev, d, r, k, n, stream)
    ev = HipEvents()
    torch.cuda.synchronize()

    for t in range(W):
        job.step(grad_sets[t % G], batched)
    torch.cuda.synchronize()

    # ---- steady loop: long enough for the clocks to settle -----------------
    steady = None
    if args.steady_steps > 0:
        S = args.steady_steps
        ms_s, fused_s = timed_loop(job, torch, ev, grad_sets, S, batched, trace_every=TE)
        tenth = max(1, len(fused_s) // 10)
        steady = {"steps": S, "ms_per_step": round(ms_s, 4), "region_ms": round(ms_s * S, 1),
                  "value": round(n * 4.0 * d / (ms_s * 1e-3) / 1e9, 2), "unit": "GB/s",
                  "k_fused_ms_first_tenth": round(mean(fused_s[:tenth]), 5),
                  "k_fused_ms_last_tenth": round(mean(fused_s[-tenth:]), 5),
                  "k_fused_ms_mean": round(mean(fused_s), 5)}
        job.check_stats("steady loop")

    # ---- timed region: EXACTLY K steps between two synchronisations --------
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    ms_per_step, fused_ms = timed_loop(job, torch, ev, grad_sets, K, batched, trace_every=TE)
    t_wall1 = time.perf_counter()
    stats = job.check_stats("timed region")
    vectors_per_launch = n if batched else 1

    # ---- outside the timed region: the split of a step into its two calls
    #      (three more event records per step cost the stream ~2%) -----------
    legs = min(K, 20)
    enc_ms_vector, agg_ms_call, _ = split_loop(job, torch, grad_sets, legs, batched)
    job.check_stats("split leg")

    # ---- one rtopk_encode call per worker (the latency of a single call) ---
    per_call = None
    if batched and not args.no_per_call_leg:
        ms_call, _, ms_step = split_loop(job, torch, grad_sets, legs, False)
        _, fused_single = timed_loop(job, torch, ev, grad_sets, legs, False)
        job.check_stats("per-call leg")
        per_call = {"encode_ms_per_call": round(ms_call, 4),
                    "encode_gradient_GBps": round(4.0 * d / (ms_call * 1e-3) / 1e9, 2),
                    "encode_pct_hbm_peak_at_12d": round(100.0 * 12.0 * d / (ms_call * 1e-3) / 1e9
                                                        / HBM_PEAK_GBPS, 2),
                    "k_fused_ms": round(mean(fused_single), 5),
                    "k_fused_frac": round(12.0 * d / (mean(fused_single) * 1e-3) / 1e9
                                          / HBM_PEAK_GBPS, 4),
                    "ms_per_step": round(ms_step, 4),
                    "value": round(n * 4.0 * d / (ms_step * 1e-3) / 1e9, 2), "unit": "GB/s"}

    # ---- the bare stream: residual += gradient over the same n buffer pairs,
    #      same accesses and grid as the dominant kernel, nothing else --------
    rounds = 10
    for w in range(n):
        rt.diag_stream_add(grad_sets[0][w], job.residual[w], stream)
    c0, c1 = (torch.cuda.Event(enable_timing=True) for _ in range(2))
    c0.record(stream)
    for q in range(rounds):
        for w in range(n):
            rt.diag_stream_add(grad_sets[q % G][w], job.residual[w], stream)
    c1.record(stream)
    torch.cuda.synchronize()
    add_ms = c0.elapsed_time(c1) / (rounds * n)
    stream_add = {"what": "residual += gradient, 12 d bytes per launch, launches back to back "
                          f"over the {n} workers' buffers",
                  "ms_per_launch": round(add_ms, 5),
                  "achieved": round(12.0 * d / (add_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                  "frac": round(12.0 * d / (add_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
    for m in job.residual:
        m.zero_()                                  # the sums above are no residuals

    # ---- the master's fused updates on the last step's messages -------------
    idx, val = job.idx, job.val
    upd_ws = torch.empty(rt.aggregate_update_workspace_bytes(d, n, k), dtype=torch.uint8,
                         device=dev)
    omegas = [torch.randn(d, dtype=torch.float32, device=dev) for _ in range(4)]
    upd = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    upd_calls = 5 * len(omegas)
    for om in omegas:
        rt.aggregate_update(idx, val, n, k, 0.1, r / k, om, upd_ws, stream)
    upd[0].record(stream)
    for c in range(upd_calls):
        rt.aggregate_update(idx, val, n, k, 0.1, r / k, omegas[c % len(omegas)], upd_ws, stream)
    upd[1].record(stream)
    torch.cuda.synchronize()
    upd_ms_call = upd[0].elapsed_time(upd[1]) / upd_calls
    vels = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(len(omegas))]
    for om, ve in zip(omegas, vels):
        rt.aggregate_update_momentum(idx, val, n, k, 0.1, r / k, 0.9, om, ve, stream)
    upd[0].record(stream)
    for c in range(upd_calls):
        rt.aggregate_update_momentum(idx, val, n, k, 0.1, r / k, 0.9, omegas[c % len(omegas)],
                                     vels[c % len(omegas)], stream)
    upd[1].record(stream)
    torch.cuda.synchronize()
    mom_ms_call = upd[0].elapsed_time(upd[1]) / upd_calls
    del omegas, vels

    if args.copy_calibration > 0:
        src = grad_sets[0][0]
        for _ in range(args.copy_calibration):
            job.out.copy_(src)
        torch.cuda.synchronize()

    fused_ms_avg = mean(fused_ms)
    value = n * 4.0 * d / (ms_per_step * 1e-3) / 1e9
    launch_bytes = vectors_per_launch * 12 * d
    achieved = launch_bytes / (fused_ms_avg * 1e-3) / 1e9
    traffic = traffic_from_profile(d, vectors_per_launch)
    ws_bytes = job.ws_bytes
    result = {
        "metric": METRIC,
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.config.name, "d": d, "r": r, "k": k, "workers": n,
                   "step": (f"1 x rtopk_encode_batch ({n} workers) + 1 x rtopk_aggregate"
                            if batched else f"{n} x rtopk_encode + 1 x rtopk_aggregate")
                           + f", one stream; {G} gradient sets resident in HBM, step s uses set "
                             f"s mod {G} on the evolving residuals under a fresh step number",
                   "encode_workspace_bytes_per_vector": ws_bytes},
        "timed_region_ms": round(ms_per_step * K, 2),
        "steady": steady,
        "encode_gradient_GBps": round(4.0 * d / (enc_ms_vector * 1e-3) / 1e9, 2),
        "encode_ms_per_vector": round(enc_ms_vector, 4),
        "encode_pct_hbm_peak_at_12d": round(100.0 * 12.0 * d / (enc_ms_vector * 1e-3) / 1e9
                                            / HBM_PEAK_GBPS, 2),
        "aggregate_GBps": round(4.0 * d / (agg_ms_call * 1e-3) / 1e9, 2),
        "aggregate_ms_per_call": round(agg_ms_call, 4),
        "aggregate_update_ms_per_call": round(upd_ms_call, 4),
        "aggregate_update_momentum_ms_per_call": round(mom_ms_call, 4),
        "aggregate_update_momentum_GBps": round(16.0 * d / (mom_ms_call * 1e-3) / 1e9, 2),
        "per_call": per_call,
        "wall_ms_per_step": round((t_wall1 - t_wall0) * 1e3 / K, 4),
        "last_encode": {"path": stats["path"], "superset": stats["superset_size"],
                        "boundary_list": stats["boundary_list_size"],
                        "key_list": stats["key_list_size"]},
        "roofline": {
            "kernel": "k_fused",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": traffic,
            "traffic_source": TRAFFIC_PROFILE if traffic is not None else None,
            "bytes_per_launch": launch_bytes,
            "vectors_per_launch": vectors_per_launch,
            "avg_launch_ms": round(fused_ms_avg, 5),
            "launches": len(fused_ms),
            "launches_bracketed": f"every {TE}th step of the timed region" if TE > 1 else "every step of the timed region",
            "stream_add_calibration": stream_add,
        },
    }
    del grad_sets, job
    torch.cuda.empty_cache()
    if args.configs.strip().lower() not in ("", "none"):
        which = [int(c) for c in args.configs.split(",") if int(c) != args.config]
        result["configs"] = other_configs(rt, torch, dev, stream, ev, which, args.configs_steps, 2)
    ev.close()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, max(1, min(args.cpu_sample, n)))
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
