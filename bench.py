#!/usr/bin/env python3
"""Benchmark of the rTop-k hot path on one MI355X.

One *step* is one pass of the whole hot path over one batch of synthetic
input: the n workers' fresh d-element gradients go through the
error-compensated rTop-k sparsifier (``rtopk_encode_batch``: one call, shared
kernel launches, every worker computed exactly as by ``rtopk_encode``) and the
master runs ``rtopk_aggregate`` on the n messages. The workload is the
ResNet-50-sized configuration (d = 25,557,032, r = 0.5% d, k = 0.1% d, n = 8
workers) that the headline metric is quoted on. All gradients of the warm-up
and timed steps are resident in HBM before the clock starts; everything runs
on one stream. ``--sequential`` times n separate ``rtopk_encode`` calls per
step instead; by default that variant runs once more after the timed region
and is reported as ``per_call`` (the latency of a single call). Inside the timed
region the stream carries, besides the work, only the two HIP events around the
dominant kernel of every step; the split of a step into encode and aggregate
time (``encode_ms_per_vector``, ``aggregate_ms_per_call``) comes from a second
pass over the same steps with an event after each call.

Prints ONE JSON line:
  value      = gradient bytes consumed per second over whole steps
               (n * 4d bytes per step / seconds per step), GB/s
  roofline   = the dominant kernel (fused residual add + candidate append):
               algorithmic bytes per launch (12 d per vector in the launch)
               over its mean duration, measured with HIP events on the launch
               stream, against the 8 TB/s HBM peak
  cpu_baseline = the CPU oracle, one thread, timed on a bounded sample of the
               same workload
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "rTop-k encode gradient GB/s and % of HBM peak at d=25.6M; aggregate GB/s"

# HBM bytes per launch of the dominant kernel (k_fused at d = 25,557,032) from
# two rocprofv3 --pmc runs, FETCH_SIZE then WRITE_SIZE, each scaled by a device
# copy of known size in the same run; the summary and the commands are in
# profiles/k_fused_cfg3_hbm_traffic.txt. Only valid for the default workload.
SINGLE_KERNEL_TRAFFIC_BYTES = 309_655_484       # one vector per launch (--sequential)
BATCH_KERNEL_TRAFFIC_BYTES = 2_476_223_559   # the default: 8 workers per launch


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
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload configuration (1-5; 6 = the federated update vector)")
    ap.add_argument("--workers", type=int, default=0, help="override the workload's worker count")
    ap.add_argument("--sequential", action="store_true",
                    help="the timed steps call rtopk_encode once per worker instead of "
                         "rtopk_encode_batch once per step")
    ap.add_argument("--trace-stride", type=int, default=0, metavar="N",
                    help="with --sequential: bracket every N-th launch of the dominant kernel "
                         "with HIP events (default: the number of workers, i.e. one launch per "
                         "step, a different worker each step; 1 = every launch). The two event "
                         "records cost the stream a few microseconds per traced launch.")
    ap.add_argument("--no-per-call-leg", action="store_true",
                    help="skip the extra pass that times one rtopk_encode call per worker")
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

    import numpy as np
    import torch
    import paper_2005_10761_amd as rt
    from workloads import Workload, philox_seed_for_worker

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    rt.load_library()
    dev = torch.device("cuda:0")
    wl = Workload(args.config)
    d, r, k = wl.d, wl.r, wl.k
    n = args.workers or wl.n_workers
    K, W = args.steps, args.warmup
    total_steps = K + W
    batched = not args.sequential

    # ---- inputs: every gradient of every step resident in HBM ------------
    grads = [[torch.from_numpy(wl.gradient(w, t)).to(dev) for w in range(n)]
             for t in range(total_steps)]
    residual = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
    idx = torch.empty(n * k, dtype=torch.int32, device=dev)
    val = torch.empty(n * k, dtype=torch.float32, device=dev)
    out_i = [idx[w * k:(w + 1) * k] for w in range(n)]
    out_v = [val[w * k:(w + 1) * k] for w in range(n)]
    seeds = [philox_seed_for_worker(w) for w in range(n)]
    out = torch.empty(d, dtype=torch.float32, device=dev)
    ws_bytes = rt.encode_workspace_bytes(d, r, k)
    ws = torch.empty(n * ws_bytes, dtype=torch.uint8, device=dev)   # one slice per worker
    ws_of = [ws[w * ws_bytes:(w + 1) * ws_bytes] for w in range(n)]
    stream = torch.cuda.Stream(device=dev)                           # default priority
    torch.cuda.synchronize()

    def one_step(t: int, step_no: int, as_batch: bool, trace=None, phase=None):
        """The n workers' encodes (one batched call, or n calls) and the
        master's average, all on one stream."""
        if phase is not None:
            phase[0].record(stream)
        if as_batch:
            if trace is not None and trace[0] is not None:
                rt.trace_next_encode(rt.STAGES["fused"], *trace[0])
            rt.encode_batch(grads[t], residual, r, k, seeds, step_no, out_i, out_v, ws, stream)
        else:
            for w in range(n):
                if trace is not None and trace[w] is not None:
                    rt.trace_next_encode(rt.STAGES["fused"], *trace[w])
                rt.encode(grads[t][w], residual[w], r, k, seeds[w], step_no, out_i[w], out_v[w],
                          ws_of[w], stream)
        if phase is not None:
            phase[1].record(stream)
        rt.aggregate(idx, val, n, k, out, None, stream)
        if phase is not None:
            phase[2].record(stream)

    def check_stats():
        last = None
        for w in range(n):
            last = rt.encode_stats(ws_of[w], stream)
            if last["error_flags"] != 0:
                print(f"bench.py: encode of worker {w} reported error flags {last}",
                      file=sys.stderr)
                return None
        return last

    for t in range(W):
        one_step(t, t, batched)
    torch.cuda.synchronize()

    # ---- timed region: K steps, events on the launch stream ----------------
    ev = HipEvents()
    if batched:
        fused_pairs = [[(ev.new(), ev.new())] for _ in range(K)]
        vectors_per_launch = n
    else:
        stride = args.trace_stride if args.trace_stride > 0 else n
        offset = 0 if stride == 1 else 1             # n | stride would always pick worker 0
        fused_pairs = [[(ev.new(), ev.new()) if (s_ * (n + offset) + w) % stride == 0 else None
                        for w in range(n)] for s_ in range(K)]
        vectors_per_launch = 1
    t_begin = torch.cuda.Event(enable_timing=True)
    t_end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    t_begin.record(stream)
    for s_ in range(K):
        one_step(W + s_, W + s_, batched, trace=fused_pairs[s_])
    t_end.record(stream)
    torch.cuda.synchronize()
    t_wall1 = time.perf_counter()
    total_ms = t_begin.elapsed_time(t_end)
    fused_ms = [ev.elapsed_ms(*pair) for row in fused_pairs for pair in row if pair is not None]
    ev.close()
    stats = check_stats()
    if stats is None:
        return 4

    # ---- outside the timed region: the same K steps again with an event after
    #      the encode and after the aggregate of every step, for the split of a
    #      step into its two calls (three more event records per step cost the
    #      stream ~2% and are kept out of the timed region); fresh step numbers,
    #      see below ----------------------------------------------------------
    phase = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(K)]
    one_step(W, 2 * total_steps + 1, batched)
    for s_ in range(K):
        one_step(W + s_, 2 * total_steps + 2 + s_, batched, phase=phase[s_])
    torch.cuda.synchronize()
    enc_ms_vector = sum(p[0].elapsed_time(p[1]) for p in phase) / (K * n)
    agg_ms_call = sum(p[1].elapsed_time(p[2]) for p in phase) / K
    if check_stats() is None:
        return 4

    # ---- outside the timed region: the same K steps once more, one
    #      rtopk_encode call per worker (the latency of a single call). The
    #      gradients of step t again, on top of the residuals as they are now,
    #      under step numbers not used before: sampling keys that already decided
    #      what left these residuals would not be independent of the top-r set. ---
    per_call = None
    if batched and not args.no_per_call_leg:
        edge = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(K)]
        one_step(W, total_steps, False)
        for s_ in range(K):
            one_step(W + s_, total_steps + 1 + s_, False, phase=edge[s_])
        torch.cuda.synchronize()
        ms_call = sum(p[0].elapsed_time(p[1]) for p in edge) / (K * n)
        ms_step = edge[0][0].elapsed_time(edge[-1][2]) / K
        if check_stats() is None:
            return 4
        per_call = {"encode_ms_per_call": round(ms_call, 4),
                    "encode_gradient_GBps": round(4.0 * d / (ms_call * 1e-3) / 1e9, 2),
                    "encode_pct_hbm_peak_at_12d": round(100.0 * 12.0 * d / (ms_call * 1e-3) / 1e9
                                                        / HBM_PEAK_GBPS, 2),
                    "ms_per_step": round(ms_step, 4),
                    "value": round(n * 4.0 * d / (ms_step * 1e-3) / 1e9, 2), "unit": "GB/s"}

    # ---- outside the timed region: the master's fused update on the last
    #      step's messages (averaging and weight step in one call) ------------
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
    # ... and with momentum (a dense pass over weights and velocity)
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
        src = grads[0][0]
        for _ in range(args.copy_calibration):
            out.copy_(src)
        torch.cuda.synchronize()

    ms_per_step = total_ms / K
    fused_ms_avg = sum(fused_ms) / len(fused_ms)
    value = n * 4.0 * d / (ms_per_step * 1e-3) / 1e9
    launch_bytes = vectors_per_launch * 12 * d
    achieved = launch_bytes / (fused_ms_avg * 1e-3) / 1e9
    traffic = None
    if args.config == 3:
        traffic = (BATCH_KERNEL_TRAFFIC_BYTES if batched and n == wl.n_workers
                   else None if batched else SINGLE_KERNEL_TRAFFIC_BYTES)
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
                           + ", one stream"},
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
            "bytes_per_launch": launch_bytes,
            "vectors_per_launch": vectors_per_launch,
            "avg_launch_ms": round(fused_ms_avg, 5),
            "launches": len(fused_ms),
        },
    }
    del grads
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, max(1, min(args.cpu_sample, n)))
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
