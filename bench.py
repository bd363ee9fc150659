#!/usr/bin/env python3
"""Benchmark of the rTop-k hot path on one MI355X.

One *step* is one pass of the whole hot path over one batch of synthetic
input: n workers each run ``rtopk_encode`` (error-compensated rTop-k
sparsification of a fresh d-element gradient) and the master runs
``rtopk_aggregate`` on the n messages. The workload is the ResNet-50-sized
configuration (d = 25,557,032, r = 0.5% d, k = 0.1% d, n = 8 workers) that the
headline metric is quoted on. All gradients of the warm-up and timed steps are
resident in HBM before the clock starts.

By default everything runs on one stream, one kernel at a time. The n workers
of a step are independent (Algorithm 1 runs them on n nodes), so with
``--streams S`` their encodes are dealt to S HIP streams, each with its own
workspace; the kernel durations measured then include whatever ran beside them.
After the timed region the same steps are run once more on two streams and
reported as ``two_stream`` (a secondary figure; ``value`` is the one-stream one).

Prints ONE JSON line:
  value      = gradient bytes consumed per second over whole steps
               (n * 4d bytes per step / seconds per step), GB/s
  roofline   = the dominant kernel (fused residual add + candidate append):
               algorithmic bytes per launch (12 d) over its mean duration,
               measured with HIP events on the launch stream (one launch per
               step by default, see --trace-stride), against the 8 TB/s HBM peak
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
DOMINANT_KERNEL_TRAFFIC_BYTES = 309_655_484


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
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload configuration (1-5)")
    ap.add_argument("--workers", type=int, default=None, help="override the worker count")
    ap.add_argument("--streams", type=int, default=1,
                    help="HIP streams the simulated workers are dealt to (each with its own "
                         "workspace); 1 = strictly one kernel at a time")
    ap.add_argument("--trace-stride", type=int, default=0, metavar="N",
                    help="bracket every N-th launch of the dominant kernel with HIP events "
                         "(default: the number of workers, i.e. one launch per step, a "
                         "different worker each step; 1 = every launch). The two event "
                         "records cost the stream a few microseconds per traced launch.")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="after the timed region, also run N plain device copies of d floats "
                         "(4d bytes read + 4d bytes written each): a kernel of known HBM "
                         "traffic to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters with")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap-leg", action="store_true",
                    help="skip the extra two-stream pass that is reported as `two_stream`")
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
    S = max(1, min(args.streams, n))
    total_steps = K + W

    # ---- inputs: every gradient of every step resident in HBM ------------
    grads = [[torch.from_numpy(wl.gradient(w, t)).to(dev) for w in range(n)]
             for t in range(total_steps)]
    residual = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
    idx = torch.empty(n * k, dtype=torch.int32, device=dev)
    val = torch.empty(n * k, dtype=torch.float32, device=dev)
    out = torch.empty(d, dtype=torch.float32, device=dev)
    ws_bytes = rt.encode_workspace_bytes(d, r, k)
    ws = [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in range(S)]
    streams = [torch.cuda.Stream(device=dev) for _ in range(S)]     # default priority
    joined = [torch.cuda.Event() for _ in range(S)]
    released = torch.cuda.Event()
    torch.cuda.synchronize()

    def one_step(t: int, trace=None, phase=None):
        """n encodes dealt round-robin to the streams, then the master's
        average on stream 0 once every stream has finished its encodes; the
        next step's encodes start after the average (it reads the messages
        they overwrite)."""
        for s in range(1, S):
            streams[s].wait_event(released)
        if phase is not None:
            phase[0].record(streams[0])
        for w in range(n):
            s = w % S
            if trace is not None and trace[w] is not None:
                rt.trace_next_encode(rt.STAGES["fused"], *trace[w])
            rt.encode(grads[t][w], residual[w], r, k, philox_seed_for_worker(w), t,
                      idx[w * k:(w + 1) * k], val[w * k:(w + 1) * k], ws[s], streams[s])
        for s in range(1, S):
            joined[s].record(streams[s])
            streams[0].wait_event(joined[s])
        if phase is not None:
            phase[1].record(streams[0])
        rt.aggregate(idx, val, n, k, out, None, streams[0])
        if phase is not None:
            phase[2].record(streams[0])
        released.record(streams[0])

    released.record(streams[0])
    for t in range(W):
        one_step(t)
    torch.cuda.synchronize()

    # ---- timed region: K steps, events on the launch streams ---------------
    ev = HipEvents()
    stride = args.trace_stride if args.trace_stride > 0 else n
    offset = 0 if stride == 1 else 1             # n | stride would always pick worker 0
    fused_pairs = [[(ev.new(), ev.new()) if (s_ * (n + offset) + w) % stride == 0 else None
                    for w in range(n)] for s_ in range(K)]
    phase = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(K)]
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    for s_ in range(K):
        one_step(W + s_, trace=fused_pairs[s_], phase=phase[s_])
    torch.cuda.synchronize()
    t_wall1 = time.perf_counter()
    total_ms = phase[0][0].elapsed_time(phase[-1][2])
    enc_ms_call = sum(p[0].elapsed_time(p[1]) for p in phase) / (K * n)
    agg_ms_call = sum(p[1].elapsed_time(p[2]) for p in phase) / K
    fused_ms = [ev.elapsed_ms(*pair) for row in fused_pairs for pair in row if pair is not None]
    ev.close()

    # ---- outside the timed region: the same K steps once more with the
    #      workers dealt to two streams, no launch bracketed (the n encodes of
    #      a step are independent; the short kernels of one overlap the
    #      streaming kernel of the next). Reported beside the headline only. ---
    overlap = None
    if S == 1 and n > 1 and not args.no_overlap_leg:
        S2 = 2
        streams2 = [streams[0], torch.cuda.Stream(device=dev)]
        ws2 = [ws[0], torch.empty(ws_bytes, dtype=torch.uint8, device=dev)]
        joined2, released2 = torch.cuda.Event(), torch.cuda.Event()
        edge = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))

        def overlapped_step(t: int, step_no: int):
            streams2[1].wait_event(released2)
            for w in range(n):
                s = w % S2
                # the gradients of step t again, on top of the residuals as they are now,
                # under a step number not used before (fresh sampling keys: keys that
                # already decided what left these residuals would not be independent
                # of the top-r set any more)
                rt.encode(grads[t][w], residual[w], r, k, philox_seed_for_worker(w),
                          step_no, idx[w * k:(w + 1) * k], val[w * k:(w + 1) * k],
                          ws2[s], streams2[s])
            joined2.record(streams2[1])
            streams2[0].wait_event(joined2)
            rt.aggregate(idx, val, n, k, out, None, streams2[0])
            released2.record(streams2[0])

        released2.record(streams2[0])
        overlapped_step(W, total_steps)               # warm-up of the second workspace
        edge[0].record(streams2[0])
        for s_ in range(K):
            overlapped_step(W + s_, total_steps + 1 + s_)
        edge[1].record(streams2[0])
        torch.cuda.synchronize()
        ms2 = edge[0].elapsed_time(edge[1]) / K
        overlap = {"streams": S2, "ms_per_step": round(ms2, 4),
                   "value": round(n * 4.0 * d / (ms2 * 1e-3) / 1e9, 2), "unit": "GB/s"}
        for w_ in ws2:
            st2 = rt.encode_stats(w_)
            if st2["error_flags"] != 0:
                print(f"bench.py: encode reported error flags {st2}", file=sys.stderr)
                return 4
        overlap["last_encode_path"] = st2["path"]
        del ws2

    # ---- outside the timed region: the master's fused update on the last
    #      step's messages (averaging and weight step in one call) ------------
    upd_ws = torch.empty(rt.aggregate_update_workspace_bytes(d, n, k), dtype=torch.uint8,
                         device=dev)
    omegas = [torch.randn(d, dtype=torch.float32, device=dev) for _ in range(4)]
    upd = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    upd_calls = 5 * len(omegas)
    with torch.cuda.stream(streams[0]):
        for om in omegas:
            rt.aggregate_update(idx, val, n, k, 0.1, r / k, om, upd_ws, streams[0])
        upd[0].record(streams[0])
        for c in range(upd_calls):
            rt.aggregate_update(idx, val, n, k, 0.1, r / k, omegas[c % len(omegas)], upd_ws,
                                streams[0])
        upd[1].record(streams[0])
    torch.cuda.synchronize()
    upd_ms_call = upd[0].elapsed_time(upd[1]) / upd_calls
    del omegas

    if args.copy_calibration > 0:
        src = grads[0][0]
        for _ in range(args.copy_calibration):
            out.copy_(src)
        torch.cuda.synchronize()

    for s in range(S):
        stats = rt.encode_stats(ws[s])
        if stats["error_flags"] != 0:
            print(f"bench.py: encode reported error flags {stats}", file=sys.stderr)
            return 4

    ms_per_step = total_ms / K
    fused_ms_avg = sum(fused_ms) / len(fused_ms)
    value = n * 4.0 * d / (ms_per_step * 1e-3) / 1e9
    achieved = 12.0 * d / (fused_ms_avg * 1e-3) / 1e9
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
                   "streams": S,
                   "step": f"{n} x rtopk_encode on {S} stream(s) + 1 x rtopk_aggregate"},
        "encode_gradient_GBps": round(4.0 * d / (enc_ms_call * 1e-3) / 1e9, 2),
        "encode_ms_per_call": round(enc_ms_call, 4),
        "encode_pct_hbm_peak_at_12d": round(100.0 * 12.0 * d / (enc_ms_call * 1e-3) / 1e9
                                            / HBM_PEAK_GBPS, 2),
        "aggregate_GBps": round(4.0 * d / (agg_ms_call * 1e-3) / 1e9, 2),
        "aggregate_ms_per_call": round(agg_ms_call, 4),
        "aggregate_update_ms_per_call": round(upd_ms_call, 4),
        "two_stream": overlap,
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
            "traffic": DOMINANT_KERNEL_TRAFFIC_BYTES if args.config == 3 else None,
            "bytes_per_launch": 12 * d,
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
