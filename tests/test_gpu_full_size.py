"""GPU parity at the benchmark's full sizes, in the launch configuration the
benchmark times (same entry points, same workspace sizing)."""
import numpy as np
import pytest

import oracle
from workloads import Workload, philox_seed_for_worker

pytestmark = pytest.mark.gpu


def _u():
    from tests import gpu_util
    return gpu_util


def test_full_size_cfg1_five_steps_bit_exact():
    """Workload 1 as stated: one worker, five steps with error feedback."""
    u = _u()
    wl = Workload(1)
    d, r, k = wl.d, wl.r, wl.k
    gw = u.GpuWorker(d, r, k)
    res = np.zeros(d, np.float32)
    seed = philox_seed_for_worker(0)
    for t in range(wl.steps):
        g = wl.gradient(0, t)
        print(f"cfg1 d={d} step={t}", flush=True)
        got = gw.encode(g, seed, t)
        oi, ov, res = oracle.encode(g, res, r, k, seed, t)
        u.assert_encode_equal(got, (oi, ov, res), f"cfg1 t={t}")
        assert gw.stats["path"] == 0
        out = u.gpu_aggregate(oi, ov, 1, d)
        assert np.array_equal(u.bits(out), u.bits(oracle.aggregate_f32(oi, ov, 1, d)))


class _Batch:
    """Device state of the n workers of one configuration, stepped with one
    rtopk_encode_batch call per step exactly as bench.py launches it (one
    workspace slice per worker, messages back to back), then rtopk_aggregate."""

    def __init__(self, u, d, r, k, n, keep_previous_residual=False):
        import torch
        self.u, self.rt, self.torch = u, u.rt, torch
        self.d, self.r, self.k, self.n = d, r, k, n
        dev = u.DEV
        self.stride = self.rt.encode_workspace_bytes(d, r, k)
        self.ws = torch.empty(n * self.stride, dtype=torch.uint8, device=dev)
        self.resid = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
        self.prev = ([torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
                     if keep_previous_residual else None)
        self.idx = torch.empty(n * k, dtype=torch.int32, device=dev)
        self.val = torch.empty(n * k, dtype=torch.float32, device=dev)
        self.out_i = [self.idx[w * k:(w + 1) * k] for w in range(n)]
        self.out_v = [self.val[w * k:(w + 1) * k] for w in range(n)]
        self.seeds = [philox_seed_for_worker(w) for w in range(n)]
        self.out = torch.empty(d, dtype=torch.float32, device=dev)

    def step(self, grads, t):
        """grads: the n workers' gradients of step t, on the device."""
        if self.prev is not None:
            for w in range(self.n):
                self.prev[w].copy_(self.resid[w])
        self.rt.encode_batch(grads, self.resid, self.r, self.k, self.seeds, t, self.out_i,
                             self.out_v, self.ws)
        self.rt.aggregate(self.idx, self.val, self.n, self.k, self.out)
        self.torch.cuda.synchronize()

    def stats(self, w):
        st = self.rt.encode_stats(self.ws[w * self.stride:(w + 1) * self.stride])
        assert st["error_flags"] == 0, (w, st)
        return st

    def message(self, w):
        return (self.out_i[w].cpu().numpy().view(np.uint32), self.out_v[w].cpu().numpy(),
                self.resid[w].cpu().numpy())

    def check_aggregate_bits(self):
        """The dense average the device just formed against the oracle's binary32
        worker-order variant of the device's messages."""
        ai, av = self.idx.cpu().numpy().view(np.uint32), self.val.cpu().numpy()
        got = self.out.cpu().numpy()
        assert np.array_equal(self.u.bits(got),
                              self.u.bits(oracle.aggregate_f32(ai, av, self.n, self.d)))
        return ai, av, got

    def check_properties(self, w, grad, t):
        """What Definitions 1 and 3 and Algorithm 1 fix at any size, checked on
        the device with plain torch reductions for worker w after step t
        (needs keep_previous_residual): the message has k strictly ascending
        indices and carries a = g + m at those indices, the residual is a with
        exactly those positions cleared, the reported threshold is the r-th
        largest magnitude and every sent coordinate lies at or above it."""
        torch = self.torch
        st = self.stats(w)
        idx = self.out_i[w].to(torch.int64) & 0xFFFFFFFF
        assert bool((idx[1:] > idx[:-1]).all()) and int(idx[-1]) < self.d
        a = grad + self.prev[w]                                   # one binary32 add per coordinate
        assert torch.equal(self.out_v[w].view(torch.int32), a[idx].view(torch.int32))
        mag = a.view(torch.int32) & 0x7FFFFFFF
        T = st["threshold_bits"]
        c_gt = int((mag > T).sum())
        c_ge = c_gt + int((mag == T).sum())
        assert c_gt == st["count_greater"] and c_gt < self.r <= c_ge, (w, t, c_gt, c_ge, st)
        assert st["count_greater"] + st["ties_taken"] == self.r
        sent_mag = mag[idx]
        assert bool((sent_mag >= T).all())
        assert int((sent_mag == T).sum()) <= st["ties_taken"]
        a[idx] = 0.0                                              # finite a - a = +0
        assert torch.equal(a.view(torch.int32), self.resid[w].view(torch.int32)), (w, t)
        del a, mag


@pytest.mark.parametrize("cfg,follow", [(2, 3), (3, 5), (4, 2)])
def test_full_size_configs_as_stated_batched_all_steps(cfg, follow, progress):
    """Workloads 2, 3 and 4 as stated: all workers (8, 8, 4) in one
    rtopk_encode_batch per step for all ten steps with error feedback, each
    step followed by rtopk_aggregate at that n. Against the oracle: every
    worker at step 0, worker `follow` through all ten steps (its oracle run
    carries its own residual and overlaps the device work), and the dense
    average of every step bit for bit against the binary32 worker-order sum
    of the device's messages (1e-6 against the binary64 mean at the last step)."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    u = _u()
    wl = Workload(cfg)
    d, r, k, n, steps = wl.d, wl.r, wl.k, wl.n_workers, wl.steps
    b = _Batch(u, d, r, k, n)
    ref_m = np.zeros(d, np.float32)
    pool = ThreadPoolExecutor(max_workers=max(2, n))
    for t in range(steps):
        progress(f"cfg{cfg} d={d} n={n} step {t}: inputs")
        host = {}
        grads = []
        for w in range(n):
            g = wl.gradient(w, t)
            if w == follow or t == 0:
                host[w] = g
            grads.append(torch.from_numpy(g).to(u.DEV))
        # the oracle steps run on the host cores while the device works
        chain = pool.submit(oracle.encode, host[follow], ref_m, r, k, b.seeds[follow], t)
        others = {w: pool.submit(oracle.encode, host[w], np.zeros(d, np.float32), r, k,
                                 b.seeds[w], 0) for w in host if w != follow}
        progress(f"cfg{cfg} step {t}: gpu")
        b.step(grads, t)
        for w in range(n):
            st = b.stats(w)
            assert st["path"] == 0, (w, t, st)
        got = {w: b.message(w) for w in host}
        ai, av, dense = b.check_aggregate_bits()
        if t == steps - 1:
            u.assert_aggregate_close(dense, ai, av, n, d, oracle.aggregate(ai, av, n, d))
        progress(f"cfg{cfg} step {t}: oracle")
        oi, ov, ref_m = chain.result()
        u.assert_encode_equal(got[follow], (oi, ov, ref_m), f"cfg{cfg} worker {follow} step {t}")
        for w, fut in others.items():
            u.assert_encode_equal(got[w], fut.result(), f"cfg{cfg} worker {w} step 0")
        del grads, host, got
    pool.shutdown()


def test_stress_sweep_as_stated_nine_points_sixteen_workers(progress):
    """Workload 5 as stated: d = 2^28, k/d in {0.01, 0.1, 1}% x r/k in {2, 5, 10},
    16 workers encoded in ONE rtopk_encode_batch per step and then aggregated
    (rtopk_aggregate at n = 16), 3 steps per sweep point from a zero residual.
    Against the oracle: one worker per sweep point (a different one each)
    over all three steps, so that its later steps run on a fed-back
    residual; the nine oracle chains run side by side on the host cores while
    the device works. All sixteen workers of every step are checked on the
    device by the properties the definitions fix at any size; the dense
    average of the last step of every point bit for bit against the binary32
    worker-order sum of the device's messages."""
    import queue
    import torch
    from concurrent.futures import ThreadPoolExecutor, wait, FIRST_COMPLETED
    from workloads.gradients import STRESS_K_FRACS, STRESS_R_OVER_K
    u = _u()
    wl = Workload(5)
    d, n, steps, oracle_steps = wl.d, wl.n_workers, wl.steps, wl.steps
    points = []
    for num, den in STRESS_K_FRACS:
        for ratio in STRESS_R_OVER_K:
            k = (d * num + den - 1) // den
            points.append((ratio * k, k))
    follow = [(5 * p + 1) % n for p in range(len(points))]       # 1, 6, 11, 0, 5, 10, 15, 4, 9
    pool = ThreadPoolExecutor(max_workers=len(points))
    host = {}
    done = queue.Queue()                  # the oracle threads' step reports, printed by this thread

    def report():
        while not done.empty():
            progress(done.get())

    def chain(p):
        r, k = points[p]
        w = follow[p]
        m = np.zeros(d, np.float32)
        outs = []
        for t in range(oracle_steps):
            oi, ov, m = oracle.encode(host[(w, t)], m, r, k, philox_seed_for_worker(w), t)
            outs.append((oi, ov, m))
            done.put(f"stress point {p} (r={r} k={k}): oracle step {t} of worker {w} done")
        return outs

    # inputs: the gradient of (worker, step) is the same for every sweep point;
    # all 48 stay on the device, the followed workers' also on the host
    progress(f"stress d={d}: inputs for the oracle chains")
    for t in range(oracle_steps):
        for w in sorted(set(follow)):
            host[(w, t)] = wl.gradient(w, t)
    chains = [pool.submit(chain, p) for p in range(len(points))]
    dev_g = {}
    for t in range(steps):
        for w in range(n):
            g = host[(w, t)] if (w, t) in host else wl.gradient(w, t)
            dev_g[(w, t)] = torch.from_numpy(g).to(u.DEV)
            if w % 4 == 3:
                progress(f"stress: inputs of step {t}, workers up to {w}, on the device")
                report()
    got = {}
    for p, (r, k) in enumerate(points):
        b = _Batch(u, d, r, k, n, keep_previous_residual=True)
        for t in range(steps):
            progress(f"stress point {p} (r={r} k={k}) step {t}: gpu")
            report()
            grads = [dev_g[(w, t)] for w in range(n)]
            b.step(grads, t)
            for w in range(n):
                b.check_properties(w, grads[w], t)
            if t < oracle_steps:
                got[(p, t)] = b.message(follow[p])
        b.check_aggregate_bits()
        del b
        torch.cuda.empty_cache()
    del dev_g
    # what is left of the oracle chains: every finished step is reported as it comes
    left = set(chains)
    while left:
        finished, left = wait(left, timeout=20, return_when=FIRST_COMPLETED)
        report()
    for p in range(len(points)):
        outs = chains[p].result()
        for t in range(oracle_steps):
            u.assert_encode_equal(got[(p, t)], outs[t],
                                  f"stress point {p} worker {follow[p]} step {t}")
    pool.shutdown()


def test_full_size_run_of_equal_magnitudes_at_the_threshold():
    """cfg3's sizes, but the vector is a frozen tensor's (all zeros) and then a
    ternary one: the threshold lies in a run of millions of equal magnitudes.
    Bit-exact against the oracle, over two steps with error feedback, and
    resolved from the per-chunk counts (path bit 2), not by the slow selection."""
    u = _u()
    wl = Workload(3)
    d, r, k = wl.d, wl.r, wl.k
    rng = np.random.default_rng(17)
    for name, g in (("zeros", np.zeros(d, np.float32)),
                    ("ternary", rng.integers(-1, 2, d).astype(np.float32))):
        w = u.GpuWorker(d, r, k)
        res = np.zeros(d, np.float32)
        for t in range(2):
            print(f"{name} d={d} step={t}", flush=True)
            got = w.encode(g, 5, t)
            oi, ov, res = oracle.encode(g, res, r, k, 5, t)
            u.assert_encode_equal(got, (oi, ov, res), f"{name} t={t}")
            assert w.stats["path"] == 4 and w.stats["error_flags"] == 0, w.stats
        del w


def test_periodic_vector_does_not_mislead_the_sampled_estimate():
    """d = 2^24 with a period close to the length of the sampling strata (1024
    elements): the sample's offsets inside the strata are hashed from (stratum,
    seed, step), so a periodic layout is sampled fairly: the ordinary path
    decides (path 0) for every worker and step, and the message is the oracle's."""
    u = _u()
    d = 1 << 24
    r, k = 100_000, 10_000
    i = np.arange(d, dtype=np.float64)
    g = (np.sin(i * (2 * np.pi / 1024.0)) ** 9 + 0.05 * np.sin(i * (2 * np.pi / 37.0))).astype(np.float32)
    for seed in (1, 2):
        w = u.GpuWorker(d, r, k)
        res = np.zeros(d, np.float32)
        for t in range(2):
            print(f"periodic d={d} seed={seed} step={t}", flush=True)
            got = w.encode(g, seed, t)
            oi, ov, res = oracle.encode(g, res, r, k, seed, t)
            u.assert_encode_equal(got, (oi, ov, res), f"periodic seed {seed} step {t}")
            assert w.stats["path"] == 0, w.stats
        del w


def test_largest_vector_the_index_type_allows():
    """d = 2^32 - 1, the largest length a 32-bit index addresses (chunks of
    131072 elements, 51 GB streamed). Inputs are drawn on the device; what the
    definition fixes is checked with plain torch reductions over the whole
    vector, and the k-subset itself with the oracle's Philox keys of the r
    members: the threshold is the r-th largest magnitude, the message is the k
    members with the smallest (key, index) in index order with the values of
    a = g + m, and the residual is a with exactly those k positions cleared.
    The aggregate of that one message (n = 1) is the message scattered."""
    import torch
    import paper_2005_10761_amd as rt
    u = _u()
    dev = u.DEV
    d = 2 ** 32 - 1
    r, k = 200_000, 20_000
    seed, step = 0x9E3779B97F4A7C15, 2 ** 40 + 7
    gen = torch.Generator(device=dev)
    gen.manual_seed(2005_10761)
    print(f"largest d={d}: inputs", flush=True)
    g = torch.randn(d, device=dev, generator=gen)
    g.mul_(g.abs()).mul_(1e-3)                               # heavier tail than a normal
    m = torch.randn(d, device=dev, generator=gen).mul_(1e-3)
    a = g + m                                                # one binary32 add per coordinate
    ws = torch.empty(rt.encode_workspace_bytes(d, r, k), dtype=torch.uint8, device=dev)
    oi = torch.empty(k, dtype=torch.int32, device=dev)
    ov = torch.empty(k, dtype=torch.float32, device=dev)
    print("largest: encode", flush=True)
    rt.encode(g, m, r, k, seed, step, oi, ov, ws)
    torch.cuda.synchronize()
    st = rt.encode_stats(ws)
    assert st["error_flags"] == 0 and st["path"] == 0, st
    del ws, g
    idx = oi.to(torch.int64) & 0xFFFFFFFF
    assert bool((idx[1:] > idx[:-1]).all()) and int(idx[-1]) < d
    assert torch.equal(ov.view(torch.int32), a[idx].view(torch.int32))

    print("largest: threshold and members", flush=True)
    T = st["threshold_bits"]
    piece = 2 ** 30
    c_gt = c_ge = 0
    above, ties = [], []
    for lo in range(0, d, piece):
        mag = a[lo:lo + piece].view(torch.int32) & 0x7FFFFFFF
        gt, eq = mag > T, mag == T
        c_gt += int(gt.sum())
        c_ge += int(gt.sum()) + int(eq.sum())
        above.append(torch.nonzero(gt).flatten() + lo)
        ties.append(torch.nonzero(eq).flatten() + lo)
        del mag, gt, eq
    assert c_gt == st["count_greater"] and c_gt < r <= c_ge, (c_gt, c_ge, st)
    members = torch.cat(above + [torch.cat(ties)[:r - c_gt]]).cpu().numpy()
    assert members.size == r
    keys = np.array([oracle.key64(seed, step, int(i)) for i in members], dtype=np.uint64)
    order = np.lexsort((members, keys))
    want_idx = np.sort(members[order[:k]])
    assert np.array_equal(idx.cpu().numpy(), want_idx)

    print("largest: residual", flush=True)
    a[idx] = 0.0                                             # a - a = +0 for the finite values sent
    for lo in range(0, d, piece):
        assert torch.equal(a[lo:lo + piece].view(torch.int32), m[lo:lo + piece].view(torch.int32)), lo
    del a

    print("largest: aggregate of the one message", flush=True)
    rt.aggregate(oi, ov, 1, k, m)                            # m reused as the dense output
    torch.cuda.synchronize()
    assert torch.equal(m[idx].view(torch.int32), ov.view(torch.int32))
    m[idx] = 0.0
    for lo in range(0, d, piece):
        assert int(torch.count_nonzero(m[lo:lo + piece].view(torch.int32))) == 0, lo
