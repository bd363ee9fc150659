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


@pytest.mark.parametrize("cfg,n_workers,steps", [(1, 1, 5), (2, 2, 2), (3, 2, 2), (4, 1, 2)])
def test_full_size_configs_bit_exact(cfg, n_workers, steps):
    u = _u()
    wl = Workload(cfg)
    d, r, k = wl.d, wl.r, wl.k
    gw = [u.GpuWorker(d, r, k) for _ in range(n_workers)]
    res = [np.zeros(d, np.float32) for _ in range(n_workers)]
    for t in range(steps):
        mi, mv = [], []
        for w in range(n_workers):
            g = wl.gradient(w, t)
            seed = philox_seed_for_worker(w)
            print(f"cfg{cfg} d={d} worker={w} step={t}", flush=True)
            got = gw[w].encode(g, seed, t)
            oi, ov, res[w] = oracle.encode(g, res[w], r, k, seed, t)
            u.assert_encode_equal(got, (oi, ov, res[w]), f"cfg{cfg} w={w} t={t}")
            assert gw[w].stats["path"] == 0
            mi.append(oi)
            mv.append(ov)
        ai, av = np.concatenate(mi), np.concatenate(mv)
        out = u.gpu_aggregate(ai, av, n_workers, d)
        u.assert_aggregate_close(out, ai, av, n_workers, d, oracle.aggregate(ai, av, n_workers, d))
        assert np.array_equal(u.bits(out), u.bits(oracle.aggregate_f32(ai, av, n_workers, d)))


def test_stress_size_properties_and_one_oracle_call():
    """d = 2^28: one full oracle comparison (k = 0.1% d, r = 5k), then the
    properties that hold at any size for a second sweep point."""
    u = _u()
    wl = Workload(5)
    d = wl.d
    k = (d + 999) // 1000
    r = 5 * k
    g = wl.gradient(0, 0)
    print(f"stress d={d} r={r} k={k}: gpu", flush=True)
    w = u.GpuWorker(d, r, k)
    got = w.encode(g, 42, 0)
    print("stress: oracle", flush=True)
    want = oracle.encode(g, np.zeros(d, np.float32), r, k, 42, 0)
    u.assert_encode_equal(got, want, "stress")
    del w
    # second sweep point, properties only: k = 1% d, r = 10k
    k2 = (d + 99) // 100
    r2 = 10 * k2
    print(f"stress d={d} r={r2} k={k2}: gpu, properties", flush=True)
    w2 = u.GpuWorker(d, r2, k2)
    gi, gv, gm = w2.encode(g, 43, 1)
    st = w2.stats
    assert gi.size == k2 and np.all(np.diff(gi.astype(np.int64)) > 0)
    assert np.array_equal(u.bits(gv), u.bits(g[gi]))
    mag = u.bits(g) & 0x7FFFFFFF
    assert np.all(mag[gi] >= st["threshold_bits"])
    assert int((mag > st["threshold_bits"]).sum()) == st["count_greater"]
    assert st["count_greater"] + st["ties_taken"] == r2
    sent = np.zeros(d, bool)
    sent[gi] = True
    assert np.all(u.bits(gm[sent]) == 0)
    assert np.array_equal(u.bits(gm[~sent]), u.bits(g[~sent]))


@pytest.mark.parametrize("cfg,second_step_members", [(2, (0, 3, 7)), (3, (1, 6))])
def test_full_size_batched_step_as_the_benchmark_launches_it(cfg, second_step_members):
    """One rtopk_encode_batch over the workload's 8 workers (workspace slices,
    messages back to back, then rtopk_aggregate), as bench.py's timed step does
    it: every member of step 0 against the oracle, some members of step 1."""
    import torch
    u = _u()
    rt = u.rt
    wl = Workload(cfg)
    d, r, k, n = wl.d, wl.r, wl.k, wl.n_workers
    dev = u.DEV
    stride = rt.encode_workspace_bytes(d, r, k)
    ws = torch.empty(n * stride, dtype=torch.uint8, device=dev)
    grads = [torch.empty(d, dtype=torch.float32, device=dev) for _ in range(n)]
    resid = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
    idx = torch.empty(n * k, dtype=torch.int32, device=dev)
    val = torch.empty(n * k, dtype=torch.float32, device=dev)
    out_i = [idx[w * k:(w + 1) * k] for w in range(n)]
    out_v = [val[w * k:(w + 1) * k] for w in range(n)]
    seeds = [philox_seed_for_worker(w) for w in range(n)]
    ref_m = [np.zeros(d, np.float32) for _ in range(n)]
    for t, members in ((0, tuple(range(n))), (1, second_step_members)):
        gs = {}
        for w in range(n):
            g = wl.gradient(w, t)
            grads[w].copy_(torch.from_numpy(g))
            if w in members:
                gs[w] = g
        print(f"cfg{cfg} batched step {t}: gpu", flush=True)
        rt.encode_batch(grads, resid, r, k, seeds, t, out_i, out_v, ws)
        torch.cuda.synchronize()
        for w in members:
            print(f"cfg{cfg} batched step {t}: oracle, worker {w}", flush=True)
            st = rt.encode_stats(ws[w * stride:(w + 1) * stride])
            assert st["error_flags"] == 0 and st["path"] == 0, (w, st)
            oi, ov, ref_m[w] = oracle.encode(gs[w], ref_m[w], r, k, seeds[w], t)
            got = (out_i[w].cpu().numpy().view(np.uint32), out_v[w].cpu().numpy(),
                   resid[w].cpu().numpy())
            u.assert_encode_equal(got, (oi, ov, ref_m[w]), f"cfg{cfg} member {w} step {t}")
        out = torch.empty(d, dtype=torch.float32, device=dev)
        rt.aggregate(idx, val, n, k, out)
        torch.cuda.synchronize()
        ai, av = idx.cpu().numpy().view(np.uint32), val.cpu().numpy()
        assert np.array_equal(u.bits(out.cpu().numpy()), u.bits(oracle.aggregate_f32(ai, av, n, d)))


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
