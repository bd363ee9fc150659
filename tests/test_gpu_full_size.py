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
