"""GPU parity: the HIP path (through the C ABI) against the CPU oracle.

Bar: indices, sent values and residual bit-exact; the aggregated average
within 1e-6 relative of the oracle's binary64 mean (tolerance stated in
``gpu_util.assert_aggregate_close``) and bit-exact against the oracle's
binary32 worker-order variant.
"""
import numpy as np
import pytest

import oracle
from workloads import Workload, philox_seed_for_worker

pytestmark = pytest.mark.gpu


def _u():
    from tests import gpu_util
    return gpu_util


def _check(g, m, r, k, seed, step, offset=0, what=""):
    u = _u()
    got = u.gpu_encode_once(g, m, r, k, seed, step, offset=offset)
    want = oracle.encode(g, m, r, k, seed, step)
    u.assert_encode_equal(got, want, what or f"d={len(g)} r={r} k={k}")
    return got[3]


# --------------------------------------------------------------------------
# small adversarial inputs
# --------------------------------------------------------------------------
def test_tiny_sizes_every_r_k():
    rng = np.random.default_rng(1)
    alphabet = np.array([0.0, -0.0, 1.0, -1.0, 2.0, 0.5, 1e-45, -1e-45, 3.5], np.float32)
    for d in (1, 2, 3, 5, 7):
        g = alphabet[rng.integers(0, alphabet.size, d)]
        m = alphabet[rng.integers(0, alphabet.size, d)]
        for r in range(1, d + 1):
            for k in range(1, r + 1):
                _check(g, m, r, k, 42 + r, k)


@pytest.mark.parametrize("d", [63, 64, 255, 257, 4095, 4096, 4097, 3 * 4096 + 17, 100_003])
@pytest.mark.parametrize("offset", [0, 1])
def test_random_values_ragged_sizes_and_misaligned_pointers(d, offset):
    rng = np.random.default_rng(d)
    g = (rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 0, d)).astype(np.float32)
    m = (rng.standard_normal(d) * 1e-2).astype(np.float32)
    r = max(1, d // 50)
    k = max(1, r // 7)
    st = _check(g, m, r, k, 7, 3, offset=offset)
    assert st["count_greater"] + st["ties_taken"] == r


def test_degenerate_value_patterns():
    rng = np.random.default_rng(3)
    d = 20_000
    cases = {
        "all_equal": np.full(d, 0.75, np.float32),
        "all_zero": np.zeros(d, np.float32),
        "signed_zero_mix": np.where(rng.random(d) < 0.5, 0.0, -0.0).astype(np.float32),
        "denormals": (rng.integers(1, 50, d) * np.float32(1e-45) *
                      rng.choice([-1, 1], d)).astype(np.float32),
        "two_levels": rng.choice([1.0, -1.0, 2.0], d).astype(np.float32),
        "mostly_zero": np.where(rng.random(d) < 0.001, rng.standard_normal(d), 0.0).astype(np.float32),
    }
    for name, g in cases.items():
        m = np.zeros(d, np.float32)
        for r, k in ((200, 20), (d // 2, 1), (d, d // 3), (1, 1), (d, d), (777, 777)):
            _check(g, m, r, k, 11, 2, what=f"{name} r={r} k={k}")


def test_ties_straddling_the_threshold_take_lowest_indices():
    d = 50_000
    rng = np.random.default_rng(4)
    g = rng.standard_normal(d).astype(np.float32) * 0.1
    tie_pos = rng.choice(d, 3000, replace=False)
    g[tie_pos] = np.where(rng.random(3000) < 0.5, 5.0, -5.0)     # 3000 ties on top
    big = rng.choice(np.setdiff1d(np.arange(d), tie_pos), 100, replace=False)
    g[big] = 9.0 + rng.random(100).astype(np.float32)
    m = np.zeros(d, np.float32)
    st = _check(g, m, 1100, 1100, 1, 1)          # r = k: the selection itself is visible
    assert st["count_greater"] == 100 and st["ties_taken"] == 1000
    _check(g, m, 1100, 300, 1, 1)


def test_long_run_of_equal_magnitudes_at_the_threshold():
    """The threshold lies in a run of equal magnitudes far longer than the short
    list of the deciding bin: the last member is found from per-chunk counts
    (path bit 2), not by the slow selection over all candidates (bit 0)."""
    d = 300_000
    g = np.full(d, -2.5, np.float32)
    g[::1000] = 3.0
    m = np.zeros(d, np.float32)
    st = _check(g, m, 5000, 500, 9, 9)
    assert st["path"] == 4 and st["count_greater"] == 300 and st["ties_taken"] == 4700
    st = _check(np.zeros(d, np.float32), m, 1000, 10, 9, 9)
    assert st["path"] == 4
    rng = np.random.default_rng(31)
    for case, (g, r, k) in enumerate((
            (rng.integers(-1, 2, d).astype(np.float32), 9_000, 900),            # ternary
            ((rng.integers(0, 2, d) * 2 - 1).astype(np.float32) * 0.125, d // 2, d // 8),  # signs
            (np.where(rng.random(d) < 0.01, rng.standard_normal(d), 0.0).astype(np.float32),
             10_000, 2_500),                                                     # fewer nonzeros than r
            (np.round(rng.standard_normal(d) * 1.5).astype(np.float32), 30_000, 30_000),  # few levels, r = k
            (np.round(rng.standard_normal(d) * 1.5).astype(np.float32), 250_000, 1),
    )):
        st = _check(g, np.zeros(d, np.float32), r, k, 77, case)
        assert st["path"] == 4, (case, st)
    # error feedback on top: the residual of step 0 moves the run's members out of the run
    g = np.full(d, 0.5, np.float32)
    m = np.zeros(d, np.float32)
    for t in range(3):
        want = oracle.encode(g, m, 2_000, 400, 5, t)
        got = _u().gpu_encode_once(g, m, 2_000, 400, 5, t)
        _u().assert_encode_equal(got, want, f"t={t}")
        assert got[3]["path"] == 4, (t, got[3])
        m = want[2]
    # the run ends in the very last chunk, and in the very first entry
    g = np.zeros(d, np.float32)
    st = _check(g, m * 0, d - 1, 7, 3, 3)
    assert st["path"] == 4 and st["ties_taken"] == d - 1
    st = _check(g, m * 0, 1, 1, 3, 3)
    assert st["ties_taken"] == 1


def test_seeded_sweep_of_tie_heavy_vectors():
    """Eighty seeded cases of vectors that are mostly ties (a few levels, sparse,
    quantised, constant with outliers, piecewise constant, signs of one or two
    neighbouring magnitudes) with every kind of (r, k): all paths, bit-exact."""
    rng = np.random.default_rng(20051076)
    paths = set()
    for case in range(80):
        d = int(rng.choice([30_000, 65_536, 100_003, 262_144]))
        kind = case % 6
        if kind == 0:
            nl = int(rng.integers(1, 7))
            lv = rng.choice([0.0, 0.5, 1.0, -1.0, 2.0, 3.0, -0.25, 1e-30, 1e-40], nl, replace=False)
            g = rng.choice(lv, d, p=rng.dirichlet(np.ones(nl) * 0.7))
        elif kind == 1:
            g = np.where(rng.random(d) < 10.0 ** rng.uniform(-4, -0.5), rng.standard_normal(d), 0.0)
        elif kind == 2:
            q = 10.0 ** rng.uniform(-0.5, 1.0)
            g = np.round(rng.standard_normal(d) * q) / q
        elif kind == 3:
            g = np.full(d, rng.choice([0.0, 0.75, -3.0]))
            sel = rng.random(d) < 10.0 ** rng.uniform(-5, -2)
            g[sel] = rng.standard_normal(int(sel.sum())) * 10
        elif kind == 4:
            cuts = np.sort(rng.integers(0, d, int(rng.integers(2, 40))))
            g = np.zeros(d)
            for a, b in zip(np.r_[0, cuts], np.r_[cuts, d]):
                g[a:b] = rng.choice([0.0, 1.0, -1.0, 0.5, 2.0])
        else:
            g = (rng.integers(0, 2, d) * 2 - 1) * rng.choice(
                [1.0, 1.0 + 2.0 ** -23], d, p=[0.9, 0.1] if case % 2 else [1.0, 0.0])
        g = g.astype(np.float32)
        m = np.zeros(d, np.float32) if case % 3 else rng.choice([0.0, 0.5, -0.5], d).astype(np.float32)
        mode = (case // 6) % 6
        if mode == 0:
            r = int(rng.integers(1, d + 1)); k = int(rng.integers(1, r + 1))
        elif mode == 1:
            r = max(1, d // 200); k = max(1, r // 5)
        elif mode == 2:
            r = int(rng.integers(1, d + 1)); k = r
        elif mode == 3:
            r = d - int(rng.integers(0, 3)); k = int(rng.integers(1, r + 1))
        elif mode == 4:
            r = int(rng.integers(1, 2000)); k = int(rng.integers(1, r + 1))
        else:
            r = max(1, d // 10); k = max(1, r // 10)
        st = _check(g, m, r, k, int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 2 ** 40)),
                    what=f"case {case} d={d} kind={kind} mode={mode} r={r} k={k}")
        paths.add(st["path"])
    assert {0, 4} <= paths, paths


def test_crowded_deciding_bin_with_two_magnitudes_takes_the_slow_selection():
    """Two neighbouring patterns share the deciding bin and fill it beyond the
    short list: no run of equal magnitudes, the exact selection over all
    candidates decides (path bit 0)."""
    d = 200_000
    rng = np.random.default_rng(8)
    one = np.float32(1.0)
    g = np.where(rng.random(d) < 0.5, one, np.nextafter(one, np.float32(2.0))).astype(np.float32)
    g *= rng.choice(np.array([-1.0, 1.0], np.float32), d)
    st = _check(g, np.zeros(d, np.float32), 120_000, 20_000, 4, 4)
    assert st["path"] & 1 and not st["path"] & 4, st


def test_special_cases_top_k_and_random_k():
    rng = np.random.default_rng(5)
    d = 30_011
    g = rng.standard_normal(d).astype(np.float32)
    m = np.zeros(d, np.float32)
    _check(g, m, 300, 300, 1, 0)      # r = k : top-k
    _check(g, m, d, 300, 1, 0)        # r = d : random-k
    _check(g, m, d, d, 1, 0)          # everything is sent
    _check(g, m, 300, 1, 1, 0)


def test_non_finite_values_are_ordered_by_bit_pattern():
    d = 5000
    rng = np.random.default_rng(6)
    g = rng.standard_normal(d).astype(np.float32)
    g[10] = np.inf
    g[20] = -np.inf
    g[30] = np.nan
    m = np.zeros(d, np.float32)
    u = _u()
    gi, gv, gm, _ = u.gpu_encode_once(g, m, 50, 50, 1, 1)
    wi, wv, wm = oracle.encode(g, m, 50, 50, 1, 1)
    assert np.array_equal(gi, wi) and {10, 20, 30} <= set(gi.tolist())
    assert np.array_equal(u.bits(gv), u.bits(wv))
    sent = np.zeros(d, bool)
    sent[gi] = True
    assert np.array_equal(u.bits(gm[~sent]), u.bits(wm[~sent]))
    assert np.array_equal(np.isnan(gm[sent]), np.isnan(wm[sent]))


def test_seed_and_step_use_all_64_bits():
    rng = np.random.default_rng(8)
    d = 9000
    g = rng.standard_normal(d).astype(np.float32)
    m = np.zeros(d, np.float32)
    seen = set()
    for seed, step in ((1, 1), (1 + (1 << 32), 1), (1, 1 + (1 << 32)), ((1 << 64) - 1, (1 << 63) + 5)):
        u = _u()
        got = u.gpu_encode_once(g, m, 900, 90, seed, step)
        u.assert_encode_equal(got, oracle.encode(g, m, 900, 90, seed, step))
        seen.add(tuple(got[0].tolist()))
    assert len(seen) == 4


# --------------------------------------------------------------------------
# the exact fallbacks behind the two statistical shortcuts
# --------------------------------------------------------------------------
@pytest.mark.parametrize("d,offset", [(5_000, 0), (70_001, 1), (300_000, 0), (300_001, 1),
                                      (3_000_017, 0)])
def test_fallback_paths_give_the_same_message(d, offset):
    """Ordinary input, but the sampled threshold estimate and/or the key window
    are made to miss: the message and the residual must not change, only the
    path the library reports."""
    import paper_2005_10761_amd as rt
    u = _u()
    wl = Workload(2, d=d)
    g = wl.gradient(0, 0)
    m = (np.random.default_rng(d).standard_normal(d) * 1e-3).astype(np.float32)
    want = oracle.encode(g, m, wl.r, wl.k, 99, 7)
    plain = u.gpu_encode_once(g, m, wl.r, wl.k, 99, 7, offset=offset)
    u.assert_encode_equal(plain, want, "no fallback")
    assert plain[3]["path"] == 0
    # from 256 chunks of 1024 elements on, the exact selection over all candidates runs on
    # many workgroups (path bit 3); shorter vectors leave it to one
    wide = 8 if (d + 1023) // 1024 >= 256 else 0
    for force, bits in ((rt.FORCE_ESTIMATE_MISS, 3), (rt.FORCE_KEY_WINDOW_MISS, 1),
                        (rt.FORCE_ESTIMATE_MISS | rt.FORCE_KEY_WINDOW_MISS, 3)):
        got = u.gpu_encode_once(g, m, wl.r, wl.k, 99, 7, offset=offset, force=force)
        u.assert_encode_equal(got, want, f"force={force}")
        assert got[3]["path"] == bits | wide, got[3]
    # the bracket ends below the threshold: exact by whichever path the sizes take
    got = u.gpu_encode_once(g, m, wl.r, wl.k, 99, 7, offset=offset, force=rt.FORCE_BRACKET_LOW)
    u.assert_encode_equal(got, want, "bracket too low")
    # the request is consumed by one call
    again = u.gpu_encode_once(g, m, wl.r, wl.k, 99, 7, offset=offset)
    assert again[3]["path"] == 0


def test_fallback_paths_with_ties_and_special_cases():
    import paper_2005_10761_amd as rt
    rng = np.random.default_rng(12)
    d = 40_000
    g = rng.choice([0.0, 1.0, -1.0, 2.0, 0.5], d).astype(np.float32)
    m = np.zeros(d, np.float32)
    for r, k in ((500, 50), (d, 1000), (3000, 3000), (1, 1)):
        for force in (rt.FORCE_ESTIMATE_MISS, rt.FORCE_KEY_WINDOW_MISS):
            got = _u().gpu_encode_once(g, m, r, k, 5, 5, force=force)
            _u().assert_encode_equal(got, oracle.encode(g, m, r, k, 5, 5), f"r={r} k={k} f={force}")


def test_exact_fallbacks_on_many_workgroups_long_vectors():
    """Inputs that the statistical shortcuts cannot decide, at lengths where the
    exact selection over all candidates is spread over the finalize kernel's
    workgroups (path bit 3): two neighbouring magnitudes filling the vector
    (the deciding bin holds millions of entries of two values), a few levels
    with noise in the last bits, a vector with a period close to the sampling
    strata; each also with the threshold estimate and the key window made to
    miss, with r = k (no keys) and r = d (no magnitudes), misaligned, and with
    error feedback over two steps."""
    import paper_2005_10761_amd as rt
    u = _u()
    rng = np.random.default_rng(31)
    d = 2_500_003
    one = np.float32(1.0)
    two = np.where(rng.random(d) < 0.5, one, np.nextafter(one, np.float32(2.0))).astype(np.float32)
    two *= rng.choice(np.array([-1.0, 1.0], np.float32), d)
    levels = (rng.integers(1, 4, d).astype(np.float32)
              * (1.0 + rng.integers(0, 64, d).astype(np.float32) * np.float32(2.0 ** -23)))
    periodic = (np.sin(np.arange(d, dtype=np.float64) * (2 * np.pi / 152.6)) ** 7).astype(np.float32)
    cases = [("two magnitudes", two, 900_000, 100_000, 0, 0, 9),
             ("two magnitudes, misaligned", two, 900_000, 100_000, 0, 1, 9),
             ("two magnitudes, top-k", two, 1_300_000, 1_300_000, 0, 0, 9),
             ("levels with noise", levels, 1_000_000, 50_000, 0, 0, None),
             ("periodic", periodic, 25_000, 2_500, 0, 0, None),
             ("periodic, estimate miss", periodic, 25_000, 2_500, rt.FORCE_ESTIMATE_MISS, 0, 11),
             # (a window miss is certain before the short lists are read when k exceeds what
             # they can add; otherwise one workgroup finds out and finishes alone: bit 0 only)
             ("periodic, window miss", periodic, 250_000, 100_000, rt.FORCE_KEY_WINDOW_MISS, 3, 9),
             ("periodic, window miss, small k", periodic, 25_000, 2_500, rt.FORCE_KEY_WINDOW_MISS, 0, None),
             ("random-k, window miss", two, d, 40_000, rt.FORCE_KEY_WINDOW_MISS, 0, 11),
             # the workgroups decide at check-in that they are not all resident: one of
             # them runs the selection alone (bit 0 without bit 3)
             ("estimate miss, check-in aborted", periodic, 25_000, 2_500,
              rt.FORCE_ESTIMATE_MISS | rt.FORCE_CHECK_IN_ABORT, 0, 3),
             ("window miss, check-in aborted", periodic, 250_000, 100_000,
              rt.FORCE_KEY_WINDOW_MISS | rt.FORCE_CHECK_IN_ABORT, 0, 1),
             # the bracket ends below the r-th largest magnitude: it lies in the one bin
             # that holds everything above the linear bins
             ("bracket too low", levels, 1_000_000, 50_000, rt.FORCE_BRACKET_LOW, 0, None),
             ("bracket too low, periodic", periodic, 250_000, 100_000, rt.FORCE_BRACKET_LOW, 1, 9),
             ("bracket too low, top-k", periodic, 30_000, 30_000, rt.FORCE_BRACKET_LOW, 0, 9)]
    for name, g, r, k, force, offset, want_path in cases:
        print(f"wide: {name} d={d} r={r} k={k}", flush=True)
        w = u.GpuWorker(d, r, k, offset=offset)
        res = np.zeros(d, np.float32)
        for t in range(2):
            got = w.encode(g, 77, t, force=force)
            oi, ov, res = oracle.encode(g, res, r, k, 77, t)
            u.assert_encode_equal(got, (oi, ov, res), f"{name} step {t}")
            if want_path is not None and t == 0:
                assert w.stats["path"] == want_path, (name, w.stats)
        del w


def test_chunks_that_keep_more_than_their_slice_are_read_from_the_vector():
    """A chunk of the vector owns a slice of the candidate buffer an eighth of
    its own length; where more of its elements are candidates (a layer that
    holds most of the top r) the later kernels read the chunk from the vector
    itself. Regions dense in candidates next to sparse ones, ties inside the
    dense region, a dense region at the ragged end; the ordinary path decides
    (path 0) and the message is the oracle's."""
    u = _u()
    rng = np.random.default_rng(32)
    for d, lo, hi, r, k in ((400_003, 100_000, 140_000, 50_000, 5_000),
                            (400_003, 390_000, 400_003, 12_000, 12_000),
                            (1_000_000, 0, 300_000, 250_000, 1_000),
                            (70_000, 1_000, 3_000, 2_500, 300)):
        g = (rng.standard_normal(d) * 1e-3).astype(np.float32)
        g[lo:hi] = (rng.standard_normal(hi - lo) * 5.0).astype(np.float32)      # the hot layer
        g[lo:hi:7] = np.float32(3.0)                                            # ties inside it
        res = np.zeros(d, np.float32)
        w = u.GpuWorker(d, r, k)
        for t in range(2):
            print(f"hot layer d={d} [{lo},{hi}) r={r} k={k} step {t}", flush=True)
            got = w.encode(g, 5, t)
            oi, ov, res = oracle.encode(g, res, r, k, 5, t)
            u.assert_encode_equal(got, (oi, ov, res), f"hot layer d={d} step {t}")
            # (in the last case all members sit in two chunks: their keys inside the window
            # overflow one classify workgroup's list, and the one-workgroup selection decides)
            if t == 0 and d > 100_000:
                assert w.stats["path"] == 0, w.stats
        del w


def test_batch_of_members_that_all_need_the_exact_fallback():
    """Several members of one batched call run the many-workgroup selection at
    the same time (each on its own part of the workspace), next to members on
    the ordinary path."""
    import torch
    u = _u()
    rt = u.rt
    dev = u.DEV
    d, r, k = 1_200_000, 300_000, 30_000
    rng = np.random.default_rng(33)
    one = np.float32(1.0)
    gs = []
    for i in range(5):
        if i == 2:
            gs.append(Workload(3, d=d, r=r, k=k).gradient(0, 0))
        else:
            v = np.where(rng.random(d) < 0.3 + 0.1 * i, one, np.nextafter(one, np.float32(2.0)))
            gs.append((v * rng.choice(np.array([-1.0, 1.0]), d)).astype(np.float32))
    n = len(gs)
    stride = rt.encode_workspace_bytes(d, r, k)
    ws = torch.empty(n * stride, dtype=torch.uint8, device=dev)
    ws.fill_(0xC3)
    grads = [torch.from_numpy(g).to(dev) for g in gs]
    resid = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
    out_i = [torch.full((k,), -1, dtype=torch.int32, device=dev) for _ in range(n)]
    out_v = [torch.full((k,), float("nan"), dtype=torch.float32, device=dev) for _ in range(n)]
    seeds = [200 + i for i in range(n)]
    rt.encode_batch(grads, resid, r, k, seeds, 3, out_i, out_v, ws)
    torch.cuda.synchronize()
    for i in range(n):
        st = rt.encode_stats(ws[i * stride:(i + 1) * stride])
        assert st["error_flags"] == 0, (i, st)
        assert st["path"] == (0 if i == 2 else 9), (i, st)
        want = oracle.encode(gs[i], np.zeros(d, np.float32), r, k, seeds[i], 3)
        got = (out_i[i].cpu().numpy().view(np.uint32), out_v[i].cpu().numpy(), resid[i].cpu().numpy())
        u.assert_encode_equal(got, want, f"member {i}")


# --------------------------------------------------------------------------
# multi-step error feedback, several workers, aggregate
# --------------------------------------------------------------------------
def _run_config(cfg, d, n_workers, steps, r=None, k=None, check_aggregate=True):
    u = _u()
    wl = Workload(cfg, d=d, r=r, k=k)
    d, r, k = wl.d, wl.r, wl.k
    gw = [u.GpuWorker(d, r, k) for _ in range(n_workers)]
    res = [np.zeros(d, np.float32) for _ in range(n_workers)]
    for t in range(steps):
        msgs_i, msgs_v = [], []
        for w in range(n_workers):
            g = wl.gradient(w, t)
            seed = philox_seed_for_worker(w)
            got = gw[w].encode(g, seed, t)
            oi, ov, res[w] = oracle.encode(g, res[w], r, k, seed, t)
            u.assert_encode_equal(got, (oi, ov, res[w]), f"cfg{cfg} d={d} w={w} t={t}")
            msgs_i.append(oi)
            msgs_v.append(ov)
        if check_aggregate:
            ai, av = np.concatenate(msgs_i), np.concatenate(msgs_v)
            out = u.gpu_aggregate(ai, av, n_workers, d)
            u.assert_aggregate_close(out, ai, av, n_workers, d, oracle.aggregate(ai, av, n_workers, d))
            assert np.array_equal(u.bits(out), u.bits(oracle.aggregate_f32(ai, av, n_workers, d)))
    return gw


@pytest.mark.parametrize("cfg,d,n,steps", [(1, 150_001, 1, 5), (2, 400_003, 4, 3), (3, 300_000, 4, 3),
                                           (4, 660_340, 2, 3), (5, 500_009, 3, 2)])
def test_scaled_down_configs_with_error_feedback(cfg, d, n, steps):
    _run_config(cfg, d, n, steps)


def test_stress_sweep_points_scaled_down():
    d = 1 << 20
    for k_num, k_den in ((1, 10000), (1, 1000), (1, 100)):
        for ratio in (2, 5, 10):
            k = max(1, (d * k_num + k_den - 1) // k_den)
            _run_config(5, d, 2, 2, r=ratio * k, k=k)


def test_same_call_twice_gives_identical_bytes():
    u = _u()
    wl = Workload(2, d=777_777)
    g = wl.gradient(0, 0)
    a = u.gpu_encode_once(g, np.zeros(wl.d, np.float32), wl.r, wl.k, 5, 6)
    b = u.gpu_encode_once(g, np.zeros(wl.d, np.float32), wl.r, wl.k, 5, 6)
    u.assert_encode_equal(a, b[:3])


def test_resume_from_residual_and_step():
    u = _u()
    wl = Workload(3, d=250_000)
    straight = u.GpuWorker(wl.d, wl.r, wl.k)
    outs = [straight.encode(wl.gradient(0, t), 42, t) for t in range(5)]
    first = u.GpuWorker(wl.d, wl.r, wl.k)
    for t in range(2):
        mid = first.encode(wl.gradient(0, t), 42, t)
    resumed = u.GpuWorker(wl.d, wl.r, wl.k, residual=mid[2])
    for t in range(2, 5):
        got = resumed.encode(wl.gradient(0, t), 42, t)
        u.assert_encode_equal(got, outs[t])


# --------------------------------------------------------------------------
# aggregate on its own
# --------------------------------------------------------------------------
def test_aggregate_special_cases():
    u = _u()
    d = 10_000
    idx = np.array([3, 9, 4096, 9999], np.uint32)
    val = np.array([1.5, -2.0, 1e-40, 7.0], np.float32)
    out = u.gpu_aggregate(idx, val, 1, d)
    want = np.zeros(d, np.float32)
    want[idx] = val
    assert np.array_equal(u.bits(out), u.bits(want))
    # every worker sends the same pairs, n a power of two
    n = 8
    sv = np.array([0.5, -3.25, 96.0, 1.0], np.float32)
    out = u.gpu_aggregate(np.tile(idx, n), np.tile(sv, n), n, d)
    assert np.array_equal(out[idx], sv) and np.count_nonzero(out) == 4
    # one sender out of n: correctly rounded v / n
    rng = np.random.default_rng(9)
    for n in (3, 5, 7, 16):
        k = 1500
        ii = np.arange(n * k, dtype=np.uint32) * 3
        vv = rng.standard_normal(n * k).astype(np.float32)
        out = u.gpu_aggregate(ii, vv, n, 3 * n * k + 5)
        assert np.array_equal(u.bits(out[ii]), u.bits((vv.astype(np.float64) / n).astype(np.float32)))


@pytest.mark.parametrize("d,n,k", [(5000, 3, 100), (4096 * 5 + 3, 16, 700), (1_000_003, 8, 10_000),
                                   (70, 70, 5), (100_000, 130, 50)])
def test_aggregate_random_messages(d, n, k):
    u = _u()
    rng = np.random.default_rng(d + n)
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = (rng.standard_normal((n, k)) * 10.0 ** rng.uniform(-3, 1, (n, k))).astype(np.float32)
    out = u.gpu_aggregate(idx, val, n, d)
    u.assert_aggregate_close(out, idx, val, n, d, oracle.aggregate(idx, val, n, d))
    assert np.array_equal(u.bits(out), u.bits(oracle.aggregate_f32(idx, val, n, d)))


def test_aggregate_crowded_messages():
    """Messages whose entries cluster in a few tiles (the top coordinates of one
    layer): one worker's slice of a tile runs to hundreds or thousands of pairs,
    fetched several 64-pair groups at a time. Contiguous runs, a run that ends
    exactly at a group boundary, a run up to the very end of the list, repeated
    indices inside a long run; dense aggregate and the momentum form."""
    u = _u()
    rng = np.random.default_rng(41)
    d = 300_000
    cases = []
    for n, k, lo, span in ((3, 5000, 10_000, 5000),        # contiguous: 2048 pairs per tile and worker
                           (8, 4000, 123_456, 9000),       # ~900 per tile
                           (2, 64 * 9, 4096, 64 * 9),      # 1 + 8 groups exactly
                           (2, 64 * 17, 2048 * 7, 2048),   # repeated indices: longer than the tile is wide
                           (5, 3000, d - 3500, 3500)):     # up to the end of the vector and of the list
        if span >= k:
            idx = np.stack([np.sort(rng.choice(span, k, replace=False)) + lo for _ in range(n)])
        else:
            idx = np.stack([np.sort(rng.integers(0, span, k)) + lo for _ in range(n)])
        val = rng.standard_normal((n, k)).astype(np.float32)
        cases.append((idx.astype(np.uint32), val, n))
    for idx, val, n in cases:
        out = u.gpu_aggregate(idx, val, n, d)
        assert np.array_equal(u.bits(out), u.bits(oracle.aggregate_f32(idx, val, n, d)))
        omega = rng.standard_normal(d).astype(np.float32)
        vel = rng.standard_normal(d).astype(np.float32)
        gw, gv = u.gpu_aggregate_update_momentum(idx, val, n, d, 0.25, 1.5, 0.9, omega, vel, 0)
        ww, wv = oracle.aggregate_update_momentum_f32(idx, val, n, d, 0.25, 1.5, 0.9, omega, vel)
        assert np.array_equal(u.bits(gw), u.bits(ww)) and np.array_equal(u.bits(gv), u.bits(wv))
        got = u.gpu_aggregate_update(idx, val, n, d, 0.25, 1.5, omega)
        assert np.array_equal(u.bits(got), u.bits(oracle.aggregate_update_f32(idx, val, n, d, 0.25, 1.5, omega)))


def test_aggregate_repeated_index_inside_one_message_is_added_again():
    u = _u()
    d, n = 9000, 2
    idx = np.array([[5, 5, 5, 4100, 4100, 8999], [5, 6, 6, 4100, 8999, 8999]], np.uint32)
    val = np.array([[1, 2, 3, 4, 5, 6], [7, 8, 9, 10, 11, 12]], np.float32) * np.float32(0.1)
    out = u.gpu_aggregate(idx, val, n, d)
    assert np.array_equal(u.bits(out), u.bits(oracle.aggregate_f32(idx, val, n, d)))


# --------------------------------------------------------------------------
# both master lines in one step: omega -= eta * scale * average
# --------------------------------------------------------------------------
def _check_update(u, idx, val, n, d, eta, scale, omega, offset=0):
    got = u.gpu_aggregate_update(idx, val, n, d, eta, scale, omega, offset=offset)
    u.assert_update_close(got, idx, val, n, d, eta, scale, omega,
                          oracle.aggregate_update(idx, val, n, d, eta, scale, omega))
    want32 = oracle.aggregate_update_f32(idx, val, n, d, eta, scale, omega)
    assert np.array_equal(u.bits(got), u.bits(want32))
    return got


def test_update_special_cases():
    u = _u()
    d = 10_000
    idx = np.array([3, 9, 4096, 9999], np.uint32)
    val = np.array([1.5, -2.0, 1e-40, 7.0], np.float32)
    rng = np.random.default_rng(3)
    omega = rng.standard_normal(d).astype(np.float32)
    omega[::5] = -0.0
    omega[7] = np.float32(np.inf)
    omega.view(np.uint32)[11] = 0x7FA00001          # a signalling NaN nobody touches
    omega.view(np.uint32)[4097] = 0xFFC12345        # a quiet NaN with a payload, same
    got = _check_update(u, idx, val, 1, d, 0.25, 1.0, omega)
    untouched = np.setdiff1d(np.arange(d), idx)
    assert np.array_equal(u.bits(got[untouched]), u.bits(omega[untouched]))
    # eta = 0 and a message that cancels leave the weights bit for bit
    got = u.gpu_aggregate_update(idx, val, 1, d, 0.0, 1.0, omega)
    assert np.array_equal(u.bits(got), u.bits(omega))
    cidx = np.array([[5, 4100], [5, 4100]], np.uint32)
    cval = np.array([[1.5, -2.0], [-1.5, 2.0]], np.float32)
    got = u.gpu_aggregate_update(cidx, cval, 2, d, 0.5, 3.0, omega)
    assert np.array_equal(u.bits(got), u.bits(omega))
    # the single-rounding case: 1 - (1 + 2^-12)^2 needs the unrounded product
    v = np.float32(1.0 + 2.0 ** -12)
    got = u.gpu_aggregate_update(np.array([2], np.uint32), np.array([v]), 1, 3, float(v), 1.0,
                                 np.ones(3, np.float32))
    assert float(got[2]) == -(2.0 ** -11 + 2.0 ** -24) and got[0] == 1 and got[1] == 1


@pytest.mark.parametrize("d,n,k,offset", [(5000, 3, 100, 0), (4096 * 5 + 3, 16, 700, 0),
                                          (1_000_003, 8, 10_000, 0), (1_000_003, 5, 300, 1),
                                          (70, 70, 5, 0), (100_000, 130, 50, 0), (1, 1, 1, 0),
                                          (2048, 2, 2048, 0), (300_000, 8, 3, 3),
                                          # many entries per tile: the scanning path, with
                                          # whole-tile vector accesses, misaligned, ragged end
                                          (8192, 3, 5000, 0), (8192, 3, 5000, 1),
                                          (2048 * 2 + 100, 2, 2000, 0), (50_000, 20, 9000, 0)])
def test_update_random_messages(d, n, k, offset):
    u = _u()
    rng = np.random.default_rng(d + n)
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = (rng.standard_normal((n, k)) * 10.0 ** rng.uniform(-3, 1, (n, k))).astype(np.float32)
    omega = rng.standard_normal(d).astype(np.float32)
    eta, scale = float(np.float32(0.05)), float(np.float32(n * 1.0))
    print(f"update d={d} n={n} k={k} offset={offset}", flush=True)
    _check_update(u, idx, val, n, d, eta, scale, omega, offset=offset)


def test_master_sums_add_workers_in_order_from_zero():
    """The cases that pin the order of the oracle's binary32 sums (2^24, 1 and
    -2^24 for one coordinate: 0 in worker order, 1/3 backwards), through all
    three master entry points; few workers and entries (the register path of
    the fused update) and the same coordinate inside a crowded tile (its
    scanning path)."""
    u = _u()
    big = np.float32(2.0 ** 24)
    d = 6000
    rng = np.random.default_rng(23)
    for vals in ((big, 1.0, -big), (1.0, big, -big), (big, -big, 1.0), (-big, 1.0, big)):
        for fill in (0, 300):                       # other entries of each worker in the same tile
            rows = []
            for w in range(3):
                others = np.sort(rng.choice(np.arange(2100, 4000), fill, replace=False))
                rows.append(np.sort(np.concatenate([[2077], others])))
            idx = np.stack(rows).astype(np.uint32)
            val = rng.standard_normal(idx.shape).astype(np.float32)
            for w in range(3):
                val[w, np.searchsorted(idx[w], 2077)] = vals[w]
            want = oracle.aggregate_f32(idx, val, 3, d)
            assert float(want[2077]) in (0.0, float(np.float32(1.0) / np.float32(3.0)))
            out = u.gpu_aggregate(idx, val, 3, d)
            assert np.array_equal(u.bits(out), u.bits(want)), (vals, fill)
            omega = np.ones(d, np.float32)
            got = u.gpu_aggregate_update(idx, val, 3, d, -1.0, 1.0, omega)
            assert np.array_equal(u.bits(got), u.bits(oracle.aggregate_update_f32(idx, val, 3, d, -1.0, 1.0, omega)))
            gw, gv = u.gpu_aggregate_update_momentum(idx, val, 3, d, -1.0, 1.0, 0.5, omega, omega)
            ww, wv = oracle.aggregate_update_momentum_f32(idx, val, 3, d, -1.0, 1.0, 0.5, omega, omega)
            assert np.array_equal(u.bits(gw), u.bits(ww)) and np.array_equal(u.bits(gv), u.bits(wv))


def test_update_moves_a_weight_only_where_the_average_is_not_zero():
    """A sum that is not zero but whose quotient by n underflows to zero leaves
    the weight's bits alone (a signalling not-a-number stays signalling), on the
    register path, on the scanning path (more than 64 entries of a worker in
    the tile) and with more than 16 workers."""
    u = _u()
    tiny = np.float32(2.0 ** -149)
    d = 5000
    for n, fill in ((3, 0), (3, 200), (17, 0)):
        rng = np.random.default_rng(n + fill)
        rows = []
        for w in range(n):
            others = np.sort(rng.choice(np.arange(100, 2000), fill, replace=False))
            rows.append(np.sort(np.concatenate([[7, 40], others])))
        idx = np.stack(rows).astype(np.uint32)
        val = rng.standard_normal(idx.shape).astype(np.float32)
        val[:, 0] = 0.0
        val[0, 0] = tiny                                   # coordinate 7: sum 2^-149, average 0
        val[:, 1] = 0.0
        val[n - 1, 1] = np.float32(2.0 ** -140)            # coordinate 40: a denormal average
        omega = rng.standard_normal(d).astype(np.float32)
        omega.view(np.uint32)[7] = 0x7FA00001
        omega[40] = 0.0
        want = oracle.aggregate_update_f32(idx, val, n, d, 1.0, 1.0, omega)
        assert int(u.bits(want)[7]) == 0x7FA00001 and want[40] != omega[40]
        got = u.gpu_aggregate_update(idx, val, n, d, 1.0, 1.0, omega)
        assert np.array_equal(u.bits(got), u.bits(want)), (n, fill)


def test_update_clustered_messages_leave_far_tiles_alone():
    # all entries inside two narrow ranges far apart; everything between them
    # and around them must come back bit for bit
    u = _u()
    rng = np.random.default_rng(17)
    d, n, k = 3_000_000, 8, 4000
    idx = np.stack([np.concatenate([
        np.sort(rng.choice(np.arange(700_000, 706_000), k // 2, replace=False)),
        np.sort(rng.choice(np.arange(2_900_000, 2_999_999), k // 2, replace=False))])
        for _ in range(n)]).astype(np.uint32)
    val = rng.standard_normal((n, k)).astype(np.float32)
    omega = rng.standard_normal(d).astype(np.float32)
    got = _check_update(u, idx, val, n, d, 0.1, 5.0, omega)
    far = np.ones(d, bool)
    far[idx.reshape(-1)] = False
    assert np.array_equal(u.bits(got[far]), u.bits(omega[far]))


def test_update_repeated_index_inside_one_message_is_added_again():
    u = _u()
    d, n = 9000, 2
    idx = np.array([[5, 5, 5, 4100, 4100, 8999], [5, 6, 6, 4100, 8999, 8999]], np.uint32)
    val = np.array([[1, 2, 3, 4, 5, 6], [7, 8, 9, 10, 11, 12]], np.float32) * np.float32(0.1)
    omega = np.linspace(-1, 1, d).astype(np.float32)
    _check_update(u, idx, val, n, d, 0.3, 1.0, omega)


def test_training_loop_of_algorithm_1_on_the_device_matches_the_oracle():
    """Nodes encode, the master averages and steps; three rounds, weights and
    residuals carried on both sides."""
    u = _u()
    d, r, k, n, eta = 200_003, 2000, 400, 5, 0.1
    rng = np.random.default_rng(23)
    w_gpu = rng.standard_normal(d).astype(np.float32)
    w_ref = w_gpu.copy()
    workers = [u.GpuWorker(d, r, k) for _ in range(n)]
    res = [np.zeros(d, np.float32) for _ in range(n)]
    for t in range(3):
        mi, mv = [], []
        for w in range(n):
            g = (rng.standard_normal(d) * 0.01 + 0.001 * w_ref).astype(np.float32)
            gi, gv, _ = workers[w].encode(g, 42 + w, t)
            oi, ov, res[w] = oracle.encode(g, res[w], r, k, 42 + w, t)
            assert np.array_equal(gi, oi) and np.array_equal(u.bits(gv), u.bits(ov))
            mi.append(oi)
            mv.append(ov)
        ai, av = np.stack(mi), np.stack(mv)
        w_gpu = u.gpu_aggregate_update(ai, av, n, d, eta, r / k, w_gpu)
        w_ref = oracle.aggregate_update_f32(ai, av, n, d, eta, r / k, w_ref)
        assert np.array_equal(u.bits(w_gpu), u.bits(w_ref))


# --------------------------------------------------------------------------
# per-step (r, k): the warm-up of the experiments section raises the sparsity
# step by step; one worker, one workspace sized for the densest step
# --------------------------------------------------------------------------
def test_warmup_schedule_of_r_and_k_with_one_workspace():
    u = _u()
    wl = Workload(3, d=400_003)
    d, n = wl.d, 5
    kept = [0.25, 0.0625, 0.015625, 0.004, 0.001, 0.001]       # fraction of d sent per step
    sched = []
    for f in kept:
        k = int(np.ceil(f * d))
        sched.append((min(d, n * k), k))                        # k / r = 1 / n, capped at d
    r_ws, k_ws = max(sched, key=lambda rk: rt_ws(u, d, *rk))
    w = u.GpuWorker(d, r_ws, max(k for _, k in sched))
    assert all(rt_ws(u, d, r, k) <= w.ws.numel() for r, k in sched)
    res = np.zeros(d, np.float32)
    for t, (r, k) in enumerate(sched):
        g = wl.gradient(0, t)
        print(f"schedule step {t}: r={r} k={k}", flush=True)
        got = w.encode(g, 42, t, r=r, k=k)
        oi, ov, res = oracle.encode(g, res, r, k, 42, t)
        u.assert_encode_equal(got, (oi, ov, res), f"schedule t={t} r={r} k={k}")


def rt_ws(u, d, r, k):
    return u.rt.encode_workspace_bytes(d, r, k)


# --------------------------------------------------------------------------
# several vectors in one call: every member exactly as if encoded alone
# --------------------------------------------------------------------------
@pytest.mark.parametrize("n,d,misalign", [(3, 150_001, None), (8, 70_000, None), (17, 20_011, None),
                                          (4, 90_004, 2),
                                          # chunk counts around the walking kernels' share-out of a
                                          # batch (2048 wavefronts of up to 16 chunks): 2,930 and 5,860
                                          # chunks, and 20 members in launches of 16 + 4
                                          (4, 3_000_003, None), (5, 6_000_001, 1), (20, 2_200_000, None)])
def test_batch_members_match_the_oracle_one_by_one(n, d, misalign):
    import torch
    u = _u()
    rt = u.rt
    r, k = max(2, d // 100), max(1, d // 1000)
    wl = Workload(3, d=d, r=r, k=k)
    dev = u.DEV
    stride = rt.encode_workspace_bytes(d, r, k)
    ws = torch.empty(n * stride, dtype=torch.uint8, device=dev)
    ws.fill_(0xA5)
    offs = [1 if i == misalign else 0 for i in range(n)]      # one member off 16-byte alignment
    g_store = [torch.empty(d + 4, dtype=torch.float32, device=dev) for _ in range(n)]
    m_store = [torch.zeros(d + 4, dtype=torch.float32, device=dev) for _ in range(n)]
    grads = [g_store[i][offs[i]:offs[i] + d] for i in range(n)]
    resid = [m_store[i][offs[i]:offs[i] + d] for i in range(n)]
    idx = torch.full((n * k,), -1, dtype=torch.int32, device=dev)
    val = torch.full((n * k,), float("nan"), dtype=torch.float32, device=dev)
    out_i = [idx[i * k:(i + 1) * k] for i in range(n)]
    out_v = [val[i * k:(i + 1) * k] for i in range(n)]
    seeds = [philox_seed_for_worker(i) + (1 << 40) * i for i in range(n)]
    ref_m = [np.zeros(d, np.float32) for _ in range(n)]
    for t in range(2):
        gs = [wl.gradient(i, t) for i in range(n)]
        for i in range(n):
            grads[i].copy_(torch.from_numpy(gs[i]))
        print(f"batch n={n} d={d} step={t}", flush=True)
        rt.encode_batch(grads, resid, r, k, seeds, t, out_i, out_v, ws)
        torch.cuda.synchronize()
        for i in range(n):
            st = rt.encode_stats(ws[i * stride:(i + 1) * stride])
            assert st["error_flags"] == 0 and st["count_greater"] + st["ties_taken"] == r, (i, st)
            oi, ov, ref_m[i] = oracle.encode(gs[i], ref_m[i], r, k, seeds[i], t)
            got = (out_i[i].cpu().numpy().view(np.uint32), out_v[i].cpu().numpy(),
                   resid[i].cpu().numpy())
            u.assert_encode_equal(got, (oi, ov, ref_m[i]), f"member {i} step {t}")
        # the messages sit back to back: the master's average takes them as they are
        out = torch.empty(d, dtype=torch.float32, device=dev)
        rt.aggregate(idx, val, n, k, out)
        torch.cuda.synchronize()
        want = oracle.aggregate_f32(idx.cpu().numpy().view(np.uint32), val.cpu().numpy(), n, d)
        assert np.array_equal(u.bits(out.cpu().numpy()), u.bits(want))


@pytest.mark.parametrize("n,d,r,k,force", [(5, 37, 9, 4, 0), (2, 1, 1, 1, 0), (3, 5000, 5000, 17, 0),
                                           (4, 30_000, 600, 600, 0), (3, 60_000, 900, 90, 1),
                                           (3, 60_000, 900, 90, 2), (6, 4097, 300, 30, 3)])
def test_batch_small_sizes_special_shapes_and_forced_fallbacks(n, d, r, k, force):
    """Tiny vectors, r = d, r = k, and the exact fallback paths forced for every
    member of a batched call."""
    import torch
    u = _u()
    rt = u.rt
    dev = u.DEV
    rng = np.random.default_rng(1000 * n + d)
    stride = rt.encode_workspace_bytes(d, r, k)
    ws = torch.empty(n * stride, dtype=torch.uint8, device=dev)
    ws.fill_(0x5A)
    gs = [(rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 0, d)).astype(np.float32) for _ in range(n)]
    ms = [(rng.standard_normal(d) * 1e-2).astype(np.float32) for _ in range(n)]
    grads = [torch.from_numpy(g).to(dev) for g in gs]
    resid = [torch.from_numpy(m).to(dev) for m in ms]
    out_i = [torch.full((k,), -1, dtype=torch.int32, device=dev) for _ in range(n)]
    out_v = [torch.full((k,), float("nan"), dtype=torch.float32, device=dev) for _ in range(n)]
    seeds = [7 + 13 * i for i in range(n)]
    if force:
        rt.force_next_encode(force)
    rt.encode_batch(grads, resid, r, k, seeds, 5, out_i, out_v, ws)
    torch.cuda.synchronize()
    for i in range(n):
        st = rt.encode_stats(ws[i * stride:(i + 1) * stride])
        assert st["error_flags"] == 0, (i, st)
        if force & 1:
            assert st["path"] & 2, (i, st)
        if force & 2 and r > k:
            assert st["path"] & 1, (i, st)
        want = oracle.encode(gs[i], ms[i], r, k, seeds[i], 5)
        got = (out_i[i].cpu().numpy().view(np.uint32), out_v[i].cpu().numpy(), resid[i].cpu().numpy())
        u.assert_encode_equal(got, want, f"member {i}")


def test_batch_rejects_bad_arguments():
    import torch
    u = _u()
    rt = u.rt
    d, r, k = 1000, 10, 2
    dev = u.DEV
    g = torch.zeros(d, dtype=torch.float32, device=dev)
    m = torch.zeros(d, dtype=torch.float32, device=dev)
    oi = torch.zeros(k, dtype=torch.int32, device=dev)
    ov = torch.zeros(k, dtype=torch.float32, device=dev)
    ws = torch.empty(rt.encode_workspace_bytes(d, r, k), dtype=torch.uint8, device=dev)
    with pytest.raises(rt.RtopkError):        # workspace for one member, two members
        rt.encode_batch([g, g], [m, m.clone()], r, k, [1, 2], 0, [oi, oi.clone()], [ov, ov.clone()], ws)
    with pytest.raises(rt.RtopkError):        # gradient and residual are the same buffer
        rt.encode_batch([g], [g], r, k, [1], 0, [oi], [ov], ws)
    with pytest.raises(ValueError):
        rt.encode_batch([g], [m], r, k, [1, 2], 0, [oi], [ov], ws)


# --------------------------------------------------------------------------
# master with momentum: velocity = mu velocity + scale average; omega -= eta velocity
# --------------------------------------------------------------------------
@pytest.mark.parametrize("d,n,k,offset", [(5000, 3, 100, 0), (4096 * 5 + 3, 16, 700, 0),
                                          (1_000_003, 8, 10_000, 0), (300_007, 5, 300, 1),
                                          (70, 70, 5, 0), (100_000, 130, 50, 0), (1, 1, 1, 0),
                                          (2048, 2, 2048, 0)])
def test_momentum_update_random_messages(d, n, k, offset):
    u = _u()
    rng = np.random.default_rng(3 * d + n)
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = (rng.standard_normal((n, k)) * 10.0 ** rng.uniform(-3, 1, (n, k))).astype(np.float32)
    omega = rng.standard_normal(d).astype(np.float32)
    vel = (rng.standard_normal(d) * 0.1).astype(np.float32)
    eta, scale, mu = float(np.float32(0.05)), float(np.float32(n)), float(np.float32(0.9))
    print(f"momentum d={d} n={n} k={k} offset={offset}", flush=True)
    gw, gv = u.gpu_aggregate_update_momentum(idx, val, n, d, eta, scale, mu, omega, vel, offset)
    ww, wv = oracle.aggregate_update_momentum_f32(idx, val, n, d, eta, scale, mu, omega, vel)
    assert np.array_equal(u.bits(gv), u.bits(wv)) and np.array_equal(u.bits(gw), u.bits(ww))
    w64, v64 = oracle.aggregate_update_momentum(idx, val, n, d, eta, scale, mu, omega, vel)
    dense = np.zeros(d)
    np.add.at(dense, idx.reshape(-1).astype(np.int64), np.abs(val.reshape(-1).astype(np.float64)) / n)
    size_v = mu * np.abs(vel.astype(np.float64)) + scale * dense
    assert np.all(np.abs(gv.astype(np.float64) - v64) <= 1e-6 * size_v + 1e-30)
    assert np.all(np.abs(gw.astype(np.float64) - w64)
                  <= 1e-6 * (np.abs(omega.astype(np.float64)) + eta * size_v) + 1e-30)


def test_momentum_update_special_cases():
    u = _u()
    x = np.float32(1.0 + 2.0 ** -12)
    one_idx = np.array([2], np.uint32)
    # the single-rounding cases of the oracle's pins, at coordinate 2 of 5
    w0, v0 = np.full(5, 5.0, np.float32), np.full(5, x, np.float32)
    gw, gv = u.gpu_aggregate_update_momentum(one_idx, np.array([-1.0], np.float32), 1, 5, 0.0, 1.0,
                                             float(x), w0, v0)
    assert float(gv[2]) == 2.0 ** -11 + 2.0 ** -24 and np.all(gw == 5.0)
    gw, gv = u.gpu_aggregate_update_momentum(one_idx, np.array([x]), 1, 5, float(x), 1.0, 0.0,
                                             np.ones(5, np.float32), np.full(5, 9.0, np.float32))
    assert float(gv[2]) == float(x) and float(gw[2]) == -(2.0 ** -11 + 2.0 ** -24)
    assert np.all(gv[[0, 1, 3, 4]] == 0.0) and np.all(gw[[0, 1, 3, 4]] == 1.0)


def test_momentum_training_loop_on_the_device_matches_the_oracle():
    u = _u()
    d, r, k, n = 150_001, 1500, 300, 4
    rng = np.random.default_rng(29)
    w_gpu = rng.standard_normal(d).astype(np.float32)
    v_gpu = np.zeros(d, np.float32)
    w_ref, v_ref = w_gpu.copy(), v_gpu.copy()
    workers = [u.GpuWorker(d, r, k) for _ in range(n)]
    res = [np.zeros(d, np.float32) for _ in range(n)]
    for t in range(3):
        mi, mv = [], []
        for w in range(n):
            g = (rng.standard_normal(d) * 0.01 + 0.001 * w_ref).astype(np.float32)
            gi, gv, _ = workers[w].encode(g, 42 + w, t)
            oi, ov, res[w] = oracle.encode(g, res[w], r, k, 42 + w, t)
            assert np.array_equal(gi, oi) and np.array_equal(u.bits(gv), u.bits(ov))
            mi.append(oi)
            mv.append(ov)
        ai, av = np.stack(mi), np.stack(mv)
        w_gpu, v_gpu = u.gpu_aggregate_update_momentum(ai, av, n, d, 0.1, 1.0, 0.9, w_gpu, v_gpu)
        w_ref, v_ref = oracle.aggregate_update_momentum_f32(ai, av, n, d, 0.1, 1.0, 0.9, w_ref, v_ref)
        assert np.array_equal(u.bits(w_gpu), u.bits(w_ref))
        assert np.array_equal(u.bits(v_gpu), u.bits(v_ref))


# --------------------------------------------------------------------------
# the federated setting's update vector: dense, smooth, r = 5% and k = 1% of d
# --------------------------------------------------------------------------
def test_federated_update_vector_five_nodes():
    u = _u()
    wl = Workload(6, d=400_009)
    d, r, k, n = wl.d, wl.r, wl.k, wl.n_workers
    assert n == 5 and abs(r - n * k) < n                      # k / r = 1 / n up to the ceilings
    gw = [u.GpuWorker(d, r, k) for _ in range(n)]
    res = [np.zeros(d, np.float32) for _ in range(n)]
    omega = np.zeros(d, np.float32)
    for t in range(3):
        mi, mv = [], []
        for w in range(n):
            g = wl.gradient(w, t)
            got = gw[w].encode(g, philox_seed_for_worker(w), t)
            oi, ov, res[w] = oracle.encode(g, res[w], r, k, philox_seed_for_worker(w), t)
            u.assert_encode_equal(got, (oi, ov, res[w]), f"federated w={w} t={t}")
            assert gw[w].stats["path"] == 0
            mi.append(oi)
            mv.append(ov)
        ai, av = np.stack(mi), np.stack(mv)
        got_w = u.gpu_aggregate_update(ai, av, n, d, 1.0, 1.0, omega)
        omega = oracle.aggregate_update_f32(ai, av, n, d, 1.0, 1.0, omega)
        assert np.array_equal(u.bits(got_w), u.bits(omega))


# --------------------------------------------------------------------------
# r = d (the random-k operator): no magnitude decides anything
# --------------------------------------------------------------------------
@pytest.mark.parametrize("d,k,offset,force", [(300_003, 300, 0, 0), (300_003, 1, 0, 0),
                                              (300_003, 30_000, 1, 0), (70_001, 70_001, 0, 0),
                                              (5, 2, 0, 0), (1_048_576, 1049, 0, 0),
                                              (120_000, 1200, 0, 2), (120_000, 1200, 3, 1),
                                              (120_000, 1200, 0, 3)])
def test_random_k_is_the_r_equals_d_case(d, k, offset, force):
    u = _u()
    rng = np.random.default_rng(d + k)
    g1 = (rng.standard_normal(d) * 10.0 ** rng.uniform(-4, 0, d)).astype(np.float32)
    g1[rng.random(d) < 0.3] = 0.0                       # magnitudes must not matter, zeros included
    m0 = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    print(f"random-k d={d} k={k} offset={offset} force={force}", flush=True)
    w = u.GpuWorker(d, d, k, residual=m0, offset=offset)
    res = m0
    for t in range(2):
        g = g1 if t == 0 else (g1 * np.float32(0.5))
        got = w.encode(g, 77, t, force=force if t == 0 else 0)
        oi, ov, res = oracle.encode(g, res, d, k, 77, t)
        u.assert_encode_equal(got, (oi, ov, res), f"random-k t={t}")
        st = w.stats
        if t == 0 and force & 2 and k < d:
            assert st["path"] & 2, st                   # the window missed: the vector itself was walked
        if not force or t == 1:
            assert st["path"] == 0, st
        # the k-subset is a uniform one: it does not follow the magnitudes
    mags = np.abs(g1 + m0)
    sent = np.zeros(d, bool)
    sent[oi] = True
    if 100 <= k <= d // 10:
        assert abs(np.median(mags[sent]) - np.median(mags)) <= 0.5 * np.median(mags) + 1e-3


# --------------------------------------------------------------------------
# seeded random sweep over sizes and value patterns, all entry points
# --------------------------------------------------------------------------
def test_seeded_random_sweep_of_sizes_and_value_patterns():
    import torch
    u = _u()
    rt = u.rt
    dev = u.DEV
    rng = np.random.default_rng(20240607)
    for case in range(180):
        d = int(rng.choice([1, 2, 3, 7, 64, 65, 255, 256, 257, 1000, 1023, 1025, 4095, 4097, 9000]))
        r = int(rng.integers(1, d + 1))
        k = int(rng.integers(1, r + 1))
        if case % 7 == 0:
            r = d
        if case % 11 == 0:
            k = r
        n = int(rng.integers(1, 5))
        pattern = case % 6
        gs, ms = [], []
        for i in range(n):
            if pattern == 0:
                g = rng.standard_normal(d)
            elif pattern == 1:                      # few distinct magnitudes: ties everywhere
                g = rng.choice([-2.0, -1.0, 0.0, 1.0, 2.0], d)
            elif pattern == 2:                      # mostly zero
                g = rng.standard_normal(d) * (rng.random(d) < 0.1)
            elif pattern == 3:                      # wide dynamic range with denormals
                g = rng.standard_normal(d) * 10.0 ** rng.uniform(-44, 3, d)
            elif pattern == 4:                      # one value
                g = np.full(d, 0.75)
            else:                                   # infinities and not-a-number values
                g = rng.standard_normal(d)
                odd = rng.random(d) < 0.02
                g[odd] = rng.choice([np.inf, -np.inf, np.nan], int(odd.sum()))
            gs.append(g.astype(np.float32))
            ms.append((rng.standard_normal(d) * (0.0 if pattern in (1, 4) else 1e-3)).astype(np.float32))
        seeds = [int(rng.integers(0, 2 ** 63)) for _ in range(n)]
        step = int(rng.integers(0, 2 ** 40))
        stride = rt.encode_workspace_bytes(d, r, k)
        ws = torch.empty(n * stride, dtype=torch.uint8, device=dev)
        grads = [torch.from_numpy(g).to(dev) for g in gs]
        resid = [torch.from_numpy(m).to(dev) for m in ms]
        idx = torch.full((n * k,), -1, dtype=torch.int32, device=dev)
        val = torch.full((n * k,), float("nan"), dtype=torch.float32, device=dev)
        out_i = [idx[i * k:(i + 1) * k] for i in range(n)]
        out_v = [val[i * k:(i + 1) * k] for i in range(n)]
        what = f"case {case}: d={d} r={r} k={k} n={n} pattern={pattern}"
        print(what, flush=True)
        rt.encode_batch(grads, resid, r, k, seeds, step, out_i, out_v, ws)
        torch.cuda.synchronize()
        for i in range(n):
            st = rt.encode_stats(ws[i * stride:(i + 1) * stride])
            assert st["error_flags"] == 0, (what, i, st)
            want = oracle.encode(gs[i], ms[i], r, k, seeds[i], step)
            got = (out_i[i].cpu().numpy().view(np.uint32), out_v[i].cpu().numpy(),
                   resid[i].cpu().numpy())
            u.assert_encode_equal(got, want, f"{what} member {i}")
        ai = idx.cpu().numpy().view(np.uint32)
        av = val.cpu().numpy()
        # sums of several not-a-number values may keep either payload: same_floats
        out = u.gpu_aggregate(ai, av, n, d)
        assert u.same_floats(out, oracle.aggregate_f32(ai, av, n, d)), what
        omega = rng.standard_normal(d).astype(np.float32)
        vel = rng.standard_normal(d).astype(np.float32)
        gw = u.gpu_aggregate_update(ai, av, n, d, 0.125, 2.0, omega)
        assert u.same_floats(gw, oracle.aggregate_update_f32(ai, av, n, d, 0.125, 2.0, omega)), what
        gw, gv = u.gpu_aggregate_update_momentum(ai, av, n, d, 0.125, 2.0, 0.5, omega, vel)
        ww, wv = oracle.aggregate_update_momentum_f32(ai, av, n, d, 0.125, 2.0, 0.5, omega, vel)
        assert u.same_floats(gw, ww) and u.same_floats(gv, wv), what


def test_batch_with_members_on_different_paths():
    """One batched call whose members take different paths: ordinary vectors
    next to a frozen tensor's zeros, a ternary vector and a vector with two
    neighbouring magnitudes crowding the deciding bin. Every member as alone."""
    import torch
    u = _u()
    rt = u.rt
    dev = u.DEV
    d, r, k = 250_000, 20_000, 2_000
    rng = np.random.default_rng(77)
    one = np.float32(1.0)
    two_mags = np.where(rng.random(d) < 0.5, one, np.nextafter(one, np.float32(2.0))).astype(np.float32)
    gs = [Workload(3, d=d, r=r, k=k).gradient(0, 0),
          np.zeros(d, np.float32),
          rng.integers(-1, 2, d).astype(np.float32),
          two_mags,
          Workload(2, d=d, r=r, k=k).gradient(1, 3)]
    want_path = [0, 4, 4, 1, 0]
    n = len(gs)
    ms = [np.zeros(d, np.float32) for _ in range(n)]
    stride = rt.encode_workspace_bytes(d, r, k)
    ws = torch.empty(n * stride, dtype=torch.uint8, device=dev)
    ws.fill_(0x3C)
    grads = [torch.from_numpy(g).to(dev) for g in gs]
    resid = [torch.from_numpy(m).to(dev) for m in ms]
    out_i = [torch.full((k,), -1, dtype=torch.int32, device=dev) for _ in range(n)]
    out_v = [torch.full((k,), float("nan"), dtype=torch.float32, device=dev) for _ in range(n)]
    seeds = [100 + i for i in range(n)]
    for t in range(2):
        rt.encode_batch(grads, resid, r, k, seeds, t, out_i, out_v, ws)
        torch.cuda.synchronize()
        for i in range(n):
            st = rt.encode_stats(ws[i * stride:(i + 1) * stride])
            assert st["error_flags"] == 0, (t, i, st)
            if t == 0:
                assert st["path"] == want_path[i], (i, st)
            want = oracle.encode(gs[i], ms[i], r, k, seeds[i], t)
            got = (out_i[i].cpu().numpy().view(np.uint32), out_v[i].cpu().numpy(),
                   resid[i].cpu().numpy())
            u.assert_encode_equal(got, want, f"step {t} member {i}")
            ms[i] = want[2]


def test_two_streams_with_their_own_workspaces_do_not_disturb_each_other():
    """Calls on different streams share nothing but the library's per-device
    launch width: with distinct workspaces, residuals and outputs they may
    overlap freely (both streams at the default priority)."""
    import torch
    u = _u()
    rt = u.rt
    dev = u.DEV
    d = 1_500_000
    wl = Workload(3, d=d)
    r, k = wl.r, wl.k
    streams = [torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)]
    gs = [wl.gradient(w, 0) for w in range(2)]
    ms = [np.zeros(d, np.float32) for _ in range(2)]
    grads = [torch.from_numpy(g).to(dev) for g in gs]
    resid = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(2)]
    ws = [torch.empty(rt.encode_workspace_bytes(d, r, k), dtype=torch.uint8, device=dev) for _ in range(2)]
    oi = [torch.empty(k, dtype=torch.int32, device=dev) for _ in range(2)]
    ov = [torch.empty(k, dtype=torch.float32, device=dev) for _ in range(2)]
    torch.cuda.synchronize()
    for t in range(3):
        for w in range(2):                                   # enqueue both before either finishes
            rt.encode(grads[w], resid[w], r, k, 42 + w, t, oi[w], ov[w], ws[w], stream=streams[w])
        torch.cuda.synchronize()
        for w in range(2):
            want = oracle.encode(gs[w], ms[w], r, k, 42 + w, t)
            got = (oi[w].cpu().numpy().view(np.uint32), ov[w].cpu().numpy(), resid[w].cpu().numpy())
            u.assert_encode_equal(got, want, f"step {t} stream {w}")
            ms[w] = want[2]


def test_exact_fallbacks_of_three_streams_at_once():
    """Three streams force the selection over all candidates at the same time.
    Each call's finalize grid wants every compute unit; the grids first agree
    among their own workgroups whether all of them are running, and a grid that
    cannot get there falls back to one workgroup. Whichever way each call goes,
    its message is the oracle's."""
    import torch
    u = _u()
    rt = u.rt
    dev = u.DEV
    d = 1_500_000
    wl = Workload(3, d=d)
    r, k = wl.r, wl.k
    n = 3
    streams = [torch.cuda.Stream(device=dev) for _ in range(n)]
    gs = [wl.gradient(w, 0) for w in range(n)]
    ms = [np.zeros(d, np.float32) for _ in range(n)]
    grads = [torch.from_numpy(g).to(dev) for g in gs]
    resid = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
    ws = [torch.empty(rt.encode_workspace_bytes(d, r, k), dtype=torch.uint8, device=dev) for _ in range(n)]
    oi = [torch.empty(k, dtype=torch.int32, device=dev) for _ in range(n)]
    ov = [torch.empty(k, dtype=torch.float32, device=dev) for _ in range(n)]
    torch.cuda.synchronize()
    for t, force in enumerate((rt.FORCE_KEY_WINDOW_MISS, rt.FORCE_ESTIMATE_MISS)):
        for w in range(n):                                   # enqueue all before any finishes
            rt.force_next_encode(force)
            rt.encode(grads[w], resid[w], r, k, 7 + w, t, oi[w], ov[w], ws[w], stream=streams[w])
        torch.cuda.synchronize()
        for w in range(n):
            st = rt.encode_stats(ws[w])
            assert st["error_flags"] == 0 and st["path"] & 1, st
            want = oracle.encode(gs[w], ms[w], r, k, 7 + w, t)
            got = (oi[w].cpu().numpy().view(np.uint32), ov[w].cpu().numpy(), resid[w].cpu().numpy())
            u.assert_encode_equal(got, want, f"step {t} stream {w} path {st['path']}")
            ms[w] = want[2]


def test_a_barrier_that_gives_up_ends_the_call_with_the_error_flag():
    """Failure handling of the many-workgroup selection, forced from the host:
    its bounded waits give up at once. Every kernel still ends, the error flag
    says that the outputs are invalid (in the statistics and in the first word
    of the workspace), and the next call on the same buffers is clean again."""
    u = _u()
    rt = u.rt
    d = 1_500_000
    wl = Workload(3, d=d)
    g = wl.gradient(0, 0)
    w = u.GpuWorker(d, wl.r, wl.k)
    w.encode(g, 5, 0, check_stats=False,
             force=rt.FORCE_KEY_WINDOW_MISS | rt.FORCE_BARRIER_TIMEOUT)
    assert w.stats["error_flags"] & 8, w.stats
    # a fresh residual (the failed call's is invalid), the same workspace
    w.residual.zero_()
    got = w.encode(g, 5, 0)
    want = oracle.encode(g, np.zeros(d, np.float32), wl.r, wl.k, 5, 0)
    u.assert_encode_equal(got, want, "after a failed call")
    assert w.stats["error_flags"] == 0 and w.stats["path"] == 0, w.stats


def test_test_hooks_belong_to_the_calling_host_thread():
    """rtopk_force_next_encode (like rtopk_trace_next_encode) is remembered per
    host thread: a request made on one thread must not reach another thread's
    call, and is still there for the first thread's own next call."""
    import threading
    import paper_2005_10761_amd as rt
    u = _u()
    d = 60_000
    wl = Workload(2, d=d)
    g = wl.gradient(0, 0)
    m = np.zeros(d, np.float32)
    want = oracle.encode(g, m, wl.r, wl.k, 9, 1)
    asked, other_done = threading.Event(), threading.Event()
    seen = {}

    def first():
        rt.force_next_encode(rt.FORCE_ESTIMATE_MISS)
        asked.set()
        other_done.wait(60)
        seen["first"] = u.gpu_encode_once(g, m, wl.r, wl.k, 9, 1)

    def second():
        asked.wait(60)
        seen["second"] = u.gpu_encode_once(g, m, wl.r, wl.k, 9, 1)
        other_done.set()

    ts = [threading.Thread(target=first), threading.Thread(target=second)]
    for t in ts:
        t.start()
    for t in ts:
        t.join(120)
    assert set(seen) == {"first", "second"}
    u.assert_encode_equal(seen["second"], want, "other thread")
    u.assert_encode_equal(seen["first"], want, "requesting thread")
    assert seen["second"][3]["path"] == 0 and seen["first"][3]["path"] & 2, (seen["second"][3], seen["first"][3])


# --------------------------------------------------------------------------
# the whole step inside a captured HIP graph
# --------------------------------------------------------------------------
def test_step_captured_in_a_hip_graph_replays_bit_exactly():
    """The library allocates nothing, clears what it needs with its own kernels
    and never synchronises: a step (batched encode + aggregate + fused update)
    can be captured into a HIP graph. Every replay, with eager work and
    synchronisations in between, must give the oracle's result again."""
    import torch
    import paper_2005_10761_amd as rt
    u = _u()
    dev = u.DEV
    n, d = 3, 200_003
    wl = Workload(2, d=d)
    r, k = wl.r, wl.k
    gs = [wl.gradient(w, 0) for w in range(n)]
    m0 = [(np.random.default_rng(w).standard_normal(d) * 1e-3).astype(np.float32) for w in range(n)]
    seeds = [philox_seed_for_worker(w) for w in range(n)]
    want = [oracle.encode(gs[w], m0[w], r, k, seeds[w], 11) for w in range(n)]
    wi = np.concatenate([w_[0] for w_ in want])
    wv = np.concatenate([w_[1] for w_ in want])
    omega0 = np.random.default_rng(99).standard_normal(d).astype(np.float32)

    stride = rt.encode_workspace_bytes(d, r, k)
    ws = torch.empty(n * stride, dtype=torch.uint8, device=dev)
    wsu = torch.empty(rt.aggregate_update_workspace_bytes(d, n, k), dtype=torch.uint8, device=dev)
    g = [torch.from_numpy(x).to(dev) for x in gs]
    m = [torch.from_numpy(x).to(dev) for x in m0]
    m_init = [t.clone() for t in m]
    idx = torch.empty(n * k, dtype=torch.int32, device=dev)
    val = torch.empty(n * k, dtype=torch.float32, device=dev)
    oi = [idx[i * k:(i + 1) * k] for i in range(n)]
    ov = [val[i * k:(i + 1) * k] for i in range(n)]
    out = torch.empty(d, dtype=torch.float32, device=dev)
    omega = torch.from_numpy(omega0).to(dev)
    omega_init = omega.clone()

    def step():
        rt.encode_batch(g, m, r, k, seeds, 11, oi, ov, ws)
        rt.aggregate(idx, val, n, k, out)
        rt.aggregate_update(idx, val, n, k, 0.5, 1.0, omega, wsu)

    def reset():
        for t, t0 in zip(m, m_init):
            t.copy_(t0)
        omega.copy_(omega_init)
        idx.fill_(-1)
        val.fill_(float("nan"))
        out.fill_(float("nan"))
        ws.fill_(0x5A)

    def check(what):
        torch.cuda.synchronize()
        for w in range(n):
            got = (oi[w].cpu().numpy().view(np.uint32), ov[w].cpu().numpy(), m[w].cpu().numpy())
            u.assert_encode_equal(got, want[w], f"{what} worker {w}")
        assert np.array_equal(u.bits(out.cpu().numpy()), u.bits(oracle.aggregate_f32(wi, wv, n, d))), what
        assert np.array_equal(u.bits(omega.cpu().numpy()),
                              u.bits(oracle.aggregate_update_f32(wi, wv, n, d, 0.5, 1.0, omega0))), what

    reset()
    step()                                        # eager, also the first call on this device
    check("eager")
    reset()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        reset()                                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        check(f"replay {rep}")


def test_training_loop_replayed_from_one_graph_with_the_step_on_the_device():
    """Algorithm 1's loop as ONE captured graph replayed every iteration: the
    batched encode reads the step number from device memory
    (rtopk_encode_batch_device_step), the master's weight step uses the entry
    point that needs no workspace, and the last node of the graph advances the
    step. Residuals and weights carry over from replay to replay; only the
    gradients are refreshed (eagerly) in between. Every iteration must match
    the oracle run with step = 5, 6, 7, 8 on its own carried residuals: a
    graph that replayed one fixed step number would draw the same subset again
    and fail at the second iteration."""
    import torch
    import paper_2005_10761_amd as rt
    u = _u()
    dev = u.DEV
    n, d, first_step, iters = 3, 150_001, 5, 4
    wl = Workload(3, d=d)
    r, k = wl.r, wl.k
    seeds = [philox_seed_for_worker(w) for w in range(n)]
    stride = rt.encode_workspace_bytes(d, r, k)
    ws = torch.empty(n * stride, dtype=torch.uint8, device=dev)
    g = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
    m = [torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(n)]
    idx = torch.empty(n * k, dtype=torch.int32, device=dev)
    val = torch.empty(n * k, dtype=torch.float32, device=dev)
    oi = [idx[i * k:(i + 1) * k] for i in range(n)]
    ov = [val[i * k:(i + 1) * k] for i in range(n)]
    omega0 = np.random.default_rng(7).standard_normal(d).astype(np.float32)
    omega = torch.from_numpy(omega0).to(dev)
    step_dev = torch.full((1,), first_step, dtype=torch.int64, device=dev)
    eta, scale = 0.25, float(r) / float(k)

    def one_iteration():
        rt.encode_batch_device_step(g, m, r, k, seeds, step_dev, oi, ov, ws)
        rt.aggregate_update_static(idx, val, n, k, eta, scale, omega)
        step_dev.add_(1)

    # first use of the library's built-in scratch array outside the capture
    # (harmless values: a zero step leaves the weights as they are)
    rt.aggregate_update_static(torch.zeros(n * k, dtype=torch.int32, device=dev),
                               torch.zeros(n * k, dtype=torch.float32, device=dev), n, k, 0.0, 1.0,
                               omega.clone())
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_iteration()
    # the capture enqueued nothing: state is still the initial one
    assert int(step_dev.item()) == first_step

    ref_m = [np.zeros(d, np.float32) for _ in range(n)]
    ref_w = omega0
    for it in range(iters):
        t = first_step + it
        grads = [wl.gradient(w, t) for w in range(n)]
        for w in range(n):
            g[w].copy_(torch.from_numpy(grads[w]))            # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        msgs_i, msgs_v = [], []
        for w in range(n):
            wi, wv, ref_m[w] = oracle.encode(grads[w], ref_m[w], r, k, seeds[w], t)
            got = (oi[w].cpu().numpy().view(np.uint32), ov[w].cpu().numpy(), m[w].cpu().numpy())
            u.assert_encode_equal(got, (wi, wv, ref_m[w]), f"iteration {it} worker {w}")
            msgs_i.append(wi)
            msgs_v.append(wv)
        ref_w = oracle.aggregate_update_f32(np.concatenate(msgs_i), np.concatenate(msgs_v), n, d,
                                            eta, scale, ref_w)
        assert np.array_equal(u.bits(omega.cpu().numpy()), u.bits(ref_w)), it
        assert int(step_dev.item()) == t + 1
    # the same call issued eagerly with a 64-bit step on the device equals the by-value entry point
    big_step = 2 ** 40 + 3
    step_dev.fill_(big_step)
    m2 = [torch.from_numpy(x).to(dev) for x in ref_m]
    rt.encode_batch_device_step(g, m2, r, k, seeds, step_dev, oi, ov, ws)
    torch.cuda.synchronize()
    for w in range(n):
        wi, wv, wm = oracle.encode(grads[w], ref_m[w], r, k, seeds[w], big_step)
        got = (oi[w].cpu().numpy().view(np.uint32), ov[w].cpu().numpy(), m2[w].cpu().numpy())
        u.assert_encode_equal(got, (wi, wv, wm), f"64-bit device step, worker {w}")


def test_debug_build_checks_the_preconditions_of_the_master_entry_points():
    """The library built with RTOPK_DEBUG_CHECKS refuses a message with an index
    at or beyond d, or a slice that does not ascend, with RTOPK_EINVAL and
    writes nothing; a valid message gives the release build's bits."""
    import ctypes
    import os
    import torch
    import paper_2005_10761_amd as rt
    from paper_2005_10761_amd import build as hip_build
    u = _u()
    assert rt.load_library().rtopk_debug_checks() == 0
    assert os.path.exists(hip_build.DEBUG_LIB_PATH), "run __graft_entry__.build() first"
    dbg = ctypes.CDLL(hip_build.DEBUG_LIB_PATH)
    assert dbg.rtopk_debug_checks() == 1
    vp, u32, u64, f32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float
    dbg.rtopk_aggregate.argtypes = [vp, vp, u32, u64, u64, vp, vp, u64, vp]
    dbg.rtopk_aggregate_update_static.argtypes = [vp, vp, u32, u64, u64, f32, f32, vp, vp]
    dbg.rtopk_aggregate_update_momentum.argtypes = [vp, vp, u32, u64, u64, f32, f32, f32, vp, vp, vp]
    d, n, k = 10_000, 2, 4
    rng = np.random.default_rng(5)
    good = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = rng.standard_normal((n, k)).astype(np.float32)
    past_end = good.copy()
    past_end[1, k - 1] = d
    unsorted = good.copy()
    unsorted[0, 1], unsorted[0, 2] = good[0, 2], good[0, 1]
    tv = torch.from_numpy(val.reshape(-1)).to(u.DEV)
    omega = rng.standard_normal(d).astype(np.float32)
    for name, idx, want_rc in (("good", good, 0), ("index == d", past_end, -1),
                               ("descending pair", unsorted, -1)):
        ti = torch.from_numpy(idx.reshape(-1).view(np.int32)).to(u.DEV)
        out = torch.full((d,), 7.0, dtype=torch.float32, device=u.DEV)
        tw = torch.from_numpy(omega).to(u.DEV)
        tvel = torch.zeros(d, dtype=torch.float32, device=u.DEV)
        rc = dbg.rtopk_aggregate(ti.data_ptr(), tv.data_ptr(), n, k, d, out.data_ptr(), None, 0, None)
        rc2 = dbg.rtopk_aggregate_update_static(ti.data_ptr(), tv.data_ptr(), n, k, d, 0.5, 1.0,
                                                tw.data_ptr(), None)
        rc3 = dbg.rtopk_aggregate_update_momentum(ti.data_ptr(), tv.data_ptr(), n, k, d, 0.5, 1.0,
                                                  0.0, tw.clone().data_ptr(), tvel.data_ptr(), None)
        torch.cuda.synchronize()
        assert (rc, rc2, rc3) == (want_rc,) * 3, (name, rc, rc2, rc3)
        if want_rc == 0:
            assert np.array_equal(u.bits(out.cpu().numpy()), u.bits(oracle.aggregate_f32(idx, val, n, d)))
            assert np.array_equal(u.bits(tw.cpu().numpy()),
                                  u.bits(oracle.aggregate_update_f32(idx, val, n, d, 0.5, 1.0, omega)))
        else:
            assert bool((out == 7.0).all()) and np.array_equal(u.bits(tw.cpu().numpy()), u.bits(omega))


def test_streaming_calibration_kernel_adds_in_place():
    import torch
    import paper_2005_10761_amd as rt
    u = _u()
    rng = np.random.default_rng(1)
    for d in (1, 255, 1024, 70_001, 3_000_017):
        g = rng.standard_normal(d).astype(np.float32)
        m = rng.standard_normal(d).astype(np.float32)
        tg, tm = torch.from_numpy(g).to(u.DEV), torch.from_numpy(m).to(u.DEV)
        rt.diag_stream_add(tg, tm)
        torch.cuda.synchronize()
        assert np.array_equal(u.bits(tm.cpu().numpy()), u.bits(g + m)), d
