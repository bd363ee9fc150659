"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is checked against things it does not itself define: published
known answers of the generator, a definition-level brute force on tiny
inputs, special cases that reduce to library routines (stable argsort,
torch.topk), exact invariants of Algorithm 1, the closed form in the proof
that rTop-k is a compression operator, and the inclusion probabilities that
Definition 3's uniform k-subset implies.
"""
import itertools
import os

import numpy as np
import pytest
from scipy import stats

import oracle
from tests import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


# --------------------------------------------------------------------------
# generator
# --------------------------------------------------------------------------
def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], tuple(w[6:10])))
    assert len(rows) == 3
    return rows


@pytest.mark.parametrize("ctr,key,expect", _kat_rows())
def test_philox_known_answers(ctr, key, expect):
    assert oracle.philox4x32_10(ctr, key) == expect
    assert brute.philox4x32_10(ctr, key) == expect


def test_key64_layout_matches_independent_typing():
    # counter = (index, 0, step_lo, step_hi), key = (seed_lo, seed_hi),
    # K = out0 << 32 | out1 -- including seeds and steps above 2^32
    rng = np.random.default_rng(7)
    for _ in range(200):
        seed = int(rng.integers(0, 1 << 63)) * 2 + int(rng.integers(0, 2))
        step = int(rng.integers(0, 1 << 63)) * 2 + int(rng.integers(0, 2))
        index = int(rng.integers(0, 1 << 32))
        assert oracle.key64(seed, step, index) == brute.key64(seed, step, index)
    o = oracle.philox4x32_10((5, 0, 9, 0), (42, 0))
    assert oracle.key64(42, 9, 5) == (o[0] << 32) | o[1]


# --------------------------------------------------------------------------
# brute force on tiny d: every (r, k), ties, signed zeros, denormals
# --------------------------------------------------------------------------
ALPHABET = np.array([0.0, -0.0, 1.0, -1.0, 1.0, 2.0, -2.0, 0.5, 1e-45, -1e-45, 3.5, -3.5],
                    dtype=np.float32)


@pytest.mark.parametrize("d", [1, 2, 5, 8])
def test_encode_equals_brute_force(d):
    rng = np.random.default_rng(100 + d)
    n_vec = 12 if d == 8 else 20
    for trial in range(n_vec):
        g = ALPHABET[rng.integers(0, ALPHABET.size, d)]
        m = ALPHABET[rng.integers(0, ALPHABET.size, d)] if trial % 2 else np.zeros(d, np.float32)
        for r in range(1, d + 1):
            for k in range(1, r + 1):
                seed = int(rng.integers(0, 1 << 40))
                step = int(rng.integers(0, 1 << 34))
                oi, ov, om = oracle.encode(g, m, r, k, seed, step)
                bi, bv, bm = brute.encode(g, m, r, k, seed, step)
                assert np.array_equal(oi, bi), (g, m, r, k, seed, step)
                assert np.array_equal(bits(ov), bits(bv))
                assert np.array_equal(bits(om), bits(bm))


def test_top_r_equals_brute_force_with_heavy_ties():
    rng = np.random.default_rng(5)
    small = np.array([0.0, -0.0, 1.0, -1.0, 2.0], dtype=np.float32)
    for _ in range(60):
        d = int(rng.integers(1, 10))
        a = small[rng.integers(0, small.size, d)]
        for r in range(1, d + 1):
            got = oracle.top_r(a, r)
            assert tuple(sorted(got.tolist())) == brute.top_r_set(a.tolist(), r)
            # pi itself: non-increasing magnitude, index ascending inside ties
            mags = [brute.mag_bits(float(a[i])) for i in got]
            assert all(mags[j] > mags[j + 1] or (mags[j] == mags[j + 1] and got[j] < got[j + 1])
                       for j in range(r - 1))


# --------------------------------------------------------------------------
# special cases that reduce to library routines
# --------------------------------------------------------------------------
def test_r_equals_k_is_top_k_stable_argsort():
    rng = np.random.default_rng(11)
    d = 5000
    g = rng.standard_normal(d).astype(np.float32)
    g[rng.integers(0, d, 500)] = 0.25          # ties
    g[rng.integers(0, d, 500)] = -0.25
    m = rng.standard_normal(d).astype(np.float32) * 0.1
    a = g + m
    mag = bits(a) & 0x7FFFFFFF
    order = np.argsort(-(mag.astype(np.int64)), kind="stable")
    for k in (1, 17, 400, 4999, 5000):
        oi, ov, om = oracle.encode(g, m, k, k, 3, 4)
        assert np.array_equal(oi, np.sort(order[:k]).astype(np.uint32))
        assert np.array_equal(bits(ov), bits(a[oi]))


def test_top_r_matches_torch_topk_on_distinct_magnitudes():
    import torch
    rng = np.random.default_rng(12)
    d = 20000
    mags = rng.permutation(d).astype(np.float32) + 1.0
    a = mags * rng.choice([-1.0, 1.0], d).astype(np.float32)
    for r in (1, 10, 777, d):
        want = torch.topk(torch.from_numpy(np.abs(a)), r).indices.numpy()
        got = oracle.top_r(a, r)
        assert np.array_equal(got, want.astype(np.uint32))


def test_r_equals_d_is_random_k_over_all_coordinates():
    rng = np.random.default_rng(13)
    d = 48
    g = rng.standard_normal(d).astype(np.float32)
    m = np.zeros(d, np.float32)
    for k in (1, 7, 47, 48):
        for seed, step in ((42, 0), (42, 1), (1 << 35, 1 << 33)):
            oi, _, _ = oracle.encode(g, m, d, k, seed, step)
            assert oi.tolist() == brute.random_k_subset(range(d), k, seed, step)


# --------------------------------------------------------------------------
# invariants of Definition 3 and Algorithm 1
# --------------------------------------------------------------------------
@pytest.mark.parametrize("d,r,k", [(1000, 100, 10), (4097, 41, 41), (333, 333, 5), (64, 1, 1)])
def test_invariants(d, r, k):
    rng = np.random.default_rng(d + r + k)
    g = (rng.standard_normal(d) * 10.0 ** rng.uniform(-3, 0, d)).astype(np.float32)
    g[rng.integers(0, d, d // 10)] = 0.0
    m = (rng.standard_normal(d) * 1e-2).astype(np.float32)
    a = g + m
    idx, val, m2 = oracle.encode(g, m, r, k, 99, 5)
    assert idx.size == k and np.all(np.diff(idx.astype(np.int64)) > 0)
    top = set(oracle.top_r(a, r).tolist())
    assert set(idx.tolist()) <= top
    # top-r set dominates its complement
    mag = (bits(a) & 0x7FFFFFFF).astype(np.int64)
    inside = np.zeros(d, bool)
    inside[list(top)] = True
    if r < d:
        assert mag[inside].min() >= mag[~inside].max()
        thr = mag[inside].min()
        tie_in = np.flatnonzero(inside & (mag == thr))
        tie_out = np.flatnonzero(~inside & (mag == thr))
        if tie_out.size:
            assert tie_in.max() < tie_out.min()
    # values pass through unmodified; memory holds exactly what was not sent
    assert np.array_equal(bits(val), bits(a[idx]))
    sent = np.zeros(d, bool)
    sent[idx] = True
    assert np.array_equal(bits(m2[~sent]), bits(a[~sent]))
    assert np.all(bits(m2[sent]) == 0)
    ghat = np.zeros(d, np.float32)
    ghat[idx] = val
    assert np.all(m2 + ghat == a)              # m^{t+1} + ghat^t = g^t + m^t


def test_domain_of_definition_3_is_enforced():
    g = np.ones(8, np.float32)
    m = np.zeros(8, np.float32)
    for r, k in ((4, 0), (4, 5), (9, 2), (0, 0)):
        with pytest.raises(ValueError):
            oracle.encode(g, m, r, k, 1, 1)


def test_memory_makes_a_small_constant_gradient_get_sent():
    # error compensation: what is not sent is carried over, so a persistent
    # small component keeps growing in memory until it is selected.
    rng = np.random.default_rng(21)
    d, r, k, j = 200, 10, 5, 7
    m = np.zeros(d, np.float32)
    sent_at = None
    for t in range(4000):
        g = rng.standard_normal(d).astype(np.float32)
        g[j] = 0.05
        idx, val, m = oracle.encode(g, m, r, k, 1, t)
        if j in idx.tolist():
            sent_at = t
            break
    assert sent_at is not None and sent_at > 5
    assert m[j] == 0.0


# --------------------------------------------------------------------------
# uniformity of U (Definition 3) and the compression-operator closed form
# --------------------------------------------------------------------------
def _inclusion_counts(vary, n_draws, d=256, r=64, k=16):
    rng = np.random.default_rng(31)
    base = rng.permutation(d).astype(np.float32) + 1.0
    a = base * rng.choice([-1.0, 1.0], d).astype(np.float32)
    top = np.sort(oracle.top_r(a, r))
    pos = {int(i): p for p, i in enumerate(top)}
    m = np.zeros(d, np.float32)
    single = np.zeros(r, np.int64)
    pair = np.zeros((r, r), np.int64)
    for t in range(n_draws):
        seed, step = (1000 + t, 3) if vary == "seed" else (77, t)
        idx, _, _ = oracle.encode(a, m, r, k, seed, step)
        p = np.array([pos[int(i)] for i in idx])
        single[p] += 1
        pair[np.ix_(p, p)] += 1
    return single, pair


@pytest.mark.parametrize("vary", ["seed", "step"])
def test_each_top_r_member_is_included_with_probability_k_over_r(vary):
    r, k, N = 64, 16, 20000
    single, pair = _inclusion_counts(vary, N, r=r, k=k)
    assert single.sum() == N * k
    p = k / r
    # for a fixed-size uniform subset the inclusion counts have covariance
    # that shrinks the Pearson statistic by (r-1)/r; then it is ~ chi2(r-1)
    x2 = ((r - 1) / r) * np.sum((single - N * p) ** 2) / (N * p * (1 - p))
    lo, hi = stats.chi2.ppf([1e-5, 1 - 1e-5], r - 1)
    assert lo < x2 < hi, x2
    # pairs: P(i and j both in U) = k(k-1) / (r(r-1))
    off = pair[~np.eye(r, dtype=bool)]
    pp = k * (k - 1) / (r * (r - 1))
    z = (off - N * pp) / np.sqrt(N * pp * (1 - pp))
    assert np.abs(z).max() < 6.0
    assert abs(off.mean() / N - pp) < 1e-9     # exact: every draw has k(k-1) ordered pairs


def test_expected_squared_error_matches_closed_form():
    # proof that rTop-k is a compression operator:
    # E||w - rTop_k(w)||^2 = (1 - k/r) sum_{j<=r} w_j^2 + sum_{j>r} w_j^2 <= (1 - k/d)||w||^2
    rng = np.random.default_rng(41)
    d, r, k, N = 400, 50, 10, 6000
    w = (rng.standard_normal(d) * 10.0 ** rng.uniform(-2, 0, d)).astype(np.float32)
    m = np.zeros(d, np.float32)
    w64 = w.astype(np.float64)
    srt = np.sort(w64 ** 2)[::-1]
    closed = (1 - k / r) * srt[:r].sum() + srt[r:].sum()
    assert closed <= (1 - k / d) * (w64 ** 2).sum() + 1e-12
    errs = np.empty(N)
    mean_vec = np.zeros(d)
    for t in range(N):
        idx, val, _ = oracle.encode(w, m, r, k, 5000 + t, 0)
        gh = np.zeros(d)
        gh[idx] = val
        errs[t] = ((w64 - gh) ** 2).sum()
        mean_vec += gh
    se = errs.std(ddof=1) / np.sqrt(N)
    assert abs(errs.mean() - closed) < 5 * se, (errs.mean(), closed, se)
    # E[rTop_k(w)] = (k/r) top_r(w)
    top = oracle.top_r(w, r)
    want = np.zeros(d)
    want[top] = w64[top] * k / r
    sd = np.sqrt((k / r) * (1 - k / r) / N) * np.abs(w64) + 1e-12
    assert np.all(np.abs(mean_vec / N - want) < 6 * sd)


# --------------------------------------------------------------------------
# master: ghat = (1/n) sum_i ghat_i
# --------------------------------------------------------------------------
def test_aggregate_single_worker_is_a_scatter():
    d = 50
    idx = np.array([3, 9, 10, 49], np.uint32)
    val = np.array([1.5, -2.0, 1e-40, 7.0], np.float32)
    for fn in (oracle.aggregate, oracle.aggregate_f32):
        out = fn(idx, val, 1, d)
        want = np.zeros(d, np.float32)
        want[idx] = val
        assert np.array_equal(bits(out), bits(want))


def test_aggregate_disjoint_supports_divide_by_n_not_by_senders():
    d, n, k = 64, 4, 3
    idx = np.arange(n * k, dtype=np.uint32)
    val = (np.arange(n * k) + 1).astype(np.float32)
    for fn in (oracle.aggregate, oracle.aggregate_f32):
        out = fn(idx, val, n, d)
        want = np.zeros(d, np.float32)
        want[idx] = val / np.float32(n)
        assert np.array_equal(out, want)
        assert np.all(out[n * k:] == 0)


def test_aggregate_identical_messages_power_of_two_n_returns_the_value():
    d, n = 32, 8
    one_idx = np.array([1, 5, 30], np.uint32)
    one_val = np.array([0.1, -3.3, 1e-3], np.float32)
    idx = np.tile(one_idx, n)
    # binary64 accumulation of 8 binary32 values is exact, so the mean is v
    out = oracle.aggregate(idx, np.tile(one_val, n), n, d)
    assert np.array_equal(out[one_idx], one_val)
    # in binary32 the partial sums 3v, 5v, ... round unless v has a short mantissa
    short_val = np.array([0.5, -3.25, 96.0], np.float32)
    out = oracle.aggregate_f32(idx, np.tile(short_val, n), n, d)
    assert np.array_equal(out[one_idx], short_val)


def test_aggregate_equals_dense_mean_and_f32_variant_is_close():
    rng = np.random.default_rng(51)
    d, n, k = 300, 5, 40
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = rng.standard_normal((n, k)).astype(np.float32)
    dense = np.zeros((n, d), np.float64)
    for w in range(n):
        dense[w, idx[w]] = val[w]
    want = dense.sum(axis=0) / n                     # the formula, on dense vectors
    abs_sum = np.abs(dense).sum(axis=0) / n
    out64 = oracle.aggregate(idx, val, n, d)
    out32 = oracle.aggregate_f32(idx, val, n, d)
    assert np.array_equal(out64, want.astype(np.float32))
    tol = 1e-6 * np.maximum(np.abs(want), abs_sum)
    assert np.all(np.abs(out32.astype(np.float64) - want) <= tol)
    untouched = np.setdiff1d(np.arange(d), idx.reshape(-1))
    assert np.all(bits(out64[untouched]) == 0) and np.all(bits(out32[untouched]) == 0)


def test_aggregate_f32_divides_by_n_with_one_correct_rounding():
    # a coordinate sent by exactly one of n workers must come out as the
    # correctly rounded quotient v / n (not v times a rounded reciprocal)
    rng = np.random.default_rng(52)
    k = 4000
    for n in (3, 5, 7, 11):
        d = n * k
        idx = np.arange(d, dtype=np.uint32)
        val = (rng.standard_normal(d) * 10.0 ** rng.uniform(-6, 3, d)).astype(np.float32)
        want = (val.astype(np.float64) / n).astype(np.float32)
        assert np.any(want != val * (np.float32(1.0) / np.float32(n)))
        for fn in (oracle.aggregate, oracle.aggregate_f32):
            assert np.array_equal(bits(fn(idx, val, n, d)), bits(want))


def test_aggregate_rejects_out_of_range_index():
    with pytest.raises(ValueError):
        oracle.aggregate(np.array([4], np.uint32), np.array([1.0], np.float32), 1, 4)


def test_encode_then_aggregate_matches_brute_force_end_to_end():
    rng = np.random.default_rng(61)
    d, r, k, n = 9, 5, 2, 3
    res = [np.zeros(d, np.float32) for _ in range(n)]
    for t in range(3):
        msgs_i, msgs_v, dense = [], [], np.zeros(d, np.float64)
        for w in range(n):
            g = rng.standard_normal(d).astype(np.float32)
            bi, bv, bm = brute.encode(g, res[w], r, k, 42 + w, t)
            oi, ov, om = oracle.encode(g, res[w], r, k, 42 + w, t)
            assert np.array_equal(oi, bi) and np.array_equal(bits(om), bits(bm))
            res[w] = om
            msgs_i.append(oi)
            msgs_v.append(ov)
            dense[bi] += bv.astype(np.float64)
        out = oracle.aggregate(np.concatenate(msgs_i), np.concatenate(msgs_v), n, d)
        assert np.array_equal(out, (dense / n).astype(np.float32))


# --------------------------------------------------------------------------
# master, both lines: omega <- omega - eta * scale * (1/n) sum_i ghat_i
# --------------------------------------------------------------------------
def test_aggregate_update_worked_example_by_hand():
    # two workers, six weights, all numbers dyadic so that every step is exact:
    # worker 0 sends (1, 0.5), (4, -2); worker 1 sends (1, 1.5), (3, 4)
    # mean = [0, 1, 0, 2, -1, 0]
    idx = np.array([1, 4, 1, 3], np.uint32)
    val = np.array([0.5, -2.0, 1.5, 4.0], np.float32)
    omega = np.array([1, 2, 3, 4, 5, 6], np.float32)
    for fn in (oracle.aggregate_update, oracle.aggregate_update_f32):
        # eta = 1/2, as printed in Algorithm 1 (scale 1)
        assert np.array_equal(fn(idx, val, 2, 6, 0.5, 1.0, omega),
                              np.array([1, 1.5, 3, 3, 5.5, 6], np.float32))
        # the same with what was kept divided by a kept fraction of 1/2
        assert np.array_equal(fn(idx, val, 2, 6, 0.5, 2.0, omega),
                              np.array([1, 1, 3, 2, 6, 6], np.float32))
        # a step against the gradient direction's sign: eta < 0 moves the other way
        assert np.array_equal(fn(idx, val, 2, 6, -0.25, 1.0, omega),
                              np.array([1, 2.25, 3, 4.5, 4.75, 6], np.float32))


def test_aggregate_update_reduces_to_the_average_and_to_the_identity():
    rng = np.random.default_rng(71)
    d, n, k = 500, 6, 30
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = rng.standard_normal((n, k)).astype(np.float32)
    omega = rng.standard_normal(d).astype(np.float32)
    omega[::7] = -0.0
    zero = np.zeros(d, np.float32)
    # from zero weights with eta = -1 the update is the average itself
    assert np.array_equal(oracle.aggregate_update(idx, val, n, d, -1.0, 1.0, zero),
                          oracle.aggregate(idx, val, n, d))
    assert np.array_equal(oracle.aggregate_update_f32(idx, val, n, d, -1.0, 1.0, zero),
                          oracle.aggregate_f32(idx, val, n, d))
    # eta = 0 leaves every weight as it is; so does a coordinate nobody sent
    assert np.array_equal(oracle.aggregate_update(idx, val, n, d, 0.0, 1.0, omega), omega)
    out32 = oracle.aggregate_update_f32(idx, val, n, d, 0.3, 5.0, omega)
    out64 = oracle.aggregate_update(idx, val, n, d, 0.3, 5.0, omega)
    untouched = np.setdiff1d(np.arange(d), idx.reshape(-1))
    assert np.array_equal(bits(out32[untouched]), bits(omega[untouched]))
    assert np.array_equal(bits(out64[untouched]), bits(omega[untouched]))
    touched = np.unique(idx.reshape(-1))
    assert np.all(out64[touched] != omega[touched])


def test_aggregate_update_equals_the_dense_formula_and_f32_variant_is_close():
    rng = np.random.default_rng(72)
    d, n, k = 400, 5, 60
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = (rng.standard_normal((n, k)) * 10.0 ** rng.uniform(-3, 1, (n, k))).astype(np.float32)
    omega = rng.standard_normal(d).astype(np.float32)
    eta, scale = float(np.float32(0.05)), float(np.float32(2.5))
    dense = np.zeros((n, d), np.float64)
    for w in range(n):
        for j in range(k):                           # ghat_w as a dense vector, entry by entry
            dense[w, idx[w, j]] += float(val[w, j])
    ghat = dense.sum(axis=0) / n
    want = omega.astype(np.float64) - eta * scale * ghat
    out64 = oracle.aggregate_update(idx, val, n, d, eta, scale, omega)
    assert np.array_equal(out64, want.astype(np.float32))
    out32 = oracle.aggregate_update_f32(idx, val, n, d, eta, scale, omega)
    size = np.abs(omega.astype(np.float64)) + eta * scale * np.abs(dense).sum(axis=0) / n
    assert np.all(np.abs(out32.astype(np.float64) - want) <= 1e-6 * size)
    # the order of the two scalars matters to nobody: (eta, scale) and (eta * scale, 1)
    swapped = oracle.aggregate_update(idx, val, n, d, eta * scale, 1.0, omega)
    assert np.array_equal(swapped, out64)


def test_aggregate_update_f32_uses_one_rounding_for_multiply_and_subtract():
    # omega = 1, mean = 1 + 2^-12, c = 1 + 2^-12: the product 1 + 2^-11 + 2^-24
    # needs 25 bits. Fused: 1 - that = -(2^-11 + 2^-24), exact in binary32.
    # A rounded product (1 + 2^-11, the tie goes to even) would give -2^-11.
    v = np.float32(1.0 + 2.0 ** -12)
    out = oracle.aggregate_update_f32(np.array([0], np.uint32), np.array([v], np.float32), 1, 1,
                                      float(v), 1.0, np.array([1.0], np.float32))
    assert float(out[0]) == -(2.0 ** -11 + 2.0 ** -24)
    out64 = oracle.aggregate_update(np.array([0], np.uint32), np.array([v], np.float32), 1, 1,
                                    float(v), 1.0, np.array([1.0], np.float32))
    assert float(out64[0]) == -(2.0 ** -11 + 2.0 ** -24)


def test_scale_r_over_k_makes_the_sent_vector_unbiased_for_the_top_r_part():
    # The estimator in the proof of the estimation upper bound divides the
    # subsampled vector by its subsampling fraction. Here the fraction is k/r:
    # over many independent draws (steps) the mean of (r/k) * rTop_k(x) must
    # approach top_r(x). One worker, zero weights, eta = -1: the update is
    # scale * ghat.
    rng = np.random.default_rng(73)
    d, r, k, N = 120, 40, 8, 3000
    x = rng.standard_normal(d).astype(np.float32)
    top = oracle.top_r(x, r)
    want = np.zeros(d, np.float64)
    want[top] = x[top]
    acc = np.zeros(d, np.float64)
    zero = np.zeros(d, np.float32)
    for t in range(N):
        oi, ov, _ = oracle.encode(x, zero, r, k, 99, t)
        acc += oracle.aggregate_update(oi, ov, 1, d, -1.0, r / k, zero)
    sd = np.sqrt((r / k - 1.0) / N) * np.abs(want)   # sd of the mean of (r/k) * x * Bernoulli(k/r)
    assert np.all(np.abs(acc / N - want) <= 6 * sd)
    assert np.any(np.abs(acc / N - want * k / r) > 6 * sd)   # and the unscaled mean is not


def test_aggregate_update_rejects_out_of_range_index_and_wrong_length():
    one = np.array([1.0], np.float32)
    with pytest.raises(ValueError):
        oracle.aggregate_update(np.array([4], np.uint32), one, 1, 4, 0.1, 1.0, np.zeros(4, np.float32))
    with pytest.raises(ValueError):
        oracle.aggregate_update(np.array([1], np.uint32), one, 1, 4, 0.1, 1.0, np.zeros(3, np.float32))


def test_aggregate_update_binary64_is_the_master_line_for_every_coordinate():
    # Algorithm 1's master lines, omega - eta * ghat, are applied to every
    # coordinate, also where ghat = 0: nobody sent coordinate 1 and the two
    # entries at 2 cancel. A negative zero stays (-0 - (+0) = -0) with a
    # positive step and becomes +0 with a negative one (-0 - (-0) = +0); a
    # signalling not-a-number comes out quiet, as from any arithmetic operation.
    omega = np.array([1.0, 0.0, -0.0, 4.0], np.float32)
    omega.view(np.uint32)[1] = 0x7FA00001
    idx = np.array([0, 2, 2, 3], np.uint32)
    val = np.array([1.0, 2.5, -2.5, 2.0], np.float32)
    out = oracle.aggregate_update(idx, val, 2, 4, 0.5, 1.0, omega)
    assert list(bits(out)) == [bits(np.float32(0.75)), 0x7FE00001, 0x80000000,
                               bits(np.float32(3.5))]
    out = oracle.aggregate_update(idx, val, 2, 4, -0.5, 1.0, omega)
    assert list(bits(out)) == [bits(np.float32(1.25)), 0x7FE00001, 0x00000000,
                               bits(np.float32(4.5))]


def test_aggregate_update_f32_copies_coordinates_the_average_does_not_move():
    # the binary32 reading: where the average is zero the weight keeps its
    # bits, a signalling not-a-number and a negative zero included, whatever
    # the sign of the step; nobody sent coordinate 1, the two entries at 2 cancel
    omega = np.array([1.0, 0.0, -0.0, 4.0], np.float32)
    omega.view(np.uint32)[1] = 0x7FA00001
    idx = np.array([0, 2, 2, 3], np.uint32)
    val = np.array([1.0, 2.5, -2.5, 2.0], np.float32)
    out = oracle.aggregate_update_f32(idx, val, 2, 4, 0.5, 1.0, omega)
    assert list(bits(out)) == [bits(np.float32(0.75)), 0x7FA00001, 0x80000000,
                               bits(np.float32(3.5))]
    out = oracle.aggregate_update_f32(idx, val, 2, 4, -0.5, 1.0, omega)
    assert list(bits(out)) == [bits(np.float32(1.25)), 0x7FA00001, 0x80000000,
                               bits(np.float32(4.5))]
    # the test is on the AVERAGE: a sum of 2^-149 divided by 3 rounds to zero,
    # so the weight is copied although something was sent for it
    tiny = np.array([2.0 ** -149], np.float32)
    w = np.array([0.0], np.float32)
    w.view(np.uint32)[0] = 0x7FA00001
    out = oracle.aggregate_update_f32(np.array([0, 0, 0], np.uint32),
                                      np.array([tiny[0], 0.0, 0.0], np.float32), 3, 1, 1.0, 1.0, w)
    assert int(bits(out)[0]) == 0x7FA00001
    # ... while with n = 1 the same entry moves a weight: 0 + 2^-149
    out = oracle.aggregate_update_f32(np.array([0], np.uint32), tiny, 1, 1, -1.0, 1.0,
                                      np.zeros(1, np.float32))
    assert int(bits(out)[0]) == 1


# --------------------------------------------------------------------------
# order of the binary32 additions: from +0, workers 0, 1, 2, ..., entries of
# one message in position order
# --------------------------------------------------------------------------
def test_f32_sums_add_workers_in_order_from_zero():
    # One coordinate sent by three workers: 2^24, 1, -2^24. In worker order
    # fl(2^24 + 1) = 2^24 (the tie goes to even), then - 2^24 = 0: average 0.
    # Backwards, fl(-2^24 + 1) = -(2^24 - 1) is exact, + 2^24 = 1: average 1/3.
    # (1, 2^24, -2^24) in order also gives 0; (2^24, -2^24, 1) gives 1/3: so
    # neither a reversed nor a rotated order passes all three cases.
    big = np.float32(2.0 ** 24)
    third = np.float32(1.0) / np.float32(3.0)
    d = 5
    idx = np.array([3, 3, 3], np.uint32)
    cases = [((big, 1.0, -big), 0.0), ((1.0, big, -big), 0.0), ((big, -big, 1.0), third),
             ((-big, 1.0, big), third)]
    for vals, want in cases:
        val = np.array(vals, np.float32)
        out = oracle.aggregate_f32(idx, val, 3, d)
        assert float(out[3]) == float(want), (vals, out[3])
        assert np.all(bits(np.delete(out, 3)) == 0)
        # binary64 holds every partial sum exactly: always 1/3, correctly rounded
        assert float(oracle.aggregate(idx, val, 3, d)[3]) == float(np.float32(1.0 / 3.0))
        # the weight step built on the same sum: omega = 1, eta = -1 adds the average
        one = np.ones(d, np.float32)
        upd = oracle.aggregate_update_f32(idx, val, 3, d, -1.0, 1.0, one)
        assert float(upd[3]) == float(np.float32(1.0) + np.float32(want))
        # ... and with momentum from rest (mu = 0): velocity = the average
        w, v = oracle.aggregate_update_momentum_f32(idx, val, 3, d, -1.0, 1.0, 0.0, one,
                                                    np.zeros(d, np.float32))
        assert float(v[3]) == float(want) and float(w[3]) == float(np.float32(1.0) + np.float32(want))


def test_f32_sums_add_the_entries_of_one_message_in_position_order():
    # the same index three times inside ONE message (never produced by the
    # encoder, but defined: it is added again), next to a second worker
    big = np.float32(2.0 ** 24)
    idx = np.array([2, 2, 2, 0, 1, 4], np.uint32)        # worker 0: 2, 2, 2; worker 1: 0, 1, 4
    for vals, want in (((big, 1.0, -big), 0.0), ((-big, 1.0, big), 0.5)):
        val = np.array(list(vals) + [8.0, 8.0, 8.0], np.float32)
        out = oracle.aggregate_f32(idx, val, 2, 5)
        assert [float(x) for x in out] == [4.0, 4.0, want, 0.0, 4.0]


def test_f32_sum_starts_from_positive_zero():
    # -0 sent by every worker: +0 + (-0) = +0, so the average is +0, not -0
    idx = np.array([1, 1], np.uint32)
    val = np.array([-0.0, -0.0], np.float32)
    assert list(bits(oracle.aggregate_f32(idx, val, 2, 3))) == [0, 0, 0]


# --------------------------------------------------------------------------
# master with momentum: v <- mu v + scale * ghat ; omega <- omega - eta v
# --------------------------------------------------------------------------
def test_momentum_update_worked_example_by_hand():
    # the hand example of the plain update, with a velocity: mean = [0, 1, 0, 2, -1, 0]
    idx = np.array([1, 4, 1, 3], np.uint32)
    val = np.array([0.5, -2.0, 1.5, 4.0], np.float32)
    omega = np.array([1, 2, 3, 4, 5, 6], np.float32)
    vel = np.array([2, 0, -4, 1, 0, 8], np.float32)
    for fn in (oracle.aggregate_update_momentum, oracle.aggregate_update_momentum_f32):
        w, v = fn(idx, val, 2, 6, 0.5, 1.0, 0.5, omega, vel)
        # v' = 0.5 v + mean = [1, 1, -2, 2.5, -1, 4]; w' = w - 0.5 v'
        assert np.array_equal(v, np.array([1, 1, -2, 2.5, -1, 4], np.float32))
        assert np.array_equal(w, np.array([0.5, 1.5, 4, 2.75, 5.5, 4], np.float32))
        w, v = fn(idx, val, 2, 6, 0.25, 2.0, 0.0, omega, vel)
        # mu = 0, scale = 2: v' = 2 mean; w' = w - 0.25 v'
        assert np.array_equal(v, np.array([0, 2, 0, 4, -2, 0], np.float32))
        assert np.array_equal(w, np.array([1, 1.5, 3, 3, 5.5, 6], np.float32))


def test_momentum_update_reduces_to_the_plain_update_and_matches_the_closed_form():
    rng = np.random.default_rng(81)
    d, n, k = 300, 4, 40
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = rng.standard_normal((n, k)).astype(np.float32)
    omega = rng.standard_normal(d).astype(np.float32)
    zero = np.zeros(d, np.float32)
    eta, scale = float(np.float32(0.125)), 2.0            # dyadic: eta * scale is exact
    # mu = 0: the weights move as in the plain update, whatever the old velocity was
    w, v = oracle.aggregate_update_momentum(idx, val, n, d, eta, scale, 0.0, omega,
                                            rng.standard_normal(d).astype(np.float32))
    assert np.array_equal(w, oracle.aggregate_update(idx, val, n, d, eta, scale, omega))
    assert np.array_equal(v, (scale * oracle.aggregate(idx, val, n, d).astype(np.float64))
                          .astype(np.float32))
    # the same message T times from rest: v_T = g (1 - mu^T) / (1 - mu),
    # w_T = w_0 - eta g (T - mu (1 - mu^T) / (1 - mu)) / (1 - mu)
    mu, T = 0.5, 6
    g = scale * oracle.aggregate(idx, val, n, d).astype(np.float64)
    w, v = omega.astype(np.float64), zero.astype(np.float64)
    w32, v32 = omega, zero
    for _ in range(T):
        w32, v32 = oracle.aggregate_update_momentum(idx, val, n, d, eta, scale, mu, w32, v32)
    v_T = g * (1 - mu ** T) / (1 - mu)
    w_T = omega.astype(np.float64) - eta * g * (T - mu * (1 - mu ** T) / (1 - mu)) / (1 - mu)
    assert np.allclose(v32, v_T, rtol=1e-6, atol=1e-7)
    assert np.allclose(w32, w_T, rtol=1e-5, atol=1e-6)
    # nothing sent anywhere near coordinate i: the velocity only decays there
    untouched = np.setdiff1d(np.arange(d), idx.reshape(-1))
    vel = rng.standard_normal(d).astype(np.float32)
    w, v = oracle.aggregate_update_momentum(idx, val, n, d, eta, scale, 0.25, omega, vel)
    assert np.array_equal(v[untouched], (0.25 * vel[untouched].astype(np.float64)).astype(np.float32))
    assert np.array_equal(w[untouched], (omega[untouched].astype(np.float64)
                                         - eta * 0.25 * vel[untouched].astype(np.float64))
                          .astype(np.float32))


def test_momentum_update_f32_variant_is_close_and_uses_the_stored_velocity():
    rng = np.random.default_rng(82)
    d, n, k = 400, 5, 60
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = (rng.standard_normal((n, k)) * 10.0 ** rng.uniform(-3, 1, (n, k))).astype(np.float32)
    omega = rng.standard_normal(d).astype(np.float32)
    vel = rng.standard_normal(d).astype(np.float32)
    eta, scale, mu = float(np.float32(0.05)), float(np.float32(2.5)), float(np.float32(0.9))
    w64, v64 = oracle.aggregate_update_momentum(idx, val, n, d, eta, scale, mu, omega, vel)
    w32, v32 = oracle.aggregate_update_momentum_f32(idx, val, n, d, eta, scale, mu, omega, vel)
    dense = np.zeros(d)
    np.add.at(dense, idx.reshape(-1).astype(np.int64), np.abs(val.reshape(-1).astype(np.float64)) / n)
    size_v = mu * np.abs(vel.astype(np.float64)) + scale * dense
    assert np.all(np.abs(v32.astype(np.float64) - v64) <= 1e-6 * size_v + 1e-30)
    assert np.all(np.abs(w32.astype(np.float64) - w64)
                  <= 1e-6 * (np.abs(omega.astype(np.float64)) + eta * size_v) + 1e-30)
    # the weight step uses the velocity as stored (rounded to binary32)
    want_w = np.array([np.float32(float(omega[i]) - eta * float(v32[i])) for i in range(d)])
    assert np.all(np.abs(w32.astype(np.float64) - want_w) <= 6e-8 * (np.abs(want_w) + 1e-30) + 1e-37)


def test_momentum_update_f32_uses_one_rounding_per_fused_step():
    x = np.float32(1.0 + 2.0 ** -12)      # x * x = 1 + 2^-11 + 2^-24 needs 25 bits
    one_idx, one_val = np.array([0], np.uint32), np.array([-1.0], np.float32)
    # velocity step: mu * v + u with mu = v = x, u = -1 -> 2^-11 + 2^-24 exactly when fused
    w, v = oracle.aggregate_update_momentum_f32(one_idx, one_val, 1, 1, 0.0, 1.0, float(x),
                                                np.array([5.0], np.float32), np.array([x]))
    assert float(v[0]) == 2.0 ** -11 + 2.0 ** -24 and float(w[0]) == 5.0
    # weight step: w - eta * v' with eta = v' = x (mu = 0, the message is x), w = 1
    w, v = oracle.aggregate_update_momentum_f32(one_idx, np.array([x]), 1, 1, float(x), 1.0, 0.0,
                                                np.array([1.0], np.float32), np.array([9.0], np.float32))
    assert float(v[0]) == float(x) and float(w[0]) == -(2.0 ** -11 + 2.0 ** -24)
