"""Host-side checks of the synthetic input generators (no GPU)."""
import numpy as np

from workloads import CONFIGS, Workload, ceil_fraction


def test_counts_follow_the_printed_configuration():
    # the first benchmark configuration prints r = 10,486 and k = 1,049 for
    # d = 2^20: the ceilings of 1% and 0.1% of d
    w = Workload(1)
    assert (w.d, w.r, w.k) == (1 << 20, 10486, 1049)
    assert ceil_fraction(25_557_032, 5, 1000) == 127_786
    assert ceil_fraction(25_557_032, 1, 1000) == 25_558
    # Section IV's example: 99.9% compression with n = 5 nodes is k = 0.1% d,
    # r = 0.5% d, i.e. k / r = 1 / n
    c = CONFIGS[3]
    assert c.r_frac[0] * c.k_frac[1] == 5 * c.k_frac[0] * c.r_frac[1]


def test_streams_are_seeded_and_distinct():
    for cfg in (1, 2, 3, 4, 5, 6):
        w = Workload(cfg, d=40_000)
        a = w.gradient(0, 0)
        assert a.dtype == np.float32 and a.shape == (40_000,)
        assert np.array_equal(a, Workload(cfg, d=40_000).gradient(0, 0))
        assert not np.array_equal(a, w.gradient(1, 0))
        assert not np.array_equal(a, w.gradient(0, 1))
        assert 1 <= w.k <= w.r <= w.d


def test_structure_of_the_language_model_stand_in():
    w = Workload(4, d=660_340)
    g = w.gradient(2, 3)
    emb = g[: w.emb_len].reshape(w.emb_rows, w.row_len)
    on = np.any(emb != 0, axis=1)
    assert on.sum() == w.hot_rows == w.emb_rows // 20
    assert np.all(g[w.emb_len:] != 0)


def test_segment_sizes_sum_to_d():
    for cfg in (2, 3):
        w = Workload(cfg, d=100_003)
        assert int(w.segment_sizes.sum()) == w.d and w.segment_sizes.min() >= 1
