"""Synthetic stand-ins for the gradient vectors of the five benchmark workloads.

The method was evaluated on gradients of image classifiers and of a two-layer
LSTM language model (Section IV). Those datasets and models are not available
here, so each configuration below borrows only a parameter count and a
qualitative value structure (per-layer scale spread, a few hot coordinates,
row-sparse embedding gradients, heavy tails) and draws the numbers from a
seeded generator.

Recipe shared by all configurations
  * ``numpy.random.Generator(PCG64(SeedSequence([...])))``, float64 arithmetic,
    one final cast to float32.
  * *Structure* (per-element or per-segment scales, segment sizes, the outlier
    mask) depends on the configuration only and is reused for every worker and
    step. *Noise* is redrawn for every (worker, step).
  * Vectors are produced in fixed chunks of ``CHUNK`` elements, each chunk with
    its own seed, so the bytes do not depend on how many threads generate them.

No arithmetic of the sparsifier lives here apart from ``ceil_fraction``, the
exact integer ceiling that turns "r = 1% of d" into a count.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Callable, Optional, Tuple

import numpy as np

CHUNK = 1 << 21

_TAG_STRUCT = 0x5752
_TAG_NOISE = 0x4E4F
_TAG_ROWS = 0x524F


def ceil_fraction(d: int, num: int, den: int) -> int:
    """ceil(d * num / den) in exact integer arithmetic."""
    return (d * num + den - 1) // den


def philox_seed_for_worker(worker: int) -> int:
    """Seed handed to the sparsifier for simulated worker ``worker``."""
    return 42 + worker


@dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    d: int
    r_frac: Tuple[int, int]
    k_frac: Tuple[int, int]
    n_workers: int
    steps: int
    note: str


CONFIGS = {
    1: Config(1, "cfg1-logscale-1M", 1 << 20, (1, 100), (1, 1000), 1, 5,
              "N(0,1) times a per-element scale, log-uniform in [1e-3, 1]"),
    2: Config(2, "cfg2-resnet18-sized", 11_173_962, (1, 100), (1, 1000), 8, 10,
              "62 segments, per-segment scale log-uniform [1e-4,1e-1] times N(0,1); "
              "0.5% of entries times 20"),
    3: Config(3, "cfg3-resnet50-sized", 25_557_032, (5, 1000), (1, 1000), 8, 10,
              "161 segments, Laplace(0,b) with per-segment b log-uniform [1e-5,1e-2]"),
    4: Config(4, "cfg4-lstm-lm", 66_034_000, (1, 100), (1, 1000), 4, 10,
              "10k x 1500 embedding with 5% nonzero rows N(0,1e-2); rest N(0,1e-3)"),
    5: Config(5, "cfg5-stress-student-t", 1 << 28, (1, 1000), (1, 10000), 16, 3,
              "Student-t(nu=3) times 1e-3; the sweep over k/d and r/k is applied by the caller"),
    # Not one of the five benchmark configurations: the update vector of the
    # federated setting (the change of the weights over one local epoch rather
    # than one minibatch gradient; Section IV), which is dense and smooth, at the
    # ResNet-18 size, with the sizes the experiments use for five nodes at 99%
    # compression: k = 1% of d and k / r = 1 / 5.
    6: Config(6, "cfg6-federated-delta-resnet18-sized", 11_173_962, (5, 100), (1, 100), 5, 5,
              "62 segments, per-segment scale log-uniform [1e-4,1e-2] times N(0,1); no zeros, "
              "no outliers"),
}

# k/d and r/k points of the stress sweep.
STRESS_K_FRACS = ((1, 10000), (1, 1000), (1, 100))
STRESS_R_OVER_K = (2, 5, 10)


def _n_threads() -> int:
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        avail = os.cpu_count() or 1
    return max(1, min(16, avail))


def _rng(*words: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(words))))


def _segment_sizes(rng: np.random.Generator, d: int, nseg: int, alpha: float) -> np.ndarray:
    """nseg sizes >= 1 that sum to d, proportional to a Dirichlet(alpha) draw."""
    nseg = min(nseg, d)
    p = rng.dirichlet(np.full(nseg, alpha))
    spare = d - nseg
    raw = p * spare
    base = np.floor(raw).astype(np.int64)
    short = spare - int(base.sum())
    if short > 0:
        order = np.argsort(-(raw - base), kind="stable")
        base[order[:short]] += 1
    return base + 1


def _fill_chunks(out: np.ndarray, fn: Callable[[int, int, int], np.ndarray]) -> None:
    d = out.shape[0]
    spans = [(c, lo, min(lo + CHUNK, d)) for c, lo in enumerate(range(0, d, CHUNK))]

    def work(span):
        c, lo, hi = span
        out[lo:hi] = fn(c, lo, hi)

    nt = _n_threads()
    if nt == 1 or len(spans) == 1:
        for s in spans:
            work(s)
    else:
        with ThreadPoolExecutor(max_workers=nt) as pool:
            list(pool.map(work, spans))


class Workload:
    """One configuration: sizes, (r, k) and a seeded gradient stream.

    ``d`` may be overridden to get a smaller vector with the same structure
    (tests use that); ``r``/``k`` default to the configuration's percentages
    of the actual ``d`` and may be overridden too.
    """

    def __init__(self, cfg: int, d: Optional[int] = None,
                 r: Optional[int] = None, k: Optional[int] = None):
        self.config = CONFIGS[cfg]
        self.cfg = cfg
        self.d = int(d) if d is not None else self.config.d
        if self.d < 1:
            raise ValueError("d must be >= 1")
        self.k = int(k) if k is not None else max(1, ceil_fraction(self.d, *self.config.k_frac))
        self.r = int(r) if r is not None else max(self.k, ceil_fraction(self.d, *self.config.r_frac))
        self.n_workers = self.config.n_workers
        self.steps = self.config.steps
        self._scale: Optional[np.ndarray] = None
        self._build_structure()

    # ----- structure, drawn once per configuration -------------------------
    def _build_structure(self) -> None:
        cfg, d = self.cfg, self.d
        if cfg == 1:
            scale = np.empty(d, dtype=np.float32)

            def fn(c, lo, hi):
                u = _rng(cfg, 0, _TAG_STRUCT, c).random(hi - lo)
                return np.power(10.0, -3.0 + 3.0 * u)

            _fill_chunks(scale, fn)
            self._scale = scale
        elif cfg in (2, 3, 6):
            rng = _rng(cfg, _TAG_STRUCT)
            nseg, lo_e, hi_e = {2: (62, -4.0, -1.0), 3: (161, -5.0, -2.0), 6: (62, -4.0, -2.0)}[cfg]
            sizes = _segment_sizes(rng, d, nseg, 0.3)
            seg_scale = np.power(10.0, lo_e + (hi_e - lo_e) * rng.random(sizes.shape[0]))
            scale = np.repeat(seg_scale, sizes).astype(np.float64)
            if cfg == 2:
                n_out = ceil_fraction(d, 5, 1000)
                hot = rng.choice(d, size=min(n_out, d), replace=False)
                scale[hot] *= 20.0
            self.segment_sizes = sizes
            self.segment_scales = seg_scale
            self._scale = scale.astype(np.float32)
        elif cfg == 4:
            full_d, full_emb, row = 66_034_000, 15_000_000, 1500
            if d >= 100 * row:
                self.row_len = row
                self.emb_rows = max(1, (d * full_emb // full_d) // row)
            else:
                self.row_len = max(1, d // 64)
                self.emb_rows = max(1, (d * full_emb // full_d) // self.row_len)
            self.emb_len = self.emb_rows * self.row_len
            self.hot_rows = max(1, self.emb_rows // 20)
        elif cfg == 5:
            pass
        else:  # pragma: no cover
            raise ValueError(cfg)

    # ----- noise, redrawn per (worker, step) -------------------------------
    def gradient(self, worker: int, step: int) -> np.ndarray:
        """The float32 gradient of simulated worker ``worker`` at ``step``."""
        cfg, d = self.cfg, self.d
        out = np.empty(d, dtype=np.float32)
        if cfg in (1, 2, 6):
            scale = self._scale

            def fn(c, lo, hi):
                z = _rng(cfg, worker, step, _TAG_NOISE, c).standard_normal(hi - lo)
                return z * scale[lo:hi].astype(np.float64)
        elif cfg == 3:
            scale = self._scale

            def fn(c, lo, hi):
                z = _rng(cfg, worker, step, _TAG_NOISE, c).laplace(0.0, 1.0, hi - lo)
                return z * scale[lo:hi].astype(np.float64)
        elif cfg == 4:
            rows = _rng(cfg, worker, step, _TAG_ROWS).choice(
                self.emb_rows, size=self.hot_rows, replace=False)
            row_on = np.zeros(self.emb_rows, dtype=bool)
            row_on[rows] = True
            emb_len, row_len = self.emb_len, self.row_len

            def fn(c, lo, hi):
                z = _rng(cfg, worker, step, _TAG_NOISE, c).standard_normal(hi - lo)
                pos = np.arange(lo, hi, dtype=np.int64)
                in_emb = pos < emb_len
                on = np.zeros(hi - lo, dtype=bool)
                on[in_emb] = row_on[pos[in_emb] // row_len]
                sd = np.where(in_emb, np.where(on, 1e-2, 0.0), 1e-3)
                return z * sd
        elif cfg == 5:
            def fn(c, lo, hi):
                z = _rng(cfg, worker, step, _TAG_NOISE, c).standard_t(3.0, hi - lo)
                return z * 1e-3
        else:  # pragma: no cover
            raise ValueError(cfg)
        _fill_chunks(out, fn)
        return out

    def describe(self) -> dict:
        return {"workload": self.config.name, "d": self.d, "r": self.r, "k": self.k,
                "n_workers": self.n_workers, "steps": self.steps}
