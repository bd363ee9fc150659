"""Helpers for the GPU parity tests: run the HIP path through the C ABI and
hand back numpy arrays to compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2005_10761_amd as rt

DEV = torch.device("cuda:0")


def bits(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


class GpuWorker:
    """Device-side state of one simulated worker: residual, message buffers,
    workspace. ``offset`` shifts grad/residual off 16-byte alignment."""

    def __init__(self, d: int, r: int, k: int, residual=None, offset: int = 0):
        self.d, self.r, self.k, self.offset = d, r, k, offset
        self._res_store = torch.zeros(d + offset, dtype=torch.float32, device=DEV)
        self.residual = self._res_store[offset:]
        if residual is not None:
            self.residual.copy_(torch.from_numpy(np.ascontiguousarray(residual, np.float32)))
        self._g_store = torch.empty(d + offset, dtype=torch.float32, device=DEV)
        self.grad = self._g_store[offset:]
        self.idx = torch.full((k,), -1, dtype=torch.int32, device=DEV)
        self.val = torch.full((k,), float("nan"), dtype=torch.float32, device=DEV)
        self.ws = torch.empty(rt.encode_workspace_bytes(d, r, k), dtype=torch.uint8, device=DEV)
        # poison the workspace: the library must not depend on its contents
        self.ws.fill_(0xA5)

    def encode(self, g: np.ndarray, seed: int, step: int, check_stats: bool = True,
               force: int = 0, r: int = None, k: int = None):
        """``r``/``k`` override the sizes of this call only (they must not need
        more workspace or a longer message than the worker was built for)."""
        r = self.r if r is None else r
        k = self.k if k is None else k
        assert k <= self.k and rt.encode_workspace_bytes(self.d, r, k) <= self.ws.numel()
        self.grad.copy_(torch.from_numpy(np.ascontiguousarray(g, np.float32)))
        if force:
            rt.force_next_encode(force)
        rt.encode(self.grad, self.residual, r, k, seed, step, self.idx, self.val, self.ws)
        st = rt.encode_stats(self.ws)
        # the error flags are also the first word of the workspace
        assert int(self.ws[:4].view(torch.int32).item()) == st["error_flags"], st
        if check_stats:
            assert st["error_flags"] == 0, st
        self.stats = st
        return (self.idx[:k].cpu().numpy().view(np.uint32).copy(),
                self.val[:k].cpu().numpy().copy(),
                self.residual.cpu().numpy().copy())


def gpu_encode_once(g, m, r, k, seed, step, offset=0, force=0):
    w = GpuWorker(len(g), r, k, residual=m, offset=offset)
    out = w.encode(g, seed, step, force=force)
    return out + (w.stats,)


def gpu_aggregate(idx: np.ndarray, val: np.ndarray, n: int, d: int) -> np.ndarray:
    idx = np.ascontiguousarray(idx, np.uint32).reshape(-1)
    val = np.ascontiguousarray(val, np.float32).reshape(-1)
    k = idx.size // n
    ti = torch.from_numpy(idx.view(np.int32)).to(DEV)
    tv = torch.from_numpy(val).to(DEV)
    out = torch.full((d,), float("nan"), dtype=torch.float32, device=DEV)
    rt.aggregate(ti, tv, n, k, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_aggregate_update(idx: np.ndarray, val: np.ndarray, n: int, d: int, eta: float,
                         scale: float, omega: np.ndarray, offset: int = 0) -> np.ndarray:
    """``offset`` (in elements) shifts omega off its 16-byte alignment."""
    idx = np.ascontiguousarray(idx, np.uint32).reshape(-1)
    val = np.ascontiguousarray(val, np.float32).reshape(-1)
    k = idx.size // n
    ti = torch.from_numpy(idx.view(np.int32)).to(DEV)
    tv = torch.from_numpy(val).to(DEV)
    buf = torch.zeros(d + offset, dtype=torch.float32, device=DEV)
    tw = buf[offset:]
    tw.copy_(torch.from_numpy(np.ascontiguousarray(omega, np.float32)))
    ws = torch.empty(rt.aggregate_update_workspace_bytes(d, n, k), dtype=torch.uint8, device=DEV)
    ws.fill_(0xA5)                                   # whatever the workspace held must not matter
    rt.aggregate_update(ti, tv, n, k, eta, scale, tw, ws)
    torch.cuda.synchronize()
    return tw.cpu().numpy()


def gpu_aggregate_update_momentum(idx, val, n, d, eta, scale, mu, omega, velocity, offset=0):
    """``offset`` (in elements) shifts omega and velocity off their 16-byte alignment."""
    idx = np.ascontiguousarray(idx, np.uint32).reshape(-1)
    val = np.ascontiguousarray(val, np.float32).reshape(-1)
    k = idx.size // n
    ti = torch.from_numpy(idx.view(np.int32)).to(DEV)
    tv = torch.from_numpy(val).to(DEV)
    wbuf = torch.zeros(d + offset, dtype=torch.float32, device=DEV)
    vbuf = torch.zeros(d + offset, dtype=torch.float32, device=DEV)
    tw, tvel = wbuf[offset:], vbuf[offset:]
    tw.copy_(torch.from_numpy(np.ascontiguousarray(omega, np.float32)))
    tvel.copy_(torch.from_numpy(np.ascontiguousarray(velocity, np.float32)))
    rt.aggregate_update_momentum(ti, tv, n, k, eta, scale, mu, tw, tvel)
    torch.cuda.synchronize()
    return tw.cpu().numpy(), tvel.cpu().numpy()


def assert_update_close(got, idx, val, n, d, eta, scale, omega, want64):
    """|gpu - ref| <= 1e-6 * (|omega| + |eta scale| sum_w |v_w| / n)."""
    size = np.zeros(d)
    np.add.at(size, np.asarray(idx).reshape(-1).astype(np.int64),
              np.abs(np.asarray(val, np.float64).reshape(-1)) / n)
    with np.errstate(invalid="ignore"):             # not-a-number weights are compared below
        size = np.abs(omega.astype(np.float64)) + abs(eta * scale) * size
    fin = np.isfinite(omega) & np.isfinite(want64)   # the rest is compared bit for bit elsewhere
    assert np.all(np.abs(got[fin].astype(np.float64) - want64[fin].astype(np.float64))
                  <= 1e-6 * size[fin])
    assert np.array_equal(np.isnan(got), np.isnan(want64))
    assert np.array_equal(got[~fin & ~np.isnan(got)], want64[~fin & ~np.isnan(got)])


def same_floats(a, b) -> bool:
    """Bit for bit, except that two not-a-number values count as equal whatever
    their payloads: which payload survives a sum of several is the hardware's choice."""
    a = np.ascontiguousarray(a, np.float32)
    b = np.ascontiguousarray(b, np.float32)
    na, nb = np.isnan(a), np.isnan(b)
    return bool(np.array_equal(na, nb) and np.array_equal(bits(a)[~na], bits(b)[~nb]))


def assert_encode_equal(got, want, what=""):
    gi, gv, gm = got[:3]
    wi, wv, wm = want
    assert np.array_equal(gi, wi), f"{what}: indices differ"
    assert np.array_equal(bits(gv), bits(wv)), f"{what}: values differ"
    assert np.array_equal(bits(gm), bits(wm)), f"{what}: residual differs"


def assert_aggregate_close(got, idx, val, n, d, want64):
    """|gpu - ref| <= 1e-6 * max(|ref|, sum_w |v_w| / n): relative to the mean,
    or to the mean of absolute contributions when those cancel."""
    scale = np.zeros(d)
    np.add.at(scale, np.asarray(idx).reshape(-1).astype(np.int64),
              np.abs(np.asarray(val, np.float64).reshape(-1)) / n)
    g = got.astype(np.float64)
    w = want64.astype(np.float64)
    assert np.all(np.abs(g - w) <= 1e-6 * np.maximum(np.abs(w), scale))
