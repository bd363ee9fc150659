"""ctypes binding of the CPU oracle (``rtopk_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product
package never does. The oracle is plain C compiled with gcc; ``build()``
compiles it, ``lib()`` loads it (building it first if it is missing or older
than its source).

Every function takes and returns numpy arrays; nothing here touches a GPU.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rtopk_oracle.c")
_SO = os.path.join(_HERE, "librtopk_oracle.so")
_LIB = None

_u32p = ctypes.POINTER(ctypes.c_uint32)
_f32p = ctypes.POINTER(ctypes.c_float)


def build() -> str:
    """Compile the oracle with gcc (strict IEEE arithmetic, no contraction)."""
    cmd = ["gcc", "-O2", "-std=c11", "-fno-fast-math", "-ffp-contract=off",
           "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


def lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        if not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
            build()
        L = ctypes.CDLL(_SO)
        L.rtopk_oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.rtopk_oracle_philox4x32_10.restype = None
        L.rtopk_oracle_key64.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32]
        L.rtopk_oracle_key64.restype = ctypes.c_uint64
        L.rtopk_oracle_top_r.argtypes = [_f32p, ctypes.c_uint64, ctypes.c_uint64, _u32p]
        L.rtopk_oracle_top_r.restype = ctypes.c_int
        L.rtopk_oracle_encode.argtypes = [
            _f32p, _f32p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_uint64, ctypes.c_uint64, _u32p, _f32p]
        L.rtopk_oracle_encode.restype = ctypes.c_int
        for name in ("rtopk_oracle_aggregate", "rtopk_oracle_aggregate_f32"):
            fn = getattr(L, name)
            fn.argtypes = [_u32p, _f32p, ctypes.c_uint32, ctypes.c_uint64,
                           ctypes.c_uint64, _f32p]
            fn.restype = ctypes.c_int
        L.rtopk_oracle_aggregate_update.argtypes = [
            _u32p, _f32p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_double, ctypes.c_double, _f32p, _f32p]
        L.rtopk_oracle_aggregate_update.restype = ctypes.c_int
        L.rtopk_oracle_aggregate_update_f32.argtypes = [
            _u32p, _f32p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_float, ctypes.c_float, _f32p, _f32p]
        L.rtopk_oracle_aggregate_update_f32.restype = ctypes.c_int
        for name, ft in (("rtopk_oracle_aggregate_update_momentum", ctypes.c_double),
                         ("rtopk_oracle_aggregate_update_momentum_f32", ctypes.c_float)):
            fn = getattr(L, name)
            fn.argtypes = [_u32p, _f32p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint64,
                           ft, ft, ft, _f32p, _f32p, _f32p, _f32p]
            fn.restype = ctypes.c_int
        _LIB = L
    return _LIB


def _f32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"{what}: oracle returned {rc}")


def philox4x32_10(ctr, key) -> Tuple[int, int, int, int]:
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (ctypes.c_uint32 * 4)()
    lib().rtopk_oracle_philox4x32_10(c, k, o)
    return tuple(int(x) for x in o)


def key64(seed: int, step: int, index: int) -> int:
    return int(lib().rtopk_oracle_key64(seed, step, index))


def top_r(a: np.ndarray, r: int) -> np.ndarray:
    """pi(1..r) of Definition 1 for the float32 vector ``a``."""
    a = _f32(a)
    out = np.empty(r, dtype=np.uint32)
    rc = lib().rtopk_oracle_top_r(a.ctypes.data_as(_f32p), a.size, r,
                                  out.ctypes.data_as(_u32p))
    _check(rc, "top_r")
    return out


def encode(grad: np.ndarray, residual: np.ndarray, r: int, k: int,
           seed: int, step: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One node step of Algorithm 1. Returns (out_idx, out_val, new_residual);
    the input arrays are left untouched."""
    g = _f32(grad)
    m = _f32(residual).copy()
    if g.shape != m.shape or g.ndim != 1:
        raise ValueError("grad and residual must be 1-D and of equal length")
    k_alloc = max(int(k), 1)
    out_idx = np.empty(k_alloc, dtype=np.uint32)
    out_val = np.empty(k_alloc, dtype=np.float32)
    rc = lib().rtopk_oracle_encode(
        g.ctypes.data_as(_f32p), m.ctypes.data_as(_f32p), g.size, r, k, seed, step,
        out_idx.ctypes.data_as(_u32p), out_val.ctypes.data_as(_f32p))
    _check(rc, "encode")
    return out_idx, out_val, m


def _aggregate(fn_name: str, idx: np.ndarray, val: np.ndarray, n: int, d: int) -> np.ndarray:
    idx = np.ascontiguousarray(idx, dtype=np.uint32).reshape(-1)
    val = _f32(val).reshape(-1)
    if idx.size != val.size or n < 1 or idx.size % n != 0:
        raise ValueError("idx/val must hold n messages of equal length")
    k = idx.size // n
    out = np.empty(d, dtype=np.float32)
    rc = getattr(lib(), fn_name)(idx.ctypes.data_as(_u32p), val.ctypes.data_as(_f32p),
                                 n, k, d, out.ctypes.data_as(_f32p))
    _check(rc, fn_name)
    return out


def aggregate(idx: np.ndarray, val: np.ndarray, n: int, d: int) -> np.ndarray:
    """Master step of Algorithm 1, binary64 accumulation, one rounding."""
    return _aggregate("rtopk_oracle_aggregate", idx, val, n, d)


def aggregate_f32(idx: np.ndarray, val: np.ndarray, n: int, d: int) -> np.ndarray:
    """The same average in binary32, workers added in order 0..n-1."""
    return _aggregate("rtopk_oracle_aggregate_f32", idx, val, n, d)


def _aggregate_update(fn_name: str, idx, val, n: int, d: int, eta: float, scale: float,
                      omega: np.ndarray) -> np.ndarray:
    idx = np.ascontiguousarray(idx, dtype=np.uint32).reshape(-1)
    val = _f32(val).reshape(-1)
    omega = _f32(omega).reshape(-1)
    if idx.size != val.size or n < 1 or idx.size % n != 0 or omega.size != d:
        raise ValueError("idx/val must hold n messages of equal length, omega d weights")
    k = idx.size // n
    out = np.empty(d, dtype=np.float32)
    rc = getattr(lib(), fn_name)(idx.ctypes.data_as(_u32p), val.ctypes.data_as(_f32p), n, k, d,
                                 eta, scale, omega.ctypes.data_as(_f32p),
                                 out.ctypes.data_as(_f32p))
    _check(rc, fn_name)
    return out


def aggregate_update(idx, val, n: int, d: int, eta: float, scale: float,
                     omega: np.ndarray) -> np.ndarray:
    """Both master lines of Algorithm 1: omega - eta * scale * mean, binary64, one rounding."""
    return _aggregate_update("rtopk_oracle_aggregate_update", idx, val, n, d, eta, scale, omega)


def aggregate_update_f32(idx, val, n: int, d: int, eta: float, scale: float,
                         omega: np.ndarray) -> np.ndarray:
    """The same update in binary32: worker-order sum, / n, fma(-(eta * scale), mean, omega)."""
    return _aggregate_update("rtopk_oracle_aggregate_update_f32", idx, val, n, d, eta, scale,
                             omega)


def _aggregate_update_momentum(fn_name, idx, val, n, d, eta, scale, mu, omega, velocity):
    idx = np.ascontiguousarray(idx, dtype=np.uint32).reshape(-1)
    val = _f32(val).reshape(-1)
    omega = _f32(omega).reshape(-1)
    velocity = _f32(velocity).reshape(-1)
    if (idx.size != val.size or n < 1 or idx.size % n != 0 or omega.size != d
            or velocity.size != d):
        raise ValueError("idx/val must hold n messages of equal length, omega and velocity d values")
    k = idx.size // n
    w_out = np.empty(d, dtype=np.float32)
    v_out = np.empty(d, dtype=np.float32)
    rc = getattr(lib(), fn_name)(idx.ctypes.data_as(_u32p), val.ctypes.data_as(_f32p), n, k, d,
                                 eta, scale, mu, omega.ctypes.data_as(_f32p),
                                 velocity.ctypes.data_as(_f32p), w_out.ctypes.data_as(_f32p),
                                 v_out.ctypes.data_as(_f32p))
    _check(rc, fn_name)
    return w_out, v_out


def aggregate_update_momentum(idx, val, n: int, d: int, eta: float, scale: float, mu: float,
                              omega: np.ndarray, velocity: np.ndarray):
    """v <- mu v + scale * mean; omega <- omega - eta v; binary64. Returns (omega, velocity)."""
    return _aggregate_update_momentum("rtopk_oracle_aggregate_update_momentum", idx, val, n, d,
                                      eta, scale, mu, omega, velocity)


def aggregate_update_momentum_f32(idx, val, n: int, d: int, eta: float, scale: float, mu: float,
                                  omega: np.ndarray, velocity: np.ndarray):
    """The same in binary32: u = scale * mean, v' = fma(mu, v, u), omega' = fma(-eta, v', omega)."""
    return _aggregate_update_momentum("rtopk_oracle_aggregate_update_momentum_f32", idx, val, n, d,
                                      eta, scale, mu, omega, velocity)
