"""ctypes binding of the C ABI in ``include/rtopk.h`` (same names, same
argument order). Tensors are passed as raw device pointers; no arithmetic of
the method happens here."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librtopk.so")
_LIB: Optional[ctypes.CDLL] = None

# what include/rtopk.h declares ...
EXPORTS = ("rtopk_encode_workspace_bytes", "rtopk_aggregate_workspace_bytes", "rtopk_encode",
           "rtopk_encode_batch", "rtopk_encode_batch_device_step",
           "rtopk_aggregate", "rtopk_aggregate_update", "rtopk_aggregate_update_workspace_bytes",
           "rtopk_aggregate_update_momentum", "rtopk_aggregate_update_static",
           "rtopk_strerror", "rtopk_version")
# ... and include/rtopk_diag.h
DIAG_EXPORTS = ("rtopk_encode_stats", "rtopk_trace_next_encode", "rtopk_force_next_encode",
                "rtopk_diag_stream_add", "rtopk_debug_checks")


class RtopkError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


class EncodeStats(ctypes.Structure):
    _fields_ = [("error_flags", ctypes.c_uint32), ("path", ctypes.c_uint32),
                ("threshold_bits", ctypes.c_uint32), ("boundary_list_size", ctypes.c_uint32),
                ("count_greater", ctypes.c_uint64), ("ties_taken", ctypes.c_uint64),
                ("superset_size", ctypes.c_uint64), ("key_list_size", ctypes.c_uint64)]


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load ``librtopk.so``. There is no fallback: a missing library is an error."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2005_10761_amd.build` "
            "(hipcc, gfx950). The rTop-k path has no CPU or PyTorch fallback.")
    L = ctypes.CDLL(_LIB_PATH)
    u64, u32, vp = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p
    L.rtopk_encode_workspace_bytes.argtypes = [u64, u64, u64, ctypes.POINTER(u64)]
    L.rtopk_encode_workspace_bytes.restype = ctypes.c_int
    L.rtopk_aggregate_workspace_bytes.argtypes = [u64, u32, u64, ctypes.POINTER(u64)]
    L.rtopk_aggregate_workspace_bytes.restype = ctypes.c_int
    L.rtopk_encode.argtypes = [vp, vp, u64, u64, u64, u64, u64, vp, vp, vp, u64, vp]
    L.rtopk_encode.restype = ctypes.c_int
    L.rtopk_encode_batch.argtypes = [u32, vp, vp, u64, u64, u64, vp, u64, vp, vp, vp, u64, vp]
    L.rtopk_encode_batch.restype = ctypes.c_int
    L.rtopk_encode_batch_device_step.argtypes = [u32, vp, vp, u64, u64, u64, vp, vp, vp, vp, vp,
                                                 u64, vp]
    L.rtopk_encode_batch_device_step.restype = ctypes.c_int
    L.rtopk_diag_stream_add.argtypes = [vp, vp, u64, vp]
    L.rtopk_diag_stream_add.restype = ctypes.c_int
    L.rtopk_debug_checks.argtypes = []
    L.rtopk_debug_checks.restype = ctypes.c_int
    L.rtopk_aggregate.argtypes = [vp, vp, u32, u64, u64, vp, vp, u64, vp]
    L.rtopk_aggregate.restype = ctypes.c_int
    L.rtopk_aggregate_update_workspace_bytes.argtypes = [u64, u32, u64, ctypes.POINTER(u64)]
    L.rtopk_aggregate_update_workspace_bytes.restype = ctypes.c_int
    L.rtopk_aggregate_update.argtypes = [vp, vp, u32, u64, u64, ctypes.c_float, ctypes.c_float,
                                         vp, vp, u64, vp]
    L.rtopk_aggregate_update.restype = ctypes.c_int
    L.rtopk_aggregate_update_static.argtypes = [vp, vp, u32, u64, u64, ctypes.c_float,
                                                ctypes.c_float, vp, vp]
    L.rtopk_aggregate_update_static.restype = ctypes.c_int
    L.rtopk_aggregate_update_momentum.argtypes = [vp, vp, u32, u64, u64, ctypes.c_float,
                                                  ctypes.c_float, ctypes.c_float, vp, vp, vp]
    L.rtopk_aggregate_update_momentum.restype = ctypes.c_int
    L.rtopk_encode_stats.argtypes = [vp, vp, ctypes.POINTER(EncodeStats)]
    L.rtopk_encode_stats.restype = ctypes.c_int
    L.rtopk_trace_next_encode.argtypes = [ctypes.c_int, vp, vp]
    L.rtopk_trace_next_encode.restype = ctypes.c_int
    L.rtopk_force_next_encode.argtypes = [ctypes.c_uint]
    L.rtopk_force_next_encode.restype = ctypes.c_int
    L.rtopk_strerror.argtypes = [ctypes.c_int]
    L.rtopk_strerror.restype = ctypes.c_char_p
    L.rtopk_version.argtypes = []
    L.rtopk_version.restype = ctypes.c_int
    _LIB = L
    return L


def strerror(code: int) -> str:
    return load_library().rtopk_strerror(int(code)).decode()


def version() -> int:
    return int(load_library().rtopk_version())


def encode_workspace_bytes(d: int, r: int, k: int) -> int:
    out = ctypes.c_uint64(0)
    rc = load_library().rtopk_encode_workspace_bytes(d, r, k, ctypes.byref(out))
    if rc:
        raise RtopkError(rc, "rtopk_encode_workspace_bytes")
    return int(out.value)


def aggregate_workspace_bytes(d: int, n: int, k: int) -> int:
    out = ctypes.c_uint64(0)
    rc = load_library().rtopk_aggregate_workspace_bytes(d, n, k, ctypes.byref(out))
    if rc:
        raise RtopkError(rc, "rtopk_aggregate_workspace_bytes")
    return int(out.value)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream
    return h if h else None


def _need(t: torch.Tensor, dtype, name: str) -> None:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous {dtype} tensor on the GPU")


def encode(grad: torch.Tensor, residual: torch.Tensor, r: int, k: int, seed: int, step: int,
           out_idx: torch.Tensor, out_val: torch.Tensor, workspace: torch.Tensor,
           stream=None) -> None:
    """rtopk_encode: enqueue one node-side step of Algorithm 1. ``residual`` is
    updated in place; ``out_idx`` (int32 storage holding uint32 values) and
    ``out_val`` receive the message."""
    _need(grad, torch.float32, "grad")
    _need(residual, torch.float32, "residual")
    _need(out_idx, torch.int32, "out_idx")
    _need(out_val, torch.float32, "out_val")
    d = grad.numel()
    if residual.numel() != d or out_idx.numel() < k or out_val.numel() < k:
        raise ValueError("residual must have d elements, out_idx/out_val at least k")
    rc = load_library().rtopk_encode(
        _ptr(grad), _ptr(residual), d, r, k, seed & (2**64 - 1), step & (2**64 - 1),
        _ptr(out_idx), _ptr(out_val), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc:
        raise RtopkError(rc, "rtopk_encode")


def encode_batch(grads, residuals, r: int, k: int, seeds, step: int, out_idx, out_val,
                 workspace: torch.Tensor, stream=None) -> None:
    """rtopk_encode_batch: one node-side step of Algorithm 1 for every member of
    a list of equally sized vectors, in shared kernel launches. ``grads``,
    ``residuals``, ``out_idx``, ``out_val`` are sequences of tensors (as for
    :func:`encode`), ``seeds`` a sequence of ints; ``workspace`` holds
    ``len(grads)`` slices of ``encode_workspace_bytes(d, r, k)`` bytes."""
    n = len(grads)
    if n < 1 or not (len(residuals) == len(seeds) == len(out_idx) == len(out_val) == n):
        raise ValueError("grads, residuals, seeds, out_idx, out_val must have the same length >= 1")
    d = grads[0].numel()
    for g, m, oi, ov in zip(grads, residuals, out_idx, out_val):
        _need(g, torch.float32, "grad")
        _need(m, torch.float32, "residual")
        _need(oi, torch.int32, "out_idx")
        _need(ov, torch.float32, "out_val")
        if g.numel() != d or m.numel() != d or oi.numel() < k or ov.numel() < k:
            raise ValueError("every member needs d gradient and residual elements and k outputs")
    vp_arr = ctypes.c_void_p * n
    seeds_arr = (ctypes.c_uint64 * n)(*[s & (2**64 - 1) for s in seeds])
    rc = load_library().rtopk_encode_batch(
        n, vp_arr(*[_ptr(t) for t in grads]), vp_arr(*[_ptr(t) for t in residuals]), d, r, k,
        seeds_arr, step & (2**64 - 1), vp_arr(*[_ptr(t) for t in out_idx]),
        vp_arr(*[_ptr(t) for t in out_val]), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc:
        raise RtopkError(rc, "rtopk_encode_batch")


def encode_batch_device_step(grads, residuals, r: int, k: int, seeds, step_device: torch.Tensor,
                             out_idx, out_val, workspace: torch.Tensor, stream=None) -> None:
    """rtopk_encode_batch_device_step: as :func:`encode_batch`, with the step
    number read from ``step_device`` (one int64 on the GPU) when the kernels run."""
    n = len(grads)
    if n < 1 or not (len(residuals) == len(seeds) == len(out_idx) == len(out_val) == n):
        raise ValueError("grads, residuals, seeds, out_idx, out_val must have the same length >= 1")
    _need(step_device, torch.int64, "step_device")
    d = grads[0].numel()
    for g, m, oi, ov in zip(grads, residuals, out_idx, out_val):
        _need(g, torch.float32, "grad")
        _need(m, torch.float32, "residual")
        _need(oi, torch.int32, "out_idx")
        _need(ov, torch.float32, "out_val")
        if g.numel() != d or m.numel() != d or oi.numel() < k or ov.numel() < k:
            raise ValueError("every member needs d gradient and residual elements and k outputs")
    vp_arr = ctypes.c_void_p * n
    seeds_arr = (ctypes.c_uint64 * n)(*[s & (2**64 - 1) for s in seeds])
    rc = load_library().rtopk_encode_batch_device_step(
        n, vp_arr(*[_ptr(t) for t in grads]), vp_arr(*[_ptr(t) for t in residuals]), d, r, k,
        seeds_arr, _ptr(step_device), vp_arr(*[_ptr(t) for t in out_idx]),
        vp_arr(*[_ptr(t) for t in out_val]), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc:
        raise RtopkError(rc, "rtopk_encode_batch_device_step")


def diag_stream_add(grad: torch.Tensor, residual: torch.Tensor, stream=None) -> None:
    """rtopk_diag_stream_add: residual += grad, streamed as the encoder's dominant kernel streams."""
    _need(grad, torch.float32, "grad")
    _need(residual, torch.float32, "residual")
    if grad.numel() != residual.numel():
        raise ValueError("grad and residual must have the same length")
    rc = load_library().rtopk_diag_stream_add(_ptr(grad), _ptr(residual), grad.numel(),
                                              _stream_handle(stream))
    if rc:
        raise RtopkError(rc, "rtopk_diag_stream_add")


def aggregate(idx: torch.Tensor, val: torch.Tensor, n: int, k: int, out: torch.Tensor,
              workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """rtopk_aggregate: enqueue the master's averaging step. ``idx``/``val`` hold
    the n messages back to back; ``out`` (d elements) is fully overwritten."""
    _need(idx, torch.int32, "idx")
    _need(val, torch.float32, "val")
    _need(out, torch.float32, "out")
    if idx.numel() < n * k or val.numel() < n * k:
        raise ValueError("idx/val must hold n*k entries")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load_library().rtopk_aggregate(_ptr(idx), _ptr(val), n, k, out.numel(), _ptr(out),
                                        _ptr(workspace), ws_bytes, _stream_handle(stream))
    if rc:
        raise RtopkError(rc, "rtopk_aggregate")


def aggregate_update_workspace_bytes(d: int, n: int, k: int) -> int:
    out = ctypes.c_uint64(0)
    rc = load_library().rtopk_aggregate_update_workspace_bytes(d, n, k, ctypes.byref(out))
    if rc:
        raise RtopkError(rc, "rtopk_aggregate_update_workspace_bytes")
    return out.value


def aggregate_update(idx: torch.Tensor, val: torch.Tensor, n: int, k: int, eta: float,
                     scale: float, omega: torch.Tensor, workspace: torch.Tensor,
                     stream=None) -> None:
    """rtopk_aggregate_update: enqueue omega -= eta * scale * (average of the n
    messages), in place on ``omega`` (d elements)."""
    _need(idx, torch.int32, "idx")
    _need(val, torch.float32, "val")
    _need(omega, torch.float32, "omega")
    if idx.numel() < n * k or val.numel() < n * k:
        raise ValueError("idx/val must hold n*k entries")
    rc = load_library().rtopk_aggregate_update(_ptr(idx), _ptr(val), n, k, omega.numel(),
                                               eta, scale, _ptr(omega), _ptr(workspace),
                                               workspace.numel() * workspace.element_size(),
                                               _stream_handle(stream))
    if rc:
        raise RtopkError(rc, "rtopk_aggregate_update")


STATIC_SCRATCH_BYTES = 16 << 20


def aggregate_update_static(idx: torch.Tensor, val: torch.Tensor, n: int, k: int, eta: float,
                            scale: float, omega: torch.Tensor, stream=None) -> None:
    """rtopk_aggregate_update_static: as :func:`aggregate_update`, with the
    library's built-in scratch array in place of a workspace."""
    _need(idx, torch.int32, "idx")
    _need(val, torch.float32, "val")
    _need(omega, torch.float32, "omega")
    if idx.numel() < n * k or val.numel() < n * k:
        raise ValueError("idx/val must hold n*k entries")
    rc = load_library().rtopk_aggregate_update_static(_ptr(idx), _ptr(val), n, k, omega.numel(),
                                                      eta, scale, _ptr(omega),
                                                      _stream_handle(stream))
    if rc:
        raise RtopkError(rc, "rtopk_aggregate_update_static")


def aggregate_update_momentum(idx: torch.Tensor, val: torch.Tensor, n: int, k: int, eta: float,
                              scale: float, mu: float, omega: torch.Tensor,
                              velocity: torch.Tensor, stream=None) -> None:
    """rtopk_aggregate_update_momentum: enqueue velocity = mu * velocity + scale *
    (average of the n messages); omega -= eta * velocity, both in place."""
    _need(idx, torch.int32, "idx")
    _need(val, torch.float32, "val")
    _need(omega, torch.float32, "omega")
    _need(velocity, torch.float32, "velocity")
    if idx.numel() < n * k or val.numel() < n * k or velocity.numel() != omega.numel():
        raise ValueError("idx/val must hold n*k entries; omega and velocity the same d")
    rc = load_library().rtopk_aggregate_update_momentum(
        _ptr(idx), _ptr(val), n, k, omega.numel(), eta, scale, mu, _ptr(omega), _ptr(velocity),
        _stream_handle(stream))
    if rc:
        raise RtopkError(rc, "rtopk_aggregate_update_momentum")


STAGES = {"prepare": 1, "fused": 2, "classify": 3, "finalize": 4, "emit": 5, "all": 100}


def trace_next_encode(stage: int, ev_begin: int, ev_end: int) -> None:
    """rtopk_trace_next_encode: raw hipEvent_t handles, recorded around ``stage``
    of the next encode issued from this thread."""
    rc = load_library().rtopk_trace_next_encode(stage, ev_begin, ev_end)
    if rc:
        raise RtopkError(rc, "rtopk_trace_next_encode")


FORCE_ESTIMATE_MISS = 1
FORCE_KEY_WINDOW_MISS = 2
FORCE_CHECK_IN_ABORT = 4
FORCE_BRACKET_LOW = 8
FORCE_BARRIER_TIMEOUT = 16


def force_next_encode(flags: int) -> None:
    """rtopk_force_next_encode: make the next encode from this thread take an
    exact fallback path (test hook)."""
    rc = load_library().rtopk_force_next_encode(flags)
    if rc:
        raise RtopkError(rc, "rtopk_force_next_encode")


def encode_stats(workspace: torch.Tensor, stream=None) -> dict:
    st = EncodeStats()
    rc = load_library().rtopk_encode_stats(_ptr(workspace), _stream_handle(stream),
                                           ctypes.byref(st))
    if rc:
        raise RtopkError(rc, "rtopk_encode_stats")
    return {name: int(getattr(st, name)) for name, _ in EncodeStats._fields_}
