"""MI355X-native rTop-k gradient sparsification: Python binding of ``librtopk.so``.

The package is argument marshalling only. Every step of the hot path runs in
the hand-written gfx950 kernels behind the C ABI declared in
``include/rtopk.h``; PyTorch supplies device memory and streams and nothing
else. There is no CPU fallback: if the compiled library is missing the import
of :mod:`paper_2005_10761_amd.binding` symbols fails loudly at first use.
"""
from .binding import (RtopkError, aggregate, aggregate_update, aggregate_update_momentum, aggregate_update_static, STATIC_SCRATCH_BYTES,
                      aggregate_update_workspace_bytes,
                      aggregate_workspace_bytes, encode, encode_batch, encode_batch_device_step,
                      diag_stream_add,
                      encode_stats, encode_workspace_bytes, library_path, load_library,
                      strerror, trace_next_encode, version, STAGES, force_next_encode,
                      FORCE_ESTIMATE_MISS, FORCE_KEY_WINDOW_MISS, FORCE_CHECK_IN_ABORT, FORCE_BRACKET_LOW, FORCE_BARRIER_TIMEOUT)

__all__ = ["RtopkError", "aggregate", "aggregate_update", "aggregate_update_momentum", "aggregate_update_static", "STATIC_SCRATCH_BYTES", "aggregate_update_workspace_bytes", "aggregate_workspace_bytes", "encode", "encode_batch", "encode_batch_device_step", "diag_stream_add", "encode_stats",
           "encode_workspace_bytes", "library_path", "load_library", "strerror", "trace_next_encode", "version", "STAGES",
           "force_next_encode", "FORCE_ESTIMATE_MISS", "FORCE_KEY_WINDOW_MISS", "FORCE_CHECK_IN_ABORT", "FORCE_BRACKET_LOW", "FORCE_BARRIER_TIMEOUT"]
