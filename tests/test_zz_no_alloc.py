"""rtopk_aggregate_update_static, the entry point that allocates nothing and
keeps its tile-start table in a device array inside the library, against
rtopk_aggregate_update (which takes the table's memory as a workspace): the
same weights bit for bit, on two calls in a row, the second with a smaller
input, so that whatever the first call left in the shared array is seen not
to matter. Also against the oracle's binary32 variant, and the size limit."""
import ctypes

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


def _messages(rng, d, n, k):
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.uint32)
    val = (rng.standard_normal((n, k)) * 10.0 ** rng.uniform(-3, 1, (n, k))).astype(np.float32)
    return idx, val


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    import torch
    from tests import gpu_util as u
    rt = u.rt
    rng = np.random.default_rng(2005_10761)
    # first a large call (8 workers, 3 M coordinates: 1,466 tiles), then a small one
    for d, n, k, eta, scale in ((3_000_017, 8, 20_000, 0.1, 5.0), (70_001, 3, 900, 0.25, 1.0)):
        print(f"static update d={d} n={n} k={k}", flush=True)
        idx, val = _messages(rng, d, n, k)
        omega = rng.standard_normal(d).astype(np.float32)
        want = u.gpu_aggregate_update(idx, val, n, d, eta, scale, omega)
        ti = torch.from_numpy(idx.reshape(-1).view(np.int32)).to(u.DEV)
        tv = torch.from_numpy(val.reshape(-1)).to(u.DEV)
        tw = torch.from_numpy(omega).to(u.DEV)
        rt.aggregate_update_static(ti, tv, n, k, eta, scale, tw)
        torch.cuda.synchronize()
        got = tw.cpu().numpy()
        assert np.array_equal(u.bits(got), u.bits(want))
        assert np.array_equal(u.bits(got), u.bits(oracle.aggregate_update_f32(idx, val, n, d, eta,
                                                                              scale, omega)))


def test_static_scratch_entry_point_rejects_sizes_beyond_its_array():
    import torch
    from tests import gpu_util as u
    rt = u.rt
    lib = rt.load_library()
    one_i = torch.zeros(1, dtype=torch.int32, device=u.DEV)
    one_v = torch.zeros(1, dtype=torch.float32, device=u.DEV)
    # (ceil(d / 2048) + 1) * n * 4 bytes: 2^28 coordinates with 32 workers need 16 MiB + 128 B
    d, n = 1 << 28, 32
    assert rt.aggregate_update_workspace_bytes(d, n, 1) > rt.STATIC_SCRATCH_BYTES
    assert rt.aggregate_update_workspace_bytes(d, 31, 1) <= rt.STATIC_SCRATCH_BYTES
    # the size check comes before any launch: the (too short) buffers are never touched
    rc = lib.rtopk_aggregate_update_static(one_i.data_ptr(), one_v.data_ptr(), n, 1, d,
                                           ctypes.c_float(0.1), ctypes.c_float(1.0),
                                           one_v.data_ptr(), None)
    assert rc == -4 and "built-in scratch" in rt.strerror(rc)
    rc = lib.rtopk_aggregate_update_static(None, one_v.data_ptr(), 1, 1, 10, ctypes.c_float(0.1),
                                           ctypes.c_float(1.0), one_v.data_ptr(), None)
    assert rc == -1
