"""The C-ABI library loads and exports every symbol include/*.h declares;
host-side argument checks (no kernel is launched, no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2005_10761_amd as rt
from paper_2005_10761_amd.binding import DIAG_EXPORTS, EXPORTS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header="rtopk.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(rtopk_[a-z_0-9]+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    lib = rt.load_library()
    declared = _declared_symbols()
    assert declared == set(EXPORTS)
    diag = _declared_symbols("rtopk_diag.h")
    assert diag == set(DIAG_EXPORTS) and not (diag & declared)
    for name in declared | diag:
        assert getattr(lib, name) is not None
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["rtopk.h", "rtopk_diag.h"]


def test_version_and_strerror():
    assert rt.version() >= 100
    assert rt.strerror(0) == "ok"
    for code in (-1, -2, -3, -99):
        assert isinstance(rt.strerror(code), str) and rt.strerror(code)


def test_workspace_queries_validate_definition_3_domain():
    assert rt.encode_workspace_bytes(1 << 20, 10486, 1049) > 0
    assert rt.encode_workspace_bytes(1, 1, 1) > 0
    for d, r, k in ((10, 5, 0), (10, 5, 6), (10, 11, 5), (1 << 32, 5, 5), (0, 0, 0)):
        with pytest.raises(rt.RtopkError) as e:
            rt.encode_workspace_bytes(d, r, k)
        assert e.value.code == -1
    assert rt.aggregate_workspace_bytes(1000, 4, 10) >= 0
    with pytest.raises(rt.RtopkError):
        rt.aggregate_workspace_bytes(1000, 0, 10)


def test_encode_rejects_bad_arguments_before_launching():
    lib = rt.load_library()
    u64 = ctypes.c_uint64
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: checks fail first
    fake2 = ctypes.c_void_p(0x100000)
    # null pointers
    assert lib.rtopk_encode(None, fake, 8, 4, 2, 0, 0, fake, fake, fake, u64(1 << 30), None) == -1
    # k > r
    assert lib.rtopk_encode(fake, fake2, 8, 4, 5, 0, 0, fake, fake, fake, u64(1 << 30), None) == -1
    # grad overlaps residual
    assert lib.rtopk_encode(fake, fake, 8, 4, 2, 0, 0, fake, fake, fake, u64(1 << 30), None) == -1
    # workspace too small / null / misaligned
    assert lib.rtopk_encode(fake, fake2, 8, 4, 2, 0, 0, fake, fake, fake, u64(16), None) == -2
    assert lib.rtopk_encode(fake, fake2, 8, 4, 2, 0, 0, fake, fake, None, u64(1 << 30), None) == -2
    assert lib.rtopk_encode(fake, fake2, 8, 4, 2, 0, 0, fake, fake, ctypes.c_void_p(0x1010),
                            u64(1 << 30), None) == -2
    # aggregate
    assert lib.rtopk_aggregate(None, fake, 2, 3, 10, fake, None, u64(0), None) == -1
    assert lib.rtopk_aggregate(fake, fake, 0, 3, 10, fake, None, u64(0), None) == -1


def test_master_updates_and_batch_reject_bad_arguments_before_launching():
    lib = rt.load_library()
    u64 = ctypes.c_uint64
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: checks fail first
    fake2 = ctypes.c_void_p(0x100000)
    big = u64(1 << 30)
    # fused weight step: null pointers, no workers, workspace missing / small / misaligned
    assert lib.rtopk_aggregate_update(None, fake, 2, 3, 10, 0.1, 1.0, fake, fake, big, None) == -1
    assert lib.rtopk_aggregate_update(fake, fake, 0, 3, 10, 0.1, 1.0, fake, fake, big, None) == -1
    assert lib.rtopk_aggregate_update(fake, fake, 2, 3, 10, 0.1, 1.0, fake2, None, big, None) == -2
    assert lib.rtopk_aggregate_update(fake, fake, 2, 3, 10, 0.1, 1.0, fake2, fake, u64(8), None) == -2
    assert lib.rtopk_aggregate_update(fake, fake, 2, 3, 10, 0.1, 1.0, fake2,
                                      ctypes.c_void_p(0x1010), big, None) == -2
    assert rt.aggregate_update_workspace_bytes(10_000, 4, 10) == 256     # 4 workers x 6 rows x 4 B
    with pytest.raises(rt.RtopkError):
        rt.aggregate_update_workspace_bytes(10_000, 0, 10)
    # with momentum: null pointers, weights and velocity in one buffer
    assert lib.rtopk_aggregate_update_momentum(fake, fake, 2, 3, 10, 0.1, 1.0, 0.9, None, fake2,
                                               None) == -1
    assert lib.rtopk_aggregate_update_momentum(fake, fake, 2, 3, 10, 0.1, 1.0, 0.9, fake2, fake2,
                                               None) == -1
    # batched encode: no members, a null member pointer, overlap inside a member, workspace
    # that holds one member instead of two
    one = rt.encode_workspace_bytes(8, 4, 2)
    vp2 = ctypes.c_void_p * 2
    seeds = (u64 * 2)(1, 2)
    ok_g, ok_m = vp2(0x1000, 0x3000), vp2(0x100000, 0x300000)
    outs = vp2(0x5000, 0x7000)
    assert lib.rtopk_encode_batch(0, ok_g, ok_m, 8, 4, 2, seeds, 0, outs, outs, fake, big, None) == -1
    assert lib.rtopk_encode_batch(2, vp2(0x1000, None), ok_m, 8, 4, 2, seeds, 0, outs, outs, fake,
                                  big, None) == -1
    assert lib.rtopk_encode_batch(2, ok_g, vp2(0x100000, 0x3000), 8, 4, 2, seeds, 0, outs, outs,
                                  fake, big, None) == -1
    assert lib.rtopk_encode_batch(2, ok_g, ok_m, 8, 4, 2, seeds, 0, outs, outs, fake, u64(one),
                                  None) == -2
    assert lib.rtopk_encode_batch(2, ok_g, ok_m, 8, 5, 6, seeds, 0, outs, outs, fake, big, None) == -1
