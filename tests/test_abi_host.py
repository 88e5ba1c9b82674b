"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and
rejects bad arguments before touching the GPU (so these run without one)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ev():
    import paper_2605_27390_amd as ev
    return ev


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            src = open(os.path.join(inc, fn)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names |= set(re.findall(r"\b(evospec_[a-z_]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol(ev):
    syms = declared_symbols()
    assert "evospec_active_gather" in syms and "evospec_active_lmhead_topk" in syms
    assert len(syms) >= 11
    for s in syms:
        assert hasattr(ev.lib, s), f"{s} declared in include/ but not exported"
    assert ev.version() == 210


def test_status_strings(ev):
    for code in range(11):
        assert ev.status_string(code) and ev.status_string(code) != "unknown status"
    assert ev.status_string(99) == "unknown status"


def test_workspace_bytes(ev):
    a = ev.workspace_bytes(60, 36864, 4096, 10)
    b = ev.workspace_bytes(60, 151936, 4096, 10)
    assert 0 < a < b
    assert ev.workspace_bytes(60, 36864, 4096, 20) > a
    assert ev.workspace_bytes(128, 36864, 4096, 10) == a           # 64-row passes reuse the scratch
    assert ev.workspace_bytes(960, 36864, 4104, 10) == a           # hidden size not a multiple of 64: passes
    # from 129 rows on one launch keeps a partial per 128 active rows and draft row
    big = ev.workspace_bytes(960, 36864, 4096, 10)
    assert big >= 288 * 960 * (10 * 8 + 8)
    seg = ev.workspace_bytes_segmented(960, 32768, 2048, 16, 4096, 10)
    assert seg >= 256 * 960 * (10 * 8 + 8) + ev.workspace_bytes(64, 2048, 4096, 10)
    seg_small = ev.workspace_bytes_segmented(128, 32768, 2048, 4, 4096, 10)
    assert seg_small >= 2 * ev.workspace_bytes(64, 32768, 4096, 10)
    out = ctypes.c_size_t(0)
    L = ev.lib
    assert L.evospec_workspace_bytes(1, 10, 64, 1, None) == 1
    assert L.evospec_workspace_bytes(1, 10, 60, 1, ctypes.byref(out)) == 2       # d % 8
    assert L.evospec_workspace_bytes(1, 0, 64, 1, ctypes.byref(out)) == 2
    assert L.evospec_workspace_bytes(-1, 10, 64, 1, ctypes.byref(out)) == 2
    assert L.evospec_workspace_bytes(1, 10, 64, 0, ctypes.byref(out)) == 3
    assert L.evospec_workspace_bytes(1, 10, 64, 11, ctypes.byref(out)) == 3      # k > V_act
    assert L.evospec_workspace_bytes(1, 1000, 64, 65, ctypes.byref(out)) == 3    # k > K_MAX


def test_matrix_bytes(ev):
    # row-major: rows x d; packed: rows to a multiple of 16, d to a multiple of 256
    assert ev.matrix_bytes(36864, 4096, ev.ROW_MAJOR) == 36864 * 4096 * 2
    assert ev.matrix_bytes(36864, 4096, ev.PACKED) == 36864 * 4096 * 2
    assert ev.matrix_bytes(33, 72, ev.ROW_MAJOR) == 33 * 72 * 2
    assert ev.matrix_bytes(33, 72, ev.PACKED) == 48 * 256 * 2
    assert ev.matrix_bytes(0, 64, ev.PACKED) == 0
    out = ctypes.c_size_t(0)
    L = ev.lib
    assert L.evospec_matrix_bytes(10, 64, 0, None) == 1
    assert L.evospec_matrix_bytes(10, 60, 0, ctypes.byref(out)) == 2
    assert L.evospec_matrix_bytes(-1, 64, 0, ctypes.byref(out)) == 2
    assert L.evospec_matrix_bytes(10, 64, 2, ctypes.byref(out)) == 9


def test_head_argument_errors_need_no_gpu(ev):
    L = ev.lib
    buf = ctypes.create_string_buffer(4096 + 64)
    base = ctypes.addressof(buf)
    al = ctypes.c_void_p((base + 15) // 16 * 16)          # a 16-byte aligned host address (never dereferenced)
    mis = ctypes.c_void_p(al.value + 2)
    f = L.evospec_active_lmhead_topk
    big = 1 << 30
    # every call below fails validation on the host: nothing is ever launched on these host addresses
    assert f(None, 4, 64, al, None, 100, 0, 5, al, al, al, al, big, None) == 1
    assert f(al, 4, 64, None, None, 100, 0, 5, al, al, al, al, big, None) == 1
    assert f(al, 4, 64, al, None, 100, 0, 5, None, al, al, al, big, None) == 1
    assert f(al, 4, 64, al, None, 100, 0, 5, al, al, al, None, big, None) == 1
    assert f(al, 4, 60, al, None, 100, 0, 5, al, al, al, al, big, None) == 2
    assert f(al, -1, 64, al, None, 100, 0, 5, al, al, al, al, big, None) == 2
    assert f(al, 4, 64, al, None, 0, 0, 5, al, al, al, al, big, None) == 2
    assert f(al, 4, 64, al, None, 100, 0, 0, al, al, al, al, big, None) == 3
    assert f(al, 4, 64, al, None, 100, 0, 101, al, al, al, al, big, None) == 3
    assert f(al, 4, 64, al, None, 100, 0, 65, al, al, al, al, big, None) == 3
    assert f(mis, 4, 64, al, None, 100, 0, 5, al, al, al, al, big, None) == 4
    assert f(al, 4, 64, mis, None, 100, 0, 5, al, al, al, al, big, None) == 4
    assert f(al, 4, 64, al, None, 100, 0, 5, al, al, al, mis, big, None) == 4
    assert f(al, 4, 64, al, None, 100, 0, 5, al, al, al, al, 16, None) == 5
    assert f(al, 0, 64, al, None, 100, 0, 5, al, al, al, al, 0, None) == 0             # M == 0: no-op
    g = L.evospec_active_lmhead_partials
    assert g(al, 65, 64, al, None, 100, 0, 5, al, big, None) == 2                       # one 64-row pass only
    assert g(al, 4, 64, al, None, 100, 0, 5, al, 16, None) == 5
    assert g(al, 4, 64, al, None, 100, 2, 5, al, big, None) == 9                     # unknown layout
    assert f(al, 4, 64, al, None, 100, 7, 5, al, al, al, al, big, None) == 9
    assert f(al, 4, 64, al, None, 100, 1, 5, al, al, al, al, 16, None) == 5            # packed: same checks


def test_static_scratch_entry_rejects_on_the_host(ev):
    """The no-allocation variant: same argument checks as the workspace variant, and shapes whose
    scratch need exceeds the fixed array are refused before any HIP call."""
    L = ev.lib
    buf = ctypes.create_string_buffer(4096 + 64)
    al = ctypes.c_void_p((ctypes.addressof(buf) + 15) // 16 * 16)
    f = L.evospec_active_lmhead_topk_static
    assert f(al, 4, 60, al, None, 100, 0, 5, al, al, al, None) == 2
    assert f(al, 4, 64, al, None, 100, 0, 0, al, al, al, None) == 3
    assert f(al, 0, 64, al, None, 100, 0, 5, al, al, al, None) == 0             # M == 0: no-op
    cap = ev.STATIC_SCRATCH_BYTES
    assert ev.workspace_bytes(60, 36864, 4096, 10) <= cap                       # the headline shape fits
    assert ev.workspace_bytes(60, 151936, 4096, 10) > cap
    assert f(al, 60, 4096, al, None, 151936, 0, 10, al, al, al, None) == 10
    assert ev.workspace_bytes(960, 36864, 4096, 10) > cap
    assert f(al, 960, 4096, al, None, 36864, 0, 10, al, al, al, None) == 10
    assert "EVOSPEC_STATIC_SCRATCH_BYTES" in ev.status_string(10)


def test_gather_argument_errors_need_no_gpu(ev):
    L = ev.lib
    buf = ctypes.create_string_buffer(256)
    al = ctypes.c_void_p((ctypes.addressof(buf) + 15) // 16 * 16)
    mis = ctypes.c_void_p(al.value + 4)
    f = L.evospec_active_gather
    assert f(al, 100, 64, al, None, 0, al, al, 10, 0, None) == 0                        # n == 0: no-op
    assert f(al, 100, 64, al, None, 11, al, al, 10, 0, None) == 2                       # n > V_act without slots
    assert f(al, 100, 60, al, None, 1, al, al, 10, 0, None) == 2
    assert f(al, 0, 64, al, None, 1, al, al, 10, 0, None) == 2
    assert f(al, 100, 64, al, None, -1, al, al, 10, 0, None) == 2
    assert f(None, 100, 64, al, None, 1, al, al, 10, 0, None) == 1
    assert f(al, 100, 64, None, None, 1, al, al, 10, 0, None) == 1
    assert f(al, 100, 64, al, None, 1, None, al, 10, 0, None) == 1
    assert f(al, 100, 64, al, None, 1, al, None, 10, 0, None) == 1
    assert f(mis, 100, 64, al, None, 1, al, al, 10, 0, None) == 4
    assert f(al, 100, 64, al, None, 1, mis, al, 10, 0, None) == 4
    assert f(al, 100, 64, al, None, 1, al, al, 10, 3, None) == 9                     # unknown layout
    assert f(al, 100, 64, al, None, 11, al, al, 10, 1, None) == 2                    # packed: same checks


def test_segment_errors_need_no_gpu(ev):
    L = ev.lib
    buf = ctypes.create_string_buffer(256)
    al = ctypes.c_void_p((ctypes.addressof(buf) + 15) // 16 * 16)
    f = L.evospec_active_lmhead_topk_segmented
    big = 1 << 30

    def ro(*v):
        return (ctypes.c_int32 * len(v))(*v)

    args = lambda r, S=2, M=8: (al, M, 64, al, None, 50, al, al, 10, 0, r, S, 5, al, al, al, al, big, None)
    assert f(*args(ro(1, 4, 8))) == 6
    assert f(*args(ro(0, 4, 7))) == 6
    assert f(*args(ro(0, 9, 8))) == 6
    assert f(*args(None)) == 1
    assert f(*args(ro(0, 0, 0), M=0)) == 0
    assert f(al, 8, 64, al, None, 50, al, al, 10, 0, ro(0, 4, 8), 0, 5, al, al, al, al, big, None) == 2
    assert f(al, 8, 64, al, None, 50, al, al, 10, 0, ro(0, 4, 8), 2, 61, al, al, al, al, big, None) == 3
    assert f(al, 8, 64, al, None, 50, al, al, 10, 5, ro(0, 4, 8), 2, 5, al, al, al, al, big, None) == 9


def test_validate_ids_argument_errors(ev):
    L = ev.lib
    assert L.evospec_validate_ids(None, 0, 10, None) == 0
    assert L.evospec_validate_ids(None, 5, 10, None) == 1
    assert L.evospec_validate_ids(None, -1, 10, None) == 2
