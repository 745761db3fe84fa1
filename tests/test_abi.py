"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function that
include/hire.h declares, sizes workspaces, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2402_09360_amd", "libhire.so")
HEADER = os.path.join(ROOT, "include", "hire.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2402_09360_amd import build
        build.build()
    return C.CDLL(LIB)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)))


def test_header_declares_the_three_entry_points():
    names = declared_functions()
    for f in ("hire_ffn_step", "hire_softmax_step", "topk_select", "hire_pack_int4", "hire_ffn_workspace_bytes"):
        assert f in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


class FFNLayer(C.Structure):
    _fields_ = [("d_model", C.c_int), ("d_ff", C.c_int), ("w1u", C.c_void_p), ("w2u", C.c_void_p),
                ("scorer_kind", C.c_int), ("q4", C.c_void_p), ("q4_scale", C.c_void_p), ("lr_a", C.c_void_p),
                ("lr_b", C.c_void_p), ("r", C.c_int)]


def test_workspace_sizes_and_pack_bytes(lib):
    lib.hire_pack_int4_bytes.restype = C.c_size_t
    assert lib.hire_pack_int4_bytes(16384, 2048) == 16384 * 1024
    assert lib.hire_pack_int4_bytes(10, 48) == 0          # cols must be a multiple of 32
    lib.hire_ffn_workspace_bytes.restype = C.c_size_t
    L = FFNLayer(2048, 16384, 0x1000, 0x2000, 0, 0x3000, 0x4000, None, None, 0)
    small = lib.hire_ffn_workspace_bytes(C.byref(L), 1, 819, 3276)
    big = lib.hire_ffn_workspace_bytes(C.byref(L), 16, 819, 3276)
    assert 0 < small < big < (1 << 28)
    assert lib.hire_ffn_workspace_bytes(C.byref(L), 1, 4000, 3276) == 0     # k > k'
    assert lib.hire_ffn_workspace_bytes(C.byref(L), 65, 819, 3276) == 0     # batch too large


def test_bad_arguments_are_rejected_on_the_host(lib):
    """Nothing is enqueued on an argument error, so fake (never dereferenced) pointers are safe here."""
    f = lib.hire_ffn_step
    f.restype = C.c_int
    f.argtypes = [C.POINTER(FFNLayer), C.c_void_p, C.c_int, C.c_int, C.c_int] + [C.c_void_p] * 7 + [C.c_size_t,
                                                                                                     C.c_void_p]
    good = FFNLayer(2048, 16384, 0x10000, 0x20000, 0, 0x30000, 0x40000, None, None, 0)
    x, y, ws = 0x50000, 0x60000, 0x70000

    def call(L=good, B=1, k=819, kp=3276, x=x, y=y, ws=ws, ws_bytes=1 << 30):
        return f(C.byref(L), x, B, k, kp, y, None, None, None, None, None, ws, ws_bytes, None)

    EINVAL, ENOSPC = -1, -2
    assert call(k=4000) == EINVAL                   # k > k'
    assert call(kp=20000) == EINVAL                 # k' > d_ff
    assert call(B=0) == EINVAL and call(B=65) == EINVAL
    assert call(x=None) == EINVAL and call(y=None) == EINVAL and call(ws=None) == EINVAL
    assert call(ws_bytes=1024) == ENOSPC
    assert call(L=FFNLayer(2040, 16384, 0x10000, 0x20000, 0, 0x30000, 0x40000, None, None, 0)) == EINVAL  # d % 32
    assert call(L=FFNLayer(2048, 16384, 0x10008, 0x20000, 0, 0x30000, 0x40000, None, None, 0)) == EINVAL  # misaligned
    assert call(L=FFNLayer(2048, 16384, 0x10000, 0x20000, 0, None, 0x40000, None, None, 0)) == EINVAL     # no q4
    assert call(L=FFNLayer(2048, 16384, 0x10000, 0x20000, 1, None, None, 0x30000, 0x40000, 12)) == EINVAL  # r % 8
    t = lib.topk_select
    t.restype = C.c_int
    t.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                  C.c_void_p]
    assert t(0x1000, 1, 100, 101, 0, 0x2000, None, None, 0, None) == EINVAL
    assert t(0x1000, 1, 100000, 5000, 2, 0x2000, None, None, 0, None) == -3   # rank order beyond the sort limit
    assert t(0x1000, 1, 100000, 50, 0, 0x2000, None, 0x3000, 256, None) == ENOSPC   # long rows keep histograms
    lib.hire_topk_workspace_bytes.restype = C.c_size_t
    lib.hire_topk_workspace_bytes.argtypes = [C.c_int] * 4
    assert lib.hire_topk_workspace_bytes(2, 16384, 100, 0) == 256
    # rank order on long rows: the same histograms plus the k survivors of every row staged in index order
    assert (lib.hire_topk_workspace_bytes(2, 100000, 100, 2) ==
            lib.hire_topk_workspace_bytes(2, 100000, 100, 0) + 2 * 1024)
    assert lib.hire_topk_workspace_bytes(2, 20000, 100, 2) == 256            # short rows: one workgroup per row
    assert lib.hire_topk_workspace_bytes(2, 100000, 100, 0) > 2 * 1024 * 1024
    lib.hire_strerror.restype = C.c_char_p
    assert b"workspace" in lib.hire_strerror(ENOSPC)
