"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function that the
headers under include/ declare, sizes workspaces, and rejects bad arguments before touching the device."""
import ctypes as C
import glob
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2402_09360_amd", "libhire.so")
HEADERS = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2402_09360_amd import build
        build.build()
    return C.CDLL(LIB)


def declared_functions(headers=None):
    names = set()
    for h in headers or HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names.update(re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text))
    return sorted(names)


def test_header_declares_the_three_entry_points():
    assert [os.path.basename(h) for h in HEADERS] == ["hire.h", "hire_debug.h"]
    names = declared_functions([os.path.join(ROOT, "include", "hire.h")])
    for f in ("hire_ffn_step", "hire_softmax_step", "topk_select", "hire_pack_int4", "hire_ffn_workspace_bytes",
              "hire_ffn_step_static"):
        assert f in names
    # testing and measurement aids live in the second header, not in the product interface
    assert not [n for n in names if "debug" in n or n.startswith("hire_set_") or n == "hire_force_generic_path"]
    assert "hire_debug_fast_fallbacks" in declared_functions()


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


class FFNLayer(C.Structure):
    _fields_ = [("d_model", C.c_int), ("d_ff", C.c_int), ("w1u", C.c_void_p), ("w2u", C.c_void_p),
                ("scorer_kind", C.c_int), ("q4", C.c_void_p), ("q4_scale", C.c_void_p), ("lr_a", C.c_void_p),
                ("lr_b", C.c_void_p), ("r", C.c_int), ("lr_a_scale", C.c_void_p), ("lr_b_scale", C.c_void_p)]


def test_workspace_sizes_and_pack_bytes(lib):
    lib.hire_pack_int4_bytes.restype = C.c_size_t
    assert lib.hire_pack_int4_bytes(16384, 2048) == 16384 * 1024 + 64   # codes + the trailer with the largest scale
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


def test_newer_entry_points_size_and_reject_on_the_host(lib):
    """Group-sparse, CommonPath and sharded steps: workspace sizes grow with the work, and every argument error
    comes back before anything is enqueued (fake pointers, never dereferenced)."""
    EINVAL, ENOSPC, EUNSUPPORTED = -1, -2, -3
    L = FFNLayer(2048, 16384, 0x10000, 0x20000, 0, 0x30000, 0x40000, None, None, 0, None, None)
    x, y, ws = 0x50000, 0x60000, 0x70000
    for name, n_int in (("hire_ffn_group_workspace_bytes", 4), ("hire_ffn_shard_workspace_bytes", 4),
                        ("hire_ffn_commonpath_workspace_bytes", 5)):
        f = getattr(lib, name)
        f.restype = C.c_size_t
        f.argtypes = [C.POINTER(FFNLayer)] + [C.c_int] * n_int
    gw, sw, cw = (lib.hire_ffn_group_workspace_bytes, lib.hire_ffn_shard_workspace_bytes,
                  lib.hire_ffn_commonpath_workspace_bytes)
    assert 0 < gw(C.byref(L), 1, 816, 3264, 8) < gw(C.byref(L), 16, 816, 3264, 8)
    assert gw(C.byref(L), 1, 816, 3264, 3) == 0 and gw(C.byref(L), 1, 819, 3264, 8) == 0
    assert gw(C.byref(L), 1, 816, 3268, 8) == 0 and gw(C.byref(L), 1, 816, 3264, 32) == 0
    assert 0 < sw(C.byref(L), 1, 768, 3328, 256) < sw(C.byref(L), 4, 768, 3328, 256)
    assert sw(C.byref(L), 1, 768, 3328, 8) == 0 and sw(C.byref(L), 1, 3400, 3328, 256) == 0
    assert sw(C.byref(L), 1, 819, 3276, 256) == sw(C.byref(L), 1, 768, 3328, 256)   # quotas rounded up, same partials
    assert sw(C.byref(L), 1, 768, 3328, 0) == 0 and sw(C.byref(L), 1, 768, 3328, 100) == 0
    assert cw(C.byref(L), 0, 1, 816, 3264, 8) >= gw(C.byref(L), 1, 816, 3264, 8)
    assert cw(C.byref(L), 2736, 4, 816, 3264, 8) > cw(C.byref(L), 0, 4, 816, 3264, 8)
    assert cw(C.byref(L), -1, 1, 816, 3264, 8) == 0

    g = lib.hire_ffn_group_step
    g.restype = C.c_int
    g.argtypes = ([C.POINTER(FFNLayer), C.c_void_p] + [C.c_int] * 4 + [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p])

    def group(B=1, k=816, kp=3264, grp=8, x=x, y=y, ws=ws, ws_bytes=1 << 30):
        return g(C.byref(L), x, B, k, kp, grp, y, None, None, None, None, None, ws, ws_bytes, None)

    assert group(grp=3) == EINVAL and group(k=819) == EINVAL and group(kp=3268) == EINVAL
    assert group(grp=0) == EINVAL and group(B=0) == EINVAL and group(B=65) == EINVAL
    assert group(x=None) == EINVAL and group(y=None) == EINVAL and group(ws=None) == EINVAL
    assert group(ws_bytes=1024) == ENOSPC

    sh = lib.hire_ffn_shard_step
    sh.restype = C.c_int
    sh.argtypes = g.argtypes

    def shard(B=1, k=768, kp=3328, s=256, x=x, y=y, ws=ws, ws_bytes=1 << 30):
        return sh(C.byref(L), x, B, k, kp, s, y, None, None, None, None, None, ws, ws_bytes, None)

    assert shard(k=3400) == EINVAL and shard(kp=16500) == EINVAL and shard(s=0) == EINVAL and shard(s=100) == EINVAL
    assert shard(s=8) == EUNSUPPORTED                  # 2048 units per shard
    assert shard(B=0) == EINVAL and shard(x=None) == EINVAL and shard(y=None) == EINVAL
    assert shard(ws_bytes=64) == ENOSPC
    lowrank = FFNLayer(2048, 16384, 0x10000, 0x20000, 1, None, None, 0x30000, 0x40000, 128, None, None)
    assert sh(C.byref(lowrank), x, 1, 768, 3328, 256, y, None, None, None, None, None, ws, 1 << 30, None) in (
        EINVAL, EUNSUPPORTED)                           # int4 scorer only

    c = lib.hire_ffn_commonpath_step
    c.restype = C.c_int
    c.argtypes = ([C.POINTER(FFNLayer), C.c_void_p, C.c_void_p, C.c_int, C.c_void_p] + [C.c_int] * 4 +
                  [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p])

    def common(m1=2736, w1=0x80000, w2=0x90000, k=816, kp=3264, grp=8, ws_bytes=1 << 30):
        return c(C.byref(L), w1, w2, m1, x, 1, k, kp, grp, y, None, None, None, None, None, ws, ws_bytes, None)

    assert common(m1=-1) == EINVAL and common(w1=None) == EINVAL and common(w2=None) == EINVAL
    assert common(w1=0x80008) == EINVAL                 # misaligned dense rows
    assert common(k=819) == EINVAL and common(grp=5) == EINVAL
    assert common(ws_bytes=1024) == ENOSPC


def test_lrq_scorer_arguments_are_checked_on_the_host(lib):
    """HiRE-LRQ: both int4 factors and both scale vectors must be there, the rank a multiple of 32 up to 1024."""
    f = lib.hire_ffn_step
    f.restype = C.c_int
    f.argtypes = [C.POINTER(FFNLayer), C.c_void_p, C.c_int, C.c_int, C.c_int] + [C.c_void_p] * 7 + [C.c_size_t,
                                                                                                     C.c_void_p]

    def call(r=128, a=0x30000, b=0x40000, sa=0x50000, sb=0x60000):
        L = FFNLayer(2048, 16384, 0x10000, 0x20000, 2, None, None, a, b, r, sa, sb)
        return f(C.byref(L), 0x70000, 1, 819, 3276, 0x80000, None, None, None, None, None, 0x90000, 64, None)

    EINVAL, ENOSPC = -1, -2
    assert call() == ENOSPC                              # valid layer: only the 64-byte workspace is wrong
    assert call(r=0) == EINVAL and call(r=48) == EINVAL and call(r=2048) == EINVAL
    assert call(a=None) == EINVAL and call(b=None) == EINVAL
    assert call(sa=None) == EINVAL and call(sb=None) == EINVAL
    lib.hire_ffn_workspace_bytes.restype = C.c_size_t
    L = FFNLayer(2048, 16384, 0x10000, 0x20000, 2, None, None, 0x30000, 0x40000, 128, 0x50000, 0x60000)
    assert lib.hire_ffn_workspace_bytes(C.byref(L), 1, 819, 3276) > 0
    assert lib.hire_ffn_workspace_bytes(C.byref(L), 1, 819, 20000) == 0    # k' beyond the units
