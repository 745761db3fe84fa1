"""ctypes access to the CPU oracle (oracle/hire_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg.  Nothing here touches the GPU library.
All arrays are numpy; bf16 tensors are uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hire_oracle.c")
_LIB = os.path.join(_HERE, "libhire_oracle.so")

SCORER_INT4 = 0
SCORER_LOWRANK = 1
SCORER_LRQ = 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O3 -fopenmp, no fast-math: double sums stay sequential).  HIRE_ORACLE_LIB names
    a library built otherwise from the same source (the sanitizer build of the test suite) to load instead."""
    if os.environ.get("HIRE_ORACLE_LIB"):
        return os.environ["HIRE_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16
    return a


def quantize_rows_int4(w_bits: np.ndarray):
    """Per-row symmetric int4 codes (int8 storage, values in [-7,7]) and fp32 scales."""
    w_bits = _u16(w_bits)
    rows, cols = w_bits.shape
    q = np.empty((rows, cols), dtype=np.int8)
    s = np.empty(rows, dtype=np.float32)
    lib().hire_oracle_quantize_rows_int4(_p(w_bits, C.c_uint16), rows, cols, _p(q, C.c_int8), _p(s, C.c_float))
    return q, s


def quantize_tokens_int8(x_bits: np.ndarray):
    x_bits = _u16(x_bits)
    B, d = x_bits.shape
    xq = np.empty((B, d), dtype=np.int8)
    sx = np.empty(B, dtype=np.float32)
    lib().hire_oracle_quantize_tokens_int8(_p(x_bits, C.c_uint16), B, d, _p(xq, C.c_int8), _p(sx, C.c_float))
    return xq, sx


def scorer_int4(q: np.ndarray, scale: np.ndarray, xq: np.ndarray, relu: bool):
    q = np.ascontiguousarray(q, dtype=np.int8)
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    N, d = q.shape
    B = xq.shape[0]
    acc = np.empty((B, N), dtype=np.int32)
    key = np.empty((B, N), dtype=np.float32)
    lib().hire_oracle_scorer_int4(_p(q, C.c_int8), _p(scale, C.c_float), _p(xq, C.c_int8), B, N, d, int(relu),
                                  _p(acc, C.c_int32), _p(key, C.c_float))
    return acc, key


def scorer_lowrank(z1_bits, z2_bits, x_bits, relu: bool):
    z1_bits, z2_bits, x_bits = _u16(z1_bits), _u16(z2_bits), _u16(x_bits)
    d, r = z1_bits.shape
    N = z2_bits.shape[0]
    B = x_bits.shape[0]
    t = np.empty((B, r), dtype=np.uint16)
    key = np.empty((B, N), dtype=np.float64)
    lib().hire_oracle_scorer_lowrank(_p(z1_bits, C.c_uint16), _p(z2_bits, C.c_uint16), _p(x_bits, C.c_uint16), B, N, d,
                                     r, int(relu), _p(t, C.c_uint16), _p(key, C.c_double))
    return t, key


def topk(v: np.ndarray, k: int, rank_order: bool = False, return_margin: bool = False):
    v = np.ascontiguousarray(v, dtype=np.float64)
    idx = np.empty(k, dtype=np.int32)
    m = C.c_double(0.0)
    lib().hire_oracle_topk(_p(v, C.c_double), v.size, k, int(rank_order), _p(idx, C.c_int32), C.byref(m))
    return (idx, m.value) if return_margin else idx


def topk_f32(v: np.ndarray, k: int, relu: bool = False, rank_order: bool = False):
    v = np.ascontiguousarray(v, dtype=np.float32)
    idx = np.empty(k, dtype=np.int32)
    lib().hire_oracle_topk_f32(_p(v, C.c_float), v.size, k, int(relu), int(rank_order), _p(idx, C.c_int32))
    return idx


def union(sets: np.ndarray, N: int):
    sets = np.ascontiguousarray(sets, dtype=np.int32)
    B, m = sets.shape
    U = np.empty(min(B * m, N), dtype=np.int32)
    n = lib().hire_oracle_union(_p(sets, C.c_int32), B, m, N, _p(U, C.c_int32))
    return U[:n].copy()


def exact_scores(W_bits, x_bits, U, relu: bool):
    W_bits, x_bits = _u16(W_bits), _u16(x_bits)
    U = np.ascontiguousarray(U, dtype=np.int32)
    B, d = x_bits.shape
    h = np.empty((B, U.size), dtype=np.float64)
    lib().hire_oracle_exact_scores(_p(W_bits, C.c_uint16), _p(x_bits, C.c_uint16), _p(U, C.c_int32), U.size, B, d,
                                   int(relu), _p(h, C.c_double))
    return h


def _scorer_args(scorer):
    """scorer = ("int4", q, scale), ("lowrank", z1_bits, z2_bits) or ("lrq", q1 [r,d], s1 [r], q2 [N,r], s2 [N])
    -> (kind, arrays to keep alive, the C functions' scorer arguments q, qscale, z1, z2, r, q1, s1)."""
    if scorer[0] == "int4":
        q = np.ascontiguousarray(scorer[1], dtype=np.int8)
        s = np.ascontiguousarray(scorer[2], dtype=np.float32)
        return SCORER_INT4, (q, s), (_p(q, C.c_int8), _p(s, C.c_float), None, None, 0, None, None)
    if scorer[0] == "lrq":
        q1 = np.ascontiguousarray(scorer[1], dtype=np.int8)
        s1 = np.ascontiguousarray(scorer[2], dtype=np.float32)
        q2 = np.ascontiguousarray(scorer[3], dtype=np.int8)
        s2 = np.ascontiguousarray(scorer[4], dtype=np.float32)
        assert q1.shape[0] == q2.shape[1] == s1.size and q2.shape[0] == s2.size
        return SCORER_LRQ, (q1, s1, q2, s2), (_p(q2, C.c_int8), _p(s2, C.c_float), None, None, q1.shape[0],
                                              _p(q1, C.c_int8), _p(s1, C.c_float))
    z1, z2 = _u16(scorer[1]), _u16(scorer[2])
    return SCORER_LOWRANK, (z1, z2), (None, None, _p(z1, C.c_uint16), _p(z2, C.c_uint16), z1.shape[1], None, None)


def lrq_factors(z1_bits, z2_bits):
    """The int4 copies HiRE-LRQ scores with: Z1 [d, r] transposed to rows and Z2 [N, r], each quantised row by row.
    Returns ("lrq", q1 [r,d], s1 [r], q2 [N,r], s2 [N])."""
    z1t = np.ascontiguousarray(_u16(z1_bits).T)
    q1, s1 = quantize_rows_int4(z1t)
    q2, s2 = quantize_rows_int4(_u16(z2_bits))
    return ("lrq", q1, s1, q2, s2)


def scorer_lrq(q1, s1, q2, s2, x_bits, relu: bool):
    """HiRE-LRQ keys fp32 [B, N] and the bf16 intermediate t [B, r]."""
    q1 = np.ascontiguousarray(q1, dtype=np.int8)
    q2 = np.ascontiguousarray(q2, dtype=np.int8)
    s1 = np.ascontiguousarray(s1, dtype=np.float32)
    s2 = np.ascontiguousarray(s2, dtype=np.float32)
    x_bits = _u16(x_bits)
    r, d = q1.shape
    N = q2.shape[0]
    B = x_bits.shape[0]
    t = np.empty((B, r), dtype=np.uint16)
    key = np.empty((B, N), dtype=np.float32)
    lib().hire_oracle_scorer_lrq(_p(q1, C.c_int8), _p(s1, C.c_float), _p(q2, C.c_int8), _p(s2, C.c_float),
                                 _p(x_bits, C.c_uint16), B, N, d, r, int(relu), _p(t, C.c_uint16), _p(key, C.c_float))
    return t, key


def ffn_step(w1u_bits, w2u_bits, scorer, x_bits, k: int, kprime: int, want_acc: bool = False):
    """One HiRE-FFN step.  Returns a dict: y f32 [B,d], topk_idx [B,k] ascending, topk_val f64 [B,k],
    cand (ascending union), acc (optional int32 [B,N]), margin_kprime [B], margin_k [B]."""
    w1u_bits, w2u_bits, x_bits = _u16(w1u_bits), _u16(w2u_bits), _u16(x_bits)
    N, d = w1u_bits.shape
    B = x_bits.shape[0]
    kind, keep, sargs = _scorer_args(scorer)
    y = np.empty((B, d), dtype=np.float32)
    idx = np.empty((B, k), dtype=np.int32)
    val = np.empty((B, k), dtype=np.float64)
    U = np.empty(min(B * kprime, N), dtype=np.int32)
    acc = np.empty((B, N), dtype=np.int32) if (want_acc and kind == SCORER_INT4) else None
    mkp = np.empty(B, dtype=np.float64)
    mk = np.empty(B, dtype=np.float64)
    f = lib().hire_oracle_ffn_step
    f.restype = C.c_int
    n = f(_p(w1u_bits, C.c_uint16), _p(w2u_bits, C.c_uint16), kind, *sargs, _p(x_bits, C.c_uint16), B, d, N, k, kprime,
          _p(y, C.c_float), _p(idx, C.c_int32), _p(val, C.c_double), _p(U, C.c_int32), _p(acc, C.c_int32),
          _p(mkp, C.c_double), _p(mk, C.c_double))
    del keep
    return dict(y=y, topk_idx=idx, topk_val=val, cand=U[:n].copy(), acc=acc, margin_kprime=mkp, margin_k=mk)


def ffn_group_step(w1u_bits, w2u_bits, scorer, x_bits, k: int, kprime: int, g: int, want_acc: bool = False):
    """One group-sparse HiRE-FFN step (groups of g adjacent units; k and k' count units).  Returns a dict:
    y f32 [B,d], topk_group [B,k/g] ascending, topk_val f64 [B,k], cand (ascending union of groups),
    acc (optional int32 [B,N]), margin_kprime [B], margin_k [B]."""
    w1u_bits, w2u_bits, x_bits = _u16(w1u_bits), _u16(w2u_bits), _u16(x_bits)
    N, d = w1u_bits.shape
    B = x_bits.shape[0]
    assert g >= 1 and N % g == 0 and k % g == 0 and kprime % g == 0
    kind, keep, sargs = _scorer_args(scorer)
    y = np.empty((B, d), dtype=np.float32)
    grp = np.empty((B, k // g), dtype=np.int32)
    val = np.empty((B, k), dtype=np.float64)
    U = np.empty(min(B * (kprime // g), N // g), dtype=np.int32)
    acc = np.empty((B, N), dtype=np.int32) if (want_acc and kind == SCORER_INT4) else None
    mkp = np.empty(B, dtype=np.float64)
    mk = np.empty(B, dtype=np.float64)
    f = lib().hire_oracle_ffn_group_step
    f.restype = C.c_int
    n = f(_p(w1u_bits, C.c_uint16), _p(w2u_bits, C.c_uint16), kind, *sargs, _p(x_bits, C.c_uint16), B, d, N, k, kprime,
          g, _p(y, C.c_float), _p(grp, C.c_int32), _p(val, C.c_double), _p(U, C.c_int32), _p(acc, C.c_int32),
          _p(mkp, C.c_double), _p(mk, C.c_double))
    del keep
    assert n >= 0
    return dict(y=y, topk_group=grp, topk_val=val, cand=U[:n].copy(), acc=acc, margin_kprime=mkp, margin_k=mk)


def ffn_commonpath_step(dense_w1u_bits, dense_w2u_bits, w1u_bits, w2u_bits, scorer, x_bits, k: int, kprime: int,
                        g: int, want_acc: bool = False):
    """One CommonPath FFN step (eq. (7)): the dense units [m1, d] used by every token plus the group-sparse HiRE step
    on the other units.  Returns the group step's dict with y = dense part + sparse part."""
    dw1, dw2 = _u16(dense_w1u_bits), _u16(dense_w2u_bits)
    w1u_bits, w2u_bits, x_bits = _u16(w1u_bits), _u16(w2u_bits), _u16(x_bits)
    N, d = w1u_bits.shape
    m1 = dw1.shape[0]
    assert dw1.shape == dw2.shape and (m1 == 0 or dw1.shape[1] == d)
    B = x_bits.shape[0]
    assert g >= 1 and N % g == 0 and k % g == 0 and kprime % g == 0
    kind, keep, sargs = _scorer_args(scorer)
    y = np.empty((B, d), dtype=np.float32)
    grp = np.empty((B, k // g), dtype=np.int32)
    val = np.empty((B, k), dtype=np.float64)
    U = np.empty(min(B * (kprime // g), N // g), dtype=np.int32)
    acc = np.empty((B, N), dtype=np.int32) if (want_acc and kind == SCORER_INT4) else None
    mkp = np.empty(B, dtype=np.float64)
    mk = np.empty(B, dtype=np.float64)
    f = lib().hire_oracle_ffn_commonpath_step
    f.restype = C.c_int
    n = f(_p(dw1, C.c_uint16), _p(dw2, C.c_uint16), m1, _p(w1u_bits, C.c_uint16), _p(w2u_bits, C.c_uint16), kind,
          *sargs, _p(x_bits, C.c_uint16), B, d, N, k, kprime, g, _p(y, C.c_float), _p(grp, C.c_int32),
          _p(val, C.c_double), _p(U, C.c_int32), _p(acc, C.c_int32), _p(mkp, C.c_double), _p(mk, C.c_double))
    del keep
    assert n >= 0
    return dict(y=y, topk_group=grp, topk_val=val, cand=U[:n].copy(), acc=acc, margin_kprime=mkp, margin_k=mk)


def ffn_shard_step(w1u_bits, w2u_bits, scorer, x_bits, k: int, kprime: int, shards: int, want_acc: bool = False):
    """One HiRE-FFN step with the distributed approximate top-k of Algorithm 2 over `shards` contiguous shards of
    the hidden units (int4 scorer), per-shard quotas ceil(k'/shards) and ceil(k/shards).  Returns a dict: y f32
    [B,d], topk_idx [B, shards*ceil(k/shards)] (shard after shard, ascending), topk_val f64 of the same shape,
    cand = list of per-shard ascending unions, acc, margin_kprime [B], margin_k [B]."""
    w1u_bits, w2u_bits, x_bits = _u16(w1u_bits), _u16(w2u_bits), _u16(x_bits)
    N, d = w1u_bits.shape
    B = x_bits.shape[0]
    assert shards >= 1 and N % shards == 0
    kind, keep, sargs = _scorer_args(scorer)
    assert kind == SCORER_INT4
    qp, q = -(-kprime // shards), -(-k // shards)
    cap = min(B * qp, N // shards)
    y = np.empty((B, d), dtype=np.float32)
    idx = np.empty((B, shards * q), dtype=np.int32)
    val = np.empty((B, shards * q), dtype=np.float64)
    U = np.zeros((shards, cap), dtype=np.int32)
    nU = np.zeros(shards, dtype=np.int32)
    acc = np.empty((B, N), dtype=np.int32) if want_acc else None
    mkp = np.empty(B, dtype=np.float64)
    mk = np.empty(B, dtype=np.float64)
    f = lib().hire_oracle_ffn_shard_step
    f.restype = C.c_int
    rc = f(_p(w1u_bits, C.c_uint16), _p(w2u_bits, C.c_uint16), sargs[0], sargs[1], _p(x_bits, C.c_uint16), B, d, N, k,
           kprime, shards, _p(y, C.c_float), _p(idx, C.c_int32), _p(val, C.c_double), _p(U, C.c_int32),
           _p(nU, C.c_int32), _p(acc, C.c_int32), _p(mkp, C.c_double), _p(mk, C.c_double))
    del keep
    assert rc == 0
    return dict(y=y, topk_idx=idx, topk_val=val, cand=[U[i, :nU[i]].copy() for i in range(shards)], n_cand=nU,
                acc=acc, margin_kprime=mkp, margin_k=mk)


def softmax_step(W_bits, scorer, x_bits, k: int, kprime: int, want_acc: bool = False):
    """One HiRE-Softmax step.  Returns top_idx [B,k] (rank order), top_prob / top_logit f64 [B,k], cand, acc."""
    W_bits, x_bits = _u16(W_bits), _u16(x_bits)
    c, d = W_bits.shape
    B = x_bits.shape[0]
    kind, keep, sargs = _scorer_args(scorer)
    idx = np.empty((B, k), dtype=np.int32)
    prob = np.empty((B, k), dtype=np.float64)
    logit = np.empty((B, k), dtype=np.float64)
    U = np.empty(min(B * kprime, c), dtype=np.int32)
    acc = np.empty((B, c), dtype=np.int32) if (want_acc and kind == SCORER_INT4) else None
    mkp = np.empty(B, dtype=np.float64)
    mk = np.empty(B, dtype=np.float64)
    f = lib().hire_oracle_softmax_step
    f.restype = C.c_int
    n = f(_p(W_bits, C.c_uint16), kind, *sargs, _p(x_bits, C.c_uint16), B, d, c, k, kprime, _p(idx, C.c_int32),
          _p(prob, C.c_double), _p(logit, C.c_double), _p(U, C.c_int32), _p(acc, C.c_int32), _p(mkp, C.c_double),
          _p(mk, C.c_double))
    del keep
    return dict(top_idx=idx, top_prob=prob, top_logit=logit, cand=U[:n].copy(), acc=acc, margin_kprime=mkp,
                margin_k=mk)


def dense_ffn(w1u_bits, w2u_bits, x_bits):
    w1u_bits, w2u_bits, x_bits = _u16(w1u_bits), _u16(w2u_bits), _u16(x_bits)
    N, d = w1u_bits.shape
    B = x_bits.shape[0]
    y = np.empty((B, d), dtype=np.float64)
    lib().hire_oracle_dense_ffn(_p(w1u_bits, C.c_uint16), _p(w2u_bits, C.c_uint16), _p(x_bits, C.c_uint16), B, d, N,
                                _p(y, C.c_double))
    return y


def topk_ffn(w1u_bits, w2u_bits, x_bits, k: int):
    w1u_bits, w2u_bits, x_bits = _u16(w1u_bits), _u16(w2u_bits), _u16(x_bits)
    N, d = w1u_bits.shape
    B = x_bits.shape[0]
    y = np.empty((B, d), dtype=np.float64)
    S = np.empty((B, k), dtype=np.int32)
    lib().hire_oracle_topk_ffn(_p(w1u_bits, C.c_uint16), _p(w2u_bits, C.c_uint16), _p(x_bits, C.c_uint16), B, d, N, k,
                               _p(y, C.c_double), _p(S, C.c_int32))
    return y, S


def dense_softmax(W_bits, x_bits):
    W_bits, x_bits = _u16(W_bits), _u16(x_bits)
    c, d = W_bits.shape
    B = x_bits.shape[0]
    p = np.empty((B, c), dtype=np.float64)
    lib().hire_oracle_dense_softmax(_p(W_bits, C.c_uint16), _p(x_bits, C.c_uint16), B, d, c, _p(p, C.c_double))
    return p


def softmax_k(W_bits, x_bits, k: int):
    W_bits, x_bits = _u16(W_bits), _u16(x_bits)
    c, d = W_bits.shape
    B = x_bits.shape[0]
    p = np.empty((B, c), dtype=np.float64)
    lib().hire_oracle_softmax_k(_p(W_bits, C.c_uint16), _p(x_bits, C.c_uint16), B, d, c, k, _p(p, C.c_double))
    return p


def num_threads() -> int:
    f = lib().hire_oracle_num_threads
    f.restype = C.c_int
    return int(f())
