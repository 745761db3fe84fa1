"""Parameter-byte accounting for the HiRE step (the paper's latency proxy PS, Sec. 3.1/3.2) and the
algorithmic bytes one step has to move, which the benchmark divides by the measured time.

PS formulas (bytes of parameters touched for the top-k problem of eq. (5), d x l matrix in bf16):
    dense baseline   2 d l
    HiRE-LR          2 (d r + r l + d k')
    HiRE-Q           d l / 2 + 2 d k'
"""
from __future__ import annotations


def ps_dense(d: int, l: int) -> int:
    return 2 * d * l


def ps_hire_lr(d: int, l: int, r: int, kprime: int) -> int:
    return 2 * (d * r + r * l + d * kprime)


def ps_hire_q(d: int, l: int, kprime: int) -> int:
    return d * l // 2 + 2 * d * kprime


def scorer_bytes(kind: str, d: int, N: int, r: int = 0) -> int:
    """Scorer parameters streamed per step: int4 codes + fp32 row scales, or the two low-rank factors (bf16, or
    int4 with scales for "lrq")."""
    if kind == "int4":
        return d * N // 2 + 4 * N
    if kind == "lrq":       # both factors as int4 codes with fp32 row scales
        return (d * r + r * N) // 2 + 4 * (r + N)
    return 2 * (d * r + r * N)


def ffn_step_bytes(kind: str, d: int, N: int, B: int, n_cand: int, n_sel_union: int, r: int = 0) -> dict:
    """Algorithmic HBM bytes of one HiRE-FFN step with the union sizes the step actually produced:
    scorer + gathered W1 rows (|U| rows of 2d bytes) + gathered W2 rows (|union of S_b| rows) + x in, y out."""
    parts = {
        "scorer": scorer_bytes(kind, d, N, r),
        "w1_gather": n_cand * 2 * d,
        "w2_gather": n_sel_union * 2 * d,
        "io": B * d * 2 + B * d * 4,
    }
    parts["total"] = sum(parts.values())
    parts["dense"] = 2 * ps_dense(d, N)      # both FFN matrices
    return parts


def softmax_step_bytes(kind: str, d: int, c: int, B: int, n_cand: int, k: int, r: int = 0) -> dict:
    parts = {
        "scorer": scorer_bytes(kind, d, c, r),
        "w_gather": n_cand * 2 * d,
        "io": B * d * 2 + B * k * 12,
    }
    parts["total"] = sum(parts.values())
    parts["dense"] = ps_dense(d, c)
    return parts


def expected_union(N: int, m: int, B: int) -> float:
    """E|union| of B independent uniformly random m-subsets of N."""
    return N * (1.0 - (1.0 - m / N) ** B)
