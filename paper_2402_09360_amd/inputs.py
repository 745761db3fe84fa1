"""Seeded synthetic inputs for the HiRE decode-step path.

This module only *draws numbers*: Gaussian bf16 weight matrices and token
vectors in the shapes of a ~1B-parameter decoder.  It contains none of the
method's arithmetic (no quantiser, no scorer, no top-k), so the CPU oracle
and the HIP path can both be fed from it without sharing any code of the
method itself.  Every tensor is a numpy array; bf16 tensors are carried as
uint16 bit patterns so that both sides consume byte-identical data.

Generator: numpy's counter-based Philox bit generator keyed by the seed, so a
(seed, shape) pair names one tensor.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "f32_to_bf16_bits", "bf16_bits_to_f32", "bf16_bits_to_f64",
    "normal_bf16", "tokens", "correlated_tokens", "ffn_layer", "classifier",
    "lowrank_ffn_layer", "CONFIGS",
]


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def normal_bf16(seed: int, shape, std: float = 1.0, chunk_rows: int = 8192) -> np.ndarray:
    """N(0, std^2) samples rounded to bf16, as uint16 bits of the given shape.

    Drawn row-chunk by row-chunk from one Philox stream, so the result does
    not depend on the chunk size and large tensors never exist in fp32 whole.
    """
    shape = tuple(int(s) for s in shape)
    rng = _rng(seed)
    if len(shape) != 2:
        v = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        return f32_to_bf16_bits(v)
    rows, cols = shape
    out = np.empty(shape, dtype=np.uint16)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        v = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        v *= np.float32(std)
        out[r0:r1] = f32_to_bf16_bits(v)
    return out


def tokens(seed: int, B: int, d_model: int) -> np.ndarray:
    """B iid token vectors, entries N(0,1), bf16 bits [B, d_model]."""
    return normal_bf16(seed, (B, d_model), 1.0)


def correlated_tokens(seed: int, B: int, d_model: int, rho: float) -> np.ndarray:
    """Tokens sharing a common component: x_b = sqrt(rho) c + sqrt(1-rho) e_b.

    Stands in for several samples of one query, whose activations overlap.
    """
    rng = _rng(seed)
    c = rng.standard_normal((1, d_model), dtype=np.float32)
    e = rng.standard_normal((B, d_model), dtype=np.float32)
    x = np.float32(np.sqrt(rho)) * c + np.float32(np.sqrt(1.0 - rho)) * e
    return f32_to_bf16_bits(x)


def ffn_layer(seed: int, d_model: int, d_ff: int) -> dict:
    """One FFN layer with entries N(0, 1/d_model).

    W1 is drawn in its mathematical orientation (d_model x d_ff) and then
    transposed once into the unit-major store w1u[d_ff, d_model] (row j = u_j);
    W2 (d_ff x d_model) is already unit-major (row j = v_j).
    """
    std = float(d_model) ** -0.5
    w1_math = normal_bf16(2 * seed + 0, (d_model, d_ff), std)
    w1u = np.ascontiguousarray(w1_math.T)
    del w1_math
    w2u = normal_bf16(2 * seed + 1, (d_ff, d_model), std)
    return {"d_model": d_model, "d_ff": d_ff, "w1u": w1u, "w2u": w2u}


def classifier(seed: int, vocab: int, d_model: int) -> np.ndarray:
    """Classifier matrix, one row per class, entries N(0, 1/d_model); bf16 bits [vocab, d_model]."""
    return normal_bf16(seed, (vocab, d_model), float(d_model) ** -0.5)


def lowrank_ffn_layer(seed: int, d_model: int, d_ff: int, r: int) -> dict:
    """FFN layer whose first-layer matrix has a decaying spectrum, plus rank-r factors.

    W1 = P diag(sigma) Q^T with P (d_model x d_model) and Q (d_ff x d_model)
    orthonormal (QR of seeded Gaussians), sigma_i proportional to i^-1/2 and
    scaled so that the mean squared entry is 1/d_model.  The factors handed to
    the low-rank scorer are the leading r terms of that decomposition:
    z1 = P[:, :r] diag(sigma[:r]) (bf16 [d_model, r]) and z2 = Q[:, :r]
    (bf16 [d_ff, r]).  They are inputs to both sides, so no SVD sign or
    rotation ambiguity enters any comparison.
    """
    rng = _rng(seed)
    P, _ = np.linalg.qr(rng.standard_normal((d_model, d_model)))
    Q, _ = np.linalg.qr(rng.standard_normal((d_ff, d_model)))
    sigma = np.arange(1, d_model + 1, dtype=np.float64) ** -0.5
    sigma *= np.sqrt(float(d_ff) / np.sum(sigma ** 2))
    w1u = (Q * sigma[None, :]) @ P.T                      # [d_ff, d_model], row j = u_j
    z1 = P[:, :r] * sigma[None, :r]
    z2 = Q[:, :r]
    w2u = normal_bf16(2 * seed + 1, (d_ff, d_model), float(d_model) ** -0.5)
    return {
        "d_model": d_model, "d_ff": d_ff, "r": r,
        "w1u": f32_to_bf16_bits(w1u.astype(np.float32)),
        "w2u": w2u,
        "z1": f32_to_bf16_bits(z1.astype(np.float32)),
        "z2": f32_to_bf16_bits(z2.astype(np.float32)),
    }


# The five workload shapes.  k and k' are literals, not derived from a fraction.
CONFIGS = {
    "ffn_small": dict(kind="ffn", d_model=256, d_ff=1024, k=52, kprime=208, batches=(1,), seed=1),
    "ffn_1b": dict(kind="ffn", d_model=2048, d_ff=16384, k=819, kprime=3276, batches=(1, 4, 16), seed=2),
    "ffn_1b_lowrank": dict(kind="ffn_lr", d_model=2048, d_ff=16384, r=128, k=819, kprime=3276,
                           batches=(1, 16), seed=3),
    "softmax_1b": dict(kind="softmax", d_model=2048, vocab=256000, k=64, kprime=1024, batches=(1, 16), seed=4),
    "stack_1b": dict(kind="stack", d_model=2048, d_ff=16384, vocab=256000, layers=18, k=819, kprime=3276,
                     sm_k=64, sm_kprime=1024, batches=(64,), seed=500),
}
