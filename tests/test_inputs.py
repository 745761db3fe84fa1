"""The synthetic input generators: bf16 rounding, determinism, shapes and statistics."""
import numpy as np

from paper_2402_09360_amd import inputs as I


def test_bf16_round_to_nearest_even_brute_force():
    grid_bits = np.arange(0, 0x7F80, dtype=np.uint16)
    grid = I.bf16_bits_to_f64(grid_bits)
    rng = np.random.default_rng(1)
    vals = np.concatenate([rng.standard_normal(500).astype(np.float32),
                           ((grid[16200:16230] + grid[16201:16231]) / 2).astype(np.float32)])
    got = I.bf16_bits_to_f64(I.f32_to_bf16_bits(vals))
    for v, g in zip(vals, got):
        dist = np.abs(grid - abs(float(v)))
        best = np.flatnonzero(dist == dist.min())
        if len(best) == 2:
            best = [b for b in best if grid_bits[b] % 2 == 0]
        assert g == np.copysign(grid[best[0]], v)


def test_generators_are_deterministic_and_chunk_independent():
    a = I.normal_bf16(5, (100, 64), 0.5, chunk_rows=7)
    b = I.normal_bf16(5, (100, 64), 0.5, chunk_rows=100)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, I.normal_bf16(6, (100, 64), 0.5))


def test_layer_shapes_and_scale():
    L = I.ffn_layer(3, 128, 512)
    assert L["w1u"].shape == (512, 128) and L["w2u"].shape == (512, 128)
    for w in (L["w1u"], L["w2u"]):
        assert abs(I.bf16_bits_to_f64(w).std() * np.sqrt(128) - 1.0) < 0.02
    x = I.tokens(4, 8, 128)
    assert x.shape == (8, 128) and abs(I.bf16_bits_to_f64(x).std() - 1.0) < 0.06


def test_lowrank_layer_spectrum():
    L = I.lowrank_ffn_layer(9, 64, 256, 16)
    w = I.bf16_bits_to_f64(L["w1u"])
    assert abs((w ** 2).mean() * 64 - 1.0) < 0.02
    s = np.linalg.svd(w, compute_uv=False)
    ratio = s[:16] / s[0] * np.sqrt(np.arange(1, 17))
    assert np.all(np.abs(ratio - 1.0) < 0.05)                   # sigma_i ~ i^-1/2
    approx = I.bf16_bits_to_f64(L["z2"]) @ I.bf16_bits_to_f64(L["z1"]).T
    captured = 1.0 - ((w - approx) ** 2).sum() / (w ** 2).sum()
    want = (1.0 / np.arange(1, 17)).sum() / (1.0 / np.arange(1, 65)).sum()
    assert abs(captured - want) < 0.02


def test_correlated_tokens_share_a_component():
    x = I.bf16_bits_to_f64(I.correlated_tokens(10, 16, 4096, 0.9))
    c = np.corrcoef(x)
    off = c[~np.eye(16, dtype=bool)]
    assert abs(off.mean() - 0.9) < 0.03
