"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded bytes.
Integer and index work must be bit-exact; floats within max-rel-err 2e-3 (see hire_testlib)."""
import numpy as np
import pytest
import torch

from paper_2402_09360_amd import inputs as I
import hire_testlib as T

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hire():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2402_09360_amd import hire as H
    return H


def log(msg):
    print(msg, flush=True)


# ----------------------------------------------------------------------------
@pytest.mark.parametrize("rows,cols", [(300, 256), (1000, 2048), (77, 96)])
def test_pack_int4_bit_exact(hire, oracle, rows, cols):
    log(f"pack_int4 rows={rows} cols={cols}")
    w = I.normal_bf16(60 + rows, (rows, cols), cols ** -0.5)
    w[5, :] = 0
    q4, s = hire.hire_pack_int4(T.dev_bf16(w))
    codes = hire.hire_unpack_int4(q4, rows, cols)
    torch.cuda.synchronize()
    q_ref, s_ref = oracle.quantize_rows_int4(w)
    assert np.array_equal(s.cpu().numpy(), s_ref)
    assert np.array_equal(codes.cpu().numpy(), q_ref)


# ----------------------------------------------------------------------------
def _topk_cases(N):
    rng = np.random.default_rng(N)
    yield "normal", rng.standard_normal(N).astype(np.float32)
    yield "all_equal", np.full(N, 1.5, dtype=np.float32)
    z = np.maximum(rng.standard_normal(N), 0).astype(np.float32)
    yield "relu_zeros", z
    yield "dups", rng.integers(-3, 4, N).astype(np.float32)
    sz = np.where(rng.random(N) < 0.5, 0.0, -0.0).astype(np.float32)
    sz[N // 2] = 1.0
    yield "signed_zero", sz
    out = rng.standard_normal(N).astype(np.float32)
    out[N // 3] = 1e30
    out[N // 2] = -1e30
    yield "outliers", out
    yield "ascending", np.arange(N, dtype=np.float32)


@pytest.mark.parametrize("N", [1, 63, 1000, 16384, 20000, 70001])
def test_topk_select_matches_oracle(hire, oracle, N):
    for name, v in _topk_cases(N):
        ks = sorted({1, min(N, 2), max(1, N // 5), max(1, N - 1), N})
        for k in ks:
            for relu in (False, True):
                for rank in (False, True):
                    if rank and k > hire.MAX_RANK_ORDER_K:
                        continue
                    log(f"topk_select N={N} case={name} k={k} relu={relu} rank={rank}")
                    sc = torch.from_numpy(np.stack([v, v[::-1].copy()])).cuda()
                    idx, val = hire.topk_select(sc, k, relu=relu, rank_order=rank)
                    torch.cuda.synchronize()
                    idx, val = idx.cpu().numpy(), val.cpu().numpy()
                    for b, row in enumerate((v, v[::-1].copy())):
                        want = oracle.topk_f32(row, k, relu=relu, rank_order=rank)
                        assert np.array_equal(idx[b], want), (name, k, relu, rank, b)
                        ref = np.maximum(row, 0) if relu else row
                        assert np.array_equal(val[b], ref[want] + np.float32(0.0))


def test_topk_select_large_vocab(hire, oracle):
    rng = np.random.default_rng(5)
    v = rng.standard_normal((2, 256000)).astype(np.float32)
    for k, rank in ((1024, False), (64, True), (1024, True)):
        log(f"topk_select N=256000 k={k} rank={rank}")
        idx, val = hire.topk_select(torch.from_numpy(v).cuda(), k, rank_order=rank)
        torch.cuda.synchronize()
        for b in range(2):
            assert np.array_equal(idx[b].cpu().numpy(), oracle.topk_f32(v[b], k, rank_order=rank))


def test_topk_select_long_rows_steady_state(hire, oracle):
    """Rows beyond 32768 in index order: many workgroups per row and histograms in the workspace.  A fresh workspace
    selects by streaming once; from the second call on the histograms answer (no streaming selections counted),
    except for inputs that defeat them (all keys equal: a crowded bin), which stay exact through the fallback."""
    rng = np.random.default_rng(9)
    for N, k, B in ((70001, 700, 3), (256000, 1024, 2), (40000, 39999, 1)):
        for relu in (False, True):
            ws = hire.alloc_workspace(hire.hire_topk_workspace_bytes(B, N, k, hire.RELU if relu else 0))
            for call, kind in enumerate(("normal", "normal", "all_equal", "normal")):
                v = (rng.standard_normal((B, N)) if kind == "normal" else np.full((B, N), -2.5)).astype(np.float32)
                log(f"topk_select long rows N={N} k={k} relu={relu} call {call} ({kind})")
                idx, val = hire.topk_select(torch.from_numpy(v).cuda(), k, relu=relu, workspace=ws)
                torch.cuda.synchronize()
                for b in range(B):
                    want = oracle.topk_f32(v[b], k, relu=relu)
                    assert np.array_equal(idx[b].cpu().numpy(), want), (N, k, relu, call, b)
                    ref = np.maximum(v[b], 0) if relu else v[b]
                    assert np.array_equal(val[b].cpu().numpy(), ref[want] + np.float32(0.0))
                fb = hire.hire_debug_general_fallbacks(ws)
                log(f"  counters {fb}")
                if call == 1 and k <= N // 4:        # a k-th key far below the largest lies outside the window
                    assert fb == (0, 0, 1)


# ----------------------------------------------------------------------------
@pytest.mark.parametrize("d,N,B,k,kp", [
    (256, 1024, 1, 52, 208),        # config 1
    (96, 777, 3, 40, 160),          # ragged everything
    (64, 100, 2, 100, 100),         # k = k' = N: dense FFN
    (128, 2000, 5, 1, 1),           # k = k' = 1
    (512, 3000, 64, 150, 600),      # maximum batch
    (96, 777, 1, 40, 160),          # batch 1 (four-kernel route), ragged
    (64, 100, 1, 100, 100),         # batch 1, k = k' = N
    (128, 2000, 1, 1, 1),           # batch 1, k = k' = 1
    (2048, 16384, 1, 4000, 16384),  # batch 1, every unit is a candidate, large k
    (1024, 5000, 1, 700, 4500),     # batch 1, k' past the positive keys: the threshold sits in the ReLU zeros
])
def test_ffn_step_small(hire, oracle, d, N, B, k, kp):
    log(f"ffn_step d={d} N={N} B={B} k={k} kp={kp}")
    L = I.ffn_layer(70 + d, d, N)
    layer, scorer = T.make_ffn_layer(L)
    T.check_ffn(layer, scorer, L, I.tokens(71 + B, B, d), k, kp)


def test_ffn_step_degenerate_tokens(hire, oracle):
    """All-zero token (every key ties at zero) next to an ordinary one, and duplicated tokens."""
    d, N, k, kp = 128, 600, 20, 80
    L = I.ffn_layer(72, d, N)
    layer, scorer = T.make_ffn_layer(L)
    x = I.tokens(73, 4, d)
    x[1, :] = 0
    x[3, :] = x[0, :]
    log("ffn_step degenerate tokens")
    got, _ = T.check_ffn(layer, scorer, L, x, k, kp)
    assert not got["y"][1].any()
    assert np.array_equal(got["y"][0], got["y"][3])


def test_ffn_step_batch1_degenerate(hire, oracle):
    """Batch 1 through the four-kernel route: an all-zero token, and a layer with many identical rows
    (crowded threshold bin, ties settled by index)."""
    d, N, k, kp = 128, 600, 20, 80
    L = I.ffn_layer(74, d, N)
    L["w1u"][100:400] = L["w1u"][100]              # 300 identical units
    layer, scorer = T.make_ffn_layer(L)
    x = I.tokens(75, 1, d)
    log("ffn_step batch 1, duplicated rows")
    T.check_ffn(layer, scorer, L, x, k, kp)
    T.check_ffn(layer, scorer, L, x, 250, 350)
    log("ffn_step batch 1, zero token")
    got, _ = T.check_ffn(layer, scorer, L, np.zeros((1, d), dtype=np.uint16), k, kp)
    assert not got["y"].any() and got["cand"].tolist() == list(range(kp))


@pytest.fixture(scope="module")
def ffn_1b(hire, oracle):
    L = I.ffn_layer(2, 2048, 16384)
    layer, scorer = T.make_ffn_layer(L)
    return L, layer, scorer


@pytest.mark.parametrize("B", [1, 4, 16])
def test_ffn_step_1b_shape(hire, oracle, ffn_1b, B):
    """Config 2: d_m=2048, d_ff=16384, k=819, k'=3276, iid tokens, union across the batch."""
    L, layer, scorer = ffn_1b
    log(f"ffn_step 1B shape B={B}")
    got, want = T.check_ffn(layer, scorer, L, I.tokens(100 + B, B, 2048), 819, 3276)
    log(f"  |U|={got['n_cand']} min margin k={want['margin_k'].min():.3e} k'={want['margin_kprime'].min():.3e}")


def test_ffn_step_is_deterministic(hire, ffn_1b):
    L, layer, scorer = ffn_1b
    x = I.tokens(104, 4, 2048)
    a = T.run_ffn(layer, x, 819, 3276)
    b = T.run_ffn(layer, x, 819, 3276)
    for key in ("y", "topk_idx", "topk_val", "cand", "acc"):
        assert np.array_equal(a[key], b[key]), key


def test_ffn_step_correlated_tokens(hire, oracle, ffn_1b):
    """Tokens that share a component: the union is much smaller than B k' (Sec. 3.4.1)."""
    L, layer, scorer = ffn_1b
    x = I.correlated_tokens(105, 8, 2048, 0.9)
    log("ffn_step correlated tokens B=8")
    got, _ = T.check_ffn(layer, scorer, L, x, 819, 3276)
    assert got["n_cand"] < 0.6 * 8 * 3276


@pytest.mark.parametrize("d,N,r,B,k,kp", [(64, 500, 16, 3, 20, 80), (256, 1024, 40, 2, 52, 208),
                                          (64, 500, 16, 1, 20, 80),        # batch 1: the short kernel sequence
                                          (256, 1024, 40, 1, 52, 208),     # ... rows of 5 chunks
                                          (512, 3001, 136, 1, 300, 1200),  # ... odd N, rows longer than 16 chunks
                                          (128, 2000, 32, 1, 1, 1),
                                          (128, 600, 24, 1, 600, 600)])    # ... k = k' = N
def test_ffn_step_lowrank_small(hire, oracle, d, N, r, B, k, kp):
    log(f"ffn_step lowrank d={d} N={N} r={r} B={B}")
    L = I.lowrank_ffn_layer(80 + d, d, N, r)
    layer, scorer = T.make_ffn_layer(L, lowrank=True)
    T.check_ffn(layer, scorer, L, I.tokens(81, B, d), k, kp)


def test_ffn_step_lowrank_batch1_degenerate(hire, oracle):
    """Batch 1 with the low-rank scorer through the short kernel sequence: a zero token (every key ties at zero,
    both bounds are zero), duplicated factor rows (crowded threshold bin), and the same layer without the
    preparation (general sequence): all equal the oracle."""
    from paper_2402_09360_amd import hire as H
    d, N, r, k, kp = 128, 900, 24, 30, 120
    L = I.lowrank_ffn_layer(90, d, N, r)
    L["z2"][100:500] = L["z2"][100]
    L["w1u"][100:500] = L["w1u"][100]
    layer, scorer = T.make_ffn_layer(L, lowrank=True)
    x = I.tokens(91, 1, d)
    log("ffn_step lowrank batch 1, duplicated rows")
    T.check_ffn(layer, scorer, L, x, k, kp)
    T.check_ffn(layer, scorer, L, x, 250, 450)
    log("ffn_step lowrank batch 1, zero token")
    got, _ = T.check_ffn(layer, scorer, L, np.zeros((1, d), dtype=np.uint16), k, kp)
    assert not got["y"].any() and got["cand"].tolist() == list(range(kp))
    plain = H.FFNLayer(T.dev_bf16(L["w1u"]), T.dev_bf16(L["w2u"]), lr_a=T.dev_bf16(L["z1"]), lr_b=T.dev_bf16(L["z2"]),
                       prepare=False)
    a, b = T.run_ffn(layer, x, k, kp), T.run_ffn(plain, x, k, kp)
    for key in ("topk_idx", "cand"):
        assert np.array_equal(a[key], b[key]), key
    # the bounds are upper bounds, and tight ones
    w1 = I.bf16_bits_to_f64(L["w1u"]); z2 = I.bf16_bits_to_f64(L["z2"])
    bounds = layer.row_norm_bounds.cpu().numpy().astype(np.float64)
    true = np.array([np.sqrt((w1 * w1).sum(axis=1)).max(), np.sqrt((z2 * z2).sum(axis=1)).max()])
    assert (bounds >= true).all() and (bounds <= 1.01 * true).all(), (bounds, true)


@pytest.mark.parametrize("B", [1, 16])
def test_ffn_step_lowrank_1b_shape(hire, oracle, B):
    """Config 3: rank-128 scorer from the leading terms of a decaying-spectrum W1."""
    log(f"ffn_step lowrank 1B shape B={B} (building the layer takes a while)")
    L = _lowrank_1b()
    layer, scorer = T.make_ffn_layer(L, lowrank=True)
    got, want = T.check_ffn(layer, scorer, L, I.tokens(300 + B, B, 2048), 819, 3276)
    log(f"  |U|={got['n_cand']} min margin k'={want['margin_kprime'].min():.3e}")
    # both selections (fp64 scorer keys, activations) find their thresholds through the window histogram
    x = T.dev_bf16(I.tokens(300 + B, B, 2048))
    ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, B, 819, 3276))
    out = hire.FFNOutputs(layer, B, 819, 3276)
    for _ in range(4):
        hire.hire_ffn_step(layer, x, 819, 3276, out, ws)
    torch.cuda.synchronize()
    if B == 1:      # short kernel sequence: both selections answered from their window histograms
        assert hire.hire_debug_fast_fallbacks(ws) == (0, 0)
        marker, nonzero_key_bins, counted_h = hire.hire_debug_fast_state(ws)
        assert marker == 1 and nonzero_key_bins == 0 and 0 < counted_h <= 3276
    else:
        assert hire.hire_debug_general_fallbacks(ws) == (0, 0, 0)


# ----------------------------------------------------------------------------
# Group-sparse FFN (eq. (6)).
@pytest.mark.parametrize("d,N,B,k,kp,g", [
    (256, 1024, 1, 48, 208, 8),     # config 1's layer, groups of 8
    (256, 1024, 1, 52, 208, 1),     # groups of one: the plain step through the group entry point
    (96, 784, 3, 40, 160, 8),       # ragged row length, batch on the 4-token tiles
    (96, 784, 5, 40, 160, 4),       # 16-token tiles
    (64, 96, 2, 96, 96, 16),        # everything shortlisted and selected: dense FFN
    (128, 2000, 5, 2, 2, 2),        # one group
    (512, 3008, 64, 160, 640, 16),  # maximum batch, largest group
    (1024, 5000, 1, 700, 4500, 4),  # k' past the positive keys: group sums of zero tie
])
def test_ffn_group_step_small(hire, oracle, d, N, B, k, kp, g):
    log(f"ffn_group_step d={d} N={N} B={B} k={k} kp={kp} g={g}")
    L = I.ffn_layer(170 + d, d, N)
    layer, scorer = T.make_ffn_layer(L)
    T.check_ffn_group(layer, scorer, L, I.tokens(171 + B, B, d), k, kp, g)


def test_ffn_group_step_batch1_degenerate(hire, oracle):
    """Batch 1, groups of eight through the four-kernel route: half of the groups have all-zero keys (the shortlist
    reaches into them: ties at zero go to the lower group), many identical groups (crowded threshold bin), and an
    all-zero token."""
    d, N = 128, 4800
    L = I.ffn_layer(174, d, N)
    L["w1u"][2400:] = 0                              # groups 300..599 score zero
    L["w1u"][800:1600] = np.tile(L["w1u"][800:808], (100, 1))   # 100 identical groups
    layer, scorer = T.make_ffn_layer(L)
    x = I.tokens(175, 1, d)
    log("ffn_group_step batch 1, zero and duplicated groups")
    got, _ = T.check_ffn_group(layer, scorer, L, x, 800, 3200, 8)
    assert got["cand"].tolist()[-100:] == list(range(300, 400))
    T.check_ffn_group(layer, scorer, L, x, 8, 8, 8)
    T.check_ffn_group(layer, scorer, L, x, 4800, 4800, 8)
    log("ffn_group_step batch 1, zero token")
    got, _ = T.check_ffn_group(layer, scorer, L, np.zeros((1, d), dtype=np.uint16), 80, 320, 8)
    assert not got["y"].any() and got["cand"].tolist() == list(range(40))


def test_ffn_group_step_equals_plain_step_for_groups_of_one(hire, ffn_1b):
    L, layer, scorer = ffn_1b
    x = I.tokens(172, 4, 2048)
    a = T.run_ffn(layer, x, 819, 3276)
    b = T.run_ffn_group(layer, x, 819, 3276, 1)
    assert np.array_equal(a["topk_idx"], b["topk_group"]) and np.array_equal(a["cand"], b["cand"])
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["topk_val"], b["topk_val"])


@pytest.mark.parametrize("B", [1, 4, 16])
def test_ffn_group_step_1b_shape(hire, oracle, ffn_1b, B):
    """Config 2's layer with the paper's group size 8: 408 of 2048 groups shortlisted, 102 kept."""
    L, layer, scorer = ffn_1b
    log(f"ffn_group_step 1B shape B={B}")
    got, want = T.check_ffn_group(layer, scorer, L, I.tokens(100 + B, B, 2048), 816, 3264, 8)
    log(f"  |U_g|={got['n_cand']} min margin k={want['margin_k'].min():.3e} k'={want['margin_kprime'].min():.3e}")


@pytest.mark.parametrize("d,N,r,B,k,kp,g", [(64, 512, 16, 3, 24, 80, 8), (256, 1024, 40, 1, 52, 208, 4)])
def test_ffn_group_step_lowrank(hire, oracle, d, N, r, B, k, kp, g):
    log(f"ffn_group_step lowrank d={d} N={N} r={r} B={B} g={g}")
    L = I.lowrank_ffn_layer(180 + d, d, N, r)
    layer, scorer = T.make_ffn_layer(L, lowrank=True)
    T.check_ffn_group(layer, scorer, L, I.tokens(181, B, d), k, kp, g)


def test_ffn_group_step_rejects_bad_groups(hire, ffn_1b):
    L, layer, scorer = ffn_1b
    assert hire.hire_ffn_group_workspace_bytes(layer, 1, 816, 3264, 3) == 0      # not a power of two
    assert hire.hire_ffn_group_workspace_bytes(layer, 1, 819, 3264, 8) == 0      # k not a multiple
    assert hire.hire_ffn_group_workspace_bytes(layer, 1, 816, 3264, 32) == 0     # too large
    ws = hire.alloc_workspace(hire.hire_ffn_group_workspace_bytes(layer, 1, 816, 3264, 8))
    out = hire.FFNGroupOutputs(layer, 1, 816, 3264, 8)
    x = T.dev_bf16(I.tokens(173, 1, 2048))
    with pytest.raises(hire.HireError):
        hire.hire_ffn_group_step(layer, x, 819, 3264, 8, out, ws)
    with pytest.raises(hire.HireError):
        hire.hire_ffn_group_step(layer, x, 816, 3264, 3, out, ws)


# ----------------------------------------------------------------------------
# Sharded approximate top-k (Algorithm 2).
@pytest.mark.parametrize("d,N,B,k,kp,s", [
    (256, 1024, 1, 48, 208, 16),     # config 1's layer, 16 shards of 64 units
    (256, 1024, 1, 52, 208, 1),      # one shard: Algorithm 1 itself (counting selection over 1024 keys)
    (96, 770, 3, 35, 140, 7),        # ragged shard length 110, batch
    (64, 96, 2, 96, 96, 4),          # everything shortlisted and selected: dense FFN
    (128, 2000, 5, 50, 50, 50),      # one unit per shard and token
    (4096, 512, 2, 32, 128, 8),      # two 16-byte chunks of a packed row per lane
    (8192, 256, 1, 16, 64, 4),       # four
    (1024, 5000, 1, 700, 4500, 5),   # shortlist past the positive keys: zeros tie, lower index wins
    (512, 3008, 64, 188, 752, 47),   # maximum batch
    (256, 1024, 1, 50, 205, 16),     # quotas that do not divide: ceil(205/16) = 13 shortlisted, ceil(50/16) = 4 kept
    (96, 770, 3, 33, 141, 7),        # the same with a batch and a ragged shard length (21 and 5 per shard)
    (128, 2000, 5, 1, 51, 50),       # k below the number of shards: every shard still keeps one unit
])
def test_ffn_shard_step_small(hire, oracle, d, N, B, k, kp, s):
    log(f"ffn_shard_step d={d} N={N} B={B} k={k} kp={kp} shards={s}")
    L = I.ffn_layer(190 + d, d, N)
    layer, scorer = T.make_ffn_layer(L)
    T.check_ffn_shard(layer, scorer, L, I.tokens(191 + B, B, d), k, kp, s)


@pytest.mark.parametrize("B,s,k,kp", [(1, 256, 768, 3328), (1, 64, 832, 3264), (4, 256, 768, 3328), (16, 128, 768, 3328),
                                      (1, 256, 819, 3276), (4, 128, 819, 3276)])
def test_ffn_shard_step_1b_shape(hire, oracle, ffn_1b, B, s, k, kp):
    """Config 2's layer cut into shards, quotas k'/s and k/s: multiples of s, and the layer's own k = 819 and
    k' = 3276, whose quotas are rounded up (4 and 13 per shard at s = 256)."""
    L, layer, scorer = ffn_1b
    log(f"ffn_shard_step 1B shape B={B} shards={s}")
    got, want = T.check_ffn_shard(layer, scorer, L, I.tokens(100 + B, B, 2048), k, kp, s)
    log(f"  sum |U_i|={int(got['n_cand'].sum())} min margin k={want['margin_k'].min():.3e}")


def test_ffn_shard_step_one_shard_equals_plain_step(hire, oracle):
    L = I.ffn_layer(192, 256, 1024)
    layer, scorer = T.make_ffn_layer(L)
    x = I.tokens(193, 3, 256)
    a = T.run_ffn(layer, x, 52, 208)
    b = T.run_ffn_shard(layer, x, 52, 208, 1)
    assert np.array_equal(a["topk_idx"], b["topk_idx"]) and np.array_equal(a["cand"], b["cand"][0])
    T.assert_float_close(b["y"], a["y"], "y")


def test_ffn_shard_step_degenerate_inputs(hire, oracle):
    """Sharded step on inputs full of ties: an all-zero token inside a bundle of ordinary ones, a repeated token,
    and a layer whose shards hold many identical units (equal keys and equal activations, lower index first)."""
    d, N, k, kp, s = 128, 640, 40, 160, 8
    L = I.ffn_layer(195, d, N)
    L["w1u"][100:400] = L["w1u"][100]              # identical units across four shards
    layer, scorer = T.make_ffn_layer(L)
    x = I.tokens(196, 6, d)
    x[1, :] = 0
    x[4, :] = x[0, :]
    log("ffn_shard_step degenerate inputs, batch 6")
    got, _ = T.check_ffn_shard(layer, scorer, L, x, k, kp, s)
    assert not got["y"][1].any()
    assert np.array_equal(got["y"][0], got["y"][4])
    log("ffn_shard_step degenerate inputs, zero token alone")
    got, _ = T.check_ffn_shard(layer, scorer, L, np.zeros((1, d), dtype=np.uint16), k, kp, s)
    assert not got["y"].any()
    log("ffn_shard_step degenerate inputs, batch 1")
    T.check_ffn_shard(layer, scorer, L, x[:1], k, kp, s)


def test_ffn_shard_step_rejects_what_it_cannot_do(hire, ffn_1b):
    L, layer, scorer = ffn_1b
    assert hire.hire_ffn_shard_workspace_bytes(layer, 1, 768, 3328, 8) == 0        # 2048 units per shard
    assert hire.hire_ffn_shard_workspace_bytes(layer, 1, 3400, 3328, 256) == 0     # k above k'
    assert hire.hire_ffn_shard_workspace_bytes(layer, 1, 768, 3328, 100) == 0      # shards do not divide d_ff
    ws = hire.alloc_workspace(hire.hire_ffn_shard_workspace_bytes(layer, 1, 768, 3328, 256))
    out = hire.FFNShardOutputs(layer, 1, 768, 3328, 256)
    x = T.dev_bf16(I.tokens(194, 1, 2048))
    with pytest.raises(hire.HireError):
        hire.hire_ffn_shard_step(layer, x, 768, 3328, 8, out, ws)
    with pytest.raises(hire.HireError):
        hire.hire_ffn_shard_step(layer, x, 3400, 3328, 256, out, ws)
    with pytest.raises(hire.HireError):
        hire.hire_ffn_shard_step(layer, x, 768, 3328, 100, out, ws)


# ----------------------------------------------------------------------------
# CommonPath (eq. (7)): dense units next to the group-sparse ones.
@pytest.mark.parametrize("d,N,m1,B,k,kp,g", [
    (256, 1024, 176, 1, 32, 136, 8),    # config 1's layer, a sixth of the units dense
    (96, 784, 100, 3, 40, 160, 8),      # ragged, batch on the 4-token tiles
    (128, 640, 37, 5, 32, 96, 4),       # odd number of dense units, 16-token tiles
    (64, 200, 0, 2, 16, 64, 8),         # no dense units: the group-sparse step
    (512, 3072, 512, 64, 160, 640, 16), # maximum batch
    (64, 96, 5000, 1, 8, 32, 1),        # many more dense units than sparse ones
])
def test_ffn_commonpath_step_small(hire, oracle, d, N, m1, B, k, kp, g):
    log(f"ffn_commonpath_step d={d} N={N} m1={m1} B={B} k={k} kp={kp} g={g}")
    L = I.ffn_layer(200 + d, d, N)
    D = I.ffn_layer(201 + d, d, max(m1, 1))
    dense = (D["w1u"][:m1], D["w2u"][:m1])
    layer, scorer = T.make_ffn_layer(L)
    T.check_ffn_commonpath(layer, scorer, L, dense, I.tokens(202 + B, B, d), k, kp, g)


def test_ffn_commonpath_step_degenerate_inputs(hire, oracle):
    """CommonPath on an all-zero token (alone: the batch-1 route with the dense units folded in; and inside a
    batch) and on a layer with many identical units among both the dense and the sparse ones."""
    d, N, m1, k, kp, g = 128, 640, 120, 40, 160, 8
    L = I.ffn_layer(203, d, N)
    L["w1u"][96:400] = L["w1u"][96]
    D = I.ffn_layer(204, d, m1)
    D["w1u"][10:90] = D["w1u"][10]
    dense = (D["w1u"], D["w2u"])
    layer, scorer = T.make_ffn_layer(L)
    x = I.tokens(205, 3, d)
    x[1, :] = 0
    log("ffn_commonpath_step degenerate inputs, batch 3")
    T.check_ffn_commonpath(layer, scorer, L, dense, x, k, kp, g)
    log("ffn_commonpath_step degenerate inputs, zero token alone")
    T.check_ffn_commonpath(layer, scorer, L, dense, np.zeros((1, d), dtype=np.uint16), k, kp, g)
    log("ffn_commonpath_step degenerate inputs, batch 1")
    T.check_ffn_commonpath(layer, scorer, L, dense, x[:1], k, kp, g)


@pytest.mark.parametrize("B", [1, 4])
def test_ffn_commonpath_step_1b_shape(hire, oracle, B):
    """Config 2's shape split as in the paper's CommonPath experiment: a sixth of the 16384 units dense (2736),
    3.3 % of all units (544 = 68 groups of 8) kept from the other 13648, 272 groups shortlisted."""
    d, m1, m2 = 2048, 2736, 13648
    L = I.ffn_layer(210, d, m2)
    D = I.ffn_layer(211, d, m1)
    layer, scorer = T.make_ffn_layer(L)
    log(f"ffn_commonpath_step 1B shape B={B}")
    T.check_ffn_commonpath(layer, scorer, L, (D["w1u"], D["w2u"]), I.tokens(212 + B, B, d), 544, 2176, 8)


# ----------------------------------------------------------------------------
# HiRE-LRQ: both low-rank factors in int4.
@pytest.mark.parametrize("d,N,r,B,k,kp", [(64, 512, 32, 3, 20, 80), (256, 1024, 64, 1, 52, 208),
                                          (96, 777, 32, 17, 40, 160), (1024, 2000, 1024, 2, 30, 120)])
def test_ffn_step_lrq_small(hire, oracle, d, N, r, B, k, kp):
    log(f"ffn_step lrq d={d} N={N} r={r} B={B}")
    L = I.lowrank_ffn_layer(220 + d, d, N, r)
    layer, scorer = T.make_ffn_layer(L, lrq=True)
    T.check_ffn(layer, scorer, L, I.tokens(221, B, d), k, kp)
    if N % 8 == 0:
        T.check_ffn_group(layer, scorer, L, I.tokens(222, B, d), 8 * (k // 8), 8 * (kp // 8), 8)


@pytest.mark.parametrize("B", [1, 16])
def test_ffn_step_lrq_1b_shape(hire, oracle, B):
    """Config 3's layer with its rank-128 factors quantised to int4."""
    log(f"ffn_step lrq 1B shape B={B}")
    L = _lowrank_1b()
    layer, scorer = T.make_ffn_layer(L, lrq=True)
    got, want = T.check_ffn(layer, scorer, L, I.tokens(300 + B, B, 2048), 819, 3276)
    log(f"  |U|={got['n_cand']} min margin k'={want['margin_kprime'].min():.3e}")


@pytest.mark.parametrize("d,c,r,B,k,kp", [(64, 5000, 32, 3, 8, 100), (256, 40000, 64, 2, 64, 1024)])
def test_softmax_step_lrq_small(hire, oracle, d, c, r, B, k, kp):
    """Classifier with random low-rank factors (the scorer's quality is not at stake, only parity); the second
    case has rows beyond 32768, selected by many work-groups through the key histograms."""
    log(f"softmax_step lrq d={d} c={c} r={r} B={B}")
    W = I.classifier(230 + d, c, d)
    z1, z2 = I.normal_bf16(231, (d, r), d ** -0.5), I.normal_bf16(232, (c, r), 1.0)
    layer, scorer = T.make_softmax_layer(W, lrq=(z1, z2))
    T.check_softmax(layer, scorer, W, I.tokens(233, B, d), k, kp)


def test_lrq_steps_degenerate_tokens(hire, oracle):
    """HiRE-LRQ with an all-zero token (the intermediate t is zero and so is its int8 scale) and a repeated one,
    through the FFN and the softmax step."""
    d, N, r = 128, 1024, 32
    L = I.lowrank_ffn_layer(236, d, N, r)
    layer, scorer = T.make_ffn_layer(L, lrq=True)
    x = I.tokens(237, 4, d)
    x[2, :] = 0
    x[3, :] = x[0, :]
    log("ffn_step lrq degenerate tokens")
    got, _ = T.check_ffn(layer, scorer, L, x, 40, 160)
    assert not got["y"][2].any() and np.array_equal(got["y"][0], got["y"][3])
    T.check_ffn(layer, scorer, L, x[2:3], 40, 160)
    log("softmax_step lrq degenerate tokens")
    W = I.classifier(238, 5000, d)
    z1, z2 = I.normal_bf16(239, (d, r), d ** -0.5), I.normal_bf16(240, (5000, r), 1.0)
    sm, sm_scorer = T.make_softmax_layer(W, lrq=(z1, z2))
    T.check_softmax(sm, sm_scorer, W, x, 8, 100)
    T.check_softmax(sm, sm_scorer, W, x[2:3], 8, 100)


@pytest.mark.parametrize("B", [1, 16])
def test_softmax_step_lrq_1b_shape(hire, oracle, classifier_1b, B):
    """Config 4's classifier with rank d/4 = 512 int4 factors (the paper's rank for the softmax layer)."""
    W = classifier_1b[0]
    log(f"softmax_step lrq 1B shape B={B}")
    z1, z2 = I.normal_bf16(234, (2048, 512), 2048 ** -0.5), I.normal_bf16(235, (256000, 512), 1.0)
    layer, scorer = T.make_softmax_layer(W, lrq=(z1, z2))
    T.check_softmax(layer, scorer, W, I.tokens(400 + B, B, 2048), 64, 1024)


# ----------------------------------------------------------------------------
# Seeded random shapes through every FFN entry point and scorer.
def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    for _ in range(n):
        d = int(rng.integers(1, 11)) * 32
        g = int(rng.choice([1, 2, 4, 8, 16]))
        s = int(rng.choice([1, 2, 3, 5, 8, 16]))
        unit = g * s                                    # N, k, k' multiples of both the group and the shard count
        N = unit * int(rng.integers(max(1, 40 // unit), max(2, 1500 // unit) + 1))
        k = unit * int(rng.integers(1, max(2, N // (4 * unit)) + 1))
        kp = min(N, k * int(rng.integers(1, 5)))
        kp -= kp % unit
        kp = max(kp, k)
        B = int(rng.choice([1, 1, 2, 3, 4, 5, 9]))
        yield d, N, B, k, kp, g, s, str(rng.choice(["int4", "lowrank", "lrq"]))


@pytest.mark.parametrize("case", list(_random_cases(24, 2024)), ids=lambda c: "-".join(map(str, c)))
def test_random_shapes_all_ffn_entry_points(hire, oracle, case):
    d, N, B, k, kp, g, s, kind = case
    log(f"random case d={d} N={N} B={B} k={k} kp={kp} g={g} s={s} scorer={kind}")
    x = I.tokens(900 + B, B, d)
    if kind == "int4" or N < d:
        L = I.ffn_layer(901 + N, d, N)
        layer, scorer = T.make_ffn_layer(L)
    else:
        L = I.lowrank_ffn_layer(902 + N, d, N, 32)
        layer, scorer = T.make_ffn_layer(L, lowrank=kind == "lowrank", lrq=kind == "lrq")
    T.check_ffn(layer, scorer, L, x, k, kp)
    T.check_ffn_group(layer, scorer, L, x, k, kp, g)
    m1 = (N * 7) % 97
    D = I.ffn_layer(903 + N, d, max(m1, 1))
    T.check_ffn_commonpath(layer, scorer, L, (D["w1u"][:m1], D["w2u"][:m1]), x, k, kp, g)
    if scorer[0] == "int4" and N // s <= 1024:
        T.check_ffn_shard(layer, scorer, L, x, k, kp, s)


def _random_softmax_cases(n, seed):
    rng = np.random.default_rng(seed)
    for _ in range(n):
        d = int(rng.integers(1, 9)) * 32
        c = int(rng.integers(50, 60000))
        k = int(rng.integers(1, min(c, 300) + 1))
        kp = int(rng.integers(k, min(c, 4 * k + 50) + 1))
        yield d, c, int(rng.choice([1, 2, 3, 7])), k, kp, str(rng.choice(["int4", "lrq"]))


@pytest.mark.parametrize("case", list(_random_softmax_cases(12, 2025)), ids=lambda c: "-".join(map(str, c)))
def test_random_shapes_softmax(hire, oracle, case):
    d, c, B, k, kp, kind = case
    log(f"random softmax case d={d} c={c} B={B} k={k} kp={kp} scorer={kind}")
    W = I.classifier(910 + c, c, d)
    lrq = (I.normal_bf16(911, (d, 32), d ** -0.5), I.normal_bf16(912, (c, 32), 1.0)) if kind == "lrq" else None
    layer, scorer = T.make_softmax_layer(W, lrq=lrq)
    T.check_softmax(layer, scorer, W, I.tokens(913 + B, B, d), k, kp)


_LR_CACHE = {}


def _lowrank_1b():
    if "L" not in _LR_CACHE:
        _LR_CACHE["L"] = I.lowrank_ffn_layer(3, 2048, 16384, 128)
    return _LR_CACHE["L"]


# ----------------------------------------------------------------------------
@pytest.mark.parametrize("d,c,B,k,kp", [(64, 5000, 3, 8, 100), (256, 33333, 2, 64, 1024), (128, 300, 2, 300, 300),
                                        (64, 6000, 2, 4096, 5000)])   # the last: largest k the rank ordering takes
def test_softmax_step_small(hire, oracle, d, c, B, k, kp):
    log(f"softmax_step d={d} c={c} B={B} k={k} kp={kp}")
    W = I.classifier(90 + d, c, d)
    layer, scorer = T.make_softmax_layer(W)
    T.check_softmax(layer, scorer, W, I.tokens(91, B, d), k, kp)


# ----------------------------------------------------------------------------
# One token on a long vocabulary: the three-kernel sequence (scorer with the window of workgroup maxima, logits of a
# superset of the shortlist, final selections).
def _check_softmax_b1(hire, oracle, W, x, k, kp, expect_window, lrq=None):
    """Three steps on one workspace against the oracle, then the same step through the general kernel sequence,
    which must agree bit for bit.  expect_window: every step is served by the maxima's window (no direct selection
    from the keys is counted)."""
    layer, scorer = T.make_softmax_layer(W, lrq=lrq)
    want = oracle.softmax_step(W, scorer, x, k, kp, want_acc=True)
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(layer, 1, k, kp))
    runs = T.run_softmax(layer, x, k, kp, steps=3, ws=ws)
    for got in runs:
        T.compare_softmax(got, want)
    direct = hire.hire_debug_general_fallbacks(ws)[0]
    assert (direct == 0) == expect_window, f"{direct} steps selected from the keys directly"
    hire.hire_force_generic_path(True)
    try:
        general = T.run_softmax(layer, x, k, kp)
    finally:
        hire.hire_force_generic_path(False)
    for name in ("top_idx", "top_logit", "top_prob", "cand"):
        assert np.array_equal(general[name], runs[-1][name]), name
    return runs[-1], want


@pytest.mark.parametrize("d,c,k,kp", [
    (768, 40000, 64, 1024),      # 40 workgroups of 1024 keys, the last one ragged
    (544, 33000, 5, 40),         # token chunks that do not fill the lanes; a list far shorter than the 64 buckets
    (1024, 70001, 64, 1536),     # the largest shortlist
    (2048, 35000, 1, 1),         # a single class
    (640, 50000, 64, 64),        # everything shortlisted is kept
    (768, 262144, 64, 1024),     # the longest vocabulary the sequence takes
    (544, 32776, 7, 300),        # just past the single-work-group limit
])
def test_softmax_step_one_token_long_vocabulary(hire, oracle, d, c, k, kp):
    log(f"softmax_step one token d={d} c={c} k={k} kp={kp}")
    W = I.classifier(700 + d, c, d)
    _check_softmax_b1(hire, oracle, W, I.tokens(701 + d, 1, d), k, kp, expect_window=True)


@pytest.mark.parametrize("d,c,r,k,kp", [
    (256, 40000, 0, 16, 128),     # int4 scorer on short rows: one maximum per wave of the scorer
    (768, 40000, 64, 16, 128),    # int4 low-rank scorer, rank 64: the keys come from rows of 64 codes
    (1024, 66000, 256, 64, 1024), # rank 256
    (768, 200000, 128, 64, 768),  # 1564 maxima for k' = 768: the bound leaves 1.4 k' keys
])
def test_softmax_step_one_token_short_scorer_rows(hire, oracle, d, c, r, k, kp):
    log(f"softmax_step one token, short scorer rows d={d} c={c} r={r} k={k} kp={kp}")
    W = I.classifier(730 + d, c, d)
    lrq = (I.normal_bf16(731, (d, r), d ** -0.5), I.normal_bf16(732, (c, r), 1.0)) if r else None
    _check_softmax_b1(hire, oracle, W, I.tokens(733 + d, 1, d), k, kp, expect_window=True, lrq=lrq)


def _random_one_token_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        d = 32 * int(rng.integers(2, 65))              # 64 .. 2048
        c = int(rng.integers(32769, 120000))
        k = int(rng.integers(1, 65))
        kp = int(rng.integers(k, 1537))
        r = int(rng.choice([0, 0, 32, 96]))             # int4 scorer, or int4 low-rank factors of that rank
        cases.append((d, c, r, k, kp))
    return cases


@pytest.mark.parametrize("d,c,r,k,kp", _random_one_token_cases(8, 2402))
def test_softmax_step_one_token_random_shapes(hire, oracle, d, c, r, k, kp):
    """Seeded random shapes, one token on a long vocabulary: whichever kernel sequence the shape gets (the bound
    from the maxima where it is expected to serve, the general sequence otherwise) must match the oracle."""
    log(f"softmax_step one token, random shape d={d} c={c} r={r} k={k} kp={kp}")
    W = I.classifier(750 + d, c, d)
    lrq = (I.normal_bf16(751, (d, r), d ** -0.5), I.normal_bf16(752, (c, r), 1.0)) if r else None
    layer, scorer = T.make_softmax_layer(W, lrq=lrq)
    T.check_softmax(layer, scorer, W, I.tokens(753 + c, 1, d), k, kp)


def _random_long_row_batches(n, seed):
    rng = np.random.default_rng(seed)
    return [(32 * int(rng.integers(2, 17)), int(rng.integers(32769, 80000)), int(rng.integers(2, 25)),
             int(rng.integers(1, 65)), int(rng.integers(64, 1200))) for _ in range(n)]


@pytest.mark.parametrize("d,c,B,k,kp", _random_long_row_batches(5, 9360))
def test_softmax_step_batches_on_long_rows_random_shapes(hire, oracle, d, c, B, k, kp):
    """Seeded random shapes, batches on a long vocabulary: every token's shortlist from the bound that the scorer's
    maxima give (both below and from 16 tokens on, where filter and refine follows)."""
    log(f"softmax_step batch on long rows, random shape d={d} c={c} B={B} k={k} kp={kp}")
    W = I.classifier(760 + d, c, d)
    layer, scorer = T.make_softmax_layer(W)
    T.check_softmax(layer, scorer, W, I.tokens(761 + c, B, d), k, kp)


def test_softmax_step_one_token_without_optional_outputs(hire):
    """Only top_idx and top_prob requested: the same results as with every optional output."""
    d, c, k, kp = 768, 40000, 64, 1024
    layer, _ = T.make_softmax_layer(I.classifier(740, c, d))
    x = T.dev_bf16(I.tokens(741, 1, d))
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(layer, 1, k, kp))
    full, lean = hire.SoftmaxOutputs(layer, 1, k, kp), hire.SoftmaxOutputs(layer, 1, k, kp)
    log("softmax_step one token, optional outputs left out")
    hire.hire_softmax_step(layer, x, k, kp, full, ws)
    hire.hire_softmax_step(layer, x, k, kp, lean, ws, minimal=True)
    torch.cuda.synchronize()
    assert torch.equal(full.top_idx, lean.top_idx) and torch.equal(full.top_prob, lean.top_prob)


def test_softmax_step_one_token_equal_keys_and_logits(hire, oracle):
    """Classes repeated twenty times each, the copies spread over the vocabulary: both cuts (the k'-th key, the k-th
    logit) fall inside blocks of exactly equal values and are settled by the class index."""
    d, k, kp = 768, 50, 1000
    base = I.classifier(710, 2000, d)
    W = np.tile(base, (20, 1))                     # class j + 2000 m is a copy of class j
    log("softmax_step one token, 20 spread copies of 2000 classes")
    _check_softmax_b1(hire, oracle, W, I.tokens(711, 1, d), k, kp, expect_window=True)


def test_softmax_step_one_token_falls_back(hire, oracle):
    """Inputs the window cannot serve, selected from the keys directly: 3000 adjacent copies of one class (a work-group
    of the gathering kernel has more entries than slots), and the zero token (all keys zero, below every window)."""
    d, k, kp = 768, 32, 900
    base = I.classifier(720, 6, d)
    W = np.concatenate([I.classifier(721, 20000, d), np.repeat(base, 3000, axis=0), I.classifier(722, 2000, d)], axis=0)
    x = I.tokens(723, 1, d)
    log("softmax_step one token, 3000 adjacent copies of six classes")
    _check_softmax_b1(hire, oracle, W, x, k, kp, expect_window=False)
    log("softmax_step one token, zero token")
    _check_softmax_b1(hire, oracle, W, np.zeros((1, d), dtype=np.uint16), k, kp, expect_window=False)


@pytest.fixture(scope="module")
def classifier_1b(hire, oracle):
    log("building the 256000 x 2048 classifier")
    W = I.classifier(4, 256000, 2048)
    layer, scorer = T.make_softmax_layer(W)
    return W, layer, scorer


@pytest.mark.parametrize("B", [1, 16])
def test_softmax_step_1b_shape(hire, oracle, classifier_1b, B):
    """Config 4: vocab 256000, k'=1024, k=64."""
    W, layer, scorer = classifier_1b
    log(f"softmax_step 1B shape B={B}")
    got, want = T.check_softmax(layer, scorer, W, I.tokens(400 + B, B, 2048), 64, 1024)
    log(f"  |U|={got['n_cand']} min margin k={want['margin_k'].min():.3e}")


def test_full_stack_batch64(hire, oracle, classifier_1b):
    """Config 5: 18 FFN layers + the classifier at B=64, each layer fed its own seeded tokens."""
    W, sm_layer, sm_scorer = classifier_1b
    for l in range(18):
        log(f"stack layer {l}")
        L = I.ffn_layer(500 + l, 2048, 16384)
        layer, scorer = T.make_ffn_layer(L)
        T.check_ffn(layer, scorer, L, I.tokens(600 + l, 64, 2048), 819, 3276)
        del layer, scorer, L
    log("stack softmax")
    T.check_softmax(sm_layer, sm_scorer, W, I.tokens(700, 64, 2048), 64, 1024)


# ----------------------------------------------------------------------------
# the general kernel sequence with the int4 scorer: key histograms, their fallbacks and the workspace protocol
def test_general_route_takes_histograms(hire, oracle, ffn_1b, classifier_1b):
    """At the 1B shapes every selection finds its threshold through a histogram (the key histograms in the
    workspace for the long softmax rows, the window histogram in LDS elsewhere): no fallbacks are counted."""
    L, layer, scorer = ffn_1b
    x = T.dev_bf16(I.tokens(31, 4, 2048))
    ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, 4, 819, 3276))
    out = hire.FFNOutputs(layer, 4, 819, 3276)
    for _ in range(4):
        hire.hire_ffn_step(layer, x, 819, 3276, out, ws)
    assert hire.hire_debug_general_fallbacks(ws) == (0, 0, 0)      # short rows: one workgroup per token, window hit
    W, sm_layer, _ = classifier_1b
    x = T.dev_bf16(I.tokens(32, 16, 2048))
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(sm_layer, 16, 64, 1024))
    out = hire.SoftmaxOutputs(sm_layer, 16, 64, 1024)
    for _ in range(4):
        hire.hire_softmax_step(sm_layer, x, 64, 1024, out, ws)
    assert hire.hire_debug_general_fallbacks(ws) == (0, 0, 0)      # long rows: bound from the scorer's maxima, no histogram
    hire.hire_force_generic_path(True)
    try:
        for _ in range(4):
            hire.hire_softmax_step(sm_layer, x, 64, 1024, out, ws)
    finally:
        hire.hire_force_generic_path(False)
    assert hire.hire_debug_general_fallbacks(ws) == (0, 0, 1)      # key histograms, stamped once
    x = T.dev_bf16(I.tokens(33, 1, 2048))
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(sm_layer, 1, 64, 1024))
    out = hire.SoftmaxOutputs(sm_layer, 1, 64, 1024)
    for _ in range(4):
        hire.hire_softmax_step(sm_layer, x, 64, 1024, out, ws)
    assert hire.hire_debug_general_fallbacks(ws) == (0, 0, 0)      # one token: the short sequence, no direct selection
    hire.hire_force_generic_path(True)
    try:
        for _ in range(4):
            hire.hire_softmax_step(sm_layer, x, 64, 1024, out, ws)
    finally:
        hire.hire_force_generic_path(False)
    assert hire.hire_debug_general_fallbacks(ws) == (0, 0, 1)      # the general sequence on the same workspace


@pytest.mark.parametrize("d,c,B,k,kp", [(256, 40000, 16, 64, 1024),   # filter and refine: union of 16384 rows
                                         (128, 9000, 20, 8, 100),       # two token tiles, a short union
                                         (800, 30000, 33, 64, 512),     # three token tiles, ragged last pass
                                         (128, 300, 17, 300, 300),      # k = k' = N: every class refined
                                         (64, 5000, 64, 1, 1)])         # k = k' = 1
def test_softmax_step_filter_and_refine(hire, oracle, d, c, B, k, kp):
    """Batches of 16 and more take the bf16 filter stage and the refining selection; the exact route must agree."""
    log(f"softmax_step filter and refine d={d} c={c} B={B} k={k} kp={kp}")
    W = I.classifier(150 + B, c, d)
    layer, scorer = T.make_softmax_layer(W)
    x = I.tokens(151 + B, B, d)
    got, want = T.check_softmax(layer, scorer, W, x, k, kp)
    hire.hire_force_exact_stage(True)
    try:
        exact = T.run_softmax(layer, x, k, kp)
    finally:
        hire.hire_force_exact_stage(False)
    assert np.array_equal(exact["top_idx"], got["top_idx"])


@pytest.mark.parametrize("copies", [40, 3000])
def test_softmax_step_filter_and_refine_equal_logits(hire, oracle, copies):
    """Classes repeated many times: blocks of exactly equal logits around the k-th, settled by index; 3000 copies
    make the refined list overflow, so the selection runs in several rounds."""
    d, k, kp, B = 128, 48, 1000, 18
    base = I.classifier(160, 6, d)
    W = np.concatenate([np.repeat(base, copies, axis=0), I.classifier(161, 2000, d)], axis=0)
    layer, scorer = T.make_softmax_layer(W)
    x = I.tokens(162, B, d)
    log(f"softmax_step filter and refine, {copies} copies of six classes")
    T.check_softmax(layer, scorer, W, x, k, kp)


def test_general_route_batch_size_changes_on_one_workspace(hire, oracle):
    """A workspace sized for the largest batch serves smaller ones too; each change of batch size re-lays the
    histogram region, and results stay exact throughout."""
    d, c, k, kp = 256, 33333, 64, 1024
    W = I.classifier(77, c, d)
    layer, scorer = T.make_softmax_layer(W)
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(layer, 8, k, kp))
    for step, B in enumerate([8, 8, 3, 3, 8, 1, 8, 8]):
        log(f"batch change step {step} B={B}")
        x = I.tokens(780 + step, B, d)
        want = oracle.softmax_step(W, scorer, x, k, kp, want_acc=True)
        got = T.run_softmax(layer, x, k, kp, ws=ws)
        T.compare_softmax(got, want)


@pytest.mark.parametrize("copies", [700, 6000])
def test_softmax_step_many_equal_keys(hire, oracle, copies):
    """Rows repeated many times give blocks of equal scorer keys; the k'-th key falls inside one, and the lowest
    indices of the block are the ones taken.  700 equal keys are ranked from the threshold bin's list; 6000
    exceed the list and go through the streaming selection."""
    d, k, kp = 128, 32, 1000
    base = I.classifier(55, 12, d)
    W = np.concatenate([np.repeat(base, copies, axis=0), I.classifier(56, 500, d)], axis=0)
    layer, scorer = T.make_softmax_layer(W)
    x = I.tokens(57, 2, d)
    want = oracle.softmax_step(W, scorer, x, k, kp, want_acc=True)
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(layer, 2, k, kp))
    for got in T.run_softmax(layer, x, k, kp, steps=3, ws=ws):
        assert np.array_equal(got["cand"], want["cand"]), "candidate union differs"
        assert np.array_equal(got["top_idx"], want["top_idx"])
        T.assert_float_close(got["top_prob"], want["top_prob"], "top_prob")
    fb = hire.hire_debug_general_fallbacks(ws)
    log(f"  copies={copies}: streaming selections counted {fb}")
    if copies > 4096:
        assert fb[0] > 0


@pytest.mark.parametrize("d,N,B,k,kp", [
    (256, 4000, 24, 100, 400),      # two token tiles on the matrix cores (17..32 tokens)
    (160, 3000, 40, 60, 300),       # three token tiles, d not a multiple of 64
    (2304, 1200, 9, 50, 200),       # two K segments per row in the matrix-core scorer (d > 2048)
    (512, 70000, 3, 300, 2000),     # long rows with ReLU: counted by the selection's own pass, zeros included
    (128, 2500, 6, 700, 2400),      # k' past the positive keys: thresholds among the ReLU zeros, streaming selection
    (128, 2500, 16, 700, 2400),     # the same under filter and refine: the band reaches the zeros, fp64 selection
    (2048, 6000, 17, 300, 1200),    # filter and refine, two token tiles with a ragged second one
    (800, 5000, 33, 200, 900),      # filter and refine, three token tiles, d not a multiple of 512 (ragged last pass)
])
def test_ffn_step_batched_shapes(hire, oracle, d, N, B, k, kp):
    log(f"ffn_step batched d={d} N={N} B={B} k={k} kp={kp}")
    L = I.ffn_layer(170 + B, d, N)
    layer, scorer = T.make_ffn_layer(L)
    T.check_ffn(layer, scorer, L, I.tokens(171 + B, B, d), k, kp)


def test_long_rows_batched_with_a_zero_token(hire, oracle):
    """Long rows at batch 3 with an all-zero token in the middle: its keys are all equal (zero), the scorer's maxima
    give no bound for it, and its k' lowest-indexed units are selected from the keys directly; the other tokens go
    through the bound.  FFN (keys after the ReLU) and softmax (signed keys)."""
    d, N = 128, 40000
    x = I.tokens(185, 3, d)
    x[1] = 0
    log("ffn_step long rows, zero token in the batch")
    L = I.ffn_layer(184, d, N)
    layer, scorer = T.make_ffn_layer(L)
    T.check_ffn(layer, scorer, L, x, 50, 400)
    log("softmax_step long rows, zero token in the batch")
    W = I.classifier(186, N, d)
    sm_layer, sm_scorer = T.make_softmax_layer(W)
    T.check_softmax(sm_layer, sm_scorer, W, x, 16, 400)


def test_ffn_step_batched_duplicate_rows(hire, oracle):
    """Many identical units at batch > 1: crowded threshold bins in both selections (the k'-th key and the k-th
    activation fall inside blocks of equal values), ties settled by index."""
    d, N = 128, 3000
    L = I.ffn_layer(181, d, N)
    L["w1u"][200:1400] = L["w1u"][200]            # 1200 identical units
    layer, scorer = T.make_ffn_layer(L)
    for B in (5, 18):                             # 18: filter and refine, every copy inside the band
        x = I.tokens(182, B, d)
        for k, kp in [(50, 300), (400, 900), (1000, 1500)]:
            log(f"ffn_step batched duplicates B={B} k={k} kp={kp}")
            T.check_ffn(layer, scorer, L, x, k, kp)


@pytest.mark.parametrize("B", [1, 4])
def test_steps_with_only_the_required_outputs(hire, oracle, B):
    """The optional outputs (index lists, candidate union, counts, integer sums) may all be NULL: the library then
    keeps them in its workspace.  y, and the softmax's indices and probabilities, must not change."""
    d, N, k, kp = 256, 3000, 60, 240
    L = I.ffn_layer(190, d, N)
    x_bits = I.tokens(191 + B, B, d)
    x = T.dev_bf16(x_bits)
    for lowrank in (False, True):
        if lowrank:
            L = I.lowrank_ffn_layer(192, d, N, 32)
        layer, scorer = T.make_ffn_layer(L, lowrank=lowrank)
        want = oracle.ffn_step(L["w1u"], L["w2u"], scorer, x_bits, k, kp)
        ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, B, k, kp))
        out = hire.FFNOutputs(layer, B, k, kp)
        for step in range(3):
            out.y.fill_(float("nan"))
            hire.hire_ffn_step(layer, x, k, kp, out, ws, minimal=True)
            torch.cuda.synchronize()
            log(f"minimal ffn step B={B} lowrank={lowrank} step {step}")
            T.assert_float_close(out.y.cpu().numpy(), want["y"], "y")
    W = I.classifier(193, 40000, d)
    sm_layer, sm_scorer = T.make_softmax_layer(W)
    want = oracle.softmax_step(W, sm_scorer, x_bits, 16, 200)
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(sm_layer, B, 16, 200))
    out = hire.SoftmaxOutputs(sm_layer, B, 16, 200)
    for step in range(3):
        hire.hire_softmax_step(sm_layer, x, 16, 200, out, ws, minimal=True)
        torch.cuda.synchronize()
        log(f"minimal softmax step B={B} step {step}")
        assert np.array_equal(out.top_idx.cpu().numpy(), want["top_idx"])
        T.assert_float_close(out.top_prob.cpu().numpy(), want["top_prob"], "top_prob")


# ----------------------------------------------------------------------------
# Same inputs, same workspace, several times over: every output byte for byte, and the state that the batch-1 route
# carries in the workspace from one step to the next back where a step expects it.
def _bytes_of(out, names):
    torch.cuda.synchronize()
    return {n: getattr(out, n).cpu().numpy().copy() for n in names if getattr(out, n, None) is not None}


def _assert_same_bytes(a, b, what):
    assert a.keys() == b.keys()
    for n in a:
        assert a[n].tobytes() == b[n].tobytes(), (what, n)


@pytest.mark.parametrize("route", ["plain", "groups_of_8", "commonpath", "lowrank"])
def test_batch1_route_reruns_bit_for_bit_and_restores_its_histogram(hire, route):
    d, N = 512, 4096
    if route == "lowrank":
        L = I.lowrank_ffn_layer(143, d, N, 64)
        layer, _ = T.make_ffn_layer(L, lowrank=True)
    else:
        L = I.ffn_layer(140, d, N)
        layer, _ = T.make_ffn_layer(L)
    D = I.ffn_layer(141, d, 200)
    dw1, dw2 = T.dev_bf16(D["w1u"]), T.dev_bf16(D["w2u"])
    tokens = [T.dev_bf16(I.tokens(142 + i, 1, d)) for i in range(3)]
    if route in ("plain", "lowrank"):
        k, kp = 205, 820
        ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, 1, k, kp))
        names = ("y", "topk_idx", "topk_val", "cand_idx", "n_cand") + (("scorer_acc",) if route == "plain" else ())
        make = lambda: hire.FFNOutputs(layer, 1, k, kp, debug=True)
        run = lambda x, out: hire.hire_ffn_step(layer, x, k, kp, out, ws)
    elif route == "groups_of_8":
        k, kp = 200, 816
        ws = hire.alloc_workspace(hire.hire_ffn_group_workspace_bytes(layer, 1, k, kp, 8))
        names = ("y", "topk_group", "topk_val", "cand_group", "n_cand", "scorer_acc")
        make = lambda: hire.FFNGroupOutputs(layer, 1, k, kp, 8, debug=True)
        run = lambda x, out: hire.hire_ffn_group_step(layer, x, k, kp, 8, out, ws)
    else:
        k, kp = 200, 816
        ws = hire.alloc_workspace(hire.hire_ffn_commonpath_workspace_bytes(layer, 200, 1, k, kp, 8))
        names = ("y", "topk_group", "topk_val", "cand_group", "n_cand", "scorer_acc")
        make = lambda: hire.FFNGroupOutputs(layer, 1, k, kp, 8, debug=True)
        run = lambda x, out: hire.hire_ffn_commonpath_step(layer, dw1, dw2, x, k, kp, 8, out, ws)
    log(f"batch-1 route {route}: nine steps on one workspace, three tokens in turn")
    first = {}
    for step in range(9):
        t = step % 3
        out = make()
        run(tokens[t], out)
        got = _bytes_of(out, names)
        if t in first:
            _assert_same_bytes(got, first[t], (route, step))
        else:
            first[t] = got
        marker, nonzero_key_bins, counted_h = hire.hire_debug_fast_state(ws)
        assert marker == 1 and nonzero_key_bins == 0, (route, step, marker, nonzero_key_bins)
        assert 0 < counted_h <= kp, (route, step, counted_h)
    assert hire.hire_debug_fast_fallbacks(ws) == (0, 0)       # the histogram route ran, not the slower exact one
    assert not np.array_equal(first[0]["y"], first[1]["y"])


@pytest.mark.parametrize("B", [1, 4])
def test_sharded_step_reruns_bit_for_bit(hire, B):
    d, N, k, kp, s = 512, 4096, 192, 832, 64
    L = I.ffn_layer(150, d, N)
    layer, _ = T.make_ffn_layer(L)
    ws = hire.alloc_workspace(hire.hire_ffn_shard_workspace_bytes(layer, B, k, kp, s))
    tokens = [T.dev_bf16(I.tokens(151 + i, B, d)) for i in range(2)]
    names = ("y", "topk_idx", "topk_val", "cand_idx", "n_cand", "scorer_acc")
    log(f"sharded step B={B}: six steps on one workspace, two token sets in turn")
    first = {}
    for step in range(6):
        t = step % 2
        out = hire.FFNShardOutputs(layer, B, k, kp, s, debug=True)
        out.cand_idx.zero_()                  # entries past a shard's count are left alone by the step
        hire.hire_ffn_shard_step(layer, tokens[t], k, kp, s, out, ws)
        got = _bytes_of(out, names)
        if t in first:
            _assert_same_bytes(got, first[t], ("shard", B, step))
        else:
            first[t] = got


@pytest.mark.parametrize("B,c,d", [(1, 40000, 256), (3, 40000, 256), (2, 3000, 256),
                                   (1, 40000, 640)])   # the last: one token on the short kernel sequence
def test_softmax_step_reruns_bit_for_bit(hire, B, c, d):
    k, kp = 16, 128
    W = I.classifier(160, c, d)
    layer, _ = T.make_softmax_layer(W)
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(layer, B, k, kp))
    tokens = [T.dev_bf16(I.tokens(161 + i, B, d)) for i in range(2)]
    names = ("top_idx", "top_prob", "top_logit", "cand_idx", "n_cand", "scorer_acc")
    log(f"softmax step B={B} c={c}: six steps on one workspace, two token sets in turn")
    first = {}
    for step in range(6):
        t = step % 2
        out = hire.SoftmaxOutputs(layer, B, k, kp, debug=True)
        out.cand_idx.zero_()
        hire.hire_softmax_step(layer, tokens[t], k, kp, out, ws)
        got = _bytes_of(out, names)
        if t in first:
            _assert_same_bytes(got, first[t], ("softmax", B, c, step))
        else:
            first[t] = got


# ----------------------------------------------------------------------------
# Filter and refine of the batched exact stage (Algorithm 1, exact computation over the candidates): fp32
# approximations on the matrix cores, fp64 only around the selection threshold.
def _near_copies_layer(seed, d, N, lo, hi, tiny):
    """Units lo..hi-1 are copies of unit lo whose first `tiny` weights differ in their last two mantissa bits."""
    L = I.ffn_layer(seed, d, N)
    rng = np.random.default_rng(seed + 1)
    L["w1u"][lo:hi] = L["w1u"][lo]
    L["w1u"][lo:hi, :tiny] ^= rng.integers(0, 4, size=(hi - lo, tiny), dtype=np.uint16)
    return L


def _tokens_with_tiny_head(seed, B, d, tiny, unit_bits):
    """Tokens leaning towards one unit's weights (so its activation is positive and sizeable for all of them)
    whose first `tiny` components are 2^-18 of an ordinary one: near-copies of that unit then differ by about
    1e-9 of the activation, far below fp32 resolution (6e-8) and far above fp64 rounding."""
    x = I.bf16_bits_to_f32(I.tokens(seed, B, d))
    u = I.bf16_bits_to_f32(unit_bits)
    x = x + np.linspace(0.02, 0.12, B, dtype=np.float32)[:, None] * u[None, :] * (np.abs(x).mean() / np.abs(u).mean())
    x[:, :tiny] *= np.float32(2.0 ** -18)
    return I.f32_to_bf16_bits(x)


def test_filter_and_refine_near_copies(hire, oracle):
    """The k-th activation falls inside a block of 1200 units that agree to about 1e-9: fp32 cannot order them,
    the fp64 recomputation of the band around the threshold must, and ties between true copies go by index."""
    d, N, B, lo, hi, tiny = 512, 6000, 16, 1000, 2200, 8
    L = _near_copies_layer(190, d, N, lo, hi, tiny)
    layer, scorer = T.make_ffn_layer(L)
    x = _tokens_with_tiny_head(191, B, d, tiny, L["w1u"][lo])
    inside = 0
    for k, kp in [(300, 2000), (700, 2000), (1100, 2000), (1500, 2000), (1900, 2000)]:
        log(f"filter and refine, near copies k={k} kp={kp}")
        got, want = T.check_ffn(layer, scorer, L, x, k, kp)
        in_block = ((want["topk_idx"] >= lo) & (want["topk_idx"] < hi)).sum(axis=1)
        inside += int(((in_block > 0) & (in_block < hi - lo)).sum())
        log(f"  tokens whose threshold cuts the block: {((in_block > 0) & (in_block < hi - lo)).sum()} of {B}; "
            f"smallest margin {want['margin_k'].min():.3e}")
        hire.hire_force_exact_stage(True)
        try:
            exact = T.run_ffn(layer, x, k, kp)
        finally:
            hire.hire_force_exact_stage(False)
        assert np.array_equal(exact["topk_idx"], got["topk_idx"])
        assert np.array_equal(exact["cand"], got["cand"])
    assert inside >= 16, inside


def test_filter_and_refine_settles_ordinary_rows_from_its_list(hire, ffn_1b):
    """On ordinary inputs the band holds a few entries per token and the list in LDS settles the selection: the
    counter of selections that had to start over stays at zero."""
    L, layer, scorer = ffn_1b
    x = I.tokens(120, 16, 2048)
    ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, 16, 819, 3276))
    T.run_ffn(layer, x, 819, 3276, steps=3, ws=ws)
    fb = hire.hire_debug_general_fallbacks(ws)
    log(f"filter and refine, 1B shape B=16: counters {fb}")
    assert fb[1] == 0


@pytest.mark.parametrize("d,rows,B", [(64, 3000, 3), (2048, 4000, 20), (8192, 1500, 64), (800, 2000, 33)])
def test_filter_stage_keeps_its_error_bound_with_slack(hire, d, rows, B):
    """What the filter stage stores against the definition in fp64 (numpy): the proven distance holds with a
    factor of eight to spare, also for rows whose products cancel, and the norms are upper bounds."""
    Wb = I.normal_bf16(200 + d, (rows, d))
    xb = I.tokens(201 + d, B, d)
    Wb[0] = xb[0] ^ (np.arange(d, dtype=np.uint16) % 2 * np.uint16(0x8000))   # products cancel almost completely
    Wb[1] = xb[B - 1]                                                         # the largest activation there is
    Wb[2] = xb[B - 1] ^ np.uint16(0x8000)                                     # ... and its negative
    Wb[3] = 0
    stored, xnorm, wmax, err_c = hire.hire_debug_filter_stage(T.dev_bf16(Wb), T.dev_bf16(xb))
    stored = stored.cpu().numpy().astype(np.float64)
    W, x = I.bf16_bits_to_f64(Wb), I.bf16_bits_to_f64(xb)
    h = x @ W.T
    un, xn = np.sqrt((W * W).sum(axis=1)), np.sqrt((x * x).sum(axis=1))
    delta = err_c * xn[:, None] * un[None, :]
    assert err_c == (2.0 ** -16 if B > 32 else 2.0 ** -17)
    tiny = np.float64(np.float32(1e-45))            # the smallest positive float
    kept = stored > tiny
    worst = (np.abs(stored - h)[kept] / np.maximum(delta[kept], 1e-300)).max()
    log(f"filter stage d={d}: worst |stored - h| / delta = {worst:.4f}; kept {kept.mean():.3f}, "
        f"unsure {(stored == tiny).mean():.2e}")
    assert worst <= 1.0 / 8.0
    unsure = stored == tiny
    assert (h[unsure] <= delta[unsure] / 8).all() and (h[unsure] > -2.2 * delta[unsure] - 1e-300).all()
    zero = stored == 0.0
    assert (kept | unsure | zero).all()
    assert (h[zero] <= 0.0).all()
    assert zero[:, 3].all() or (stored[:, 3] == tiny).all()
    xg = xnorm.cpu().numpy().astype(np.float64)
    assert (xg >= xn).all() and (xg <= 1.01 * xn).all()
    assert un.max() <= wmax <= 1.01 * un.max()
