"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run a step through the
C ABI binding, run the CPU oracle on the same bytes, and compare to the stated bars:
integers (scorer sums, index sets) bit-exact; floats max-rel-err <= 2e-3 (bf16 in, wide accumulate)."""
import numpy as np
import torch

from paper_2402_09360_amd import inputs as I

FLOAT_TOL = 2e-3


def dev_bf16(bits):
    from paper_2402_09360_amd import hire
    return hire.bf16_from_bits(bits)


def assert_float_close(got, want, what):
    """Per row: max|got-want| / max|want| <= 2e-3, and elementwise within 2e-3 relative + 2e-3*rms absolute."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    g2 = got.reshape(-1, got.shape[-1])
    w2 = want.reshape(-1, want.shape[-1])
    for r in range(g2.shape[0]):
        den = np.abs(w2[r]).max()
        err = np.abs(g2[r] - w2[r]).max()
        assert err <= FLOAT_TOL * max(den, 1e-30), (what, r, err, den)
        rms = np.sqrt((w2[r] ** 2).mean())
        assert np.allclose(g2[r], w2[r], rtol=FLOAT_TOL, atol=FLOAT_TOL * rms), (what, r)


def make_ffn_layer(L, lowrank=False, lrq=False):
    """L: dict from inputs.ffn_layer / lowrank_ffn_layer -> (device layer, oracle scorer tuple)."""
    from paper_2402_09360_amd import hire
    from oracle import hire_oracle as O
    w1u, w2u = dev_bf16(L["w1u"]), dev_bf16(L["w2u"])
    if lrq:
        layer = hire.FFNLayer.with_lrq_scorer(w1u, w2u, dev_bf16(L["z1"]), dev_bf16(L["z2"]))
        return layer, O.lrq_factors(L["z1"], L["z2"])
    if lowrank:
        layer = hire.FFNLayer(w1u, w2u, lr_a=dev_bf16(L["z1"]), lr_b=dev_bf16(L["z2"]))
        return layer, ("lowrank", L["z1"], L["z2"])
    layer = hire.FFNLayer.with_int4_scorer(w1u, w2u)
    q, s = O.quantize_rows_int4(L["w1u"])
    return layer, ("int4", q, s)


def make_softmax_layer(W_bits, lrq=None):
    """lrq: (z1 bits [d, r], z2 bits [vocab, r]) for the int4 low-rank scorer; default the int4 copy of W."""
    from paper_2402_09360_amd import hire
    from oracle import hire_oracle as O
    if lrq is not None:
        layer = hire.SoftmaxLayer.with_lrq_scorer(dev_bf16(W_bits), dev_bf16(lrq[0]), dev_bf16(lrq[1]))
        return layer, O.lrq_factors(lrq[0], lrq[1])
    layer = hire.SoftmaxLayer.with_int4_scorer(dev_bf16(W_bits))
    q, s = O.quantize_rows_int4(W_bits)
    return layer, ("int4", q, s)


def run_ffn(layer, x_bits, k, kprime, debug=True, steps=1, ws=None):
    """Run `steps` steps on one workspace and return the outputs of each (a fresh workspace takes the
    histogram-free first-use route of the batch-1 kernels, later steps the histogram route)."""
    from paper_2402_09360_amd import hire
    x = dev_bf16(x_bits)
    B = x.shape[0]
    if ws is None:
        ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, B, k, kprime))
    results = []
    for _ in range(steps):
        out = hire.FFNOutputs(layer, B, k, kprime, debug=debug)
        hire.hire_ffn_step(layer, x, k, kprime, out, ws)
        torch.cuda.synchronize()
        n = int(out.n_cand.item())
        results.append(dict(y=out.y.cpu().numpy(), topk_idx=out.topk_idx.cpu().numpy(),
                            topk_val=out.topk_val.cpu().numpy(), cand=out.cand_idx.cpu().numpy()[:n], n_cand=n,
                            acc=None if out.scorer_acc is None else out.scorer_acc.cpu().numpy()))
    return results[0] if steps == 1 else results


def compare_ffn(got, want):
    if want["acc"] is not None:
        assert np.array_equal(got["acc"], want["acc"]), "integer scorer sums differ"
    assert got["n_cand"] == len(want["cand"]), ("|U|", got["n_cand"], len(want["cand"]))
    assert np.array_equal(got["cand"], want["cand"]), "candidate union differs"
    assert np.array_equal(got["topk_idx"], want["topk_idx"]), (
        "top-k index sets differ", want["margin_k"].min())
    assert_float_close(got["topk_val"], want["topk_val"], "topk_val")
    assert_float_close(got["y"], want["y"], "y")


def check_ffn(layer, scorer, L, x_bits, k, kprime):
    """Run both sides on the same bytes and compare everything the step returns.  The GPU side runs the
    step three times on one workspace (first-use route, then twice the steady-state route) and once more
    through the general kernel sequence; all must match the oracle."""
    from oracle import hire_oracle as O
    from paper_2402_09360_amd import hire
    want = O.ffn_step(L["w1u"], L["w2u"], scorer, x_bits, k, kprime, want_acc=True)
    runs = run_ffn(layer, x_bits, k, kprime, steps=3)
    for r in runs:
        compare_ffn(r, want)
    hire.hire_force_generic_path(True)
    try:
        generic = run_ffn(layer, x_bits, k, kprime, steps=3)
    finally:
        hire.hire_force_generic_path(False)
    for r in generic:
        compare_ffn(r, want)
    return runs[-1], want


def run_ffn_group(layer, x_bits, k, kprime, g, debug=True, steps=1, ws=None):
    from paper_2402_09360_amd import hire
    x = dev_bf16(x_bits)
    B = x.shape[0]
    if ws is None:
        ws = hire.alloc_workspace(hire.hire_ffn_group_workspace_bytes(layer, B, k, kprime, g))
    results = []
    for _ in range(steps):
        out = hire.FFNGroupOutputs(layer, B, k, kprime, g, debug=debug)
        hire.hire_ffn_group_step(layer, x, k, kprime, g, out, ws)
        torch.cuda.synchronize()
        n = int(out.n_cand.item())
        results.append(dict(y=out.y.cpu().numpy(), topk_group=out.topk_group.cpu().numpy(),
                            topk_val=out.topk_val.cpu().numpy(), cand=out.cand_group.cpu().numpy()[:n], n_cand=n,
                            acc=None if out.scorer_acc is None else out.scorer_acc.cpu().numpy()))
    return results[0] if steps == 1 else results


def check_ffn_group(layer, scorer, L, x_bits, k, kprime, g):
    """Group-sparse step: three steps on one workspace (batch 1 with groups of eight: first-use route, then twice
    the steady-state route of the four-kernel sequence) and three more through the general kernel sequence, all
    compared with the oracle."""
    from oracle import hire_oracle as O
    from paper_2402_09360_amd import hire
    want = O.ffn_group_step(L["w1u"], L["w2u"], scorer, x_bits, k, kprime, g, want_acc=True)
    runs = run_ffn_group(layer, x_bits, k, kprime, g, steps=3)
    hire.hire_force_generic_path(True)
    try:
        runs = runs + run_ffn_group(layer, x_bits, k, kprime, g, steps=3)
    finally:
        hire.hire_force_generic_path(False)
    for got in runs:
        if want["acc"] is not None:
            assert np.array_equal(got["acc"], want["acc"]), "integer scorer sums differ"
        assert got["n_cand"] == len(want["cand"]), ("|U_g|", got["n_cand"], len(want["cand"]))
        assert np.array_equal(got["cand"], want["cand"]), ("group union differs", want["margin_kprime"].min())
        assert np.array_equal(got["topk_group"], want["topk_group"]), ("selected groups differ", want["margin_k"].min())
        assert_float_close(got["topk_val"], want["topk_val"], "topk_val")
        assert_float_close(got["y"], want["y"], "y")
    return runs[-1], want


def check_ffn_commonpath(layer, scorer, L, dense, x_bits, k, kprime, g):
    """CommonPath step: dense = (w1u bits [m1, d], w2u bits [m1, d]) next to the sparse layer L; three steps on one
    workspace, all compared with the oracle."""
    from oracle import hire_oracle as O
    from paper_2402_09360_amd import hire
    want = O.ffn_commonpath_step(dense[0], dense[1], L["w1u"], L["w2u"], scorer, x_bits, k, kprime, g, want_acc=True)
    m1 = dense[0].shape[0]
    dw1 = dev_bf16(dense[0]) if m1 else None
    dw2 = dev_bf16(dense[1]) if m1 else None
    x = dev_bf16(x_bits)
    B = x.shape[0]
    ws = hire.alloc_workspace(hire.hire_ffn_commonpath_workspace_bytes(layer, m1, B, k, kprime, g))
    for it in range(6):   # three steps on the default route, three forced through the general kernel sequence
        out = hire.FFNGroupOutputs(layer, B, k, kprime, g, debug=True)
        hire.hire_force_generic_path(it >= 3)
        try:
            hire.hire_ffn_commonpath_step(layer, dw1, dw2, x, k, kprime, g, out, ws)
        finally:
            hire.hire_force_generic_path(False)
        torch.cuda.synchronize()
        n = int(out.n_cand.item())
        if want["acc"] is not None:
            assert np.array_equal(out.scorer_acc.cpu().numpy(), want["acc"])
        assert np.array_equal(out.cand_group.cpu().numpy()[:n], want["cand"]), "group union differs"
        assert np.array_equal(out.topk_group.cpu().numpy(), want["topk_group"]), (
            "selected groups differ", want["margin_k"].min())
        assert_float_close(out.topk_val.cpu().numpy(), want["topk_val"], "topk_val")
        assert_float_close(out.y.cpu().numpy(), want["y"], "y")
    return out, want


def run_ffn_shard(layer, x_bits, k, kprime, shards, debug=True, steps=1, ws=None):
    from paper_2402_09360_amd import hire
    x = dev_bf16(x_bits)
    B = x.shape[0]
    if ws is None:
        ws = hire.alloc_workspace(hire.hire_ffn_shard_workspace_bytes(layer, B, k, kprime, shards))
    results = []
    for _ in range(steps):
        out = hire.FFNShardOutputs(layer, B, k, kprime, shards, debug=debug)
        hire.hire_ffn_shard_step(layer, x, k, kprime, shards, out, ws)
        torch.cuda.synchronize()
        n = out.n_cand.cpu().numpy()
        cand = out.cand_idx.cpu().numpy()
        results.append(dict(y=out.y.cpu().numpy(), topk_idx=out.topk_idx.cpu().numpy(),
                            topk_val=out.topk_val.cpu().numpy(), cand=[cand[i, :n[i]] for i in range(shards)],
                            n_cand=n, acc=None if out.scorer_acc is None else out.scorer_acc.cpu().numpy()))
    return results[0] if steps == 1 else results


def check_ffn_shard(layer, scorer, L, x_bits, k, kprime, shards):
    """Sharded step (Algorithm 2): two steps on one workspace, both compared with the oracle."""
    from oracle import hire_oracle as O
    want = O.ffn_shard_step(L["w1u"], L["w2u"], scorer, x_bits, k, kprime, shards, want_acc=True)
    runs = run_ffn_shard(layer, x_bits, k, kprime, shards, steps=2)
    for got in runs:
        assert np.array_equal(got["acc"], want["acc"]), "integer scorer sums differ"
        assert np.array_equal(got["n_cand"], want["n_cand"]), "per-shard union sizes differ"
        for i in range(shards):
            assert np.array_equal(got["cand"][i], want["cand"][i]), ("candidate union differs in shard", i)
        assert np.array_equal(got["topk_idx"], want["topk_idx"]), ("selected units differ", want["margin_k"].min())
        assert_float_close(got["topk_val"], want["topk_val"], "topk_val")
        assert_float_close(got["y"], want["y"], "y")
    return runs[-1], want


def run_softmax(layer, x_bits, k, kprime, debug=True, steps=1, ws=None):
    from paper_2402_09360_amd import hire
    x = dev_bf16(x_bits)
    B = x.shape[0]
    if ws is None:
        ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(layer, B, k, kprime))
    results = []
    for _ in range(steps):
        out = hire.SoftmaxOutputs(layer, B, k, kprime, debug=debug)
        hire.hire_softmax_step(layer, x, k, kprime, out, ws)
        torch.cuda.synchronize()
        n = int(out.n_cand.item())
        results.append(dict(top_idx=out.top_idx.cpu().numpy(), top_prob=out.top_prob.cpu().numpy(),
                            top_logit=out.top_logit.cpu().numpy(), cand=out.cand_idx.cpu().numpy()[:n], n_cand=n,
                            acc=None if out.scorer_acc is None else out.scorer_acc.cpu().numpy()))
    return results[0] if steps == 1 else results


def check_softmax(layer, scorer, W_bits, x_bits, k, kprime):
    """The GPU side runs three steps on one workspace: the first selects by streaming (fresh workspace), the
    others through the key histograms.  All must match the oracle."""
    from oracle import hire_oracle as O
    want = O.softmax_step(W_bits, scorer, x_bits, k, kprime, want_acc=True)
    for got in run_softmax(layer, x_bits, k, kprime, steps=3):
        compare_softmax(got, want)
    return got, want


def compare_softmax(got, want):
    if want["acc"] is not None:
        assert np.array_equal(got["acc"], want["acc"]), "integer scorer sums differ"
    assert np.array_equal(got["cand"], want["cand"]), "candidate union differs"
    assert np.array_equal(got["top_idx"], want["top_idx"]), ("top-k ranking differs", want["margin_k"].min())
    assert_float_close(got["top_logit"], want["top_logit"], "top_logit")
    assert_float_close(got["top_prob"], want["top_prob"], "top_prob")
    assert np.allclose(got["top_prob"].sum(axis=1), 1.0, atol=1e-5)
