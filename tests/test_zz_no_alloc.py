"""hire_ffn_step_static (the entry point that allocates nothing: its scratch memory is a static device array inside
the library) against hire_ffn_step on a caller's workspace: same inputs, outputs compared to the bar of the parity
tests - every integer output bit for bit, floats within the stated tolerance (they come out identical: the same
kernels run).  Two calls in a row share the static array, the second with a smaller input; then the order is turned
round, and a step too large for the array must be refused before anything is enqueued."""
import numpy as np
import pytest
import torch

import hire_testlib as T
from paper_2402_09360_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hire():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2402_09360_amd import hire as H
    return H


def _run(hire, layer, x_bits, k, kp, static):
    x = T.dev_bf16(x_bits)
    B = x.shape[0]
    out = hire.FFNOutputs(layer, B, k, kp, debug=True)
    if static:
        hire.hire_ffn_step_static(layer, x, k, kp, out)
    else:
        ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, B, k, kp))
        hire.hire_ffn_step(layer, x, k, kp, out, ws)
    torch.cuda.synchronize()
    n = int(out.n_cand.item())
    return dict(y=out.y.cpu().numpy(), topk_idx=out.topk_idx.cpu().numpy(), topk_val=out.topk_val.cpu().numpy(),
                cand=out.cand_idx.cpu().numpy()[:n], n_cand=n, acc=out.scorer_acc.cpu().numpy())


def _same(got, want):
    assert got["n_cand"] == want["n_cand"]
    for name in ("acc", "cand", "topk_idx"):
        assert np.array_equal(got[name], want[name]), name
    T.assert_float_close(got["topk_val"], want["topk_val"], "topk_val")
    T.assert_float_close(got["y"], want["y"], "y")


def test_static_scratch_step_matches_workspace_step(hire):
    big = I.ffn_layer(91, 512, 4096)
    small = I.ffn_layer(92, 256, 1024)
    big_layer, _ = T.make_ffn_layer(big)
    small_layer, _ = T.make_ffn_layer(small)
    cases = [(big_layer, I.tokens(93, 4, 512), 205, 820),      # several tokens: the general kernel sequence
             (small_layer, I.tokens(94, 1, 256), 52, 208),     # then a smaller step: one token, three kernels
             (big_layer, I.tokens(95, 1, 512), 205, 820),      # and larger again on what the small one left behind
             (small_layer, I.tokens(96, 3, 256), 52, 208)]
    for n, (layer, x_bits, k, kp) in enumerate(cases):
        print(f"static scratch case {n}: B={x_bits.shape[0]} d={x_bits.shape[1]} k={k} k'={kp}", flush=True)
        want = _run(hire, layer, x_bits, k, kp, static=False)
        got = _run(hire, layer, x_bits, k, kp, static=True)
        _same(got, want)
        again = _run(hire, layer, x_bits, k, kp, static=True)   # steady state of the array for this shape
        _same(again, want)


def test_static_scratch_step_refuses_what_does_not_fit(hire):
    L = I.ffn_layer(97, 256, 1024)
    layer, _ = T.make_ffn_layer(L)
    # a descriptor of the ~1B layer shape at batch 64 needs about 15 MB of scratch; the check comes before any
    # pointer is used, so the small layer's buffers stand in
    import ctypes as C
    fake = hire._FFNLayer.from_buffer_copy(layer.c)
    fake.d_model, fake.d_ff = 2048, 16384
    assert hire._lib.hire_ffn_workspace_bytes(C.byref(fake), 64, 819, 3276) > hire.STATIC_SCRATCH_BYTES
    x = T.dev_bf16(I.tokens(98, 64, 2048))
    y = torch.empty((64, 2048), dtype=torch.float32, device="cuda")
    rc = hire._lib.hire_ffn_step_static(C.byref(fake), x.data_ptr(), 64, 819, 3276, y.data_ptr(), None, None, None,
                                        None, None, None)
    assert rc == hire.ENOSPC
