"""Recall of the HiRE candidate stage on synthetic layers, swept over the scorer, its rank r and the shortlist
size k' (the shape of the paper's rank / k' trade-off tables, arXiv 2402.09360 Sec. 4.3, on seeded synthetic data:
the numbers say how the method behaves on a layer with a decaying spectrum, not how the paper's model behaves).

    python -m paper_2402_09360_amd.recall_sweep [--batch B] [--steps K]

For every setting the script runs hire_ffn_step on the MI355X and compares each token's selected units with the exact
top-k of relu(W1 x) over all units (a plain fp64 matrix product, used here only as the yardstick):
recall = |S_HiRE ∩ S_exact| / k, averaged over tokens; next to it the step time (eager launches, HIP events).
Layer: d_model 2048, d_ff 16384, W1 = P diag(sigma) Q^T with sigma_i ~ i^-1/2; low-rank scorers use the leading r
terms of that decomposition.  Prints a markdown table.
"""
from __future__ import annotations

import argparse
import sys


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=4)
    ap.add_argument("--steps", type=int, default=50)
    args = ap.parse_args()

    import numpy as np
    import torch
    from paper_2402_09360_amd import hire, hiprt, inputs as I

    assert torch.cuda.is_available(), "recall_sweep needs the MI355X"
    d, N, k, B = 2048, 16384, 819, args.batch
    ranks = (32, 64, 128, 256)
    L = I.lowrank_ffn_layer(3, d, N, max(ranks))          # factors of rank 256; lower ranks are their leading columns
    w1u, w2u = hire.bf16_from_bits(L["w1u"]), hire.bf16_from_bits(L["w2u"])
    x_bits = I.tokens(700, B, d)
    x = hire.bf16_from_bits(x_bits)
    act = torch.relu(x.double() @ w1u.double().t())
    exact = [set(torch.topk(act[b], k).indices.tolist()) for b in range(B)]

    def z(r):
        return (hire.bf16_from_bits(np.ascontiguousarray(L["z1"][:, :r])),
                hire.bf16_from_bits(np.ascontiguousarray(L["z2"][:, :r])))

    settings = [("HiRE-Q (int4 copy of W1)", lambda: hire.FFNLayer.with_int4_scorer(w1u, w2u))]
    for r in ranks:
        settings.append((f"HiRE-LR r={r}", lambda r=r: hire.FFNLayer(w1u, w2u, lr_a=z(r)[0], lr_b=z(r)[1])))
    for r in ranks:
        settings.append((f"HiRE-LRQ r={r}", lambda r=r: hire.FFNLayer.with_lrq_scorer(w1u, w2u, *z(r))))

    mults = (1, 2, 4, 8)
    print(f"| scorer | " + " | ".join(f"k'={m}k: recall, us" for m in mults) + " |")
    print("|---|" + "---|" * len(mults))
    stream = torch.cuda.current_stream().cuda_stream
    ev = hiprt.Events(2)
    for name, make in settings:
        layer = make()
        cells = []
        for m in mults:
            kp = min(N, m * k)
            out = hire.FFNOutputs(layer, B, k, kp)
            ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, B, k, kp))
            for _ in range(5):
                hire.hire_ffn_step(layer, x, k, kp, out, ws)
            torch.cuda.synchronize()
            ev.record(0, stream)
            for _ in range(args.steps):
                hire.hire_ffn_step(layer, x, k, kp, out, ws, minimal=True)
            ev.record(1, stream)
            torch.cuda.synchronize()
            us = ev.elapsed_ms(0, 1) * 1e3 / args.steps
            hire.hire_ffn_step(layer, x, k, kp, out, ws)
            torch.cuda.synchronize()
            got = out.topk_idx.cpu().numpy()
            rec = float(np.mean([len(exact[b] & set(got[b].tolist())) / k for b in range(B)]))
            cells.append(f"{rec:.3f}, {us:.0f}")
        print(f"| {name} | " + " | ".join(cells) + " |", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
