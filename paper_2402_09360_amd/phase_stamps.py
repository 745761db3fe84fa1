"""Phase stamps of the selecting kernels, read from the profiling build of the library.

    python -m paper_2402_09360_amd.build --timestamps
    HIRE_LIB=$PWD/paper_2402_09360_amd/libhire_ts.so python -m paper_2402_09360_amd.phase_stamps --batch 1
    HIRE_LIB=$PWD/paper_2402_09360_amd/libhire_ts.so python -m paper_2402_09360_amd.phase_stamps --softmax

The profiling build (-DHIRE_TIMESTAMPS) makes thread 0 of workgroup 0 store the 100 MHz wall clock and the shader
clock at numbered points of the kernels; this module runs a few FFN steps of the 1B shape (d_model 2048, d_ff
16384, k 819, k' 3276, seeded synthetic weights and tokens), reads the three tables back and prints, per kernel,
the time of every stamp since the kernel's first one.  The stamps show where the time inside ONE workgroup goes;
they do not show launch latency, and a stamp's own store costs a few tens of nanoseconds.
"""
from __future__ import annotations

import argparse
import ctypes as C

import numpy as np
import torch

from . import hire, inputs as I

# stamp number -> what has happened by then (kernels of the batch-1 route, ffn_fast.hip / fast_select.h)
FAST = [
    ("k_fast_score_int4", [(30, "kernel start"), (31, "token loaded, largest |x| known"),
                            (32, "token quantised, sum |xq| known (anchors)"), (33, "integer dot products done"),
                            (34, "keys stored and counted into the window histogram")]),
    ("k_fast_gather", [(10, "kernel start"), (11, "keys, window and token requested and unpacked"),
                       (18, "everything requested has arrived (profiling build only)"),
                       (15, "window walked: threshold bin proposed"), (16, "keys above the bin counted, bin listed"),
                       (17, "bin ranked: cut known"), (12, "selection returned"),
                       (13, "this workgroup's rows listed in LDS"), (14, "rows read, activations stored and counted")]),
    ("k_fast_w2", [(24, "kernel start (row slice known)"), (20, "window walked"), (21, "counted and listed"),
                   (22, "ranked"), (25, "selection returned"), (26, "selected rows and coefficients in LDS"),
                   (27, "second-layer rows read and accumulated"), (28, "reduced over the waves, y written")]),
]
GENERAL = [
    ("k_select_nonneg<float> (top-k' of the keys)",
     [(10, "kernel start"), (11, "keys loaded, anchor known"), (12, "window histogram built"), (13, "window walked"),
      (14, "counted and listed"), (15, "ranked"), (16, "selection returned"), (17, "bitmap / outputs written")]),
    ("k_select_nonneg<double> or k_select_refine (top-k of the activations)",
     [(40, "kernel start"), (41, "values loaded, anchor known"), (42, "window histogram built"), (43, "window walked"),
      (44, "counted and listed"), (45, "ranked"), (46, "selection returned"),
      (49, "band marked (filter and refine)"), (50, "band recomputed in fp64"), (51, "band ranked"),
      (47, "outputs written")]),
]
GATHER = [
    ("k_gather_dot_bf16 (filter stage, first workgroup)",
     [(55, "kernel start"), (56, "tile's candidates known")] +
     [(1 + 6 * p + j, f"pass {p}: {what}") for p in range(4) for j, what in enumerate(
         ["start", "tokens' slab stored", "candidates' slab stored", "next pass requested, barrier passed",
          "matrix cores done", "barrier passed"])] +
     [(57, "all passes done"), (58, "norms, stored values, maxima written")]),
]


SOFTMAX_B1 = [
    ("k_sm1_gather (first workgroup)",
     [(20, "kernel start"), (21, "keys, maxima and token requested, window cleared"),
      (22, "maxima counted, window walked: lower bound of the k'-th key known"),
      (23, "own keys at or above the bound found, their logits computed and stored")]),
    ("k_sm1_final",
     [(30, "kernel start (slots requested)"), (31, "superset counted; key bins and logit range known"),
      (32, "surplus keys dropped, logits of the shortlist counted"),
      (34, "bin of the k-th logit found, selected entries listed"), (35, "ranked, indices and logits written"),
      (36, "softmax written")]),
]


def softmax_one_token(steps):
    """Config 4's classifier (256000 x 2048, k 64, k' 1024) at one token: the short kernel sequence."""
    d, N, k, kp = 2048, 256000, 64, 1024
    layer = hire.SoftmaxLayer.with_int4_scorer(hire.bf16_from_bits(I.classifier(4, N, d)))
    out = hire.SoftmaxOutputs(layer, 1, k, kp)
    ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(layer, 1, k, kp))
    x = hire.bf16_from_bits(I.tokens(600, 1, d))
    for _ in range(steps):
        hire.hire_softmax_step(layer, x, k, kp, out, ws)
    torch.cuda.synchronize()
    print(f"# phase stamps, softmax step d_model={d} vocab={N} k={k} k'={kp} batch=1, after {steps} steps on one workspace")
    show(SOFTMAX_B1, *table("hire_debug_timestamps_softmax_b1"))


def table(name):
    fn = getattr(hire._lib, name, None)
    if fn is None:
        raise SystemExit(f"{name} is not exported: load the profiling build (HIRE_LIB=.../libhire_ts.so)")
    buf = (C.c_uint64 * 128)()
    fn(buf)
    return np.array(buf[:64], dtype=np.int64), np.array(buf[64:], dtype=np.int64)


def show(kernels, ts, tc):
    for kernel, points in kernels:
        have = [(i, what) for i, what in points if ts[i] > 0]
        if not have:
            continue
        print(kernel)
        t0, prev = ts[have[0][0]], None
        for i, what in have:
            line = f"  [{i:2d}] +{(ts[i] - t0) * 0.01:7.2f} us"
            if prev is not None:
                dt = (ts[i] - ts[prev]) * 0.01
                mhz = f" at {(tc[i] - tc[prev]) / dt:5.0f} MHz" if dt > 0 else ""
                line += f"  (+{dt:5.2f}{mhz})"
            print(f"{line:52s} {what}")
            prev = i


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--steps", type=int, default=6)
    ap.add_argument("--general", action="store_true", help="batch 1 through the general kernel sequence")
    ap.add_argument("--softmax", action="store_true", help="the softmax step for one token instead of the FFN step")
    args = ap.parse_args()
    if args.softmax:
        softmax_one_token(args.steps)
        return
    d, N, k, kp, B = 2048, 16384, 819, 3276, args.batch
    L = I.ffn_layer(500, d, N)
    layer = hire.FFNLayer.with_int4_scorer(hire.bf16_from_bits(L["w1u"]), hire.bf16_from_bits(L["w2u"]))
    out = hire.FFNOutputs(layer, B, k, kp)
    ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layer, B, k, kp))
    x = hire.bf16_from_bits(I.tokens(600, B, d))
    if args.general:
        hire.hire_force_generic_path(True)
    for _ in range(args.steps):
        hire.hire_ffn_step(layer, x, k, kp, out, ws)
    torch.cuda.synchronize()
    print(f"# phase stamps, FFN step d_model={d} d_ff={N} k={k} k'={kp} batch={B}, after {args.steps} steps on one workspace")
    if B == 1 and not args.general:
        show(FAST, *table("hire_debug_timestamps_fast"))
    else:
        show(GENERAL, *table("hire_debug_timestamps_select"))
        show(GATHER, *table("hire_debug_timestamps_gather"))


if __name__ == "__main__":
    main()
