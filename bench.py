#!/usr/bin/env python3
"""Benchmark of the HiRE decode-step hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A "step" is one pass of the whole HiRE-FFN (or HiRE-Softmax) path over one batch of synthetic tokens:
scorer -> top-k' -> union -> exact scores on the candidates -> exact top-k -> second layer (or softmax).
The default workload is the batch-1 HiRE-FFN step at the ~1B-decoder shape (d_model 2048, d_ff 16384,
k = 819, k' = 3276, int4 scorer).  Weights rotate over 18 distinct seeded layers (2.7 GB) so that every
step reads HBM-cold weights rather than the Infinity Cache.  All inputs are resident in HBM before the timed
region; the K timed steps are enqueued back to back on one stream (replayed from a HIP graph so that host
launch cost does not bound them) and bracketed by device synchronisation.  Five repetitions; `value` is their
median, the minimum is reported next to it.

Prints ONE JSON line: step time, achieved algorithmic HBM bandwidth of the whole step, a list of the step's
kernels with their algorithmic bytes and durations, the roofline of the kernel that dominates the step BY TIME,
the recall of the exact dense top-k, and the CPU oracle (HiRE step and dense layer) timed on the host cores.

Kernel durations come from two places and both are reported: the average of the same kernel in the committed
`rocprofv3 --kernel-trace --stats` summary of this workload (profiles/<workload>_kernel_stats.txt: the kernel's own
duration, from which `frac` is computed so that it can be recomputed by hand from that file), and HIP events
recorded live around the kernel on its stream in this run (eager launches: they include dispatch latency and do
not add up to the step time of the graph replay).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
REPS = 5

WORKLOADS = {
    # name: (kind, scorer, batch)
    "ffn_1b_b1": ("ffn", "int4", 1),
    "ffn_1b_b4": ("ffn", "int4", 4),
    "ffn_1b_b16": ("ffn", "int4", 16),
    "ffn_1b_b64": ("ffn", "int4", 64),
    # tokens that share a component, x_b = sqrt(rho) c + sqrt(1 - rho) e_b: stands in for samples of one query,
    # whose activations overlap (Sec. 3.4.1)
    "ffn_1b_b4_rho0.9": ("ffn", "int4", 4),
    "ffn_1b_b16_rho0.9": ("ffn", "int4", 16),
    "ffn_lr_b1": ("ffn", "lowrank", 1),
    "ffn_lr_b16": ("ffn", "lowrank", 16),
    "softmax_1b_b1": ("softmax", "int4", 1),
    "softmax_1b_b16": ("softmax", "int4", 16),
    "softmax_1b_b64": ("softmax", "int4", 64),
    "ffn_small_b1": ("ffn_small", "int4", 1),
    # the full decode-step stack: 18 FFN steps and one softmax step per "step", 64 tokens
    "stack_1b_b64": ("stack", "int4", 64),
    # group-sparse FFN, groups of 8 adjacent units (k = 816 = 102 groups, k' = 3264 = 408 groups)
    "ffn_1b_g8_b1": ("ffn_g8", "int4", 1),
    "ffn_1b_g8_b4": ("ffn_g8", "int4", 4),
    "ffn_1b_g8_b16": ("ffn_g8", "int4", 16),
    # Algorithm 2's sharded top-k, 256 shards of 64 units (k = 768 = 3 per shard, k' = 3328 = 13 per shard)
    "ffn_1b_s256_b1": ("ffn_s256", "int4", 1),
    "ffn_1b_s256_b4": ("ffn_s256", "int4", 4),
    "ffn_1b_s256_b16": ("ffn_s256", "int4", 16),
    "ffn_small_s16_b1": ("ffn_small_s16", "int4", 1),   # config 1's layer, 16 shards (k = 48, k' = 208)
    # CommonPath: 2736 of the 16384 units dense, groups of 8 on the other 13648 (k = 544, k' = 2176)
    "ffn_1b_cp_b1": ("ffn_cp", "int4", 1),
    "ffn_1b_cp_b4": ("ffn_cp", "int4", 4),
    # HiRE-LRQ: the low-rank factors in int4 (FFN: config 3's rank-128 factors; softmax: rank d/4 = 512, random
    # factors - the scorer's quality is not what is timed)
    "ffn_lrq_b1": ("ffn", "lrq", 1),
    "ffn_lrq_b16": ("ffn", "lrq", 16),
    "softmax_lrq_b1": ("softmax", "lrq", 1),
    "softmax_lrq_b16": ("softmax", "lrq", 16),
}


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


# stage of the live event timing -> names (substrings) of its kernels in a rocprofv3 summary
_STAGE_KERNELS = {
    "scorer": ("k_fast_score", "k_scorer_int4", "k_lr_score", "k_lr_project", "k_lr_reduce"),
    "quantise_x": ("k_quantize_tokens",),
    "select_kprime": ("k_select<float", "k_select_nonneg<float", "k_count_f32", "k_mark_f32", "k_group_sums",
                      "k_sm1_gather<false"),
    "union": ("k_resolve_compact", "k_bitmap_compact", "k_union_compact", "k_max_resolve"),
    "gather_dot": ("k_gather_dot", "k_sm1_gather<true", "k_sm1_final"),
    "select_k": ("k_select<double", "k_select_nonneg<double", "k_select_refine"),
    "select_k_softmax": ("k_select<double",),
    "second_layer": ("k_w2_tokens", "k_w2_reduce"),
    "shard_step": ("k_ffn_shard",),
    "reduce": ("k_fast_reduce", "k_shard_reduce"),
    "select_gather": ("k_fast_gather",),
    "select_w2": ("k_fast_w2",),
}


def profiled_kernels(workload):
    """[(kernel name, calls, avg_us)] from the committed rocprofv3 --kernel-trace --stats summary of this workload
    (profiles/<workload>_kernel_stats.txt), or [] when no summary has been taken."""
    path = os.path.join(ROOT, "profiles", f"{workload}_kernel_stats.txt")
    rows = []
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 6 and line.startswith("hire::"):      # name (may contain spaces), calls, avg, min, max, pct
                rows.append((" ".join(f[:-5]), int(f[-5]), float(f[-4])))
    except (OSError, ValueError):
        return []
    return rows


def profiled_traffic(workload, names):
    """HBM bytes per launch (read + written) of the kernels whose names contain one of `names`, from the committed
    rocprofv3 --pmc summary of this workload (profiles/<workload>_hbm_traffic.txt: counters already scaled by the
    plain-copy calibration), or None when no summary has been taken."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    try:
        total = None
        for line in open(path):
            f = line.split()
            if len(f) >= 4 and line.startswith("hire::") and any(n in line for n in names):
                total = (total or 0) + int(float(f[-2])) + int(float(f[-1]))     # name, dispatches, read, written
        return total
    except OSError:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=360)
    ap.add_argument("--warmup", type=int, default=36)
    ap.add_argument("--workload", default="ffn_1b_b1", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=0, help="distinct weight sets to rotate over (0 = default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph replay")
    ap.add_argument("--exact-stage", action="store_true",
                    help="batches: every candidate's activation in fp64 instead of filter and refine (comparison run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU path (no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2402_09360_amd import cost, hire, hiprt, inputs as I

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    if args.exact_stage:
        hire.hire_force_exact_stage(True)
    kind, scorer, B = WORKLOADS[args.workload]
    K, W = args.steps, args.warmup
    rho = 0.9 if "rho0.9" in args.workload else 0.0
    stack = kind == "stack"
    if stack and args.steps == 360:
        K, W = 20, 2        # a stack step is 18 FFN steps and a softmax step

    group = 8 if kind in ("ffn_g8", "ffn_cp") else 1
    m1 = 2736 if kind == "ffn_cp" else 0
    dense = []
    # ---------------- inputs, resident in HBM ----------------
    t0 = time.time()
    host_layers = []
    classifiers, host_classifier, host_factors = [], None, None
    if kind in ("softmax", "stack"):
        sd, sN, sk, skp = 2048, 256000, 64, 1024
        n_cls = (args.layers or 2) if kind == "softmax" else 1   # 1.05 GB + 0.26 GB each; the int4 copy alone
        for l in range(n_cls):                                  # exceeds the Infinity Cache
            Wb = I.classifier(4 + 1000 * l, sN, sd)
            if scorer == "lrq":
                zz = (I.normal_bf16(40 + 1000 * l, (sd, 512), sd ** -0.5), I.normal_bf16(41 + 1000 * l, (sN, 512), 1.0))
                classifiers.append(hire.SoftmaxLayer.with_lrq_scorer(hire.bf16_from_bits(Wb), hire.bf16_from_bits(zz[0]),
                                                                     hire.bf16_from_bits(zz[1])))
            else:
                classifiers.append(hire.SoftmaxLayer.with_int4_scorer(hire.bf16_from_bits(Wb)))
            if l == 0:
                host_classifier = Wb
                host_factors = zz if scorer == "lrq" else None
            log(f"classifier {l} ready ({time.time() - t0:.1f}s)")
    layers = []
    if kind != "softmax":
        if kind == "ffn_small":
            d, N, k, kp = 256, 1024, 52, 208
        elif kind == "ffn_g8":
            d, N, k, kp = 2048, 16384, 816, 3264
        elif kind == "ffn_s256":
            d, N, k, kp = 2048, 16384, 768, 3328
        elif kind == "ffn_small_s16":
            d, N, k, kp = 256, 1024, 48, 208
        elif kind == "ffn_cp":
            d, N, k, kp = 2048, 13648, 544, 2176
        else:
            d, N, k, kp = 2048, 16384, 819, 3276
        n_layers = args.layers or 18
        for l in range(n_layers):
            if scorer == "lowrank":
                L = I.lowrank_ffn_layer(3 + 1000 * l, d, N, 128)
                layers.append(hire.FFNLayer(hire.bf16_from_bits(L["w1u"]), hire.bf16_from_bits(L["w2u"]),
                                            lr_a=hire.bf16_from_bits(L["z1"]), lr_b=hire.bf16_from_bits(L["z2"])))
            elif scorer == "lrq":
                L = I.lowrank_ffn_layer(3 + 1000 * l, d, N, 128)
                layers.append(hire.FFNLayer.with_lrq_scorer(hire.bf16_from_bits(L["w1u"]), hire.bf16_from_bits(L["w2u"]),
                                                            hire.bf16_from_bits(L["z1"]), hire.bf16_from_bits(L["z2"])))
            else:
                L = I.ffn_layer(500 + l, d, N)
                layers.append(hire.FFNLayer.with_int4_scorer(hire.bf16_from_bits(L["w1u"]),
                                                             hire.bf16_from_bits(L["w2u"])))
            if m1:
                D = I.ffn_layer(700 + l, d, m1)
                dense.append((hire.bf16_from_bits(D["w1u"]), hire.bf16_from_bits(D["w2u"])))
                if l == 0:
                    host_dense = (D["w1u"], D["w2u"])
            if l == 0:
                host_layers.append(L)
        log(f"{n_layers} FFN layers ready ({time.time() - t0:.1f}s)")
    else:
        d, N, k, kp = sd, sN, sk, skp
        n_layers = len(classifiers)
    shards = 256 if kind == "ffn_s256" else (16 if kind == "ffn_small_s16" else 1)
    make_tokens = (lambda seed: I.correlated_tokens(seed, B, d, rho)) if rho else (lambda seed: I.tokens(seed, B, d))
    x_bits = [make_tokens(600 + l) for l in range(n_layers)]
    xs = [hire.bf16_from_bits(xb) for xb in x_bits]
    sm_outs = sm_ws = None
    if kind == "softmax":
        outs = [hire.SoftmaxOutputs(classifiers[l], B, k, kp) for l in range(n_layers)]
        ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(classifiers[0], B, k, kp))
        step_fn = hire.hire_softmax_step
        layers = classifiers
    elif shards > 1:
        outs = [hire.FFNShardOutputs(layers[l], B, k, kp, shards) for l in range(n_layers)]
        ws = hire.alloc_workspace(hire.hire_ffn_shard_workspace_bytes(layers[0], B, k, kp, shards))
        step_fn = lambda layer, x, k_, kp_, out, ws_: hire.hire_ffn_shard_step(layer, x, k_, kp_, shards, out, ws_)
    elif m1:
        outs = [hire.FFNGroupOutputs(layers[l], B, k, kp, group) for l in range(n_layers)]
        ws = hire.alloc_workspace(hire.hire_ffn_commonpath_workspace_bytes(layers[0], m1, B, k, kp, group))
        dense_of = {id(layers[l]): dense[l] for l in range(n_layers)}
        step_fn = lambda layer, x, k_, kp_, out, ws_: hire.hire_ffn_commonpath_step(
            layer, dense_of[id(layer)][0], dense_of[id(layer)][1], x, k_, kp_, group, out, ws_)
    elif group > 1:
        outs = [hire.FFNGroupOutputs(layers[l], B, k, kp, group) for l in range(n_layers)]
        ws = hire.alloc_workspace(hire.hire_ffn_group_workspace_bytes(layers[0], B, k, kp, group))
        step_fn = lambda layer, x, k_, kp_, out, ws_: hire.hire_ffn_group_step(layer, x, k_, kp_, group, out, ws_)
    else:
        outs = [hire.FFNOutputs(layers[l], B, k, kp) for l in range(n_layers)]
        ws = hire.alloc_workspace(hire.hire_ffn_workspace_bytes(layers[0], B, k, kp))
        step_fn = hire.hire_ffn_step
    if stack:
        sm_outs = hire.SoftmaxOutputs(classifiers[0], B, sk, skp)
        sm_ws = hire.alloc_workspace(hire.hire_softmax_workspace_bytes(classifiers[0], B, sk, skp))
        sm_x_bits = I.tokens(699, B, sd)
        sm_x = hire.bf16_from_bits(sm_x_bits)
    torch.cuda.synchronize()

    def step(i):
        if stack:       # the whole decode-step stack: every FFN layer once, then the classifier
            for l in range(n_layers):
                step_fn(layers[l], xs[l], k, kp, outs[l], ws)
            hire.hire_softmax_step(classifiers[0], sm_x, sk, skp, sm_outs, sm_ws)
            return
        l = i % n_layers
        step_fn(layers[l], xs[l], k, kp, outs[l], ws)

    # ---------------- warm-up, then K timed steps, REPS times ----------------
    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(K):
                step(W + i)
        graph.replay()                      # one untimed replay: graph upload
        torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream
    ev = hiprt.Events(2)
    reps = []
    for _ in range(REPS):
        torch.cuda.synchronize()
        ev.record(0, stream)
        if graph is not None:
            graph.replay()
        else:
            for i in range(K):
                step(W + i)
        ev.record(1, stream)
        torch.cuda.synchronize()
        reps.append(ev.elapsed_ms(0, 1))
    rep_us = sorted(r * 1e3 / K for r in reps)
    us_per_step = rep_us[len(rep_us) // 2]      # median
    min_us = rep_us[0]

    # ---------------- union sizes the steps actually produced -> algorithmic bytes ----------------
    def ffn_bytes():
        n_cand = float(np.mean([int(o.n_cand.sum().item()) for o in outs])) * group      # rows
        n_sel = float(np.mean([len(torch.unique(o.topk_group if group > 1 else o.topk_idx)) for o in outs])) * group
        by = cost.ffn_step_bytes(scorer, d, N, B, n_cand, n_sel, r=128 if scorer in ("lowrank", "lrq") else 0)
        if m1:      # the dense units' two matrices are read whole; the dense equivalent covers them too
            by["dense_units"] = 2 * m1 * d * 2
            by["total"] += by["dense_units"]
            by["dense"] += by["dense_units"]
        return by, n_cand, n_sel

    if kind == "softmax":
        n_cand = float(np.mean([int(o.n_cand.sum().item()) for o in outs]))
        by = cost.softmax_step_bytes(scorer, d, N, B, n_cand, k, r=512 if scorer == "lrq" else 0)
        n_sel = None
    elif stack:
        fby, n_cand, n_sel = ffn_bytes()
        sm_cand = float(int(sm_outs.n_cand.sum().item()))
        sby = cost.softmax_step_bytes(scorer, sd, sN, B, sm_cand, sk)
        by = {"ffn_layer": fby["total"], "ffn_layers": n_layers * fby["total"], "softmax": sby["total"],
              "total": n_layers * fby["total"] + sby["total"], "dense": n_layers * fby["dense"] + sby["dense"]}
    else:
        by, n_cand, n_sel = ffn_bytes()
    gbps = by["total"] / (us_per_step * 1e-6) / 1e9

    # ---------------- per-stage times, live, with HIP events on the launch stream ----------------
    # the three-kernel batch-1 route (units, or groups of eight)
    fast = B == 1 and ((kind in ("ffn", "ffn_small", "ffn_g8", "ffn_cp") and scorer == "int4") or
                       (kind == "ffn" and scorer in ("lowrank", "lrq")))
    stages = hire.SOFTMAX_STAGES if kind == "softmax" else (hire.FAST_FFN_STAGES if fast else hire.FFN_STAGES)
    if shards > 1:
        stages = ("shard_step", "reduce")
    stage_us = {}
    scorer_exec_us = None
    if not stack:
        sev = hiprt.Events(hire.NUM_STAGE_EVENTS)
        acc = np.zeros(len(stages))
        S = max(2 * n_layers, 36)
        hire.hire_set_stage_events(sev.array)
        try:
            for i in range(S):
                step(i)
                sev.synchronize(len(stages))
                acc += [sev.elapsed_ms(j, j + 1) * 1e3 for j in range(len(stages))]
        finally:
            hire.hire_set_stage_events(None)
        stage_us = dict(zip(stages, (acc / S).round(3).tolist()))
        # execution span of the batch-1 scorer kernel without launch cost: per-workgroup wall clocks written by it
        if fast:
            clk = torch.zeros(2048, dtype=torch.int64, device="cuda")
            nwg = hire.hire_ffn_scorer_workgroups(N)
            hire.hire_set_scorer_clocks(clk)
            try:
                spans = []
                for i in range(S):
                    step(i)
                    torch.cuda.synchronize()
                    c = clk[:2 * nwg].view(nwg, 2)
                    spans.append(float((c[:, 1].max() - c[:, 0].min()).item()) * 0.01)
            finally:
                hire.hire_set_scorer_clocks(None)
            scorer_exec_us = round(float(np.mean(spans)), 3)

    # ---------------- kernels of the step: algorithmic bytes, durations, share of the roofline ----------------
    gather_name, w2_name = ("select_gather", "select_w2") if fast else ("gather_dot", "second_layer")
    stage_bytes = {"scorer": by.get("scorer", 0) + B * d * 2,
                   gather_name: by.get("w1_gather", by.get("w_gather", 0)) + B * d * 2,
                   w2_name: by.get("w2_gather", 0)}
    if shards > 1:      # one kernel does the whole step (plus the reduction of the partial rows)
        stage_bytes = {"shard_step": by["total"]}
    prof = profiled_kernels(args.workload)
    kernels = []
    for st in (stages if not stack else ()):
        names = _STAGE_KERNELS.get(st, ())
        rows = [r for r in prof if any(n in r[0] for n in names)]
        calls = max((r[1] for r in rows), default=0)
        # a stage may run several kernels per step: their averages, each weighted by its launches per step
        prof_us = round(sum(r[2] * r[1] / calls for r in rows), 3) if rows else None
        b = int(stage_bytes.get(st, 0))
        t = prof_us if prof_us else stage_us.get(st)
        kernels.append({"stage": st, "kernels": [r[0] for r in rows] or list(names),
                        "algorithmic_bytes": b, "rocprofv3_avg_us": prof_us, "live_event_us": stage_us.get(st),
                        "frac": round(b / (t * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if t else None,
                        "frac_from": "rocprofv3_avg_us" if prof_us else "live_event_us"})
    timed = [kq for kq in kernels if (kq["rocprofv3_avg_us"] or kq["live_event_us"])]
    roofline = None
    if timed:
        dom = max(timed, key=lambda kq: kq["rocprofv3_avg_us"] or kq["live_event_us"])      # dominant BY TIME
        dom_us = dom["rocprofv3_avg_us"] or dom["live_event_us"]
        dom_gbps = dom["algorithmic_bytes"] / (dom_us * 1e-6) / 1e9
        live = dom["live_event_us"]
        roofline = {"bound": "hbm", "kernel": dom["stage"], "kernel_names": dom["kernels"],
                    "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(dom_gbps / HBM_PEAK_GBPS, 4),
                    "traffic": profiled_traffic(args.workload, _STAGE_KERNELS.get(dom["stage"], ())),
                    "algorithmic_bytes_per_launch": dom["algorithmic_bytes"], "us_per_launch": dom_us,
                    "timing": (f"average of this kernel in profiles/{args.workload}_kernel_stats.txt (rocprofv3 "
                               "--kernel-trace --stats of this command)" if dom["rocprofv3_avg_us"] else
                               "HIP events around the kernel on its stream (eager launch, includes dispatch latency)"),
                    "live_event_us": live,
                    "frac_at_live_event_us": (round(dom["algorithmic_bytes"] / (live * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)
                                              if live else None),
                    "whole_step_frac": round(gbps / HBM_PEAK_GBPS, 4),
                    "scorer_in_kernel_clock_us": scorer_exec_us}
    elif stack:
        # the stack's dominant kernel by time in the committed summary, against the bytes one launch of it needs
        rows = sorted(prof, key=lambda r: -r[1] * r[2])
        if rows:
            name, calls, avg = rows[0]
            per_launch = {"k_gather_dot_mfma": fby["w1_gather"] + B * d * 2,
                          "k_scorer_int4_mfma": fby["scorer"] + B * d}.get(name.split("<")[0].replace("hire::", ""))
            roofline = {"bound": "hbm", "kernel": name, "achieved": (round(per_launch / (avg * 1e-6) / 1e9, 1)
                                                                       if per_launch else None),
                        "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": round(per_launch / (avg * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if per_launch else None,
                        "traffic": None, "algorithmic_bytes_per_launch": per_launch, "us_per_launch": avg,
                        "timing": f"average of this kernel in profiles/{args.workload}_kernel_stats.txt",
                        "whole_step_frac": round(gbps / HBM_PEAK_GBPS, 4)}
        else:
            roofline = {"bound": "hbm", "kernel": "whole step", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
                        "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                        "timing": "graph replay of the whole stack; no per-kernel summary committed for this workload"}

    # ---------------- the CPU oracle on the host cores, bounded sample of the same workload ----------------
    cpu = None
    recall = None
    if not args.no_cpu_baseline:
        from oracle import hire_oracle as O
        O.build()

        def timed_loop(fn, budget_s, max_n=2000):
            fn()                                # warm-up
            t1 = time.time()
            n = 0
            while n < 3 or (time.time() - t1 < budget_s and n < max_n):
                fn()
                n += 1
            return (time.time() - t1) / n * 1e6, n

        dense_fn = None
        if kind == "softmax":
            Wb = host_classifier
            ssc = O.lrq_factors(*host_factors) if scorer == "lrq" else ("int4",) + O.quantize_rows_int4(Wb)
            fn = lambda: O.softmax_step(Wb, ssc, x_bits[0], k, kp)
            dense_fn = lambda: O.softmax_k(Wb, x_bits[0], k)
        else:
            L = host_layers[0]
            if scorer == "lowrank":
                sc = ("lowrank", L["z1"], L["z2"])
            elif scorer == "lrq":
                sc = O.lrq_factors(L["z1"], L["z2"])
            else:
                sc = ("int4",) + O.quantize_rows_int4(L["w1u"])
            if m1:
                fn = lambda: O.ffn_commonpath_step(host_dense[0], host_dense[1], L["w1u"], L["w2u"], sc, x_bits[0],
                                                   k, kp, group)
            elif shards > 1:
                fn = lambda: O.ffn_shard_step(L["w1u"], L["w2u"], sc, x_bits[0], k, kp, shards)
            elif group > 1:
                fn = lambda: O.ffn_group_step(L["w1u"], L["w2u"], sc, x_bits[0], k, kp, group)
            else:
                fn = lambda: O.ffn_step(L["w1u"], L["w2u"], sc, x_bits[0], k, kp)
                dense_fn = lambda: O.dense_ffn(L["w1u"], L["w2u"], x_bits[0])
                # recall of the exact dense top-k of relu(W1 x) (layer 0, this workload's tokens)
                _, S = O.topk_ffn(L["w1u"], L["w2u"], x_bits[0], k)
                got = outs[0].topk_idx.cpu().numpy()
                recall = round(float(np.mean([len(np.intersect1d(got[b], S[b])) / k for b in range(B)])), 4)
        cpu_us, n_cpu = timed_loop(fn, 7.0 if dense_fn else 10.0)
        sample = f"{n_cpu} steps of layer 0 with this workload's tokens, weights pre-quantised"
        if stack:       # 18 FFN steps + one softmax step: one of each timed, scaled
            Wb = host_classifier
            ssc = ("int4",) + O.quantize_rows_int4(Wb)
            sm_us, n_sm = timed_loop(lambda: O.softmax_step(Wb, ssc, sm_x_bits, sk, skp), 5.0, 20)
            cpu_us = n_layers * cpu_us + sm_us
            sample = (f"{n_cpu} FFN steps of layer 0 (x {n_layers}) + {n_sm} softmax steps, weights pre-quantised")
            dense_fn = None
        cpu = {"value": round(cpu_us, 1), "unit": "us/step", "cores": O.num_threads(), "kind": "oracle", "sample": sample}
        if dense_fn is not None:
            d_us, n_d = timed_loop(dense_fn, 5.0, 200)
            cpu["dense_value"] = round(d_us, 1)
            cpu["dense_sample"] = (f"{n_d} runs of the oracle's dense layer on the same tokens (eq. (3) / eq. (1)): "
                                   "what the CPU pays without HiRE")

    result = {
        "metric": "HiRE-FFN/Softmax decode step us and achieved HBM GB/s (% of peak), 1 GPU",
        "value": round(us_per_step, 3), "unit": "us/step",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(us_per_step / 1e3, 6),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "dtype_detail": "int4 x int8 -> int32 scorer; bf16 weights/activations, fp64 accumulate "
                                         "(exact stage), fp32 accumulate (second layer)",
        "data": "synthetic",
        "config": {"workload": args.workload, "d_model": d, "rows": N, "batch": B, "k": k, "kprime": kp,
                   "scorer": scorer, "group": group, "shards": shards, "dense_units": m1, "token_correlation": rho,
                   "layers_rotated": n_layers, "steps_per_stack_step": (n_layers + 1) if stack else 1,
                   "graph_replay": graph is not None},
        "value_is": f"median of {REPS} repetitions of {K} steps", "min_us_per_step": round(min_us, 3),
        "rep_us_per_step": [round(r, 3) for r in rep_us],
        "hbm_GBps": round(gbps, 1), "hbm_frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": {kk: int(v) for kk, v in by.items()},
        "n_cand_mean": n_cand, "n_selected_union_mean": n_sel,
        "dense_equiv_us_at_peak": round(by["dense"] / (HBM_PEAK_GBPS * 1e9) * 1e6, 2),
        "recall_of_dense_topk": recall,
        "kernels": kernels,
        "stage_us_eager_nonadditive": stage_us,
        "stage_us_note": "HIP events around each stage of eager launches: every stage includes its dispatch latency, "
                         "so the stages add up to more than the step time of the graph replay",
        "streaming_selections": {"fast_route": list(hire.hire_debug_fast_fallbacks(ws)),
                                 "general_route": list(hire.hire_debug_general_fallbacks(ws))},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
