#!/usr/bin/env python3
"""Throughput of the batched dataflow-graph hot path on one MI355X.

A step is one whole forward pass over one synthetic mini-batch: host level scheduling, the
single index upload and every level kernel.  Weights, tables and inputs are resident in HBM
before the timed region; the host structure arrays (tree child indices / sequence lengths)
are consumed by the call itself, as the library's boundary defines.

Prints ONE JSON line.  `roofline` is measured live with HIP events that the library hands to
every launch on its stream (stamped with the kernel's own begin and end); `cpu_baseline` is the CPU
oracle timed on this machine's host cores on the same inputs.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0
# ceilings measured on this machine: a loop of nothing but fp32 matrix instructions on all compute
# units, and a plain streaming read by 256 workgroups
MEASURED_MFMA_TFLOPS = 155.0
MEASURED_HBM_GBS = 5800.0

# HBM bytes per launch of the dominant kernel, from the committed rocprofv3 counter summaries
# (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 KiB per dispatch, factors from a plain copy of known size; averaged over
# the launches that make up the dominant variant).  Hardware counters cannot be read from inside this process:
# the figures are those of the library as of the commit named with each and are reported with that label, not as
# live measurements; a workload without a summary reports null.
MEASURED_TRAFFIC = {  # (workload, dominant kernel) -> (bytes per launch, summary, commit the library was at)
    ("treelstm_h256_8x20", "kind=2 tile=16"): (3.43e6, "profiles/treelstm_h256_small_configs.md", "98cad87"),
    ("treelstm_h256_8x20", "kind=2 tile=6"): (3.64e6, "profiles/treelstm_h256_small_configs.md (stepwise kernel on every level)", "b76ed52"),
    ("treelstm_h256_64", "kind=2 tile=6"): (9.3e6, "profiles/treelstm_h256_small_configs.md", "e1d1bbb"),
    ("treelstm_h512_256", "kind=2 tile=64"): (80.0e6, "profiles/treelstm_h512_256_cell_level_kernel.md", "90fe6c3"),
    ("mvrnn_d64_64", "kind=14 tile=0"): (81.6e6, "profiles/mvrnn_d64_64_mvrnn_level_kernel.md", "0f6c915"),
    ("mvrnn_d64_64", "kind=3 tile=1"): (6.9e6, "profiles/mvrnn_d64_64_mvrnn_level_kernel.md (one launch per level)", "b76ed52"),
    ("lstm_h512_256", "kind=13 tile=16"): (227.9e6, "profiles/lstm_h512_256_cell_kernels.md", "2065830"),
    ("lstm_h512_256", "kind=6 tile=6"): (12.3e6, "profiles/lstm_h512_256_cell_kernels.md (one launch per step)", "138cebb"),
    ("paper_birnn_large_bs64", "kind=15 tile=16"): (24.5e6, "profiles/birnn_large_64_and_mvrnn_d128_64.md", "2065830"),
}


def bench_drnn(args, w, ctx, dev, stream):
    """Tree generation with tensor-dependent control flow (paper grid only): one step = the whole
    mini-batch, every evaluation with its launches, score copy and synchronisation.  The number
    of nodes is an outcome of the run; nothing about the trees is known beforehand."""
    import torch
    import paper_2305_10611_amd as A
    H, n_out, cap = int(w["H"]), int(w["n_out"]), int(w["cap"])
    t = {k: dev(np.asarray(w[k], np.float32)) for k in ("x0", "emb", "Wa", "ba", "Wf", "bf", "Wp", "bp", "Wo", "bo")}
    a, f, g = (torch.empty(cap, H, device="cuda") for _ in range(3))
    y = torch.empty(cap, n_out, device="cuda")

    def run(mode, ghosts):
        rc, trees, st = ctx.acrobat_drnn_forward(w, t["x0"], t, a, f, g, y, mode, ghosts, cap, stream)
        ctx.check(rc)
        return trees, st

    def timed(mode, ghosts, steps, warmup):
        for _ in range(warmup):
            run(mode, ghosts)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            trees, st = run(mode, ghosts)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, trees, st

    ms, trees, st = timed(A.TDC_FORK_JOIN, True, args.steps, args.warmup)
    n = st["n_nodes"]
    few = max(3, args.steps // 10)
    modes = {"fork_join_fibers_with_ghosts": {"ms_per_step": round(ms, 4), **st}}
    for name, mode, ghosts in (("fork_join_fibers_without_ghosts", A.TDC_FORK_JOIN, False),
                               ("one_fiber_per_instance", A.TDC_INSTANCE_FIBERS, True),
                               ("no_fibers", A.TDC_SEQUENTIAL, True)):
        m, _, s2 = timed(mode, ghosts, few if mode != A.TDC_SEQUENTIAL else 2, 1)
        modes[name] = {"ms_per_step": round(m, 4), **s2}
    th = []
    for _ in range(10):
        h0 = time.perf_counter()
        A.acrobat_drnn_schedule(w, A.TDC_FORK_JOIN, True, cap)
        th.append(time.perf_counter() - h0)
    ctx.acrobat_set_profiling(True)
    run(A.TDC_FORK_JOIN, True)
    recs = ctx.acrobat_last_profile()
    ctx.acrobat_set_profiling(False)
    t_device_ms = sum(r[3] for r in recs)
    flops = n * (3 * 2.0 * 2 * H * H + 2.0 * H * n_out)
    if args.verbose:
        for r in recs:
            print(f"batch {r[1]:>3} n {r[2]:>5} tile {r[4]:>3} {r[3] * 1e3:>8.2f} us", file=sys.stderr)
    cpu_baseline, err = None, None
    if not args.no_cpu_baseline:
        import oracle
        from workloads.generators import match_trees
        c0 = time.perf_counter()
        ref = oracle.drnn(w)
        c1 = time.perf_counter()
        cpu_baseline = {"value": round(n / (c1 - c0), 1), "unit": "nodes/s", "cores": 1, "kind": "oracle",
                        "sample": f"the whole {w['name']} batch ({n} nodes), one thread"}
        at = match_trees(trees, ref)
        err = max(float(np.abs(v[:n].cpu().numpy().astype(np.float64) - ref[k][at]).max())
                  for k, v in (("a", a), ("f", f), ("g", g), ("y", y)))
    line = {"metric": "node evals/sec", "value": round(n / (ms * 1e-3), 1), "unit": "nodes/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": w["name"], "index": -1, "nodes": n, "seed": int(w["seed"])},
            "roofline": None, "cpu_baseline": cpu_baseline, "tensor_dependent_control_flow": modes,
            "breakdown": {"t_host_program_ms": round(float(np.median(th)) * 1e3, 4), "t_device_ms": round(t_device_ms, 4),
                          "launches": len(recs), "evaluations": st["n_rounds"], "algorithmic_gflop": round(flops / 1e9, 3),
                          "max_abs_err_vs_oracle": err}}
    print(json.dumps(line), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 0..4 (2 = headline)")
    ap.add_argument("--paper-grid", default=None, metavar="MODEL:SIZE:BATCH",
                    help="instead of --config: a mini-batch shaped like the paper's grid, e.g. treelstm:small:64")
    ap.add_argument("--instances", type=int, default=None,
                    help="with --config: the same recipe with this many trees / sequences (scaling runs)")
    ap.add_argument("--profile-steps", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--verbose", action="store_true", help="per-level table on stderr")
    ap.add_argument("--two-streams", dest="overlap_streams", action="store_true", default=None,
                    help="also measure, for information, the throughput when consecutive mini-batches alternate "
                         "between two streams (reported under \"two_stream_throughput\"); the default for TreeLSTM "
                         "workloads, whose kernels never wait for each other - the single launches of the recurrences "
                         "and of MV-RNN batches want the chip to themselves (include/acrobat.h, acrobat_set_persistent)")
    ap.add_argument("--no-two-streams", dest="overlap_streams", action="store_false",
                    help="skip the two-stream measurement")
    ap.add_argument("--ablation", action="store_true",
                    help="TreeLSTM only: also time the forward pass with gather fusion switched off (explicit "
                         "gather launches), reported under \"ablation\"")
    ap.add_argument("--generic-runtime", action="store_true",
                    help="TreeLSTM only: also time the same batch through the generic dataflow-graph runtime (the "
                         "unbatched program calls invoke() per node with inline depths), reported under "
                         "\"generic_runtime\"")
    ap.add_argument("--graph-replay", action="store_true",
                    help="also time the forward call replayed from a captured HIP graph (index upload + every launch), "
                         "and what capturing and instantiating it costs; reported under \"graph_replay\"")
    ap.add_argument("--persistent", choices=("auto", "off"), default="auto",
                    help="LSTM, BiRNN and MV-RNN: off = one launch per time step / level instead of one persistent launch")
    ap.add_argument("--tuning", default=None, metavar="TILE,KSPLIT",
                    help="force one kernel variant for every cell level (acrobat_set_tuning), e.g. 64,1 or 65,1")
    ap.add_argument("--sync-probe", action="store_true",
                    help="only run the library's probe of barriers among workgroups inside one kernel (three styles, "
                         "groups on one XCD or spread) and print one JSON line per case")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="only run one plain device-to-device copy of this many MiB (a kernel of known traffic "
                         "for scaling hardware-counter readings) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (instances are independent, so more GPUs would "
              "simply take disjoint sets of trees; no collective is part of the path). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2305_10611_amd as A
    from workloads import make_config

    torch.cuda.set_device(0)
    if args.copy_calibration_mib > 0:
        n = args.copy_calibration_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_mib": args.copy_calibration_mib, "launches": 3}))
        return
    if args.sync_probe:
        ctx = A.Context(0)
        names = ("store+wg_barrier", "announce", "wait", "acquire+wg_barrier", "load")
        for groups, gsize in ((8, 32), (8, 8), (1, 256), (1, 32)):
            for same_xcd in (1, 0):
                for style in (0, 1, 2, 3):
                    if style == 2 and gsize > 32:
                        continue
                    rounds = 200 if style == 3 else 2000  # (style 3 keeps every round's payload)
                    for store, load in ((0, 0), (512, 16384)):
                        load = min(load, gsize * store // 1024 * 1024)
                        rc, us, ph = ctx.acrobat_sync_probe(groups, gsize, rounds, same_xcd, style, 1, store, load)
                        ctx.check(rc)
                        print(json.dumps({"sync_probe": {"groups": groups, "group_size": gsize, "same_xcd": same_xcd,
                                                         "style": ("counter+fences", "counter", "flag lines", "counter, write-once payload read with plain loads")[style],
                                                         "store_bytes": 4 * store, "load_bytes": 4 * load,
                                                         "us_per_round": round(us, 2),
                                                         "stale_elements": int(ph[5]),
                                                         "phase_us": {k: round(v, 2) for k, v in zip(names, ph)}}}), flush=True)
        ctx.close()
        return
    if args.paper_grid:
        from workloads.generators import paper_grid_workload
        model, size, batch = args.paper_grid.split(":")
        w = paper_grid_workload(model, size, int(batch))
        args.config = -1
    else:
        w = make_config(args.config, n_instances=args.instances)
    kind = w["kind"]
    if args.overlap_streams is None:
        args.overlap_streams = kind == "treelstm"
    ctx = A.Context(0)
    if args.persistent == "off":
        ctx.acrobat_set_persistent(False)
    if args.tuning:
        tile, ks = (int(v) for v in args.tuning.split(","))
        ctx.check(ctx.acrobat_set_tuning(tile, ks, 0))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    if kind == "drnn":
        bench_drnn(args, w, ctx, dev, stream)
        ctx.close()
        return
    n_nodes = int(w["n_nodes"])

    if kind == "treelstm":
        H, D, V = int(w["H"]), int(w["D"]), int(w["V"])
        t = {k: dev(w[k]) for k in ("emb", "W_leaf", "b_leaf", "U", "b")}
        new_out = lambda: [torch.empty(n_nodes, H, device="cuda"), torch.empty(n_nodes, H, device="cuda")]
        make_step = lambda c, o, st: (lambda: c.check(c.acrobat_treelstm_forward(
            w, H, D, V, t["emb"], t["W_leaf"], t["b_leaf"], t["U"], t["b"], o[0], o[1], st)))
        sched = A.binding.prepared_schedule_trees(w, V)  # the library call alone, arguments marshalled once
        n_leaf = int((w["left"] < 0).sum())
        flops_per = {A.binding.K_TREE_LEAF: 2.0 * D * 3 * H, A.binding.K_TREE_INTERNAL: 2.0 * 2 * H * 5 * H}
        # strict-minimum bytes per node (states + indices), weights extra per launch
        bytes_per = {A.binding.K_TREE_LEAF: 4.0 * D + 4 + 8.0 * H, A.binding.K_TREE_INTERNAL: 24.0 * H + 12}
        weight_bytes = {A.binding.K_TREE_LEAF: 12.0 * H * D, A.binding.K_TREE_INTERNAL: 40.0 * H * H}
        dominant = A.binding.K_TREE_INTERNAL
        total_flops = n_leaf * flops_per[A.binding.K_TREE_LEAF] + (n_nodes - n_leaf) * flops_per[dominant]
        dtype, bound = "f32", "mfma"
    elif kind == "mvrnn":
        d, V = int(w["d"]), int(w["V"])
        t = {k: dev(w[k]) for k in ("vec_tab", "mat_tab", "W", "WM")}
        new_out = lambda: [torch.empty(n_nodes, d, device="cuda"), torch.empty(n_nodes, d, d, device="cuda")]
        make_step = lambda c, o, st: (lambda: c.check(c.acrobat_mvrnn_forward(
            w, d, V, t["vec_tab"], t["mat_tab"], t["W"], t["WM"], o[0], o[1], 0, st)))
        sched = A.binding.prepared_schedule_trees(w, V)
        n_int = int((w["left"] >= 0).sum())
        # one launch per level (K_MVRNN_LEVEL) or one launch for all internal levels (K_MVRNN_PERSISTENT): same work per node
        node_flops, node_bytes = 4.0 * d * d + 4.0 * d * d + 4.0 * d ** 3, 12.0 * (d * d + d) + 12
        flops_per = {A.binding.K_MVRNN_LEVEL: node_flops, A.binding.K_MVRNN_PERSISTENT: node_flops}
        bytes_per = {A.binding.K_MVRNN_LEVEL: node_bytes, A.binding.K_MVRNN_PERSISTENT: node_bytes}
        weight_bytes = {A.binding.K_MVRNN_LEVEL: 16.0 * d * d, A.binding.K_MVRNN_PERSISTENT: 16.0 * d * d}
        dominant = A.binding.K_MVRNN_LEVEL
        total_flops = n_int * flops_per[dominant]
        dtype, bound = "f32", "hbm"
    elif kind == "birnn":
        H, D, n_out = int(w["H"]), int(w["D"]), int(w["n_out"])
        R = n_nodes
        n_nodes = 3 * R  # dataflow-graph nodes per token: forward cell, backward cell, output operator
        names = ("x", "fWx", "fWh", "fb", "finit", "bWx", "bWh", "bb", "binit", "C", "cb")
        t = {k: dev(np.asarray(w[k], np.float32)) for k in names}
        new_out = lambda: [torch.empty(R, H, device="cuda"), torch.empty(R, H, device="cuda"),
                           torch.empty(R, n_out, device="cuda")]
        make_step = lambda c, o, st: (lambda: c.check(c.acrobat_birnn_forward(
            w["len"], H, D, n_out, t["x"], (t["fWx"], t["fWh"], t["fb"], t["finit"]),
            (t["bWx"], t["bWh"], t["bb"], t["binit"]), t["C"], t["cb"], o[0], o[1], o[2], st)))
        sched = lambda: A.acrobat_schedule_birnn(w["len"])
        B = A.binding
        # the recurrences are one launch per step (K_RNN_STEP) or one launch for all steps of both directions
        # (K_RNN_PERSISTENT): same work per (token, direction); the persistent launch reads the weights once
        flops_per = {B.K_RNN_INPUT: 2.0 * D * H, B.K_RNN_STEP: 2.0 * H * H, B.K_RNN_PERSISTENT: 2.0 * H * H,
                     B.K_RNN_OUTPUT: 4.0 * H * n_out}
        bytes_per = {B.K_RNN_INPUT: 4.0 * D + 4.0 * H, B.K_RNN_STEP: 12.0 * H + 8, B.K_RNN_PERSISTENT: 12.0 * H,
                     B.K_RNN_OUTPUT: 8.0 * H + 4.0 * n_out}
        weight_bytes = {B.K_RNN_INPUT: 4.0 * H * D, B.K_RNN_STEP: 4.0 * H * H, B.K_RNN_PERSISTENT: 8.0 * H * H,
                        B.K_RNN_OUTPUT: 8.0 * H * n_out}
        dominant = B.K_RNN_STEP
        total_flops = R * (2 * flops_per[B.K_RNN_INPUT] + 2 * flops_per[B.K_RNN_STEP] + flops_per[B.K_RNN_OUTPUT])
        dtype, bound = "f32", "mfma"
    else:
        H, D = int(w["H"]), int(w["D"])
        t = {k: dev(w[k]) for k in ("x", "Wx", "Wh", "b")}
        new_out = lambda: [torch.empty(n_nodes, H, device="cuda"), torch.empty(n_nodes, H, device="cuda")]
        make_step = lambda c, o, st: (lambda: c.check(c.acrobat_varlen_lstm_forward(
            w["len"], H, D, t["x"], t["Wx"], t["Wh"], t["b"], o[0], o[1], st)))
        sched = lambda: A.acrobat_schedule_seqs(w["len"])
        # the recurrence is either one launch per step (K_LSTM_STEP) or one launch for all steps (K_LSTM_PERSISTENT):
        # same work per (sequence, step); the persistent launch reads the weights once
        step_flops, step_bytes = 2.0 * H * 4 * H, 16.0 * H + 8.0 * H + 8.0 * H + 8
        flops_per = {A.binding.K_LSTM_INPUT: 2.0 * D * 4 * H, A.binding.K_LSTM_STEP: step_flops,
                     A.binding.K_LSTM_PERSISTENT: step_flops}
        bytes_per = {A.binding.K_LSTM_INPUT: 4.0 * D + 16.0 * H, A.binding.K_LSTM_STEP: step_bytes,
                     A.binding.K_LSTM_PERSISTENT: step_bytes}
        weight_bytes = {A.binding.K_LSTM_INPUT: 16.0 * H * D, A.binding.K_LSTM_STEP: 16.0 * H * H,
                        A.binding.K_LSTM_PERSISTENT: 16.0 * H * H}
        dominant = A.binding.K_LSTM_STEP
        total_flops = n_nodes * (flops_per[A.binding.K_LSTM_INPUT] + flops_per[A.binding.K_LSTM_STEP])
        dtype, bound = "f32", "mfma"

    out = new_out()
    step = make_step(ctx, out, stream)

    # ---- timed region: W warm-up steps, then exactly K steps between two synchronisations
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = n_nodes / (ms_per_step * 1e-3)

    # ---- information only: the same K steps alternating between two streams (two contexts, two
    # output buffers), so that the latency-bound small levels of one mini-batch overlap the
    # compute-bound wide levels of the next.  `value` above stays the single-stream figure.
    overlap = None
    if args.overlap_streams:
        ctx2 = A.Context(0)
        s2 = torch.cuda.Stream()
        step2 = make_step(ctx2, new_out(), s2.cuda_stream)
        s2.wait_stream(torch.cuda.current_stream())
        for i in range(args.warmup):
            (step if i % 2 == 0 else step2)()
        torch.cuda.synchronize()
        o0 = time.perf_counter()
        for i in range(args.steps):
            (step if i % 2 == 0 else step2)()
        torch.cuda.synchronize()
        o1 = time.perf_counter()
        oms = (o1 - o0) * 1e3 / args.steps
        overlap = {"streams": 2, "ms_per_step": round(oms, 4), "value": round(n_nodes / (oms * 1e-3), 1)}
        ctx2.close()

    # ---- information only: the same forward call replayed from a captured graph
    graph_replay = None
    if args.graph_replay:
        gs = torch.cuda.Stream()
        gstep = make_step(ctx, out, gs.cuda_stream)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=gs, capture_error_mode="relaxed"):
            gstep()
        torch.cuda.synchronize()
        c1 = time.perf_counter()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        r0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        r1 = time.perf_counter()
        graph_replay = {"replay_ms_per_step": round((r1 - r0) * 1e3 / args.steps, 4), "eager_ms_per_step": round(ms_per_step, 4),
                        "capture_and_instantiate_ms": round((c1 - c0) * 1e3, 3)}
        del graph
        step()  # the outputs checked further down come from the eager path

    # ---- information only: gather fusion off (explicit gather launch before every level)
    ablation = None
    if args.ablation and kind == "treelstm":
        ctx.acrobat_set_gather_fusion(False)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        a0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        a1 = time.perf_counter()
        ctx.acrobat_set_gather_fusion(True)
        ams = (a1 - a0) * 1e3 / args.steps
        ablation = {"unfused_gather_ms_per_step": round(ams, 4), "fused_over_unfused_speedup": round(ams / ms_per_step, 3)}
        step()  # the outputs checked further down come from the product path

    # ---- information only: the same batch through the generic runtime (DFG construction by the unbatched
    # program + bucket scheduling + one launch per bucket), as in the activity breakdown of the paper's table 6
    generic = None
    if args.generic_runtime and kind == "treelstm":
        B = A.binding
        g = A.Dfg(ctx)
        gh, gc = new_out()
        rc, op_leaf = g.acrobat_dfg_register_op(B.EPI_TREE_LEAF, H, nseg=1, kseg=D, src0=t["emb"], ld0=D, W=t["W_leaf"],
                                                ldw=D, bias=t["b_leaf"], h=gh, c=gc, src0_rows=V, out_rows=n_nodes)
        ctx.check(rc)
        rc, op_int = g.acrobat_dfg_register_op(B.EPI_TREE_INTERNAL, H, nseg=2, kseg=H, src0=gh, ld0=H, src1=gh, ld1=H,
                                               W=t["U"], ldw=2 * H, bias=t["b"], h=gh, c=gc, cprev_src=gc,
                                               src0_rows=n_nodes, src1_rows=n_nodes, out_rows=n_nodes)
        ctx.check(rc)

        def gstep():
            g.acrobat_dfg_clear()
            ctx.check(g.acrobat_dfg_build_treelstm(w, V, op_leaf, op_int))
            ctx.check(g.acrobat_dfg_run(stream))
        for _ in range(args.warmup):
            gstep()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            gstep()
        torch.cuda.synchronize()
        g1 = time.perf_counter()
        tb = []
        for _ in range(20):
            g.acrobat_dfg_clear()
            b0 = time.perf_counter()
            g.acrobat_dfg_build_treelstm(w, V, op_leaf, op_int)
            b1 = time.perf_counter()
            g.acrobat_dfg_schedule()
            b2 = time.perf_counter()
            tb.append((b1 - b0, b2 - b1))
        gms = (g1 - g0) * 1e3 / args.steps
        same = bool(torch.equal(gh, out[0]) and torch.equal(gc, out[1]))
        generic = {"ms_per_step": round(gms, 4), "t_dfg_construction_ms": round(float(np.median([x[0] for x in tb])) * 1e3, 4),
                   "t_bucket_schedule_ms": round(float(np.median([x[1] for x in tb])) * 1e3, 4),
                   "bit_identical_to_specialised_path": same}
        g.close()

    # ---- host scheduler alone
    ts = []
    for _ in range(20):
        a0 = time.perf_counter()
        sched()
        ts.append(time.perf_counter() - a0)
    t_schedule_ms = float(np.median(ts)) * 1e3

    # ---- per-launch device times (HIP events on the launch stream, recorded by the library)
    ctx.acrobat_set_profiling(True)
    recs = []
    for _ in range(max(1, args.profile_steps)):
        step()
        recs.append(ctx.acrobat_last_profile())
    ctx.acrobat_set_profiling(False)
    n_rep = len(recs)
    per_launch = []  # (kind, level, n, tile, mean ms, ksplit)
    for i, r in enumerate(recs[0]):
        per_launch.append((r[0], r[1], r[2], r[4], float(np.mean([rr[i][3] for rr in recs])), r[5]))
    t_device_ms = sum(p[4] for p in per_launch)
    for persistent_kind in (A.binding.K_LSTM_PERSISTENT, A.binding.K_MVRNN_PERSISTENT, A.binding.K_RNN_PERSISTENT):
        if any(p[0] == persistent_kind for p in per_launch):
            dominant = persistent_kind
    K_REDUCE = A.binding.K_SPLITK_REDUCE
    t_reduce_ms = sum(p[4] for p in per_launch if p[0] == K_REDUCE)
    # dominant kernel = the variant of the dominant kind that accounts for most device time
    by_tile = {}
    for k, lv, n, tile, ms, _ in per_launch:
        if k == dominant:
            e = by_tile.setdefault(tile, [0, 0, 0.0])
            e[0] += 1
            e[1] += n
            e[2] += ms
    dom_tile = max(by_tile, key=lambda q: by_tile[q][2])
    launches, units, ms_sum = by_tile[dom_tile]
    if bound == "mfma":
        achieved = units * flops_per[dominant] / (ms_sum * 1e-3) / 1e12
        peak, unit = PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"
    else:
        achieved = (units * bytes_per[dominant] + launches * weight_bytes[dominant]) / (ms_sum * 1e-3) / 1e9
        peak, unit = PEAK_HBM_GBS, "GB/s"
    kname = f"kind={dominant} tile={dom_tile}"
    traffic, traffic_src, traffic_commit = MEASURED_TRAFFIC.get((w["name"], kname), (None, None, None))
    roofline = {"bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic, "traffic_unit": "bytes/launch",
                "traffic_source": traffic_src, "traffic_measured_at_commit": traffic_commit,
                "algorithmic_bytes_per_launch": round((units * bytes_per[dominant] + launches * weight_bytes[dominant]) / launches),
                "kernel": kname, "launches_per_step": launches,
                "units_per_step": units, "avg_launch_us": round(ms_sum / launches * 1e3, 2)}

    # ---- aggregate roofline fraction: every launch takes at least max(flops / P, bytes / B); their sum over the
    # device time says how close the whole level sequence is to the chip's two roofs
    def floor_ms(k, n, peak_tf, peak_gbs):
        return max(n * flops_per[k] / (peak_tf * 1e9), (n * bytes_per[k] + weight_bytes[k]) / (peak_gbs * 1e6))
    agg = {"datasheet": 0.0, "measured_ceilings": 0.0}
    for k, lv, n, tile, ms, ks in per_launch:
        if k in flops_per:
            agg["datasheet"] += floor_ms(k, n, PEAK_FP32_MFMA_TFLOPS, PEAK_HBM_GBS)
            agg["measured_ceilings"] += floor_ms(k, n, MEASURED_MFMA_TFLOPS, MEASURED_HBM_GBS)
    agg = {key: round(v / t_device_ms, 4) for key, v in agg.items()}
    # the dominant kernel is only part of the step: the same fraction for the whole step (every launch, the gaps
    # between them, host scheduling and upload), so that the headline figure is not mistaken for it
    if bound == "mfma":
        whole = total_flops / (ms_per_step * 1e-3) / 1e12
    else:
        whole = sum(n * bytes_per[k] + weight_bytes[k] for k, lv, n, tile, ms, ks in per_launch if k in bytes_per) / (ms_per_step * 1e-3) / 1e9
    roofline["whole_step"] = {"achieved": round(whole, 3), "frac": round(whole / peak, 4), "unit": unit,
                              "sum_of_per_launch_floors_over_device_time": agg["datasheet"]}

    if args.verbose:
        print(f"{'kind':>4} {'lvl':>4} {'n':>6} {'tile':>4} {'ks':>3} {'us':>9} {'TFLOP/s':>8} {'%MFMA':>6} {'GB/s':>8} {'%HBM':>6} {'bound':>5}",
              file=sys.stderr)
        for k, lv, n, tile, ms, ks in per_launch:
            if k == K_REDUCE or k not in flops_per:
                print(f"{'red' if k == K_REDUCE else k:>4} {lv:>4} {n:>6} {tile:>4} {ks:>3} {ms * 1e3:>9.2f}", file=sys.stderr)
                continue
            fl = n * flops_per[k]
            by = n * bytes_per[k] + weight_bytes[k]
            tf, gbs = fl / ms / 1e9, by / ms / 1e6
            which = "mfma" if fl / (PEAK_FP32_MFMA_TFLOPS * 1e9) >= by / (PEAK_HBM_GBS * 1e6) else "hbm"
            print(f"{k:>4} {lv:>4} {n:>6} {tile:>4} {ks:>3} {ms * 1e3:>9.2f} {tf:>8.2f} {100 * tf / PEAK_FP32_MFMA_TFLOPS:>6.1f} "
                  f"{gbs:>8.1f} {100 * gbs / PEAK_HBM_GBS:>6.1f} {which:>5}", file=sys.stderr)
        print(f"device sum {t_device_ms:.3f} ms, end-to-end {ms_per_step:.3f} ms/step, schedule {t_schedule_ms:.3f} ms",
              file=sys.stderr)

    # ---- the CPU oracle on this machine's host cores, same inputs, run once
    cpu_baseline = None
    err = None
    if not args.no_cpu_baseline:
        import oracle
        nt = oracle.default_threads()
        c0 = time.perf_counter()
        if kind == "treelstm":
            ref = oracle.treelstm(w, nthreads=nt)
        elif kind == "mvrnn":
            ref = oracle.mvrnn(w, nthreads=nt)
        elif kind == "birnn":
            ref = oracle.birnn(w, nthreads=nt)
        else:
            ref = oracle.varlen_lstm(w, nthreads=nt)
        c1 = time.perf_counter()
        cpu_baseline = {"value": round(n_nodes / (c1 - c0), 1), "unit": "nodes/s", "cores": nt, "kind": "oracle",
                        "sample": f"the whole {w['name']} batch ({n_nodes} nodes), evaluated once with whole "
                                  f"instances fanned out over {nt} host threads"}
        # the oracle as written, one thread, on a bounded sample: the first instances of the same batch
        if kind == "treelstm":
            k1 = min(int(w["n_trees"]), 16)
            n1 = int(w["tree_off"][k1])
            w1 = dict(w, n_trees=k1, tree_off=w["tree_off"][: k1 + 1], left=w["left"][:n1], right=w["right"][:n1],
                      token=w["token"][:n1])
            s0 = time.perf_counter()
            oracle.treelstm(w1, nthreads=1)
            s1 = time.perf_counter()
            cpu_baseline["single_thread"] = {"value": round(n1 / (s1 - s0), 1), "unit": "nodes/s", "cores": 1,
                                             "sample": f"the first {k1} trees ({n1} nodes) of the batch"}
        torch.cuda.synchronize()
        got = [o.cpu().numpy().astype(np.float64) for o in out]
        mask = slice(None) if kind != "mvrnn" else (w["left"] >= 0)
        err = max(float(np.abs(g[mask] - r[mask]).max()) for g, r in zip(got, ref))

    line = {
        "metric": "node evals/sec", "value": round(value, 1), "unit": "nodes/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": w["name"], "index": args.config, "nodes": n_nodes, "seed": int(w["seed"])},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "two_stream_throughput": overlap, "ablation": ablation, "generic_runtime": generic,
        "graph_replay": graph_replay,
        "breakdown": {"t_schedule_ms": round(t_schedule_ms, 4), "t_device_ms": round(t_device_ms, 4),
                      "t_splitk_reduce_ms": round(t_reduce_ms, 4),
                      "launches": len(per_launch), "algorithmic_gflop": round(total_flops / 1e9, 3),
                      "nodes_per_s_device": round(n_nodes / (t_device_ms * 1e-3), 1),
                      "aggregate_roofline_frac": agg,
                      "device_tflops": round(total_flops / (t_device_ms * 1e-3) / 1e12, 3),
                      "max_abs_err_vs_oracle": err},
    }
    print(json.dumps(line), flush=True)
    ctx.close()


if __name__ == "__main__":
    main()
