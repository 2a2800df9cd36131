#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: schedule + batched forward + batched backward of one
minibatch graph per step (the BiLSTM tagger workload: 64 sentences), graph arrays already
resident in HBM when the timed region starts.

Prints ONE JSON line: training instances/s (autobatched, depth-based), the roofline figures of
the dominant kernel from HIP events recorded by the library on its stream, the same graphs with
batching off (one launch per node), and the CPU oracle timed on a bounded sample.
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

from paper_1705_07860_amd import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_FP32_PEAK_TFLOPS = 157.3
R_IDX = 4  # bytes of one gathered-row index


def algorithmic_cost(g, params, batch_off, node_ids):
    """Bytes and flops the method itself must move / do for one forward+backward of this
    schedule (per-batch formulas: operands read once, results written once, one 4-byte row index
    per gathered operand row; a shared matrix is read once per batch; dW is read-modify-written
    once per parameter because its reduction is deferred over all uses).  bwd_bytes covers the
    backward step kernel (gradient pull and dX), param_bytes the deferred dW / db / dE kernels."""
    heads = node_ids[batch_off[:-1]]
    B = np.diff(batch_off).astype(np.float64)
    op = g.op[heads].astype(np.int64)
    d = g.out_dim[heads].astype(np.float64)
    ar = (g.in_off[heads + 1] - g.in_off[heads]).astype(np.float64)
    first_in = g.in_idx[np.minimum(g.in_off[heads], max(len(g.in_idx) - 1, 0))]
    k = np.where(ar > 0, g.out_dim[first_in], 0).astype(np.float64)
    fb = np.zeros(len(heads))
    bb = np.zeros(len(heads))
    fl_f = np.zeros(len(heads))
    fl_b = np.zeros(len(heads))
    un = (op == wl.OP_TANH) | (op == wl.OP_SIGMOID)
    fb[un] = (8 * d + R_IDX)[un] * B[un]
    bb[un] = (12 * d * B)[un]
    m = op == wl.OP_ADD
    fb[m] = ((4 * d * (ar + 1) + ar * R_IDX) * B)[m]
    bb[m] = (4 * d * (ar + 1) * B)[m]
    m = op == wl.OP_CMULT
    fb[m] = ((12 * d + 2 * R_IDX) * B)[m]
    bb[m] = (20 * d * B)[m]
    m = (op == wl.OP_SLICE) | (op == wl.OP_CONCAT)
    fb[m] = ((8 * d + ar * R_IDX) * B)[m]
    bb[m] = (8 * d * B)[m]
    m = (op == wl.OP_LOOKUP) | (op == wl.OP_INPUT)
    fb[m] = (8 * d * B)[m]
    bb[op == wl.OP_LOOKUP] = (16 * d * B)[op == wl.OP_LOOKUP]
    m = (op == wl.OP_PICK_NLS) | (op == wl.OP_SQNORM)
    fb[m] = ((4 * k + 4 + R_IDX) * B)[m]
    bb[m] = (8 * k * B)[m]
    m = op == wl.OP_MATVEC
    fb[m] = (4 * (d * k + k * B + d * B) + R_IDX * B)[m]
    bb[m] = (4 * (d * k + d * B + k * B))[m]                 # dX = G W in the backward step kernel
    pg = float((4 * (d * B + k * B))[m].sum())               # dW = G^T X in the deferred parameter kernels
    fl_f[m] = (2 * d * k * B)[m]
    fl_b[m] = (4 * d * k * B)[m]
    used_w = np.unique(g.param[g.op == wl.OP_MATVEC])
    dW_rmw = float(sum(8 * params.mats[int(p)].size for p in used_w))
    return dict(fwd_bytes=float(fb.sum()), bwd_bytes=float(bb.sum()), param_bytes=pg + dW_rmw,
                fwd_flops=float(fl_f.sum()), bwd_flops=float(fl_b.sum()))


# the paper's own figures for the nearest workload (Tesla K80, DyNet; throughput there includes graph
# construction and the update): context, never a target
PAPER_CONTEXT = {
    "tagger": "Table 1, BiLSTM, ByDepth on a Tesla K80: 337 sentences/s (other hardware and dimensions)",
    "tagger_char": "Table 1, BiLSTM with character model, ByDepth on a Tesla K80: 183 sentences/s (other hardware and dimensions)",
    "tree": "Table 1, TreeLSTM, ByDepth on a Tesla K80: 672 trees/s (other hardware and dimensions)",
    "parser": "Table 1, transition parser, ByDepth on a Tesla K80: 89.5 sentences/s (other hardware and dimensions)",
    "sync_tagger": "Section 4.1, same network sizes, Tesla K80: 18.3 sentences/s unbatched, 198 with agenda-based batching "
                   "(their figure includes graph construction and the update)",
    "rnn": None,
}


def stored_traffic(args, kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary (two rocprofv3 --pmc
    runs, FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size).  Counters cannot be
    read inside a timing run, so the figure is the stored one and only applies to the default
    launch configuration of the workload it was taken on; otherwise null."""
    if args.launch != "stream" or args.no_fusion or args.placement != "late" or args.mode != "depth" or args.epilogue:
        return None
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"{args.workload}_bydepth_hbm_traffic.json")
    try:
        with open(path) as f:
            k = json.load(f)["kernels"][kernel]
        return k["fetch_bytes_per_launch"] + k["write_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="tagger", choices=list(wl.CONFIGS))
    ap.add_argument("--pool", type=int, default=6, help="distinct seeded minibatches cycled through")
    ap.add_argument("--instances", type=int, default=None,
                    help="instances per minibatch (default: the configuration's own count; other values are sweep "
                         "points, not the headline workload)")
    ap.add_argument("--launch", default="stream", choices=["stream", "graph"])
    ap.add_argument("--mode", default="depth", choices=["depth", "agenda", "manual"],
                    help="batching strategy of Section 3.2: depth-based (default, the configuration the stored "
                         "profiles cover) or agenda-based; manual = Section 2's batching by hand, one batch per "
                         "statement of a program written over a batch of sentences (--workload sync_tagger only)")
    ap.add_argument("--lookahead", type=int, default=0,
                    help="minibatches scheduled ahead of the one that executes, each on a schedule stream of its own "
                         "(default: 1 for depth-based batching, 2 for agenda-based batching, whose scheduling takes longer "
                         "than its execution)")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="schedule and execute each step back to back on one stream (no overlap between steps)")
    ap.add_argument("--no-fusion", action="store_true", help="one launch per depth level")
    ap.add_argument("--epilogue", action="store_true",
                    help="fusion level 3: component-wise chains are evaluated behind the tiles of the matrix product they "
                         "read (half the forward launches of an LSTM workload, but slower launches: not the default)")
    ap.add_argument("--placement", default="late", choices=["early", "late"],
                    help="fused plans launch a batch as early as its operands / as late as its consumers allow")
    ap.add_argument("--update", action="store_true",
                    help="close every step with the gradient-descent update of Section 2 (lr 0) instead of only "
                         "zeroing the gradients; the headline metric is forward + backward, so this is off by default")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-nobatch", action="store_true", help="skip the unbatched GPU leg")
    ap.add_argument("--cpu-samples", type=int, default=12,
                    help="minibatches the CPU oracle leg runs (cycling through the pool): about 10-30 s of CPU work")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run one plain device copy of this many MiB (a kernel of known traffic, used to "
                         "scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (the path has no multi-GPU part)",
              file=sys.stderr)
        sys.exit(2)

    if args.mode == "manual" and args.workload != "sync_tagger":
        print("bench.py: --mode manual needs sentences of equal structure (--workload sync_tagger)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1705_07860_amd import binding as ob
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    cfg = wl.CONFIGS[args.workload]
    params = cfg["params"]()
    pool = max(1, min(args.pool, args.steps + args.warmup))
    graphs = [cfg["batch"](params, j, n=args.instances) for j in range(pool)]
    # device arena per context: 1 GiB holds the configurations as listed; larger sweep points get more
    arena_bytes = (1 << 30) * max(1, -(-graphs[0].n_instances // 64))
    launch = ob.OB_LAUNCH_GRAPH if args.launch == "graph" else ob.OB_LAUNCH_STREAM

    # One context per pooled minibatch, all sharing one parameter set (forks of the first) and one
    # execution stream, so the executions of consecutive steps are serial on the GPU as a training
    # loop with a parameter update in between would be.  Graph arrays are uploaded before the timed
    # region.  With pipelining (default) scheduling runs on a second stream: while step i executes,
    # the GPU already schedules step i+1 (scheduling reads only the graph, never the parameters).
    pipeline = not args.no_pipeline
    stream = torch.cuda.Stream()
    lookahead = args.lookahead if args.lookahead > 0 else (2 if args.mode == "agenda" else 1)
    lookahead = max(1, min(lookahead, max(1, pool - 2)))
    sched_streams = [torch.cuda.Stream() for _ in range(lookahead)] if pipeline else [None]
    ctxs = []
    t_up = []
    for j, g in enumerate(graphs):
        if j == 0:
            c = ob.Context(arena_bytes=arena_bytes, stream=stream, launch=launch, sched_stream=sched_streams[0],
                           mode={"agenda": ob.OB_BYAGENDA, "manual": ob.OB_MANUAL}.get(args.mode, ob.OB_BYDEPTH))
            c.set_fusion(0 if args.no_fusion else (1 if args.placement == "early" else (3 if args.epilogue else 2)))
            c.params_create(params)
            c.param_grad_zero()
        else:
            c = ctxs[0].fork(arena_bytes=arena_bytes, stream=stream, sched_stream=sched_streams[j % len(sched_streams)])
        t0 = time.perf_counter()
        c.add_bulk(g)
        if args.mode == "manual":
            c.set_manual_batches(wl.sync_tagger_manual_labels(g))
        c.upload()
        c.sync()
        torch.cuda.synchronize()
        t_up.append(time.perf_counter() - t0)
        ctxs.append(c)

    def sched(i):
        c = ctxs[i % pool]
        c.reset()
        if pipeline:
            c.schedule_async(graphs[i % pool].root)   # queued; forward() of that step collects it
        else:
            c.schedule(graphs[i % pool].root)

    def execute(i):
        c = ctxs[i % pool]
        g = graphs[i % pool]
        if not args.update:
            c.param_grad_zero()
        c.forward(g.root)
        c.backward(g.root)
        if args.update:
            c.sgd_step(0.0, zero_grad=True)    # lr 0 keeps the pooled minibatches' numbers stationary

    def run(first, count, marks=None):
        if pipeline:
            for a in range(min(lookahead, count)):
                sched(first + a)
            for i in range(first, first + count):
                if i + lookahead < first + count:
                    sched(i + lookahead)
                execute(i)
                if marks is not None:
                    marks.append(torch.cuda.Event(enable_timing=True))
                    marks[-1].record(stream)
        else:
            for i in range(first, first + count):
                sched(i)
                execute(i)
                if marks is not None:
                    marks.append(torch.cuda.Event(enable_timing=True))
                    marks[-1].record(stream)

    run(0, args.warmup)
    torch.cuda.synchronize()
    phase = dict(ms_schedule=0.0, ms_forward=0.0, ms_backward=0.0, ms_param_grads=0.0)
    launches = dict(n_launch_fwd=0, n_launch_bwd=0)
    t0 = time.perf_counter()
    run(args.warmup, args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # per-phase HIP-event times (events were recorded inside the timed region; reading them is not timed)
    per_ctx_stats = [c.stats() for c in ctxs]
    # spread of the step period: a second, untimed pass with one event per step on the execution
    # stream (the events cost a little, so they stay out of the timed pass)
    marks = []
    run(args.warmup + args.steps, args.steps, marks)
    torch.cuda.synchronize()
    periods = sorted(a.elapsed_time(b) for a, b in zip(marks[:-1], marks[1:]))
    step_period = (dict(median=round(periods[len(periods) // 2], 4), min=round(periods[0], 4), max=round(periods[-1], 4),
                        note="ms between the ends of consecutive steps on the execution stream, untimed second pass")
                   if periods else None)
    for i in range(args.steps):
        st = per_ctx_stats[(args.warmup + i) % pool]
        for k_ in phase:
            phase[k_] += st[k_]
        for k_ in launches:
            launches[k_] += st[k_]
    n_inst = sum(graphs[(args.warmup + i) % pool].n_instances for i in range(args.steps))
    n_nodes = sum(graphs[(args.warmup + i) % pool].n for i in range(args.steps))
    ms_per_step = elapsed / args.steps * 1e3
    value = n_inst / elapsed

    # algorithmic bytes / flops from the realised schedules
    cost = dict(fwd_bytes=0.0, bwd_bytes=0.0, param_bytes=0.0, fwd_flops=0.0, bwd_flops=0.0)
    for i in range(args.steps):
        j = (args.warmup + i) % pool
        if "cost" not in graphs[j].meta:
            bo, ids, bd, _ = ctxs[j].schedule_read()
            graphs[j].meta["cost"] = algorithmic_cost(graphs[j], params, bo, ids)
        for k_ in cost:
            cost[k_] += graphs[j].meta["cost"][k_]

    # Dominant kernel: the forward step interpreter (k_fwd_step) or the backward one (k_bwd_step),
    # whichever took more of the timed region.  Each kernel's launches are bracketed by HIP events on
    # the execution stream (forward: ms_forward; backward: ms_backward minus the three deferred
    # parameter-gradient kernels, which have events of their own), so the average launch duration
    # is measured live.  The other kernel is reported beside it.  Each kernel has two instantiations
    # (k_..._step<false>: any work; k_..._step<true>: launches with component-wise work only); the
    # figures cover both, as do the stored traffic numbers, and the kernel trace's per-instantiation
    # averages weighted by their call counts give the same average launch duration.
    fwd_ms, n_fwd = phase["ms_forward"], max(launches["n_launch_fwd"], 1)
    bwd_ms, n_bwd = phase["ms_backward"] - phase["ms_param_grads"], max(launches["n_launch_bwd"], 1)

    def kernel_figures(name, ms, nl, nbytes):
        ach = nbytes / (ms * 1e-3) / 1e9
        return dict(kernel=name, achieved=round(ach, 2), frac=round(ach / HBM_PEAK_GBS, 5), launches=nl,
                    avg_launch_us=round(ms * 1e3 / nl, 3), algorithmic_bytes_per_launch=round(nbytes / nl, 1),
                    traffic=stored_traffic(args, name))

    kf = kernel_figures("k_fwd_step", fwd_ms, n_fwd, cost["fwd_bytes"])
    kb = kernel_figures("k_bwd_step", bwd_ms, n_bwd, cost["bwd_bytes"])
    dom, other = (kb, kf) if bwd_ms >= fwd_ms else (kf, kb)
    roofline = dict(bound="hbm", kernel=dom["kernel"], achieved=dom["achieved"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=dom["frac"], traffic=dom["traffic"], launches=dom["launches"],
                    avg_launch_us=dom["avg_launch_us"], algorithmic_bytes_per_launch=dom["algorithmic_bytes_per_launch"],
                    other_step_kernel=other,
                    mfma=dict(fwd_tflops=round(cost["fwd_flops"] / (phase["ms_forward"] * 1e-3) / 1e12, 3),
                              bwd_tflops=round(cost["bwd_flops"] / (phase["ms_backward"] * 1e-3) / 1e12, 3),
                              peak=MFMA_FP32_PEAK_TFLOPS))

    # batch-size histogram of the first pooled minibatch's schedule (bins: 1, 2-3, 4-7, ...)
    bo0 = ctxs[0].schedule_read()[0]
    sizes = np.diff(bo0)
    bins = np.floor(np.log2(np.maximum(sizes, 1))).astype(np.int64)
    batch_hist = {f"{1 << b}-{(2 << b) - 1}": int(c) for b, c in enumerate(np.bincount(bins)) if c}

    # What bounds the step: the dependent launches (measured floor of a launch boundary on this
    # machine x launches per step) against the time the algorithmic bytes and flops would take at
    # the chip's peaks.
    floor_us = ctxs[0].test_launch_cost(2000, 0)
    n_launch_step = (launches["n_launch_fwd"] + launches["n_launch_bwd"]) / args.steps
    t_peak_ms = ((cost["fwd_bytes"] + cost["bwd_bytes"] + cost["param_bytes"]) / (HBM_PEAK_GBS * 1e9) +
                 (cost["fwd_flops"] + cost["bwd_flops"]) / (MFMA_FP32_PEAK_TFLOPS * 1e12)) / args.steps * 1e3
    launch_model = dict(launch_floor_us=round(floor_us, 3), exec_launches_per_step=round(n_launch_step, 1),
                        t_launch_ms=round(n_launch_step * floor_us * 1e-3, 4), t_at_peaks_ms=round(t_peak_ms, 4),
                        exec_ms_per_step=round((phase["ms_forward"] + phase["ms_backward"]) / args.steps, 4))

    if args.copy_calibration:
        nbytes = args.copy_calibration << 20
        src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads nbytes, writes nbytes
        torch.cuda.synchronize()
        del src, dst

    # unbatched GPU run of the same graphs (one launch per node forward, per node backward)
    nobatch = None
    if not args.no_nobatch:
        c = ob.Context(arena_bytes=arena_bytes, stream=stream, mode=ob.OB_NOBATCH, launch=ob.OB_LAUNCH_STREAM)
        c.params_create(params)
        c.param_grad_zero()
        c.add_bulk(graphs[0])
        c.upload()
        reps = 2
        for r in range(reps + 1):
            if r == 1:
                torch.cuda.synchronize()
                t1 = time.perf_counter()
            c.reset()
            c.param_grad_zero()
            c.forward(graphs[0].root)
            c.backward(graphs[0].root)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t1) / reps
        nobatch = dict(value=round(graphs[0].n_instances / dt, 2), unit="instances/s", ms_per_step=round(dt * 1e3, 2),
                       speedup_autobatch=round(value / (graphs[0].n_instances / dt), 2))
        c.close()

    cpu = None
    if not args.no_cpu:
        from oracle.interp import Oracle
        ns = max(1, args.cpu_samples)
        t1 = time.perf_counter()
        inst = 0
        for j in range(ns):
            gj = graphs[j % pool]
            o = Oracle(gj, params, "f32")
            o.forward()
            o.backward(gj.root)
            inst += gj.n_instances
        dt = time.perf_counter() - t1
        cpu = dict(value=round(inst / dt, 2), unit="instances/s", cores=1, kind="oracle",
                   sample=f"{ns} minibatches cycling through the {pool} pooled ones ({inst} instances, {dt:.1f} s), fp32 build of the "
                          f"node-at-a-time interpreter, forward+backward, 1 thread of {os.cpu_count()} host cores")

    out = {
        "metric": "training instances/sec (fwd+bwd, autobatched)",
        "value": round(value, 2), "unit": "instances/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": (f"config {cfg['index']}: {args.workload} (BASELINE.json configs[{cfg['index'] - 1}])"
                                if cfg["index"] else f"{args.workload}: the equal-length synthetic tagger of Section 4.1 "
                                                     "(not one of BASELINE.json's configs)"),
                   "instances_per_step": graphs[0].n_instances,
                   "sweep_point": (None if args.instances is None else
                                   f"{args.instances} instances per minibatch instead of the configuration's own count"),
                   "mode": "manual" if args.mode == "manual" else "by" + args.mode, "launch": args.launch,
                   "fusion": not args.no_fusion, "placement": args.placement, "update": bool(args.update),
                   "pipeline": (f"scheduling of steps i+1..i+{lookahead} overlaps execution of step i ({lookahead} schedule "
                                f"stream{'s' if lookahead > 1 else ''})") if pipeline
                   else "none (schedule, forward, backward back to back)",
                   "pool": pool, "nodes_per_step": round(n_nodes / args.steps, 1)},
        "nodes_per_s": round(n_nodes / elapsed, 1),
        "step_period_ms": step_period,
        "phase_ms_per_step": {k_: round(v / args.steps, 4) for k_, v in phase.items()},
        "launches_per_step": {k_: round(v / args.steps, 1) for k_, v in launches.items()},
        "depth_levels": per_ctx_stats[0]["n_steps"], "launch_slots": per_ctx_stats[0]["n_slots"],
        "batches": per_ctx_stats[0]["n_batches"], "batch_size_histogram": batch_hist,
        "upload_ms_host_to_hbm": round(float(np.mean(t_up)) * 1e3, 3),
        "value_including_upload": round(n_inst / (elapsed + float(np.mean(t_up)) * args.steps), 2),
        "roofline": roofline,
        "launch_model": launch_model,
        "nobatch_gpu": nobatch,
        "cpu_baseline": cpu,
        "paper_context": PAPER_CONTEXT.get(args.workload),
    }
    print(json.dumps(out))
    for c in ctxs:
        c.close()


if __name__ == "__main__":
    main()
