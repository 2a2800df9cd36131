#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step is one pass of the whole path over one minibatch: hand the graph over (ob_graph_new,
ob_add_bulk, upload to HBM), schedule it on the GPU, batched forward, batched backward.  Every
step takes a freshly generated seeded minibatch (generated on the host ahead of the timed region,
handed over inside it); parameters stay resident.  With pipelining (default) the hand-over and
the scheduling of step i+1 run on a second stream while step i executes.

Default run: the five listed configurations, the largest one (config 3, BiLSTM tagger with the
character model) as the headline with exactly --steps timed steps, the other four with fewer
steps in the `configs` object, and ONE JSON line: training instances/s (autobatched,
depth-based), nodes/s, phase times, launches, the roofline figures of the dominant step kernel
from HIP events the library records on its streams, the same graphs with batching off (one
launch per node), and the CPU oracle timed on a bounded sample.  `--workload X` measures X alone.
"""
from __future__ import annotations

import argparse
import gc
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
FIVE = ["rnn", "tagger", "tagger_char", "tree", "parser"]
HEADLINE = "tagger_char"


def algorithmic_cost(g, params, batch_off, node_ids):
    """Bytes and flops the method itself must move / do for one forward+backward of this
    schedule (per-batch formulas: operands read once, results written once, one 4-byte row index
    per gathered operand row of component-wise work; a shared matrix is read once per batch; dW is
    read-modify-written once per parameter because its reduction is deferred over all uses).
    bwd_bytes covers the backward step kernel (gradient pull and dX), param_bytes the deferred
    dW / db / dE kernels."""
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
    fb[m] = (8 * d * B)[m]
    bb[m] = (8 * d * B)[m]
    m = (op == wl.OP_LOOKUP) | (op == wl.OP_INPUT)
    fb[m] = (8 * d * B)[m]
    bb[op == wl.OP_LOOKUP] = (16 * d * B)[op == wl.OP_LOOKUP]
    m = (op == wl.OP_PICK_NLS) | (op == wl.OP_SQNORM)
    fb[m] = ((4 * k + 4) * B)[m]
    bb[m] = (8 * k * B)[m]
    m = op == wl.OP_MATVEC
    fb[m] = (4 * (d * k + k * B + d * B))[m]
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


def stored_traffic(args, workload, kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary (two rocprofv3 --pmc
    runs, FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size).  Counters cannot be
    read inside a timing run, so the figure is the stored one and only applies to the default
    launch configuration of the workload it was taken on; otherwise null."""
    if args.launch != "stream" or args.no_fusion or args.placement != "late" or args.mode != "depth" or args.instances:
        return None
    path = os.path.join(ROOT, "profiles", f"{workload}_bydepth_hbm_traffic.json")
    try:
        with open(path) as f:
            k = json.load(f)["kernels"][kernel]
        return k["fetch_bytes_per_launch"] + k["write_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def workload_label(name):
    cfg = wl.CONFIGS[name]
    if cfg["index"]:
        return f"config {cfg['index']}: {name} (BASELINE.json configs[{cfg['index'] - 1}])"
    return f"{name}: the equal-length synthetic tagger of Section 4.1 (not one of BASELINE.json's configs)"


def measure(args, ob, torch, name, steps, warmup, sustain_s, cpu_s, headline):
    """All figures of one workload.  `steps` timed steps after `warmup` untimed ones, each on a
    minibatch of its own."""
    cfg = wl.CONFIGS[name]
    params = cfg["params"]()
    t_gen = time.perf_counter()
    graphs = [cfg["batch"](params, j, n=args.instances) for j in range(warmup + steps)]
    t_gen = (time.perf_counter() - t_gen) / len(graphs)
    labels = [wl.sync_tagger_manual_labels(g) for g in graphs] if args.mode == "manual" else None
    n_g = len(graphs)
    arena_bytes = (1 << 30) * max(1, -(-graphs[0].n_instances // 64))
    launch = ob.OB_LAUNCH_GRAPH if args.launch == "graph" else ob.OB_LAUNCH_STREAM
    mode = {"agenda": ob.OB_BYAGENDA, "manual": ob.OB_MANUAL}.get(args.mode, ob.OB_BYDEPTH)

    # A ring of contexts that share one parameter set (forks of the first) and one execution
    # stream: the executions of consecutive steps are serial on the GPU, as in a training loop with
    # an update in between.  A context is reused every `pool` steps; ob_graph_new waits for that
    # context's earlier step only (long finished), so the host never waits for the GPU inside the
    # loop except for the schedule header of the step it is about to execute.
    pipeline = not args.no_pipeline
    lookahead = args.lookahead if args.lookahead > 0 else (2 if args.mode == "agenda" else 1)
    pool = max(args.pool, lookahead + 3)
    # With pipelining the schedule streams and the execution stream get disjoint compute units: scheduling
    # kernels that share units with the latency-bound execution launches slow those by about a tenth.
    raw_streams = []
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    cu_split = args.cu_split if args.cu_split >= 0 else (32 if max(g.n for g in graphs) <= 300000 else 0)
    if pipeline and 0 < cu_split < n_cu:
        def on_cus(first, count):
            raw_streams.append(ob.stream_create_on_cus(first, count))
            return torch.cuda.ExternalStream(raw_streams[-1])
        stream = on_cus(cu_split, n_cu - cu_split)
        sched_streams = [on_cus(0, cu_split) for _ in range(lookahead)]
    else:
        cu_split = 0
        stream = torch.cuda.Stream()
        sched_streams = [torch.cuda.Stream() for _ in range(lookahead)]
    ctxs = []
    for j in range(pool):
        if j == 0:
            c = ob.Context(arena_bytes=arena_bytes, stream=stream, launch=launch, mode=mode)
            c.set_fusion(0 if args.no_fusion else (1 if args.placement == "early" else 2))
            c.params_create(params)
            c.param_grad_zero()
        else:
            c = ctxs[0].fork(arena_bytes=arena_bytes, stream=stream)
        ctxs.append(c)

    host_marks = [] if os.environ.get("OB_BENCH_HOST_MARKS") else None

    def set_streams(piped):
        for j, c in enumerate(ctxs):
            c.graph_new()
            c.set_schedule_stream(sched_streams[j % lookahead] if piped else stream)

    def hand_over(i, piped):
        """graph definition + upload + scheduling of step i (queued; nothing is waited for)"""
        c = ctxs[i % pool]
        t_a = time.perf_counter()
        c.graph_new()
        t_b = time.perf_counter()
        c.add_bulk(graphs[i % n_g])
        t_c = time.perf_counter()
        if labels is not None:
            c.set_manual_batches(labels[i % n_g])
        if piped:
            c.schedule_async(graphs[i % n_g].root)
        else:
            c.schedule(graphs[i % n_g].root)
        if host_marks is not None and time.perf_counter() - t_a > 2e-3:
            print(f"slow hand-over of step {i}: graph_new {(t_b - t_a) * 1e3:.2f} add_bulk {(t_c - t_b) * 1e3:.2f} "
                  f"schedule {(time.perf_counter() - t_c) * 1e3:.2f} ms", file=sys.stderr)

    def execute(i):
        c = ctxs[i % pool]
        g = graphs[i % n_g]
        if not args.update:
            c.param_grad_zero()
        c.forward(g.root)
        c.backward(g.root)
        if args.update:
            c.sgd_step(0.0, zero_grad=True)    # lr 0 keeps the parameters, and so the timings, stationary

    def run(first, count, piped, marks=None):
        if piped:
            for a in range(min(lookahead, count)):
                hand_over(first + a, True)
            for i in range(first, first + count):
                if host_marks is not None:
                    host_marks.append(time.perf_counter())
                if i + lookahead < first + count:
                    hand_over(i + lookahead, True)
                if host_marks is not None:
                    host_marks.append(time.perf_counter())
                execute(i)
                if host_marks is not None:
                    host_marks.append(time.perf_counter())
                if marks is not None:
                    marks.append(torch.cuda.Event(enable_timing=True))
                    marks[-1].record(stream)
        else:
            for i in range(first, first + count):
                hand_over(i, False)
                execute(i)

    def timed(first, count, piped):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(first, count, piped)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # The interpreter's cyclic garbage collector stays out of the loops: a full collection walks every
    # container object of the process (tens of milliseconds here) at a moment of its own choosing.
    gc.collect()
    gc.disable()

    # Set-up, untimed: every context of the ring takes the largest minibatch once, so that its
    # page-locked graph store and the library's other host buffers have reached their steady size
    # (a training loop is in that state after its first few minibatches).
    set_streams(pipeline)
    biggest = {max(range(n_g), key=lambda j: graphs[j].n), max(range(n_g), key=lambda j: graphs[j].in_idx.size),
               max(range(n_g), key=lambda j: graphs[j].payload.size)}
    for c in ctxs:
        for j in sorted(biggest):      # most nodes, most operand references, largest input payload
            c.graph_new()
            c.add_bulk(graphs[j])
            if labels is not None:
                c.set_manual_batches(labels[j])
            c.schedule(graphs[j].root)
    torch.cuda.synchronize()

    # still set-up: the loop itself, twice around the ring and a little more, so that the runtime's own
    # pools (command buffers, copy engines, signals) have grown to what this loop needs
    run(0, 2 * pool + lookahead + 4, pipeline)
    torch.cuda.synchronize()

    # ---- the timed region: exactly `steps` steps, each with its own minibatch, hand-over included
    run(0, warmup, pipeline)
    elapsed = timed(warmup, steps, pipeline)
    if host_marks is not None:
        hm = host_marks[-3 * steps:]
        print("host ms per step (hand-over of the next, execute):",
              [(round((hm[3 * q + 1] - hm[3 * q]) * 1e3, 2), round((hm[3 * q + 2] - hm[3 * q + 1]) * 1e3, 2)) for q in range(steps)],
              file=sys.stderr)
    n_inst = sum(graphs[warmup + i].n_instances for i in range(steps))
    n_nodes = sum(graphs[warmup + i].n for i in range(steps))
    value = n_inst / elapsed

    # per-phase HIP-event times, launches and algorithmic cost of the last `cover` timed steps (a
    # context keeps the events of its latest step; reading them is not timed)
    cover = min(pool, steps)
    phase = dict(ms_upload=0.0, ms_schedule=0.0, ms_forward=0.0, ms_backward=0.0, ms_param_grads=0.0, ms_graph_build=0.0)
    launches = dict(n_launch_fwd=0, n_launch_bwd=0, n_launch_bwd_steps=0, n_launch_sched=0)
    cost = dict(fwd_bytes=0.0, bwd_bytes=0.0, param_bytes=0.0, fwd_flops=0.0, bwd_flops=0.0)
    upload_bytes = 0
    st = None
    for i in range(warmup + steps - cover, warmup + steps):
        c = ctxs[i % pool]
        st = c.stats()
        for k_ in phase:
            phase[k_] += st[k_]
        for k_ in launches:
            launches[k_] += st[k_]
        upload_bytes += st["upload_bytes"]
        bo, ids, _, _ = c.schedule_read()
        cst = algorithmic_cost(graphs[i % n_g], params, bo, ids)
        for k_ in cost:
            cost[k_] += cst[k_]
    sizes = np.diff(bo)
    bins = np.floor(np.log2(np.maximum(sizes, 1))).astype(np.int64)
    batch_hist = {f"{1 << b}-{(2 << b) - 1}": int(c_) for b, c_ in enumerate(np.bincount(bins)) if c_}

    # Dominant kernel: the forward step interpreter (k_fwd_step) or the backward one (k_bwd_step),
    # whichever took more time.  Each kernel's launches are bracketed by HIP events on the
    # execution stream (forward: ms_forward; backward: ms_backward minus the deferred
    # parameter-gradient kernels, which have an event of their own), so the average launch duration
    # is measured live.  Each kernel has two instantiations (k_..._step<false>: any work;
    # k_..._step<true>: launches with component-wise work only); the figures cover both.
    fwd_ms, n_fwd = phase["ms_forward"], max(launches["n_launch_fwd"], 1)
    bwd_ms, n_bwd = phase["ms_backward"] - phase["ms_param_grads"], max(launches["n_launch_bwd_steps"], 1)

    def kernel_figures(kname, ms, nl, nbytes):
        ach = nbytes / (ms * 1e-3) / 1e9
        return dict(kernel=kname, achieved=round(ach, 2), frac=round(ach / HBM_PEAK_GBS, 5), launches_per_step=round(nl / cover, 1),
                    avg_launch_us=round(ms * 1e3 / nl, 3), algorithmic_bytes_per_launch=round(nbytes / nl, 1),
                    traffic=stored_traffic(args, name, kname))

    kf = kernel_figures("k_fwd_step", fwd_ms, n_fwd, cost["fwd_bytes"])
    kb = kernel_figures("k_bwd_step", bwd_ms, n_bwd, cost["bwd_bytes"])
    dom, other = (kb, kf) if bwd_ms >= fwd_ms else (kf, kb)
    roofline = dict(bound="hbm", kernel=dom["kernel"], achieved=dom["achieved"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=dom["frac"], traffic=dom["traffic"], launches_per_step=dom["launches_per_step"],
                    avg_launch_us=dom["avg_launch_us"], algorithmic_bytes_per_launch=dom["algorithmic_bytes_per_launch"],
                    other_step_kernel=other,
                    whole_step=dict(algorithmic_bytes=round((cost["fwd_bytes"] + cost["bwd_bytes"] + cost["param_bytes"]) / cover, 1),
                                    gbs_over_exec_time=round((cost["fwd_bytes"] + cost["bwd_bytes"] + cost["param_bytes"]) /
                                                             ((phase["ms_forward"] + phase["ms_backward"]) * 1e-3) / 1e9, 2)),
                    mfma=dict(fwd_tflops=round(cost["fwd_flops"] / (phase["ms_forward"] * 1e-3) / 1e12, 3),
                              bwd_tflops=round(cost["bwd_flops"] / (phase["ms_backward"] * 1e-3) / 1e12, 3),
                              frac_of_peak=round((cost["fwd_flops"] + cost["bwd_flops"]) /
                                                 ((phase["ms_forward"] + phase["ms_backward"]) * 1e-3) / 1e12 /
                                                 MFMA_FP32_PEAK_TFLOPS, 5),
                              peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s fp32"))

    out = {
        "workload": workload_label(name),
        "value": round(value, 2), "unit": "instances/s", "nodes_per_s": round(n_nodes / elapsed, 1),
        "ms_per_step": round(elapsed / steps * 1e3, 4), "steps": steps, "warmup": warmup,
        "instances_per_step": graphs[0].n_instances, "nodes_per_step": round(n_nodes / steps, 1),
        "timed_region": "per step: ob_graph_new + ob_add_bulk (host arrays -> library) + upload to HBM + GPU scheduling + "
                        "forward + backward, a different seeded minibatch every step",
        "phase_ms_per_step": {k_: round(v / cover, 4) for k_, v in phase.items()},
        "launches_per_step": {k_: round(v / cover, 1) for k_, v in launches.items()},
        "upload_bytes_per_step": int(upload_bytes / cover),
        "phases_cover": f"the last {cover} timed steps",
        "depth_levels": st["n_steps"], "launch_slots": st["n_slots"], "batches": st["n_batches"],
        "batch_size_histogram": batch_hist,
        # Section 3.3: batches of the last step whose rows the forward pass never writes (SLICE batches are views of their
        # operand rows; CONCAT batches that only matrix products read are read in pieces where the pieces lie)
        "copy_elision": {"slice_view_batches": st["n_view_batches"], "slice_view_tiles": int(-(-st["view_floats"] // 1024)),
                         "concat_uncopied_batches": st["n_uncopied_batches"],
                         "concat_uncopied_tiles": int(-(-st["uncopied_floats"] // 1024)),
                         "forward_bytes_saved": int(8 * (st["view_floats"] + st["uncopied_floats"]))},
        "host_generation_ms_per_minibatch": round(t_gen * 1e3, 2),
        "roofline": roofline,
    }

    # ---- secondary figures (none of them is `value`) ----
    # step period spread: one event per step on the execution stream, untimed pass
    if pipeline and steps >= 3:
        marks = []
        run(warmup, steps, True, marks)
        torch.cuda.synchronize()
        periods = sorted(a.elapsed_time(b) for a, b in zip(marks[:-1], marks[1:]))
        out["step_period_ms"] = dict(median=round(periods[len(periods) // 2], 4), min=round(periods[0], 4),
                                     max=round(periods[-1], 4))
    # graph already resident: only reset + schedule + forward + backward per step (the figure of a
    # loop that revisits stored minibatches; upload excluded)
    torch.cuda.synchronize()
    r_steps = min(steps, 20)
    for j in range(pool):
        hand_over(j, False)
    torch.cuda.synchronize()

    def resident_step(i, piped):
        c = ctxs[i % pool]
        c.reset()
        (c.schedule_async if piped else c.schedule)(graphs[(i % pool) % n_g].root)

    def resident_run(count):
        if pipeline:
            for a in range(min(lookahead, count)):
                resident_step(a, True)
        for i in range(count):
            if pipeline:
                if i + lookahead < count:
                    resident_step(i + lookahead, True)
            else:
                resident_step(i, False)
            c = ctxs[i % pool]
            c.param_grad_zero()
            c.forward(graphs[(i % pool) % n_g].root)
            c.backward(graphs[(i % pool) % n_g].root)
    resident_run(min(pool, 4))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    resident_run(r_steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out["value_graph_resident"] = dict(value=round(r_steps * graphs[0].n_instances / dt, 2), unit="instances/s", steps=r_steps,
                                       note="minibatches already in HBM: schedule + forward + backward only")

    # serial: hand-over, scheduling, forward, backward back to back on one stream (no overlap between steps)
    s_steps = min(steps, 10)
    set_streams(False)
    run(0, 2, False)
    dt = timed(warmup, s_steps, False)
    serial_value = sum(graphs[(warmup + i) % n_g].n_instances for i in range(s_steps)) / dt
    sst = ctxs[(warmup + s_steps - 1) % pool].stats()
    out["serial"] = dict(value=round(serial_value, 2), unit="instances/s", ms_per_step=round(dt / s_steps * 1e3, 4), steps=s_steps,
                         phase_ms_last_step={k_: round(sst[k_], 4) for k_ in phase},
                         note="no pipelining: every step's hand-over, scheduling, forward and backward on one stream")
    set_streams(pipeline)

    if sustain_s > 0:
        run(0, min(warmup, 3), pipeline)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        done = 0
        chunk = max(10, min(200, int(0.25 * steps / max(elapsed, 1e-6))))
        while time.perf_counter() - t0 < sustain_s:
            run(done, chunk, pipeline)
            done += chunk
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        inst = sum(graphs[i % n_g].n_instances for i in range(done))
        out["sustained"] = dict(value=round(inst / dt, 2), unit="instances/s", steps=done, seconds=round(dt, 3),
                                note=f"same loop kept up for at least {sustain_s:g} s, cycling through the {n_g} generated minibatches "
                                     "(each handed over again every time)")

    if headline:
        floor_us = ctxs[0].test_launch_cost(2000, 0)
        n_launch_step = (launches["n_launch_fwd"] + launches["n_launch_bwd"]) / cover
        t_peak_ms = ((cost["fwd_bytes"] + cost["bwd_bytes"] + cost["param_bytes"]) / (HBM_PEAK_GBS * 1e9) +
                     (cost["fwd_flops"] + cost["bwd_flops"]) / (MFMA_FP32_PEAK_TFLOPS * 1e12)) / cover * 1e3
        out["launch_model"] = dict(launch_floor_us=round(floor_us, 3), exec_launches_per_step=round(n_launch_step, 1),
                                   t_launch_ms=round(n_launch_step * floor_us * 1e-3, 4), t_at_peaks_ms=round(t_peak_ms, 4),
                                   exec_ms_per_step=round((phase["ms_forward"] + phase["ms_backward"]) / cover, 4))

    # unbatched GPU run of the same path (one launch per node forward, one per node backward), hand-over included
    if not args.no_nobatch:
        c = ob.Context(arena_bytes=arena_bytes, stream=stream, mode=ob.OB_NOBATCH, launch=ob.OB_LAUNCH_STREAM)
        c.params_create(params)
        c.param_grad_zero()
        reps = 3 if graphs[0].n < 5000 else 1
        for r in range(reps + 1):
            if r == 1:
                torch.cuda.synchronize()
                t1 = time.perf_counter()
            g = graphs[r % n_g]
            c.graph_new()
            c.add_bulk(g)
            c.param_grad_zero()
            c.forward(g.root)
            c.backward(g.root)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t1) / reps
        nb_value = graphs[0].n_instances / dt
        out["nobatch_gpu"] = dict(value=round(nb_value, 2), unit="instances/s", ms_per_step=round(dt * 1e3, 2), steps=reps,
                                  speedup_autobatch_serial=round(serial_value / nb_value, 2),
                                  speedup_autobatch_pipelined=round(value / nb_value, 2),
                                  note="serial speed-up: both runs unpipelined, hand-over included")
        c.close()

    if not args.no_cpu:
        from oracle.interp import Oracle
        t1 = time.perf_counter()
        inst = 0
        ns = 0
        while True:
            gj = graphs[ns % n_g]
            o = Oracle(gj, params, "f32")
            o.forward()
            o.backward(gj.root)
            inst += gj.n_instances
            ns += 1
            if time.perf_counter() - t1 >= cpu_s or ns >= 4096:
                break
        dt = time.perf_counter() - t1
        out["cpu_baseline"] = dict(value=round(inst / dt, 2), unit="instances/s", cores=1, kind="oracle",
                                   sample=f"{ns} of the run's minibatches ({inst} instances, {dt:.1f} s): fp32 build of the "
                                          f"node-at-a-time interpreter, forward+backward, 1 thread of {os.cpu_count()} host cores")
    out["paper_context"] = PAPER_CONTEXT.get(name)
    out["cu_split"] = cu_split
    gc.enable()
    for c in ctxs[1:]:
        c.close()
    ctxs[0].close()
    torch.cuda.synchronize()
    for h in raw_streams:
        ob.stream_destroy(h)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all", choices=["all"] + list(wl.CONFIGS),
                    help="all (default): the five listed configurations, config 3 as the headline; or one workload alone")
    ap.add_argument("--other-steps", type=int, default=20, help="timed steps of the four non-headline configurations")
    ap.add_argument("--pool", type=int, default=8, help="contexts in the ring (a context is reused every `pool` steps)")
    ap.add_argument("--cu-split", type=int, default=-1, metavar="N",
                    help="with pipelining: the schedule streams run on compute units [0, N), the execution stream on the "
                         "rest (0: ordinary streams, every kernel anywhere on the chip; default: 32 for minibatches of "
                         "up to 300 000 nodes, whose scheduling on 32 units still hides behind their execution, else 0)")
    ap.add_argument("--instances", type=int, default=None,
                    help="instances per minibatch (default: the configuration's own count; other values are sweep "
                         "points, not the headline workload)")
    ap.add_argument("--launch", default="stream", choices=["stream", "graph"])
    ap.add_argument("--mode", default="depth", choices=["depth", "agenda", "manual"],
                    help="batching strategy of Section 3.2: depth-based (default, the configuration the stored "
                         "profiles cover) or agenda-based; manual = Section 2's batching by hand, one batch per "
                         "statement of a program written over a batch of sentences (--workload sync_tagger only)")
    ap.add_argument("--lookahead", type=int, default=0,
                    help="minibatches handed over and scheduled ahead of the one that executes, each on a schedule stream "
                         "of its own (default: 1 for depth-based batching, 2 for agenda-based batching)")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="hand over, schedule and execute each step back to back on one stream (no overlap between steps)")
    ap.add_argument("--no-fusion", action="store_true", help="one launch per depth level")
    ap.add_argument("--placement", default="late", choices=["early", "late"],
                    help="fused plans launch a batch as early as its operands / as late as its consumers allow")
    ap.add_argument("--update", action="store_true",
                    help="close every step with the gradient-descent update of Section 2 (lr 0) instead of only "
                         "zeroing the gradients; the headline metric is forward + backward, so this is off by default")
    ap.add_argument("--sustain", type=float, default=2.0, help="seconds of the sustained pass of the headline workload (0: skip)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-nobatch", action="store_true", help="skip the unbatched GPU leg")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="CPU oracle leg of the headline workload: minibatches are run until this much time has passed "
                         "(the other configurations get a quarter of it each)")
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

    t_start = time.perf_counter()
    head_name = HEADLINE if args.workload == "all" else args.workload
    head = measure(args, ob, torch, head_name, args.steps, args.warmup, args.sustain, args.cpu_seconds, True)
    configs = None
    if args.workload == "all":
        configs = {}
        for name in FIVE:
            if name == head_name:
                configs[name] = {k: head[k] for k in head if k not in ("launch_model",)}
                continue
            configs[name] = measure(args, ob, torch, name, min(args.steps, args.other_steps), min(args.warmup, 3), 0.0,
                                    args.cpu_seconds / 4, False)

    if args.copy_calibration:
        nbytes = args.copy_calibration << 20
        src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads nbytes, writes nbytes
        torch.cuda.synchronize()
        del src, dst

    lookahead = args.lookahead if args.lookahead > 0 else (2 if args.mode == "agenda" else 1)
    out = {
        "metric": "training instances/sec (fwd+bwd, autobatched)",
        "value": head["value"], "unit": "instances/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"],
                   "instances_per_step": head["instances_per_step"],
                   "sweep_point": (None if args.instances is None else
                                   f"{args.instances} instances per minibatch instead of the configuration's own count"),
                   "mode": "manual" if args.mode == "manual" else "by" + args.mode, "launch": args.launch,
                   "fusion": not args.no_fusion, "placement": args.placement, "update": bool(args.update),
                   "pipeline": (f"hand-over and scheduling of steps i+1..i+{lookahead} overlap the execution of step i "
                                f"({lookahead} schedule stream{'s' if lookahead > 1 else ''})") if not args.no_pipeline
                   else "none (hand-over, schedule, forward, backward back to back)",
                   "compute_units": (f"schedule streams on units [0, {head['cu_split']}), execution stream on the other units"
                                     if head["cu_split"] > 0 else "every stream on the whole chip"),
                   "timed_region": head["timed_region"],
                   "nodes_per_step": head["nodes_per_step"]},
    }
    for k in head:
        if k not in ("workload", "value", "unit", "ms_per_step", "steps", "warmup", "instances_per_step", "nodes_per_step",
                     "timed_region"):
            out[k] = head[k]
    if configs is not None:
        out["configs"] = configs
    out["bench_wall_s"] = round(time.perf_counter() - t_start, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
