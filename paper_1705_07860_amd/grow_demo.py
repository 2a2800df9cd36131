"""A graph that grows between evaluations (Section 3.1): 64 LSTM chains are extended by one time
step at a time, and after every step a value is read back, as a model would do that looks at
a prediction before it decides what to add next.

    python -m paper_1705_07860_amd.grow_demo [--chains 64] [--steps 40]

Prints host wall-clock times of three ways to get the same loss and gradients:
  stages   ob_forward after each extension evaluates only the new nodes
  again    the evaluation is dropped before each ob_forward, so the whole prefix is evaluated again
  oneshot  the finished graph in one forward (nothing can be read in between)
"""
from __future__ import annotations

import argparse
import time

import numpy as np

from . import binding as ob
from . import workloads as wl


def build(chains: int, steps: int, hidden: int = 256, emb: int = 128, classes: int = 50, seed: int = 1):
    """Time-major graph: all chains' nodes of step t lie before any node of step t + 1.
    Returns (params, graph, bounds): piece t is ids bounds[t] .. bounds[t + 1] - 1 (the first piece
    also holds the initial states, the last piece is the closing sum)."""
    pb = wl.ParamBuilder(np.random.default_rng(seed))
    E = pb.add("E", 1000, emb)
    wx, wh, b = wl.lstm_params(pb, "l", emb, hidden)
    ow, obias = pb.add("o.W", classes, hidden), pb.add("o.b", classes, 1)
    p = pb.done()
    rng = np.random.default_rng(seed + 1)
    g = wl.GraphBuilder(p)
    hs = [g.input(np.zeros(hidden, np.float32)) for _ in range(chains)]
    cs = [g.input(np.zeros(hidden, np.float32)) for _ in range(chains)]
    bounds, losses = [0], []
    for _ in range(steps):
        for i in range(chains):
            x = g.lookup(E, int(rng.integers(0, 1000)))
            s = g.add((g.matvec(wx, b, x), g.matvec(wh, -1, hs[i])))
            si, sf, so, sg = (g.slice(s, k * hidden, (k + 1) * hidden) for k in range(4))
            cs[i] = g.add((g.cmult(g.sigmoid(sf), cs[i]), g.cmult(g.sigmoid(si), g.tanh(sg))))
            hs[i] = g.cmult(g.sigmoid(so), g.tanh(cs[i]))
            losses.append(g.pick_nls(g.matvec(ow, obias, hs[i]), int(rng.integers(0, classes))))
        bounds.append(len(g.op))
    root = g.add(losses)
    G = g.finish(root, chains)
    bounds.append(G.n)
    return p, G, bounds


def part(G, lo: int, hi: int):
    e0, e1 = int(G.in_off[lo]), int(G.in_off[hi])
    return wl.Graph(op=G.op[lo:hi], out_dim=G.out_dim[lo:hi], in_off=G.in_off[lo:hi + 1] - e0, in_idx=G.in_idx[e0:e1],
                    param=G.param[lo:hi], bias=G.bias[lo:hi], aux0=G.aux0[lo:hi], aux1=G.aux1[lo:hi],
                    payload=G.payload, root=hi - 1)


def run_all(chains: int, steps: int, repeats: int, arena_bytes: int = 6 << 30, report=print, **sizes):
    """Runs the three ways `repeats` times on one context; returns [(kind, forward s, total s, loss)]."""
    import torch
    p, G, bounds = build(chains, steps, **sizes)
    parts = [part(G, bounds[k], bounds[k + 1]) for k in range(len(bounds) - 1)]
    report(f"{G.n} nodes, grown in {len(parts)} pieces")
    c = ob.Context(arena_bytes=arena_bytes)
    c.params_create(p)
    results = []

    def run(kind):
        c.graph_new()
        c.param_grad_zero()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        per = []
        if kind == "oneshot":
            c.add_bulk(G)
            c.forward(G.root)
        else:
            for pt in parts:
                t1 = time.perf_counter()
                c.add_bulk(pt)
                if kind == "again":
                    c.reset()
                last = c.graph_size()[0] - 1
                c.forward(last)
                c.value_read(last, 1)
                per.append(time.perf_counter() - t1)
        t_f = time.perf_counter() - t0
        c.backward(G.root)
        loss = float(c.value_read(G.root, 1)[0])
        c.sync()
        return t_f, time.perf_counter() - t0, loss, per

    for kind in ["oneshot", "stages", "again"] * repeats:
        t_f, t_all, loss, per = run(kind)
        pieces = f"; per piece: median {np.median(per) * 1e3:.2f} ms, last step {per[-2] * 1e3:.2f} ms" if per else ""
        report(f"{kind:8s} forward phase {t_f * 1e3:8.2f} ms, with backward {t_all * 1e3:8.2f} ms, loss {loss:.4f}{pieces}")
        results.append((kind, t_f, t_all, loss))
    c.close()
    return results


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--chains", type=int, default=64)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--repeats", type=int, default=3)
    args = ap.parse_args()
    run_all(args.chains, args.steps, args.repeats, report=lambda m: print(m, flush=True))


if __name__ == "__main__":
    main()
