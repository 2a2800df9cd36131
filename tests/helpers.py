"""Test-side helpers that are independent of both the oracle's C interpreter and the HIP path:
a NumPy evaluator that runs a *schedule* batch by batch, schedule validators, and the
tensor-level tolerance used by the parity tests."""
from __future__ import annotations

import numpy as np
from scipy.special import logsumexp

from paper_1705_07860_amd import workloads as wl


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |got_i - ref_i| / max(max_i |ref_i|, 1e-30): the tensor-normalised relative error."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def segment_rel_err(got: np.ndarray, ref: np.ndarray, off: np.ndarray) -> float:
    """Worst tensor-normalised relative error over the tensors ref[off[i]:off[i+1]]."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    off = np.asarray(off, np.int64)
    nz = off[1:] > off[:-1]
    starts = off[:-1][nz]
    if starts.size == 0:
        return 0.0
    err = np.maximum.reduceat(np.abs(got - ref), starts)
    mag = np.maximum(np.maximum.reduceat(np.abs(ref), starts), 1e-30)
    return float(np.max(err / mag))


def numpy_batched_forward(g, params, batch_off, node_ids):
    """Evaluate the graph batch by batch in schedule order, each batch as ONE array
    operation over the stacked operands (the W h_i -> W H conversion of Section 3.3).
    Values start as NaN, so a schedule that runs a node before its operands poisons
    the result.  Returns the list of per-node value vectors (float64)."""
    n = g.n
    vals = [None] * n
    mats = [m.astype(np.float64) for m in params.mats]
    for b in range(len(batch_off) - 1):
        ids = [int(v) for v in node_ids[batch_off[b]:batch_off[b + 1]]]
        h = ids[0]
        op = int(g.op[h])
        ar = int(g.in_off[h + 1] - g.in_off[h])
        for v in ids:
            assert int(g.op[v]) == op and int(g.in_off[v + 1] - g.in_off[v]) == ar

        def stack(slot):
            rows = []
            for v in ids:
                u = int(g.in_idx[int(g.in_off[v]) + slot])
                assert vals[u] is not None, f"node {v} scheduled before operand {u}"
                rows.append(vals[u])
            return np.stack(rows)

        if op == wl.OP_INPUT:
            out = np.stack([g.payload[int(g.aux0[v]):int(g.aux0[v]) + int(g.out_dim[v])].astype(np.float64)
                            for v in ids])
        elif op == wl.OP_LOOKUP:
            out = mats[int(g.param[h])][[int(g.aux0[v]) for v in ids], :]
        elif op == wl.OP_MATVEC:
            out = stack(0) @ mats[int(g.param[h])].T
            if int(g.bias[h]) >= 0:
                out = out + mats[int(g.bias[h])].reshape(1, -1)
        elif op == wl.OP_ADD:
            out = stack(0)
            for j in range(1, ar):
                out = out + stack(j)
        elif op == wl.OP_CMULT:
            out = stack(0) * stack(1)
        elif op == wl.OP_TANH:
            out = np.tanh(stack(0))
        elif op == wl.OP_SIGMOID:
            out = 1.0 / (1.0 + np.exp(-stack(0)))
        elif op == wl.OP_CONCAT:
            out = np.concatenate([stack(j) for j in range(ar)], axis=1)
        elif op == wl.OP_SLICE:
            out = stack(0)[:, int(g.aux0[h]):int(g.aux1[h])]
        elif op == wl.OP_PICK_NLS:
            x = stack(0)
            lab = np.asarray([int(g.aux0[v]) for v in ids])
            out = (logsumexp(x, axis=1) - x[np.arange(len(ids)), lab]).reshape(-1, 1)
        elif op == wl.OP_SQNORM:
            out = np.sum(stack(0) ** 2, axis=1, keepdims=True)
        else:
            raise AssertionError(op)
        assert out.shape == (len(ids), int(g.out_dim[h])), (out.shape, op)
        for r, v in enumerate(ids):
            vals[v] = out[r]
    return vals


def sig_string(g, v: int) -> str:
    """Signature spelled the way the paper's examples are ('slice-400x500-100:200',
    'matmul-node123-400x1'): an independent formatting used to cross-check tuple signatures."""
    op = int(g.op[v])
    ins = [int(u) for u in g.in_idx[int(g.in_off[v]):int(g.in_off[v + 1])]]
    dims = "x".join(str(int(g.out_dim[u])) for u in ins)
    s = f"{wl.OP_NAMES[op]}-out{int(g.out_dim[v])}-in{dims}"
    if op == wl.OP_MATVEC:
        s += f"-W{int(g.param[v])}-b{int(g.bias[v])}"
    if op == wl.OP_LOOKUP:
        s += f"-E{int(g.param[v])}"
    if op == wl.OP_SLICE:
        s += f"-{int(g.aux0[v])}:{int(g.aux1[v])}"
    return s


def longest_path_depths(g):
    """Depth by explicit path enumeration (memoised DFS over operands), no reliance on id order."""
    memo = {}

    def depth(v):
        if v in memo:
            return memo[v]
        ins = [int(u) for u in g.in_idx[int(g.in_off[v]):int(g.in_off[v + 1])]]
        memo[v] = 0 if not ins else 1 + max(depth(u) for u in ins)
        return memo[v]
    import sys
    sys.setrecursionlimit(100000)
    return np.asarray([depth(v) for v in range(g.n)], np.int64)


def validate_schedule(g, batch_off, node_ids, batch_depth, n=None):
    """Invariants every depth-based schedule must satisfy (Section 3.2): a partition of the
    nodes; every operand sits at a strictly smaller depth than its consumer; one signature
    per batch; no two batches share (depth, signature); canonical ordering."""
    n = g.n if n is None else n
    batch_off = np.asarray(batch_off, np.int64)
    node_ids = np.asarray(node_ids, np.int64)
    batch_depth = np.asarray(batch_depth, np.int64)
    nb = len(batch_depth)
    assert batch_off[0] == 0 and batch_off[-1] == n and len(batch_off) == nb + 1
    assert np.all(np.diff(batch_off) > 0)
    assert np.array_equal(np.sort(node_ids), np.arange(n))
    depth_of = np.empty(n, np.int64)
    for b in range(nb):
        depth_of[node_ids[batch_off[b]:batch_off[b + 1]]] = batch_depth[b]
    seen = set()
    heads = []
    for b in range(nb):
        ids = node_ids[batch_off[b]:batch_off[b + 1]]
        assert np.all(np.diff(ids) > 0), "ids inside a batch must ascend"
        sigs = {sig_string(g, int(v)) for v in ids}
        assert len(sigs) == 1, f"batch {b} mixes signatures {sigs}"
        key = (int(batch_depth[b]), sigs.pop())
        assert key not in seen, f"two batches share {key}"
        seen.add(key)
        heads.append((int(batch_depth[b]), int(ids[0])))
    assert heads == sorted(heads), "batches must ascend by (depth, smallest id)"
    for v in range(n):
        for u in g.in_idx[int(g.in_off[v]):int(g.in_off[v + 1])]:
            assert depth_of[int(u)] < depth_of[v], f"edge {u}->{v} violates depth order"
    return depth_of


def validate_agenda_schedule(g, batch_off, node_ids, n=None):
    """Replays an agenda-based schedule (Section 3.2) step by step and checks every choice
    independently of the code that made it: the batch holds every available node of its
    signature, nothing else, and no other available signature had a smaller average depth
    (exact fractions over all nodes carrying the signature; then operation class: leaf,
    component-wise / copy, per-row reduction, matrix product; then smaller first node id).
    Depths come from path enumeration, signatures from the string form."""
    from fractions import Fraction
    n = g.n if n is None else n
    depth = longest_path_depths(g)[:n]
    sig = [sig_string(g, v) for v in range(n)]
    klass = {0: 0, 1: 0, 2: 3, 9: 2, 10: 2}
    tot, cnt, first, cost = {}, {}, {}, {}
    for v in range(n):
        s = sig[v]
        tot[s] = tot.get(s, 0) + int(depth[v])
        cnt[s] = cnt.get(s, 0) + 1
        first.setdefault(s, v)
        cost[s] = klass.get(int(g.op[v]), 1)
    rank = {s: (Fraction(tot[s], cnt[s]), cost[s], first[s]) for s in tot}
    executed = np.zeros(n, bool)
    nb = len(batch_off) - 1
    assert batch_off[0] == 0 and batch_off[-1] == n
    for b in range(nb):
        ids = [int(v) for v in node_ids[batch_off[b]:batch_off[b + 1]]]
        assert ids == sorted(ids) and len(ids) > 0
        avail = [v for v in range(n) if not executed[v] and
                 all(executed[int(u)] for u in g.in_idx[int(g.in_off[v]):int(g.in_off[v + 1])])]
        s = sig[ids[0]]
        assert ids == [v for v in avail if sig[v] == s], f"batch {b} is not all available nodes of its signature"
        best = min(rank[sig[v]] for v in avail)
        assert rank[s] == best, f"batch {b}: a signature with a smaller average depth was available"
        executed[ids] = True
    assert executed.all()


def manual_schedule(labels, n=None):
    """What manual batching (Section 2) must produce from the caller's labels: batches in
    ascending label order, ids ascending inside a batch.  Returns (batch_off, node_ids)."""
    labels = np.asarray(labels, np.int64)
    labels = labels if n is None else labels[:n]
    node_ids = np.argsort(labels, kind="stable")
    cuts = np.flatnonzero(np.diff(labels[node_ids])) + 1
    batch_off = np.concatenate(([0], cuts, [len(labels)]))
    return batch_off.astype(np.int64), node_ids.astype(np.int64)


def validate_manual_labels(g, labels):
    """A labelling is usable when operands carry smaller labels than their consumers and a
    label never mixes signatures."""
    labels = np.asarray(labels, np.int64)
    assert labels.shape == (g.n,) and labels.min() >= 0
    cons = np.repeat(np.arange(g.n), np.diff(g.in_off.astype(np.int64)))
    assert np.all(labels[g.in_idx.astype(np.int64)] < labels[cons])
    sig_of = {}
    for v in range(g.n):
        assert sig_of.setdefault(int(labels[v]), sig_string(g, v)) == sig_string(g, v), f"label {labels[v]} mixes signatures"


def stage_graph(g, n0, n1):
    """Nodes [n0, n1) of g as a graph of their own (how a forward after earlier forwards sees
    them, Section 3.1): the earlier nodes they read come first, in id order, as leaves of the
    same dimension; the new nodes follow in id order.  Returns (graph, ids of the earlier nodes).
    Only the structure is filled in (no input data)."""
    from paper_1705_07860_amd.workloads import Graph
    in_off = g.in_off.astype(np.int64)
    e0, e1 = int(in_off[n0]), int(in_off[n1])
    ins = g.in_idx[e0:e1].astype(np.int64)
    proxy = np.unique(ins[ins < n0])
    P = len(proxy)
    local = np.where(ins < n0, np.searchsorted(proxy, ins), P + ins - n0)
    z = np.zeros(P, np.int32)
    return Graph(op=np.concatenate((np.zeros(P, np.uint8), g.op[n0:n1])),
                 out_dim=np.concatenate((g.out_dim[proxy], g.out_dim[n0:n1])).astype(np.uint32),
                 in_off=np.concatenate((np.zeros(P, np.int64), in_off[n0:n1 + 1] - e0)).astype(np.uint32),
                 in_idx=local.astype(np.uint32),
                 param=np.concatenate((z - 1, g.param[n0:n1])).astype(np.int32),
                 bias=np.concatenate((z - 1, g.bias[n0:n1])).astype(np.int32),
                 aux0=np.concatenate((z, g.aux0[n0:n1])).astype(np.int32),
                 aux1=np.concatenate((z, g.aux1[n0:n1])).astype(np.int32),
                 payload=np.zeros(1, np.float32), root=P + n1 - n0 - 1), proxy


def stage_schedule(schedule_fn, g, n0, n1):
    """The schedule of the stage graph in the ids of g, the stand-in leaves left out and batches
    that held nothing else dropped.  Returns (batch_off, node_ids, batch_step)."""
    sg, proxy = stage_graph(g, n0, n1)
    P = len(proxy)
    bo, ids, step = schedule_fn(sg)
    k_off, k_ids, k_step = [0], [], []
    for b in range(len(bo) - 1):
        mem = [int(v) - P + n0 for v in ids[bo[b]:bo[b + 1]] if v >= P]
        if mem:
            k_ids += mem
            k_off.append(len(k_ids))
            k_step.append(int(step[b]))
    return np.asarray(k_off, np.int64), np.asarray(k_ids, np.int64), np.asarray(k_step, np.int64)
