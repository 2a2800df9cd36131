"""Seeded synthetic workload generators: dynamic computation graphs as flat arrays.

This module holds none of the method's arithmetic (no depth, no signature, no
forward or backward evaluation).  It only *describes* graphs: a Wengert list
(Section 1, footnote on computation graphs) written as structure-of-arrays, one
per-instance loss builder per workload, and a minibatch loss that is the sum of
the per-instance losses (Section 2, Train-Batch-Naive).  Both the CPU oracle and
the HIP library consume exactly these arrays.

Graph format (node ids are dense, 0..n-1, and every operand id is smaller than
the id of the node that uses it, so id order is a topological order):

  op[n]        u8   operation code (OP_* below)
  out_dim[n]   u32  length of the node's value vector
  in_off[n+1]  u32  CSR offsets into in_idx
  in_idx[E]    u32  operand node ids, in operand-slot order
  param[n]     i32  parameter id: W of MATVEC, table of LOOKUP, else -1
  bias[n]      i32  bias parameter id of MATVEC, else -1
  aux0[n]      i32  LOOKUP: row; SLICE: lo; PICK_NLS: label; INPUT: payload offset
  aux1[n]      i32  SLICE: hi; else 0
  payload[P]   f32  concatenated INPUT vectors

Parameters are a list of row-major fp32 matrices (a bias is rows x 1).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

OP_INPUT = 0
OP_LOOKUP = 1
OP_MATVEC = 2
OP_ADD = 3
OP_CMULT = 4
OP_TANH = 5
OP_SIGMOID = 6
OP_CONCAT = 7
OP_SLICE = 8
OP_PICK_NLS = 9
OP_SQNORM = 10
OP_NAMES = ["INPUT", "LOOKUP", "MATVEC", "ADD", "CMULT", "TANH", "SIGMOID",
            "CONCAT", "SLICE", "PICK_NLS", "SQNORM"]

SEED_BASE = 170507860


@dataclass
class Graph:
    op: np.ndarray
    out_dim: np.ndarray
    in_off: np.ndarray
    in_idx: np.ndarray
    param: np.ndarray
    bias: np.ndarray
    aux0: np.ndarray
    aux1: np.ndarray
    payload: np.ndarray
    root: int
    n_instances: int = 1
    meta: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return int(self.op.shape[0])

    @property
    def n_edges(self) -> int:
        return int(self.in_idx.shape[0])


@dataclass
class Params:
    """Model parameters: row-major fp32 matrices addressed by list index."""
    mats: List[np.ndarray]
    names: List[str]

    def index(self, name: str) -> int:
        return self.names.index(name)


class ParamBuilder:
    def __init__(self, rng: np.random.Generator, std: float = 0.1):
        self.rng = rng
        self.std = std
        self.mats: List[np.ndarray] = []
        self.names: List[str] = []

    def add(self, name: str, rows: int, cols: int) -> int:
        w = (self.rng.standard_normal((rows, cols)) * self.std).astype(np.float32)
        self.mats.append(np.ascontiguousarray(w))
        self.names.append(name)
        return len(self.mats) - 1

    def done(self) -> Params:
        return Params(self.mats, self.names)


class GraphBuilder:
    """Appends nodes to Python lists; `finish` turns them into the flat arrays."""

    def __init__(self, params: Params):
        self.pshape = [m.shape for m in params.mats]
        self.op: list = []
        self.out_dim: list = []
        self.in_off: list = [0]
        self.in_idx: list = []
        self.param: list = []
        self.bias: list = []
        self.aux0: list = []
        self.aux1: list = []
        self.payload: list = []
        self.payload_len = 0

    def _node(self, op, dim, ins, param=-1, bias=-1, a0=0, a1=0) -> int:
        self.op.append(op)
        self.out_dim.append(dim)
        self.in_idx.extend(ins)
        self.in_off.append(len(self.in_idx))
        self.param.append(param)
        self.bias.append(bias)
        self.aux0.append(a0)
        self.aux1.append(a1)
        return len(self.op) - 1

    def dim(self, x: int) -> int:
        return self.out_dim[x]

    def input(self, vec) -> int:
        v = np.asarray(vec, dtype=np.float32).reshape(-1)
        off = self.payload_len
        self.payload.append(v)
        self.payload_len += v.shape[0]
        return self._node(OP_INPUT, v.shape[0], (), a0=off)

    def lookup(self, table: int, row: int) -> int:
        rows, cols = self.pshape[table]
        assert 0 <= row < rows
        return self._node(OP_LOOKUP, cols, (), param=table, a0=int(row))

    def matvec(self, w: int, b: int, x: int) -> int:
        m, k = self.pshape[w]
        assert self.out_dim[x] == k, (self.out_dim[x], k)
        if b >= 0:
            assert self.pshape[b] == (m, 1)
        return self._node(OP_MATVEC, m, (x,), param=w, bias=b)

    def add(self, xs: Sequence[int]) -> int:
        d = self.out_dim[xs[0]]
        assert all(self.out_dim[x] == d for x in xs)
        return self._node(OP_ADD, d, tuple(xs))

    def cmult(self, a: int, b: int) -> int:
        assert self.out_dim[a] == self.out_dim[b]
        return self._node(OP_CMULT, self.out_dim[a], (a, b))

    def tanh(self, x: int) -> int:
        return self._node(OP_TANH, self.out_dim[x], (x,))

    def sigmoid(self, x: int) -> int:
        return self._node(OP_SIGMOID, self.out_dim[x], (x,))

    def concat(self, xs: Sequence[int]) -> int:
        return self._node(OP_CONCAT, sum(self.out_dim[x] for x in xs), tuple(xs))

    def slice(self, x: int, lo: int, hi: int) -> int:
        assert 0 <= lo < hi <= self.out_dim[x]
        return self._node(OP_SLICE, hi - lo, (x,), a0=lo, a1=hi)

    def pick_nls(self, x: int, label: int) -> int:
        assert 0 <= label < self.out_dim[x]
        return self._node(OP_PICK_NLS, 1, (x,), a0=int(label))

    def sqnorm(self, x: int) -> int:
        return self._node(OP_SQNORM, 1, (x,))

    def finish(self, root: int, n_instances: int = 1, **meta) -> Graph:
        payload = (np.concatenate(self.payload).astype(np.float32)
                   if self.payload else np.zeros(0, np.float32))
        return Graph(
            op=np.asarray(self.op, np.uint8),
            out_dim=np.asarray(self.out_dim, np.uint32),
            in_off=np.asarray(self.in_off, np.uint32),
            in_idx=np.asarray(self.in_idx, np.uint32),
            param=np.asarray(self.param, np.int32),
            bias=np.asarray(self.bias, np.int32),
            aux0=np.asarray(self.aux0, np.int32),
            aux1=np.asarray(self.aux1, np.int32),
            payload=payload, root=int(root), n_instances=n_instances, meta=meta)


# --------------------------------------------------------------------------
# Shared sub-builders
# --------------------------------------------------------------------------

def lstm_params(pb: ParamBuilder, name: str, d_in: int, hidden: int):
    return (pb.add(name + ".Wx", 4 * hidden, d_in),
            pb.add(name + ".Wh", 4 * hidden, hidden),
            pb.add(name + ".b", 4 * hidden, 1))


def lstm_run(g: GraphBuilder, p, hidden: int, xs: Sequence[int]) -> List[int]:
    """One LSTM over the node sequence xs; 16 nodes and 8 dependency levels a step.

    gates = Wx x_t + b + Wh h_{t-1}; slices i, f, o through a sigmoid, the
    candidate through tanh; c_t = f*c_{t-1} + i*cand; h_t = o*tanh(c_t).  The
    initial h and c are zero INPUT leaves of this sequence.
    """
    wx, wh, b = p
    h = g.input(np.zeros(hidden, np.float32))
    c = g.input(np.zeros(hidden, np.float32))
    out = []
    for x in xs:
        a = g.matvec(wx, b, x)
        u = g.matvec(wh, -1, h)
        s = g.add((a, u))
        si = g.slice(s, 0, hidden)
        sf = g.slice(s, hidden, 2 * hidden)
        so = g.slice(s, 2 * hidden, 3 * hidden)
        sg = g.slice(s, 3 * hidden, 4 * hidden)
        i = g.sigmoid(si)
        f = g.sigmoid(sf)
        o = g.sigmoid(so)
        cand = g.tanh(sg)
        fc = g.cmult(f, c)
        ic = g.cmult(i, cand)
        c = g.add((fc, ic))
        tc = g.tanh(c)
        h = g.cmult(o, tc)
        out.append(h)
    return out


def bilstm_states(g: GraphBuilder, pf, pb_, hidden: int, xs: Sequence[int]):
    fwd = lstm_run(g, pf, hidden, xs)
    bwd = lstm_run(g, pb_, hidden, list(reversed(xs)))[::-1]
    return fwd, bwd


# --------------------------------------------------------------------------
# Config 1: tanh-RNN chains
# --------------------------------------------------------------------------

def rnn_params(seed: int = SEED_BASE + 100, d_in: int = 32, hidden: int = 32) -> Params:
    pb = ParamBuilder(np.random.default_rng(seed))
    pb.add("W", hidden, d_in)
    pb.add("U", hidden, hidden)
    pb.add("b", hidden, 1)
    return pb.done()


def rnn_minibatch(params: Params, seed: int = SEED_BASE + 101, n_inst: int = 8,
                  len_lo: int = 3, len_hi: int = 10, lengths=None) -> Graph:
    """h_t = tanh(W x_t + U h_{t-1} + b), loss = sum_i |h_n^(i)|^2."""
    rng = np.random.default_rng(seed)
    hidden, d_in = params.mats[0].shape
    if lengths is None:
        lengths = rng.integers(len_lo, len_hi + 1, size=n_inst)
    g = GraphBuilder(params)
    losses = []
    for n in lengths:
        h = g.input(np.zeros(hidden, np.float32))
        for _ in range(int(n)):
            x = g.input(rng.standard_normal(d_in))
            a = g.matvec(0, 2, x)
            u = g.matvec(1, -1, h)
            s = g.add((a, u))
            h = g.tanh(s)
        losses.append(g.sqnorm(h))
    root = g.add(losses)
    return g.finish(root, len(lengths), lengths=[int(x) for x in lengths], workload="rnn")


# --------------------------------------------------------------------------
# Config 2 / 3: BiLSTM tagger (optionally with a character model)
# --------------------------------------------------------------------------

def tagger_params(seed: int = SEED_BASE + 200, with_char: bool = False, vocab: int = 20000,
                  emb: int = 128, hidden: int = 256, mlp: int = 256, tags: int = 50,
                  char_vocab: int = 100, char_emb: int = 32, char_hidden: int = 64) -> Params:
    pb = ParamBuilder(np.random.default_rng(seed))
    pb.add("E", vocab, emb)
    lstm_params(pb, "fwd", emb, hidden)
    lstm_params(pb, "bwd", emb, hidden)
    pb.add("mlp.W", mlp, 2 * hidden)
    pb.add("mlp.b", mlp, 1)
    pb.add("out.W", tags, mlp)
    pb.add("out.b", tags, 1)
    if with_char:
        assert 2 * char_hidden == emb
        pb.add("Ec", char_vocab, char_emb)
        lstm_params(pb, "cfwd", char_emb, char_hidden)
        lstm_params(pb, "cbwd", char_emb, char_hidden)
    return pb.done()


def tagger_lengths(rng: np.random.Generator, n_sent: int, max_len: int = 60, p: float = 0.05):
    # L = min(max_len, 1 + G), G geometric on {0, 1, ...}; numpy's geometric starts at 1.
    return np.minimum(max_len, rng.geometric(p, size=n_sent))


def tagger_minibatch(params: Params, seed: int = SEED_BASE + 201, n_sent: int = 64,
                     with_char: bool = False, lengths=None, rare_from: int = 10000,
                     char_len_hi: int = 15) -> Graph:
    rng = np.random.default_rng(seed)
    P = params
    E = P.index("E")
    vocab, emb = P.mats[E].shape
    hidden = P.mats[P.index("fwd.Wh")].shape[1]
    tags = P.mats[P.index("out.W")].shape[0]
    pf = (P.index("fwd.Wx"), P.index("fwd.Wh"), P.index("fwd.b"))
    pbk = (P.index("bwd.Wx"), P.index("bwd.Wh"), P.index("bwd.b"))
    mw, mb = P.index("mlp.W"), P.index("mlp.b")
    ow, ob = P.index("out.W"), P.index("out.b")
    if with_char:
        Ec = P.index("Ec")
        cvocab = P.mats[Ec].shape[0]
        chid = P.mats[P.index("cfwd.Wh")].shape[1]
        cf = (P.index("cfwd.Wx"), P.index("cfwd.Wh"), P.index("cfwd.b"))
        cb = (P.index("cbwd.Wx"), P.index("cbwd.Wh"), P.index("cbwd.b"))
    if lengths is None:
        lengths = tagger_lengths(rng, n_sent)
    g = GraphBuilder(params)
    losses = []
    n_rare = 0
    for L in lengths:
        L = int(L)
        words = rng.integers(0, vocab, size=L)
        labels = rng.integers(0, tags, size=L)
        xs = []
        for w in words:
            if with_char and w >= rare_from:
                n_rare += 1
                clen = int(rng.integers(1, char_len_hi + 1))
                chars = rng.integers(0, cvocab, size=clen)
                cx = [g.lookup(Ec, int(c)) for c in chars]
                f, b = bilstm_states(g, cf, cb, chid, cx)
                xs.append(g.concat((f[-1], b[0])))
            else:
                xs.append(g.lookup(E, int(w)))
        f, b = bilstm_states(g, pf, pbk, hidden, xs)
        for t in range(L):
            z = g.concat((f[t], b[t]))
            hmid = g.tanh(g.matvec(mw, mb, z))
            sc = g.matvec(ow, ob, hmid)
            losses.append(g.pick_nls(sc, int(labels[t])))
    root = g.add(losses)
    return g.finish(root, len(lengths), lengths=[int(x) for x in lengths],
                    n_tokens=int(np.sum(lengths)), n_rare=n_rare,
                    workload="tagger_char" if with_char else "tagger")


# --------------------------------------------------------------------------
# Config 4: binary tree-LSTM classifier
# --------------------------------------------------------------------------

def tree_params(seed: int = SEED_BASE + 400, vocab: int = 20000, emb: int = 256,
                hidden: int = 256, classes: int = 5) -> Params:
    pb = ParamBuilder(np.random.default_rng(seed))
    pb.add("E", vocab, emb)
    pb.add("leaf.W", 3 * hidden, emb)
    pb.add("leaf.b", 3 * hidden, 1)
    pb.add("Ul", 5 * hidden, hidden)
    pb.add("Ur", 5 * hidden, hidden)
    pb.add("node.b", 5 * hidden, 1)
    pb.add("out.W", classes, hidden)
    pb.add("out.b", classes, 1)
    return pb.done()


def tree_minibatch(params: Params, seed: int = SEED_BASE + 401, n_trees: int = 64,
                   leaves_lo: int = 2, leaves_hi: int = 50, leaf_counts=None) -> Graph:
    rng = np.random.default_rng(seed)
    P = params
    E = P.index("E")
    vocab = P.mats[E].shape[0]
    H = P.mats[P.index("Ul")].shape[1]
    classes = P.mats[P.index("out.W")].shape[0]
    lw, lb = P.index("leaf.W"), P.index("leaf.b")
    ul, ur, nb = P.index("Ul"), P.index("Ur"), P.index("node.b")
    ow, ob = P.index("out.W"), P.index("out.b")
    if leaf_counts is None:
        leaf_counts = rng.integers(leaves_lo, leaves_hi + 1, size=n_trees)
    g = GraphBuilder(params)

    def leaf():
        x = g.lookup(E, int(rng.integers(0, vocab)))
        s = g.matvec(lw, lb, x)
        i = g.sigmoid(g.slice(s, 0, H))
        o = g.sigmoid(g.slice(s, H, 2 * H))
        u = g.tanh(g.slice(s, 2 * H, 3 * H))
        c = g.cmult(i, u)
        h = g.cmult(o, g.tanh(c))
        return h, c

    def build(n):
        # post-order: left subtree, right subtree, then the composing node
        if n == 1:
            return leaf()
        k = int(rng.integers(1, n))
        hl, cl = build(k)
        hr, cr = build(n - k)
        s = g.add((g.matvec(ul, nb, hl), g.matvec(ur, -1, hr)))
        i = g.sigmoid(g.slice(s, 0, H))
        fl = g.sigmoid(g.slice(s, H, 2 * H))
        fr = g.sigmoid(g.slice(s, 2 * H, 3 * H))
        o = g.sigmoid(g.slice(s, 3 * H, 4 * H))
        u = g.tanh(g.slice(s, 4 * H, 5 * H))
        c = g.add((g.cmult(i, u), g.cmult(fl, cl), g.cmult(fr, cr)))
        h = g.cmult(o, g.tanh(c))
        return h, c

    losses = []
    for n in leaf_counts:
        h, _ = build(int(n))
        sc = g.matvec(ow, ob, h)
        losses.append(g.pick_nls(sc, int(rng.integers(0, classes))))
    root = g.add(losses)
    return g.finish(root, len(leaf_counts), leaf_counts=[int(x) for x in leaf_counts],
                    workload="tree")


# --------------------------------------------------------------------------
# Config 5: arc-standard transition parser
# --------------------------------------------------------------------------

def parser_params(seed: int = SEED_BASE + 500, vocab: int = 20000, emb: int = 128,
                  hidden: int = 128, mlp: int = 512, actions: int = 3) -> Params:
    pb = ParamBuilder(np.random.default_rng(seed))
    pb.add("E", vocab, emb)
    lstm_params(pb, "fwd", emb, hidden)
    lstm_params(pb, "bwd", emb, hidden)
    pb.add("mlp.W", mlp, 8 * hidden)
    pb.add("mlp.b", mlp, 1)
    pb.add("out.W", actions, mlp)
    pb.add("out.b", actions, 1)
    return pb.done()


SHIFT, LEFT_ARC, RIGHT_ARC = 0, 1, 2


def parser_minibatch(params: Params, seed: int = SEED_BASE + 501, n_sent: int = 64,
                     len_lo: int = 5, len_hi: int = 50, lengths=None) -> Graph:
    """Arc-standard without composition: stack items are word positions; a sentence
    of n words takes n shifts and n-1 arcs.  At every step the features (top three
    stack items and first buffer item, read before the action) feed an MLP whose
    3-way softmax is trained on the sampled action."""
    rng = np.random.default_rng(seed)
    P = params
    E = P.index("E")
    vocab = P.mats[E].shape[0]
    hidden = P.mats[P.index("fwd.Wh")].shape[1]
    pf = (P.index("fwd.Wx"), P.index("fwd.Wh"), P.index("fwd.b"))
    pbk = (P.index("bwd.Wx"), P.index("bwd.Wh"), P.index("bwd.b"))
    mw, mb = P.index("mlp.W"), P.index("mlp.b")
    ow, ob = P.index("out.W"), P.index("out.b")
    if lengths is None:
        lengths = rng.integers(len_lo, len_hi + 1, size=n_sent)
    g = GraphBuilder(params)
    losses = []
    n_steps = 0
    for n in lengths:
        n = int(n)
        words = rng.integers(0, vocab, size=n)
        xs = [g.lookup(E, int(w)) for w in words]
        f, b = bilstm_states(g, pf, pbk, hidden, xs)
        v = [g.concat((f[t], b[t])) for t in range(n)]
        empty = g.input(np.zeros(2 * hidden, np.float32))
        stack: list = []
        buf = 0
        while not (buf == n and len(stack) == 1):
            valid = []
            if buf < n:
                valid.append(SHIFT)
            if len(stack) >= 2:
                valid.extend((LEFT_ARC, RIGHT_ARC))
            act = int(valid[int(rng.integers(0, len(valid)))])
            feats = [v[stack[-k]] if len(stack) >= k else empty for k in (1, 2, 3)]
            feats.append(v[buf] if buf < n else empty)
            z = g.concat(feats)
            hmid = g.tanh(g.matvec(mw, mb, z))
            sc = g.matvec(ow, ob, hmid)
            losses.append(g.pick_nls(sc, act))
            n_steps += 1
            if act == SHIFT:
                stack.append(buf)
                buf += 1
            elif act == LEFT_ARC:
                del stack[-2]
            else:
                del stack[-1]
    root = g.add(losses)
    return g.finish(root, len(lengths), lengths=[int(x) for x in lengths], n_steps=n_steps,
                    workload="parser")


# --------------------------------------------------------------------------
# Registry used by tests and bench
# --------------------------------------------------------------------------

# --------------------------------------------------------------------------
# Extra workload: the equal-length synthetic sequence labeler of Section 4.1
# --------------------------------------------------------------------------

def sync_tagger_params(seed: int = SEED_BASE + 600, vocab: int = 1000, emb: int = 200,
                       hidden: int = 256, tags: int = 300) -> Params:
    """Two stacked BiLSTM layers of `hidden` units per direction over `emb`-dimensional
    embeddings, then a linear layer to `tags` classes (the sizes Section 4.1 states)."""
    pb = ParamBuilder(np.random.default_rng(seed))
    pb.add("E", vocab, emb)
    lstm_params(pb, "l1f", emb, hidden)
    lstm_params(pb, "l1b", emb, hidden)
    lstm_params(pb, "l2f", 2 * hidden, hidden)
    lstm_params(pb, "l2b", 2 * hidden, hidden)
    pb.add("out.W", tags, 2 * hidden)
    pb.add("out.b", tags, 1)
    return pb.done()


def sync_tagger_minibatch(params: Params, seed: int = SEED_BASE + 601, n_sent: int = 64,
                          length: int = 40) -> Graph:
    """Every sequence has the same length (the case in which batching by hand is easiest)."""
    rng = np.random.default_rng(seed)
    P = params
    E = P.index("E")
    vocab = P.mats[E].shape[0]
    hidden = P.mats[P.index("l1f.Wh")].shape[1]
    tags = P.mats[P.index("out.W")].shape[0]
    layers = [tuple((P.index(f"{n}.Wx"), P.index(f"{n}.Wh"), P.index(f"{n}.b")) for n in pair)
              for pair in (("l1f", "l1b"), ("l2f", "l2b"))]
    ow, ob = P.index("out.W"), P.index("out.b")
    g = GraphBuilder(params)
    losses = []
    for _ in range(n_sent):
        words = rng.integers(0, vocab, size=length)
        labels = rng.integers(0, tags, size=length)
        xs = [g.lookup(E, int(w)) for w in words]
        for pf, pbk in layers:
            f, b = bilstm_states(g, pf, pbk, hidden, xs)
            xs = [g.concat((f[t], b[t])) for t in range(length)]
        for t in range(length):
            losses.append(g.pick_nls(g.matvec(ow, ob, xs[t]), int(labels[t])))
    root = g.add(losses)
    return g.finish(root, n_sent, lengths=[length] * n_sent, n_tokens=n_sent * length, workload="sync_tagger")


def sync_tagger_manual_labels(g: Graph) -> np.ndarray:
    """Batch labels as a program batched by hand over the sentences would group the nodes
    (Section 2): every sentence runs the same sequence of statements, so the k-th node of every
    sentence is one statement over a matrix with a column per sentence.  The label of a node is
    its index in its sentence's sequence; the closing sum over all losses comes last."""
    n = int(g.op.shape[0])
    per, rest = divmod(n - 1, g.n_instances)
    if rest:
        raise ValueError("sentences of different structure: no statement-wise batching")
    lab = np.arange(n, dtype=np.int32) % per
    lab[n - 1] = per
    return lab


def _sized(fn, key):
    """Minibatch generator with an optional instance count (None: the configuration's own)."""
    def batch(p, j=0, n=None, **kw):
        if n is not None:
            kw[key] = int(n)
        return fn(p, j, **kw)
    return batch


CONFIGS = {
    "rnn": dict(index=1, params=lambda: rnn_params(SEED_BASE + 100),
                batch=_sized(lambda p, j, **kw: rnn_minibatch(p, SEED_BASE + 101 + j, **kw), "n_inst")),
    "tagger": dict(index=2, params=lambda: tagger_params(SEED_BASE + 200),
                   batch=_sized(lambda p, j, **kw: tagger_minibatch(p, SEED_BASE + 201 + j, **kw), "n_sent")),
    "tagger_char": dict(index=3, params=lambda: tagger_params(SEED_BASE + 300, with_char=True),
                        batch=_sized(lambda p, j, **kw: tagger_minibatch(p, SEED_BASE + 301 + j, with_char=True, **kw),
                                     "n_sent")),
    "tree": dict(index=4, params=lambda: tree_params(SEED_BASE + 400),
                 batch=_sized(lambda p, j, **kw: tree_minibatch(p, SEED_BASE + 401 + j, **kw), "n_trees")),
    "parser": dict(index=5, params=lambda: parser_params(SEED_BASE + 500),
                   batch=_sized(lambda p, j, **kw: parser_minibatch(p, SEED_BASE + 501 + j, **kw), "n_sent")),
    # not one of the five listed configurations: Section 4.1's synthetic benchmark (index 0)
    "sync_tagger": dict(index=0, params=lambda: sync_tagger_params(SEED_BASE + 600),
                        batch=_sized(lambda p, j, **kw: sync_tagger_minibatch(p, SEED_BASE + 601 + j, **kw), "n_sent")),
}


def make(config: str, j: int = 0):
    c = CONFIGS[config]
    p = c["params"]()
    return p, c["batch"](p, j)


def random_dag(seed: int, n_nodes: int = 40, dim: int = 6, n_tables: int = 1):
    """Small random graph over every op, for oracle pins and edge-case parity."""
    rng = np.random.default_rng(seed)
    pb = ParamBuilder(rng, std=0.5)
    pb.add("E", 7, dim)
    pb.add("W", dim, dim)
    pb.add("b", dim, 1)
    pb.add("W2", 2 * dim, dim)
    pb.add("Wc", 5, dim)
    pb.add("bc", 5, 1)
    params = pb.done()
    g = GraphBuilder(params)
    vecs = {dim: [g.input(rng.standard_normal(dim)), g.lookup(0, int(rng.integers(0, 7))),
                  g.lookup(0, int(rng.integers(0, 7)))]}
    scalars = []

    def pick(d):
        pool = vecs[d]
        return pool[int(rng.integers(0, len(pool)))]

    while len(g.op) < n_nodes:
        r = int(rng.integers(0, 12))
        if r == 0:
            v = g.input(rng.standard_normal(dim))
        elif r == 1:
            v = g.lookup(0, int(rng.integers(0, 7)))
        elif r == 2:
            v = g.matvec(1, 2 if rng.integers(0, 2) else -1, pick(dim))
        elif r == 3:
            k = int(rng.integers(2, 5))
            v = g.add([pick(dim) for _ in range(k)])
        elif r == 4:
            v = g.cmult(pick(dim), pick(dim))
        elif r == 5:
            v = g.tanh(pick(dim))
        elif r == 6:
            v = g.sigmoid(pick(dim))
        elif r == 7:
            w = g.matvec(3, -1, pick(dim))
            lo = int(rng.integers(0, dim))
            v = g.slice(w, lo, lo + dim)
        elif r == 8:
            a = g.slice(pick(dim), 0, dim // 2)
            b = g.slice(pick(dim), dim // 2, dim)
            v = g.concat((a, b))
        elif r == 9:
            sc = g.matvec(4, 5, pick(dim))
            scalars.append(g.pick_nls(sc, int(rng.integers(0, 5))))
            continue
        elif r == 10:
            scalars.append(g.sqnorm(pick(dim)))
            continue
        else:
            v = g.concat((pick(dim), pick(dim)))
            v = g.matvec(1, -1, g.slice(v, 2, 2 + dim))
        vecs[dim].append(v)
    scalars.append(g.sqnorm(vecs[dim][-1]))
    root = g.add(scalars)
    return params, g.finish(root, 1, workload="random_dag")
