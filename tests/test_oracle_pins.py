"""Pins of the CPU oracle interpreter against things other than itself: hand-computed tiny
graphs, finite differences, closed forms, NumPy/SciPy library routines, a padded+masked
manual batching of the RNN (Section 2), and batch-by-batch NumPy evaluation of a schedule."""
import math

import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import schedule as S
from oracle.interp import Oracle
from paper_1705_07860_amd import workloads as wl
from tests.helpers import numpy_batched_forward, rel_err


def _params(mats):
    return wl.Params([np.asarray(m, np.float32) for m in mats], [f"p{i}" for i in range(len(mats))])


def _run(g, p):
    o = Oracle(g, p, "f64")
    o.forward()
    o.backward(g.root)
    return o


# ---------------------------------------------------------------- hand graphs (values by hand)

def test_hand_one_step_rnn_scalar():
    # w = u = 0  =>  h = tanh(b), L = tanh(b)^2, dL/db = 2 tanh(b) (1 - tanh(b)^2)
    b = 0.75   # exactly representable in fp32
    p = _params([[[0.0]], [[0.0]], [[b]]])
    g = wl.rnn_minibatch(p, lengths=[1], seed=3)
    o = _run(g, p)
    t = math.tanh(b)
    assert abs(o.value(g.root)[0] - t * t) < 1e-15
    assert abs(o.param_grad(2)[0, 0] - 2 * t * (1 - t * t)) < 1e-15
    # dL/dW = dL/ds * x, dL/dU = dL/ds * h0 = 0
    x = float(g.payload[1])
    assert abs(o.param_grad(0)[0, 0] - 2 * t * (1 - t * t) * x) < 1e-12
    assert o.param_grad(1)[0, 0] == 0.0


def test_hand_matvec_2x2_numbers():
    # W=[[1,2],[3,4]], x=[5,6], b=[.5,-.5]: y=[17.5,38.5]; L=|y|^2=1788.5
    p = _params([[[1, 2], [3, 4]], [[0.5], [-0.5]]])
    gb = wl.GraphBuilder(p)
    x = gb.input([5, 6])
    y = gb.matvec(0, 1, x)
    L = gb.sqnorm(y)
    g = gb.finish(L)
    o = _run(g, p)
    assert np.allclose(o.value(y), [17.5, 38.5], atol=0, rtol=0)
    assert o.value(L)[0] == 1788.5
    assert np.array_equal(o.node_grad(y), [35.0, 77.0])
    assert np.array_equal(o.node_grad(x), [266.0, 378.0])          # W^T dy
    assert np.array_equal(o.param_grad(0), [[175.0, 210.0], [385.0, 462.0]])  # dy x^T
    assert np.array_equal(o.param_grad(1).reshape(-1), [35.0, 77.0])


def test_hand_pick_nls():
    # x = [0, ln2, ln3]: softmax = [1/6, 1/3, 1/2]; -log p[1] = ln 3
    p = _params([])
    gb = wl.GraphBuilder(p)
    x = gb.input([0.0, math.log(2), math.log(3)])
    L = gb.pick_nls(x, 1)
    g = gb.finish(L)
    o = _run(g, p)
    xv = g.payload.astype(np.float64)
    sm = np.exp(xv) / np.exp(xv).sum()
    assert abs(o.value(L)[0] - math.log(3)) < 1e-7       # inputs are rounded to fp32
    assert np.allclose(o.node_grad(x), sm - np.array([0, 1, 0]), atol=1e-15)
    assert np.allclose(o.node_grad(x), [1 / 6, 1 / 3 - 1, 1 / 2], atol=1e-7)
    assert abs(o.node_grad(x).sum()) < 1e-15             # rows of softmax - e_y sum to zero


@pytest.mark.parametrize("margin", [0.5, 8.0, 40.0, 60.0, 100.0])
def test_pick_nls_two_classes_is_softplus_also_for_confident_rows(margin):
    # Two classes: -log softmax(x)[y] = log(1 + exp(x_other - x_y)) and the gradient is
    # (-q, q) with q = 1 / (1 + exp(x_y - x_other)) -- closed forms that stay accurate when the
    # prediction is confident (margin 60: loss = log1p(e^-60) = 8.7e-27, far below the 1e-16
    # where the textbook logsumexp(x) - x_y rounds to zero) and when it is confidently wrong.
    p = _params([])
    for label, other in ((0, 1), (1, 0)):
        for sign in (+1.0, -1.0):
            xs = [0.0, 0.0]
            xs[other] = -sign * margin          # exactly representable in fp32
            gb = wl.GraphBuilder(p)
            x = gb.input(xs)
            L = gb.pick_nls(x, label)
            g = gb.finish(L)
            o = _run(g, p)
            z = xs[other] - xs[label]
            loss = math.log1p(math.exp(z)) if z <= 0 else z + math.log1p(math.exp(-z))
            q = 1.0 / (1.0 + math.exp(-z))
            assert abs(o.value(L)[0] - loss) <= 1e-14 * loss
            want = np.zeros(2)
            want[label], want[other] = -q, q
            assert np.allclose(o.node_grad(x), want, rtol=1e-14, atol=0)


def test_pick_nls_confident_row_of_many_classes():
    # K classes, one at 0 and K - 1 at -50: loss = log1p((K-1) e^-50), label gradient
    # -(K-1) e^-50 / (1 + (K-1) e^-50), every other entry e^-50 / (1 + (K-1) e^-50)
    K = 7
    p = _params([])
    gb = wl.GraphBuilder(p)
    x = gb.input([-50.0, -50.0, 0.0] + [-50.0] * (K - 3))
    L = gb.pick_nls(x, 2)
    g = gb.finish(L)
    o = _run(g, p)
    t = (K - 1) * math.exp(-50.0)
    assert abs(o.value(L)[0] - math.log1p(t)) <= 1e-14 * math.log1p(t)
    want = np.full(K, math.exp(-50.0) / (1 + t))
    want[2] = -t / (1 + t)
    assert np.allclose(o.node_grad(x), want, rtol=1e-13, atol=0)


def test_hand_concat_slice_identity_and_fanout():
    p = _params([])
    gb = wl.GraphBuilder(p)
    a = gb.input([1.0, 2.0])
    b = gb.input([3.0, 4.0, 5.0])
    c = gb.concat((a, b))
    s = gb.slice(c, 2, 5)            # == b
    t = gb.add((a, a))               # 2a, da = 2g
    z = gb.concat((t, s))            # [2,4,3,4,5]
    w = gb.input([1.0, 10.0, 100.0, 1000.0, 10000.0])
    L1 = gb.sqnorm(gb.cmult(z, w))   # sum (z_i w_i)^2
    g = gb.finish(gb.add((L1,)))
    o = _run(g, p)
    assert np.array_equal(o.value(c), [1, 2, 3, 4, 5])
    assert np.array_equal(o.value(s), [3, 4, 5])
    assert np.array_equal(o.value(z), [2, 4, 3, 4, 5])
    wv = np.array([1.0, 10.0, 100.0, 1000.0, 10000.0])
    zv = np.array([2.0, 4, 3, 4, 5])
    assert o.value(g.root)[0] == float(np.sum((zv * wv) ** 2))
    dz = 2 * zv * wv * wv
    assert np.array_equal(o.node_grad(z), dz)
    assert np.array_equal(o.node_grad(a), 2 * dz[:2])      # through ADD(a, a)
    assert np.array_equal(o.node_grad(b), dz[2:])          # through SLICE of CONCAT
    assert np.array_equal(o.node_grad(w), 2 * zv * zv * wv)


def test_hand_sigmoid_tanh_cmult():
    p = _params([])
    gb = wl.GraphBuilder(p)
    x = gb.input([0.0])
    s = gb.sigmoid(x)               # 0.5, ds/dx = 0.25
    t = gb.tanh(x)                  # 0, dt/dx = 1
    y = gb.input([3.0])
    m = gb.cmult(s, y)              # 1.5
    q = gb.add((m, t, y))           # 4.5 ; dq/dx = 0.25*3 + 1 = 1.75 ; dq/dy = .5 + 1
    L = gb.slice(q, 0, 1)
    g = gb.finish(L)
    o = _run(g, p)
    assert o.value(q)[0] == 4.5
    assert o.node_grad(x)[0] == 1.75
    assert o.node_grad(y)[0] == 1.5


def test_unreached_nodes_have_zero_gradient():
    p = _params([])
    gb = wl.GraphBuilder(p)
    a = gb.input([1.0, 2.0])
    dead = gb.tanh(a)
    L = gb.sqnorm(a)
    g = gb.finish(L)
    o = _run(g, p)
    assert np.array_equal(o.node_grad(dead), [0, 0])
    assert np.array_equal(o.node_grad(a), [2, 4])


# ---------------------------------------------------------------- finite differences

def _fd_check(g, p, entries_per_param=None, h=1e-5, tol=1e-6, seed=0):
    o = _run(g, p)
    base = o.pdata.copy()
    rng = np.random.default_rng(seed)
    for pid in range(len(p.mats)):
        size = int(o.p_off[pid + 1] - o.p_off[pid])
        idx = np.arange(size) if entries_per_param is None or size <= entries_per_param \
            else rng.choice(size, entries_per_param, replace=False)
        fd = np.zeros(len(idx))
        for k, e in enumerate(idx):
            for sgn in (+1, -1):
                q = base.copy()
                q[o.p_off[pid] + e] += sgn * h
                o2 = Oracle(g, p, "f64")
                o2.set_params(q)
                o2.forward()
                fd[k] += sgn * o2.value(g.root)[0]
            fd[k] /= 2 * h
        an = o.param_grad(pid).reshape(-1)[idx]
        scale = max(np.max(np.abs(o.param_grad(pid))), 1e-30)
        assert np.max(np.abs(fd - an)) / scale < tol, (pid, p.names[pid], fd, an)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_finite_differences_random_dag_every_parameter_entry(seed):
    p, g = wl.random_dag(seed, n_nodes=45, dim=4)
    ops = set(int(x) for x in g.op)
    _fd_check(g, p)
    assert len(ops) >= 9


def test_finite_differences_cover_every_op():
    seen = set()
    for seed in (1, 2, 3):
        _, g = wl.random_dag(seed, n_nodes=45, dim=4)
        seen |= set(int(x) for x in g.op)
    assert seen == set(range(11))


def test_finite_differences_rnn_config():
    p, g = wl.make("rnn")
    _fd_check(g, p, entries_per_param=12, tol=1e-6)


@pytest.mark.parametrize("name", ["tagger", "tagger_char", "tree", "parser"])
def test_directional_finite_difference_small_instance_of_each_config(name):
    # <grad, delta> against (L(theta + h delta) - L(theta - h delta)) / 2h along a random direction
    c = wl.CONFIGS[name]
    p = c["params"]()
    kw = dict(with_char=True) if name == "tagger_char" else {}
    gen = {"tagger": wl.tagger_minibatch, "tagger_char": wl.tagger_minibatch,
           "tree": wl.tree_minibatch, "parser": wl.parser_minibatch}[name]
    small = {"tagger": dict(lengths=[5, 1, 9]), "tagger_char": dict(lengths=[4, 7]),
             "tree": dict(leaf_counts=[2, 7, 4]), "parser": dict(lengths=[5, 8])}[name]
    g = gen(p, seed=77, **small, **kw)
    o = _run(g, p)
    rng = np.random.default_rng(5)
    delta = rng.standard_normal(o.pdata.shape[0])
    h = 1e-6
    vals = []
    for sgn in (+1, -1):
        o2 = Oracle(g, p, "f64")
        o2.set_params(o.pdata + sgn * h * delta)
        o2.forward()
        vals.append(o2.value(g.root)[0])
    fd = (vals[0] - vals[1]) / (2 * h)
    an = float(np.dot(o.pgrad[:delta.shape[0]], delta))
    assert abs(fd - an) / max(abs(an), 1e-30) < 1e-6, (fd, an)


# ---------------------------------------------------------------- closed forms at config scale

def _zero_output_layer(p):
    mats = [m.copy() for m in p.mats]
    mats[p.index("out.W")][:] = 0
    mats[p.index("out.b")][:] = 0
    return wl.Params(mats, p.names)


@pytest.mark.parametrize("name,K", [("tagger", 50), ("tree", 5), ("parser", 3)])
def test_zero_output_layer_gives_uniform_softmax(name, K):
    p0 = wl.CONFIGS[name]["params"]()
    p = _zero_output_layer(p0)
    gen = {"tagger": lambda: wl.tagger_minibatch(p, seed=11, n_sent=6),
           "tree": lambda: wl.tree_minibatch(p, seed=11, n_trees=6),
           "parser": lambda: wl.parser_minibatch(p, seed=11, n_sent=4)}[name]
    g = gen()
    o = _run(g, p)
    loss_nodes = np.nonzero(g.op == wl.OP_PICK_NLS)[0]
    for v in loss_nodes[:50]:
        assert abs(o.value(int(v))[0] - math.log(K)) < 1e-14
    assert abs(o.value(g.root)[0] - len(loss_nodes) * math.log(K)) < 1e-9
    hist = np.bincount(g.aux0[loss_nodes], minlength=K)
    db = o.param_grad(p.index("out.b")).reshape(-1)
    assert np.allclose(db, len(loss_nodes) / K - hist, atol=1e-10)
    # nothing upstream of a zero output matrix receives gradient
    for nm in p.names:
        if nm not in ("out.W", "out.b"):
            assert not np.any(o.param_grad(p.index(nm))), nm


def test_rnn_without_recurrence_depends_only_on_last_input():
    p0 = wl.rnn_params()
    mats = [m.copy() for m in p0.mats]
    mats[1][:] = 0                                   # U = 0
    p = wl.Params(mats, p0.names)
    g = wl.rnn_minibatch(p, seed=9)
    o = _run(g, p)
    W, b = mats[0].astype(np.float64), mats[2].astype(np.float64).reshape(-1)
    tanh_nodes = np.nonzero(g.op == wl.OP_TANH)[0]
    sq = np.nonzero(g.op == wl.OP_SQNORM)[0]
    total = 0.0
    for s in sq:
        hn = int(g.in_idx[g.in_off[s]])
        add = int(g.in_idx[g.in_off[hn]])
        mv = int(g.in_idx[g.in_off[add]])            # MATVEC(W, b; x_n)
        xn = int(g.in_idx[g.in_off[mv]])
        x = g.payload[g.aux0[xn]:g.aux0[xn] + 32].astype(np.float64)
        ref = np.tanh(W @ x + b)
        assert np.allclose(o.value(hn), ref, atol=1e-14)
        total += float(ref @ ref)
    assert abs(o.value(g.root)[0] - total) < 1e-12
    assert len(tanh_nodes) == sum(g.meta["lengths"])


# ---------------------------------------------------------------- library special cases

def test_padded_masked_manual_batching_matches_rnn_config():
    """Section 2's manually batched evaluation (pad inputs to n_max, keep H as a d x b matrix,
    mask the loss at each sequence's final position) computes the same loss."""
    p, g = wl.make("rnn")
    o = _run(g, p)
    W, U, b = [m.astype(np.float64) for m in p.mats]
    lengths = g.meta["lengths"]
    nmax, B = max(lengths), len(lengths)
    X = np.zeros((nmax, 32, B))
    # payload layout per instance: h0 (32 zeros), then x_1..x_n
    off = 0
    for i, n in enumerate(lengths):
        off += 32
        for t in range(n):
            X[t, :, i] = g.payload[off:off + 32]
            off += 32
    M = np.zeros((B, nmax))
    for i, n in enumerate(lengths):
        M[i, n - 1] = 1
    H = np.zeros((32, B))
    L = 0.0
    for t in range(nmax):
        H = np.tanh(W @ X[t] + U @ H + b)            # b broadcasts over columns
        L += float(np.sum((H * M[:, t][None, :]) ** 2))
    assert abs(L - o.value(g.root)[0]) < 1e-10 * abs(L)


def test_matvec_batch_equals_numpy_gemm_and_logsumexp():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((7, 5)).astype(np.float32)
    b = rng.standard_normal((7, 1)).astype(np.float32)
    p = _params([W, b])
    gb = wl.GraphBuilder(p)
    X = rng.standard_normal((9, 5)).astype(np.float32)
    ys, ls = [], []
    for r in range(9):
        y = gb.matvec(0, 1, gb.input(X[r]))
        ys.append(y)
        ls.append(gb.pick_nls(y, r % 7))
    g = gb.finish(gb.add(ls))
    o = _run(g, p)
    Y = X.astype(np.float64) @ W.astype(np.float64).T + b.astype(np.float64).reshape(1, -1)
    for r in range(9):
        assert np.allclose(o.value(ys[r]), Y[r], atol=1e-14)
        assert abs(o.value(ls[r])[0] - (logsumexp(Y[r]) - Y[r, r % 7])) < 1e-13


@pytest.mark.parametrize("name", ["rnn", "tagger", "tagger_char", "tree", "parser"])
def test_batched_numpy_evaluation_of_schedule_equals_node_at_a_time(name, workload_cache):
    """Batched and unbatched evaluation agree (Section 4.1 footnote): run the reference
    schedule batch by batch with NumPy array ops and compare every node value."""
    p, g, o = workload_cache(name)
    bo, ids, bd = S.by_depth(g)
    vals = numpy_batched_forward(g, p, bo, ids)
    flat = np.concatenate(vals)
    assert flat.shape == o.val.shape
    assert rel_err(flat, o.val) < 1e-12
    assert abs(vals[g.root][0] - o.value(g.root)[0]) <= 1e-12 * abs(o.value(g.root)[0])


# ---------------------------------------------------------------- metamorphic

def test_permuting_and_duplicating_instances():
    p = wl.rnn_params()
    g1 = wl.rnn_minibatch(p, seed=21, lengths=[3, 5, 4])
    o1 = _run(g1, p)
    # the same three instances, duplicated: loss and gradients double
    rng_lengths = [3, 5, 4]
    gb = wl.GraphBuilder(p)
    rng = np.random.default_rng(21)
    seqs = [[rng.standard_normal(32) for _ in range(n)] for n in rng_lengths]

    def build(order):
        gb = wl.GraphBuilder(p)
        losses = []
        for i in order:
            h = gb.input(np.zeros(32))
            for x in seqs[i]:
                h = gb.tanh(gb.add((gb.matvec(0, 2, gb.input(x)), gb.matvec(1, -1, h))))
            losses.append(gb.sqnorm(h))
        return gb.finish(gb.add(losses), len(order))

    oa = _run(build([0, 1, 2]), p)
    assert abs(oa.value(build([0, 1, 2]).root)[0] - o1.value(g1.root)[0]) < 1e-12
    gp = build([2, 0, 1])
    op_ = _run(gp, p)
    assert abs(op_.value(gp.root)[0] - oa.val[-1]) < 1e-12
    assert rel_err(op_.pgrad, oa.pgrad) < 1e-12
    gd = build([0, 1, 2, 1])
    od = _run(gd, p)
    single = _run(build([1]), p)
    assert rel_err(od.pgrad, oa.pgrad + single.pgrad) < 1e-12


def test_float_build_tracks_double_build(workload_cache):
    p, g, o = workload_cache("rnn")
    o32 = Oracle(g, p, "f32")
    o32.forward()
    o32.backward(g.root)
    assert rel_err(o32.val, o.val) < 1e-5
    assert rel_err(o32.pgrad, o.pgrad) < 1e-5


def test_signature_examples_from_the_paper():
    """tests/golden/signature_examples.txt restates the signature examples of Section 3.2 and
    Appendix A; for every line two nodes that differ only in a 'must not depend on' field share
    a signature and nodes that differ in a 'must contain' field do not."""
    import os
    from oracle import schedule as S
    from paper_1705_07860_amd import workloads as wl
    path = os.path.join(os.path.dirname(__file__), "golden", "signature_examples.txt")
    rows = [ln.split("|") for ln in open(path) if ln.strip() and not ln.startswith("#")]
    kinds = [r[0].strip() for r in rows]
    assert kinds == ["tanh", "slice", "matvec", "affine"] and all(len(r) == 4 for r in rows)
    rng = np.random.default_rng(5)
    pb = wl.ParamBuilder(rng)
    A1, A2 = pb.add("A1", 256, 256), pb.add("A2", 256, 256)
    B1 = pb.add("B1", 256, 400)
    y1, y2 = pb.add("y1", 256, 1), pb.add("y2", 256, 1)
    p = pb.done()
    gb = wl.GraphBuilder(p)
    u, v = gb.input(np.ones(256)), gb.input(np.zeros(256))
    w = gb.input(np.ones(400))
    big1, big2 = gb.input(np.ones(500)), gb.input(np.zeros(500))
    nodes = dict(
        tanh_a=gb.tanh(u), tanh_b=gb.tanh(v), sig=gb.sigmoid(u),
        sl_a=gb.slice(big1, 100, 200), sl_b=gb.slice(big2, 100, 200), sl_range=gb.slice(big1, 100, 201),
        sl_size=gb.slice(gb.input(np.ones(400)), 100, 200),
        mv_a=gb.matvec(A1, -1, u), mv_b=gb.matvec(A1, -1, v), mv_param=gb.matvec(A2, -1, u), mv_size=gb.matvec(B1, -1, w),
        af_a=gb.matvec(A1, y1, u), af_b=gb.matvec(A1, y1, v), af_bias=gb.matvec(A1, y2, u), af_none=gb.matvec(A1, -1, u),
    )
    g = gb.finish(gb.sqnorm(nodes["tanh_a"]), 1)
    s = {k: S.signature(g, n) for k, n in nodes.items()}
    same = [("tanh_a", "tanh_b"), ("sl_a", "sl_b"), ("mv_a", "mv_b"), ("af_a", "af_b"), ("mv_a", "af_none")]
    differ = [("tanh_a", "sig"), ("sl_a", "sl_range"), ("sl_a", "sl_size"), ("mv_a", "mv_param"), ("mv_a", "mv_size"),
              ("af_a", "af_bias"), ("af_a", "mv_a")]
    for a, b in same:
        assert s[a] == s[b], (a, b)
    for a, b in differ:
        assert s[a] != s[b], (a, b)


def test_gradient_step_lowers_the_loss_to_first_order():
    """The oracle's update theta - lr * grad, pinned by what a gradient step must do: for a small
    lr the loss drops by lr * |grad|^2 up to second-order terms (checked at two step sizes: the
    relative gap to the linear prediction shrinks with lr)."""
    from oracle.interp import Oracle
    from paper_1705_07860_amd import workloads as wl
    p = wl.rnn_params()
    g = wl.rnn_minibatch(p, seed=11, lengths=[3, 5, 4])
    o = Oracle(g, p, "f64")
    o.forward()
    o.backward(g.root)
    loss0 = float(o.value(g.root)[0])
    g2 = float(np.sum(o.pgrad[:int(o.p_off[-1])] ** 2))
    gaps = []
    for lr in (1e-4, 1e-5):
        new = o.sgd_params(lr)
        o2 = Oracle(g, p, "f64")
        o2.set_params(np.concatenate([m.ravel() for m in new]))
        o2.forward()
        drop = loss0 - float(o2.value(g.root)[0])
        assert drop > 0
        gaps.append(abs(drop - lr * g2) / (lr * g2))
    assert gaps[0] < 1e-2 and gaps[1] < gaps[0]
