"""Pins of the oracle's reference scheduler: invariants checked by an independent validator,
the closed-form depth-based schedule of the RNN workload, brute force on tiny graphs."""
import itertools

import numpy as np
import pytest

from oracle import schedule as S
from paper_1705_07860_amd import workloads as wl
from tests.helpers import longest_path_depths, sig_string, validate_schedule


@pytest.mark.parametrize("name", ["rnn", "tagger", "tree", "parser"])
def test_schedule_invariants_on_configs(name, workload_cache):
    p, g, _ = workload_cache(name)
    bo, ids, bd = S.by_depth(g)
    depth_of = validate_schedule(g, bo, ids, bd)
    assert np.array_equal(depth_of, S.depths(g))


def test_schedule_invariants_char_config_sample():
    p = wl.tagger_params(with_char=True)
    g = wl.tagger_minibatch(p, seed=5, n_sent=6, with_char=True)
    bo, ids, bd = S.by_depth(g)
    validate_schedule(g, bo, ids, bd)
    assert np.array_equal(longest_path_depths(g), S.depths(g))


def test_closed_form_schedule_of_rnn_chains():
    """With h_t = tanh(W x_t + U h_{t-1} + b) built as MATVEC, MATVEC, ADD, TANH: depth(h_t) = 3t;
    the U-product, sum and tanh batches of step t hold #{i : n_i >= t} nodes; every W-product
    sits in one depth-1 batch; the loss nodes of unequal-length sequences land at different
    depths (the weakness of depth-based batching named in Section 3.2)."""
    lengths = [3, 7, 7, 4, 10, 3, 5, 7]
    p = wl.rnn_params()
    g = wl.rnn_minibatch(p, seed=1, lengths=lengths)
    bo, ids, bd = S.by_depth(g)
    sizes = np.diff(bo)
    by = {}
    for b in range(len(bd)):
        h = int(ids[bo[b]])
        key = (int(bd[b]), int(g.op[h]), int(g.param[h]))
        assert key not in by
        by[key] = int(sizes[b])
    nmax = max(lengths)
    assert by[(0, wl.OP_INPUT, -1)] == len(lengths) + sum(lengths)
    assert by[(1, wl.OP_MATVEC, 0)] == sum(lengths)
    for t in range(1, nmax + 1):
        alive = sum(1 for n in lengths if n >= t)
        assert by[(3 * t - 2, wl.OP_MATVEC, 1)] == alive
        assert by[(3 * t - 1, wl.OP_ADD, -1)] == alive
        assert by[(3 * t, wl.OP_TANH, -1)] == alive
    for n in set(lengths):
        assert by[(3 * n + 1, wl.OP_SQNORM, -1)] == lengths.count(n)
    last = max(3 * n + 2 for n in lengths)
    assert by[(last, wl.OP_ADD, -1)] == 1
    assert len(bd) == 1 + 1 + 3 * nmax + len(set(lengths)) + 1
    # equal lengths: the loss nodes do batch together
    g2 = wl.rnn_minibatch(p, seed=1, lengths=[6] * 5)
    bo2, ids2, bd2 = S.by_depth(g2)
    sq = [b for b in range(len(bd2)) if g2.op[ids2[bo2[b]]] == wl.OP_SQNORM]
    assert len(sq) == 1 and bo2[sq[0] + 1] - bo2[sq[0]] == 5


@pytest.mark.parametrize("seed", range(8))
def test_brute_force_grouping_on_tiny_random_graphs(seed):
    """Two nodes share a batch exactly when their longest-path depths (by path enumeration)
    and their paper-style signature strings agree; checked for every pair."""
    p, g = wl.random_dag(100 + seed, n_nodes=12, dim=4)
    bo, ids, bd = S.by_depth(g)
    depth = longest_path_depths(g)
    batch_of = np.empty(g.n, np.int64)
    for b in range(len(bd)):
        batch_of[ids[bo[b]:bo[b + 1]]] = b
    for u, v in itertools.combinations(range(g.n), 2):
        same = depth[u] == depth[v] and sig_string(g, u) == sig_string(g, v)
        assert (batch_of[u] == batch_of[v]) == same, (u, v)
    validate_schedule(g, bo, ids, bd)


def test_signature_contents():
    p = wl.tagger_params()
    g = wl.tagger_minibatch(p, seed=3, lengths=[4, 2])
    look = [v for v in range(g.n) if g.op[v] == wl.OP_LOOKUP]
    assert len({S.signature(g, v) for v in look}) == 1          # row is not in the signature
    pick = [v for v in range(g.n) if g.op[v] == wl.OP_PICK_NLS]
    assert len({S.signature(g, v) for v in pick}) == 1          # label is not in the signature
    mv = [v for v in range(g.n) if g.op[v] == wl.OP_MATVEC]
    assert {(S.signature(g, v)[3], S.signature(g, v)[4]) for v in mv} == \
        {(int(g.param[v]), int(g.bias[v])) for v in mv}          # shared A and y are in it
    sl = [v for v in range(g.n) if g.op[v] == wl.OP_SLICE]
    assert len({S.signature(g, v) for v in sl}) == 4             # the range is in it


def test_no_batching_schedule():
    p, g = wl.make("rnn")
    bo, ids, bd = S.no_batching(g)
    assert np.array_equal(np.diff(bo), np.ones(g.n))
    assert np.array_equal(ids, np.arange(g.n))


def test_permuting_instances_permutes_the_schedule():
    p = wl.rnn_params()
    ga = wl.rnn_minibatch(p, seed=2, lengths=[3, 5])
    gb = wl.rnn_minibatch(p, seed=2, lengths=[5, 3])
    boa, _, bda = S.by_depth(ga)
    bob, _, bdb = S.by_depth(gb)
    assert np.array_equal(np.diff(boa), np.diff(bob))
    assert np.array_equal(bda, bdb)


# ---------------------------------------------------------------- agenda-based batching

@pytest.mark.parametrize("seed", range(8))
def test_agenda_replay_on_tiny_random_graphs(seed):
    from tests.helpers import validate_agenda_schedule
    p, g = wl.random_dag(300 + seed, n_nodes=14, dim=4)
    bo, ids, bs = S.by_agenda(g)
    validate_schedule(g, bo, ids, bs)          # partition, one signature per batch, operands earlier
    validate_agenda_schedule(g, bo, ids)


def test_agenda_replay_on_small_workloads():
    from tests.helpers import validate_agenda_schedule
    p = wl.tagger_params()
    g = wl.tagger_minibatch(p, seed=9, lengths=[3, 1, 4])
    bo, ids, bs = S.by_agenda(g)
    validate_schedule(g, bo, ids, bs)
    validate_agenda_schedule(g, bo, ids)
    tp = wl.tree_params()
    tg = wl.tree_minibatch(tp, seed=4, leaf_counts=[3, 5, 2])
    bo, ids, bs = S.by_agenda(tg)
    validate_schedule(tg, bo, ids, bs)
    validate_agenda_schedule(tg, bo, ids)


def test_agenda_batches_the_losses_of_unequal_chains():
    """Section 3.2's motivating case: with sequences of different lengths the loss nodes become
    available at different times; their signature has the largest average depth but one, so they
    wait until the recurrence is exhausted and form ONE batch (depth-based batching needs one per
    distinct length).  Closed form for h_t = tanh(W x_t + U h_{t-1} + b) built as MATVEC, MATVEC,
    ADD, TANH: inputs, all W products, then per step U product / sum / tanh over the sequences
    still alive, then all losses, then the final sum."""
    lengths = [3, 7, 7, 4, 10, 3, 5, 7]
    p = wl.rnn_params()
    g = wl.rnn_minibatch(p, seed=1, lengths=lengths)
    bo, ids, bs = S.by_agenda(g)
    sizes = np.diff(bo).tolist()
    ops = [(int(g.op[ids[bo[b]]]), int(g.param[ids[bo[b]]])) for b in range(len(bs))]
    nmax = max(lengths)
    expect_ops = [(wl.OP_INPUT, -1), (wl.OP_MATVEC, 0)]
    expect_sizes = [len(lengths) + sum(lengths), sum(lengths)]
    for t in range(1, nmax + 1):
        alive = sum(1 for n in lengths if n >= t)
        expect_ops += [(wl.OP_MATVEC, 1), (wl.OP_ADD, -1), (wl.OP_TANH, -1)]
        expect_sizes += [alive] * 3
    expect_ops += [(wl.OP_SQNORM, -1), (wl.OP_ADD, -1)]
    expect_sizes += [len(lengths), 1]
    assert ops == expect_ops and sizes == expect_sizes
    nb_depth = len(S.by_depth(g)[2])
    assert len(bs) == nb_depth - (len(set(lengths)) - 1)


@pytest.mark.parametrize("name", ["rnn", "tagger", "tree", "parser"])
def test_agenda_invariants_on_configs(name, workload_cache):
    p, g, _ = workload_cache(name)
    bo, ids, bs = S.by_agenda(g)
    validate_schedule(g, bo, ids, bs)
    # (the heuristic does not always give fewer batches than depth-based batching: the tree
    # workload gets more)
    print(name, "batches: agenda", len(bs), "depth", len(S.by_depth(g)[2]))


def test_generators_take_an_instance_count_and_keep_their_default():
    """The benchmark's sweep asks the generators for other instance counts; without a count they
    give the configuration as listed (same arrays as before for the same seed)."""
    from paper_1705_07860_amd import workloads as wl
    for name, default in (("rnn", 8), ("tagger", 64), ("tree", 64), ("parser", 64)):
        cfg = wl.CONFIGS[name]
        p = cfg["params"]()
        g0 = cfg["batch"](p, 0)
        g1 = cfg["batch"](p, 0, n=None)
        assert g0.n_instances == default and g0.n == g1.n and np.array_equal(g0.in_idx, g1.in_idx)
        small = cfg["batch"](p, 0, n=3)
        assert small.n_instances == 3 and small.n < g0.n
        bo, ids, bd = S.by_depth(small)
        assert np.array_equal(np.sort(ids), np.arange(small.n))


def test_signature_as_the_paper_words_it_is_coarser_or_equal():
    """Section 3.2 identifies component-wise operations by their name alone; the library (and the
    reference scheduler) add operand shapes to every signature.  The printed form can only merge
    batches: every batch of the shape-aware schedule lies inside one batch of the printed one, the
    counts agree where all component-wise work of a depth has one width (RNN chains), and a graph
    with two widths at one depth shows the difference."""
    from oracle import schedule as S
    from paper_1705_07860_amd import workloads as wl
    p, g = wl.make("rnn", 0)
    a, b = S.by_depth(g), S.by_depth(g, sig=S.signature_as_printed)
    assert len(a[2]) == len(b[2]) == 31
    p = wl.Params([], [])
    gb = wl.GraphBuilder(p)
    xs = [gb.input(np.ones(4)), gb.input(np.ones(6))]
    ts = [gb.tanh(x) for x in xs]                 # same depth, two widths
    root = gb.add([gb.sqnorm(t) for t in ts])
    g = gb.finish(root, 1)
    a, b = S.by_depth(g), S.by_depth(g, sig=S.signature_as_printed)
    assert len(a[2]) == len(b[2]) + 1             # the two tanh nodes share a batch only in the printed form
    owner = {}
    for k in range(len(b[2])):
        for v in b[1][b[0][k]:b[0][k + 1]]:
            owner[int(v)] = k
    for k in range(len(a[2])):
        assert len({owner[int(v)] for v in a[1][a[0][k]:a[0][k + 1]]}) == 1
