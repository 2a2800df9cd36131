"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host logic (graph definition, validation, error codes) behaves as documented.  No compute
call is made here; a context without a device arena is enough."""
import re
from pathlib import Path

import numpy as np
import pytest

from paper_1705_07860_amd import binding as ob
from paper_1705_07860_amd import workloads as wl

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not ob.LIB_PATH.exists():
        from paper_1705_07860_amd import build
        build.build()


def test_library_exports_every_declared_symbol():
    header = (ROOT / "include" / "ob.h").read_text()
    declared = set(re.findall(r"\b(ob_[a-z_0-9]+)\s*\(", header))
    declared -= {"ob_ctx", "ob_stats"}
    L = ob.lib()
    assert len(declared) >= 30
    for name in sorted(declared):
        assert hasattr(L, name), f"{name} declared in ob.h but not exported"
    assert set(L._ob_names) == declared, "binding and header disagree"


def test_stats_record_of_the_binding_matches_the_header():
    """ob_stats_read fills a caller-owned record: the ctypes mirror must list the header's fields in the
    header's order with the header's types, or the library would write past it."""
    import ctypes
    header = (ROOT / "include" / "ob.h").read_text()
    body = re.search(r"typedef struct ob_stats \{(.*?)\} ob_stats;", header, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    ctype = {"int32_t": ctypes.c_int32, "uint64_t": ctypes.c_uint64, "float": ctypes.c_float}
    want = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        t, names = decl.split(None, 1)
        want += [(n.strip(), ctype[t]) for n in names.split(",")]
    got = [(n, t) for n, t in ob.ObStats._fields_]
    assert got == want
    assert ctypes.sizeof(ob.ObStats) == sum(ctypes.sizeof(t) for _, t in want)   # (no padding: 8-byte fields fall on 8-byte offsets)


def _host_ctx(params=None):
    c = ob.Context(arena_bytes=0)
    ids = c.params_create(params) if params is not None else []
    return c, ids


def test_adders_return_dense_ids_and_validate():
    p = wl.rnn_params()
    c, _ = _host_ctx(p)
    x = c.add_input(np.zeros(32))
    assert x == 0
    a = c.add_matvec(0, 2, x)
    u = c.add_matvec(1, -1, x)
    s = c.add_nary(wl.OP_ADD, [a, u])
    h = c.add_unary(wl.OP_TANH, s)
    L = c.add_sqnorm(h)
    assert [a, u, s, h, L] == [1, 2, 3, 4, 5]
    assert c.graph_size() == (6, 6)
    with pytest.raises(ob.ObError) as e:
        c.add_matvec(0, 2, 99)                       # forward reference
    assert e.value.code == -1
    with pytest.raises(ob.ObError) as e:
        c.add_matvec(0, 2, L)                        # 1-element operand into a 32-column matrix
    assert e.value.code == -2
    with pytest.raises(ob.ObError) as e:
        c.add_matvec(0, 1, x)                        # bias must be rows x 1
    assert e.value.code == -2
    with pytest.raises(ob.ObError) as e:
        c.add_matvec(7, -1, x)
    assert e.value.code == -1
    with pytest.raises(ob.ObError) as e:
        c.add_slice(h, 4, 40)
    assert e.value.code == -3
    with pytest.raises(ob.ObError) as e:
        c.add_pick_nls(h, 32)
    assert e.value.code == -3
    with pytest.raises(ob.ObError) as e:
        c.add_lookup(0, 32)
    assert e.value.code == -3
    with pytest.raises(ob.ObError) as e:
        c.add_nary(wl.OP_ADD, [h, L])                # dims differ
    assert e.value.code == -2
    with pytest.raises(ob.ObError) as e:
        c.add_nary(wl.OP_CMULT, [h, h, h])
    assert e.value.code == -2
    with pytest.raises(ob.ObError) as e:
        c.add_unary(wl.OP_ADD, h)
    assert e.value.code == -8
    assert c.graph_size() == (6, 6)                  # failed adds appended nothing
    assert c.add_nary(wl.OP_CONCAT, [h, L]) == 6
    c.graph_new()
    assert c.graph_size() == (0, 0)
    c.close()


@pytest.mark.parametrize("name", ["rnn", "tree"])
def test_bulk_add_equals_node_by_node(name):
    p, g = wl.make(name) if name == "rnn" else (wl.tree_params(), None)
    if g is None:
        g = wl.tree_minibatch(p, seed=3, n_trees=3)
    c, _ = _host_ctx(p)
    first = c.add_bulk(g)
    assert first == 0
    assert c.graph_size() == (g.n, g.n_edges)
    c2, _ = _host_ctx(p)
    for v in range(g.n):
        ins = [int(u) for u in g.in_idx[g.in_off[v]:g.in_off[v + 1]]]
        o = int(g.op[v])
        if o == wl.OP_INPUT:
            r = c2.add_input(g.payload[g.aux0[v]:g.aux0[v] + g.out_dim[v]])
        elif o == wl.OP_LOOKUP:
            r = c2.add_lookup(int(g.param[v]), int(g.aux0[v]))
        elif o == wl.OP_MATVEC:
            r = c2.add_matvec(int(g.param[v]), int(g.bias[v]), ins[0])
        elif o in (wl.OP_TANH, wl.OP_SIGMOID):
            r = c2.add_unary(o, ins[0])
        elif o in (wl.OP_ADD, wl.OP_CMULT, wl.OP_CONCAT):
            r = c2.add_nary(o, ins)
        elif o == wl.OP_SLICE:
            r = c2.add_slice(ins[0], int(g.aux0[v]), int(g.aux1[v]))
        elif o == wl.OP_PICK_NLS:
            r = c2.add_pick_nls(ins[0], int(g.aux0[v]))
        else:
            r = c2.add_sqnorm(ins[0])
        assert r == v
    assert c2.graph_size() == (g.n, g.n_edges)
    c.close()
    c2.close()


def test_bulk_rejects_malformed_graphs_atomically():
    p, g = wl.make("rnn")
    c, _ = _host_ctx(p)
    import copy
    bad = copy.deepcopy(g)
    bad.in_idx = bad.in_idx.copy()
    bad.in_idx[5] = g.n + 3                          # operand that does not exist
    with pytest.raises(ob.ObError) as e:
        c.add_bulk(bad)
    assert e.value.code == -1
    assert c.graph_size() == (0, 0)
    bad = copy.deepcopy(g)
    bad.out_dim = bad.out_dim.copy()
    bad.out_dim[g.n - 1] = 2                         # the loss sum is a scalar
    with pytest.raises(ob.ObError) as e:
        c.add_bulk(bad)
    assert e.value.code == -2
    bad = copy.deepcopy(g)
    bad.aux0 = bad.aux0.copy()
    bad.aux0[0] = 10 ** 6                            # INPUT payload outside the payload array
    with pytest.raises(ob.ObError) as e:
        c.add_bulk(bad)
    assert e.value.code == -3
    assert c.graph_size() == (0, 0)
    assert c.add_bulk(g) == 0
    assert c.add_bulk(g_shift(g, g.n)) == g.n        # a second bulk call refers to absolute ids
    c.close()


def g_shift(g, by):
    import copy
    h = copy.deepcopy(g)
    h.in_idx = (g.in_idx + by).astype(np.uint32)
    return h


def test_state_and_argument_errors_without_a_device():
    c, _ = _host_ctx(wl.rnn_params())
    with pytest.raises(ob.ObError) as e:
        c.forward(0)
    assert e.value.code == -1                        # no such node
    c.add_input(np.zeros(32))
    with pytest.raises(ob.ObError) as e:
        c.forward(0)
    assert e.value.code == -6                        # no device arena
    with pytest.raises(ob.ObError) as e:
        c.backward(0)
    assert e.value.code == -6
    with pytest.raises(ob.ObError) as e:
        c.value_read(0, 32)
    assert e.value.code == -6
    c.set_mode(ob.OB_BYAGENDA)
    c.set_mode(ob.OB_BYDEPTH)
    with pytest.raises(ob.ObError) as e:
        c.set_mode(17)
    assert e.value.code == -8
    with pytest.raises(ob.ObError):
        c.param_create(np.zeros((0, 3), np.float32))
    c.close()


def test_manual_batch_labels_are_checked_on_the_host():
    """Manual batching (Section 2): the library takes a labelling only if operands come from
    earlier batches and a batch holds one kind of node."""
    p = wl.rnn_params()
    c, _ = _host_ctx(p)
    x0, x1 = c.add_input(np.zeros(32)), c.add_input(np.ones(32))
    a0, a1 = c.add_matvec(0, 2, x0), c.add_matvec(0, 2, x1)
    u1 = c.add_matvec(1, -1, x1)
    t0, t1 = c.add_unary(wl.OP_TANH, a0), c.add_unary(wl.OP_TANH, a1)
    assert [x0, x1, a0, a1, u1, t0, t1] == list(range(7))
    c.set_mode(ob.OB_MANUAL)
    good = [0, 0, 1, 1, 2, 5, 5]                     # labels need not be dense
    c.set_manual_batches(good)
    for bad, why in (([0, 0, 1, 1, 2, 5], "one label short"),
                     ([0, 0, 1, 1, 2, 5, -1], "negative label"),
                     ([0, 0, 1, 1, 2, 1, 5], "tanh in the batch of its operand"),
                     ([3, 0, 1, 1, 2, 5, 5], "operand after its consumer"),
                     ([0, 0, 1, 1, 1, 5, 5], "two matrices in one batch"),
                     ([0, 0, 1, 1, 2, 5, 5, 6], "one label too many")):
        with pytest.raises(ob.ObError) as e:
            c.set_manual_batches(bad)
        assert e.value.code == -8, why
    with pytest.raises(ob.ObError) as e:
        c.forward(6)
    assert e.value.code == -6                        # labels are fine, but there is no device arena
    c.add_unary(wl.OP_SIGMOID, t1)                   # the graph grew: the labels are gone
    with pytest.raises(ob.ObError, match="no batch labels") as e:
        c.forward(7)
    assert e.value.code == -6
    c.close()


def test_statement_labels_of_the_equal_length_tagger_are_a_valid_manual_batching():
    from tests.helpers import validate_manual_labels, manual_schedule
    p = wl.sync_tagger_params(vocab=50, emb=8, hidden=4, tags=6)
    g = wl.sync_tagger_minibatch(p, n_sent=3, length=4)
    lab = wl.sync_tagger_manual_labels(g)
    validate_manual_labels(g, lab)
    bo, ids = manual_schedule(lab)
    assert np.all(np.diff(bo)[:-1] == 3) and bo[-1] - bo[-2] == 1     # every statement over the 3 sentences, then the sum
    c, _ = _host_ctx(p)
    c.add_bulk(g)
    c.set_manual_batches(lab)
    c.close()
    h = wl.tagger_minibatch(wl.tagger_params(), n_sent=3)             # unequal lengths: no such labelling
    if len(set(h.meta["lengths"])) > 1 and (h.n - 1) % 3 == 0:
        with pytest.raises(AssertionError):
            validate_manual_labels(h, wl.sync_tagger_manual_labels(h))


def test_binding_fails_loudly_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError, match="no GPU"):
        ob.Context(arena_bytes=1 << 20)
