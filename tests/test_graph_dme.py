"""Graph-level data-movement elimination (CPU only): after the fixed point every
load of a compute operator and every graph output reads materialised tensors
through one composed map, and evaluating that map on the oracle's materialised
tensors reproduces, bit for bit, the tensor the un-optimised program would have
put in front of that load."""
import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth
from tests import chains


def standin(kind, xs, shape):
    """The opaque compute operators of the test graphs (integer, so exact)."""
    if kind == "add":
        acc = xs[0].copy()
        for x in xs[1:]:
            acc = acc + x            # unsigned wrap-around
        return acc.reshape(shape)
    if kind == "rowmix":
        a, w = xs
        return (a + w[0][None, :]).reshape(shape)
    raise AssertionError(kind)


def _inputs(g, seed):
    return [synth.random_bits(g.nodes[i][1], g.elem_size, seed + i) for i in g.input_ids()]


def _check_loads(g, tensors, dme):
    mat = {i for i, n in enumerate(g.nodes) if n[0] in ("input", "compute")}
    seen = set()
    for cons, slot, m, ids in dme.loads():
        assert set(ids) <= mat, "a rewritten load still reads a tensor defined by a copy"
        want = tensors[slot] if cons < 0 else tensors[g.nodes[cons][2][slot]]
        got = B.amap_eval_host(m, [tensors[i] for i in ids])
        assert got.shape == want.shape
        assert np.array_equal(got, want), (cons, slot)
        seen.add((cons, slot))
    expect = {(c, s) for c, n in enumerate(g.nodes) if n[0] == "compute" for s in range(len(n[2]))}
    expect |= {(-1, o) for o in g.outputs}
    assert seen == expect


def test_wavenet_like_graph():
    layers, Bn, Cc, T, S = 4, 2, 8, 32, 8
    g = synth.wavenet_like_graph(layers, Bn, Cc, T, S)
    tensors = oracle.run_graph(g.nodes, _inputs(g, 5), standin)
    dme = B.GraphDME(g.nodes, g.outputs, g.elem_size)
    rep = dme.eliminate()
    _check_loads(g, tensors, dme)
    # per layer: pad, 2 taps, concat (2 pairs), transpose, reshape | reshape, transpose, 2 gate slices | skip slice
    assert rep.n_layout_ops == 11 * layers + 2
    assert rep.n_pairs == 12 * layers + layers + 1
    assert rep.n_loads == 6 * layers + 2
    # only the skip output is still copied, from one tensor per layer; the other output is a compute result
    assert rep.n_pairs_left == layers and rep.n_alias_outputs == 0
    es = g.elem_size
    skip_bytes = Bn * layers * Cc * S * es
    assert rep.moved_bytes_after == 2 * skip_bytes
    per_layer_storage = (Bn * Cc * (T + 1)) + 2 * Bn * Cc * T + 3 * Bn * 2 * Cc * T + 2 * Bn * 2 * Cc * T \
        + 2 * Bn * Cc * T + Bn * Cc * S
    dil = sum((1 << (l % 6)) - 1 for l in range(layers)) * Bn * Cc    # padding grows with the dilation
    assert rep.intermediate_bytes == (per_layer_storage * layers + dil + Bn * layers * Cc * S) * es
    assert rep.moved_bytes_before > 10 * rep.moved_bytes_after
    # the matrix-product operand is not an identity load (taps + concat + layout change): one per layer,
    # and so are the two halves of the gate
    assert rep.n_mapped_loads == 3 * layers


def test_cancelling_chain_leaves_no_copy():
    g = synth.Graph(4)
    x = g.input((3, 4, 5))
    t = g.op(("transpose", (2, 0, 1)), x)
    r = g.op(("reshape", (5, 12)), t)
    r2 = g.op(("reshape", (5, 3, 4)), r)
    back = g.op(("transpose", (1, 2, 0)), r2)
    g.output(back)
    dme = B.GraphDME(g.nodes, g.outputs, 4)
    rep = dme.eliminate()
    assert (rep.n_pairs, rep.n_pairs_left, rep.n_alias_outputs, rep.moved_bytes_after) == (4, 0, 1, 0)
    assert rep.intermediate_bytes == 4 * 60 * 4 and rep.n_rewrites == 4
    tensors = oracle.run_graph(g.nodes, _inputs(g, 1), standin)
    _check_loads(g, tensors, dme)
    (cons, slot, m, ids), = dme.loads()
    assert ids == [x] and B.amap_describe(m).n_pieces == 1


def test_reshape_of_a_whole_tensor_is_a_view():
    """A reshape changes no address: an output or an operand that is only a reshaped tensor
    needs no copy, whatever its shape says."""
    g = synth.Graph(2)
    x = g.input((4, 6))
    c = g.compute("add", [g.op(("reshape", (2, 12)), x), g.op(("reshape", (2, 12)), x)], (2, 12))
    g.output(g.op(("reshape", (3, 8)), c))
    g.output(g.op(("transpose", (1, 0)), c))            # this one does move data
    dme = B.GraphDME(g.nodes, g.outputs, 2)
    rep = dme.eliminate()
    assert (rep.n_alias_outputs, rep.n_pairs_left, rep.n_mapped_loads) == (1, 1, 0)
    assert rep.moved_bytes_after == 2 * 24 * 2
    _check_loads(g, oracle.run_graph(g.nodes, _inputs(g, 3), standin), dme)


def test_several_consumers_and_chains_through_compute():
    g = synth.Graph(2)
    a = g.input((4, 6))
    b = g.input((4, 6))
    at = g.op(("transpose", (1, 0)), a)                 # read by two compute operators and an output
    bt = g.op(("transpose", (1, 0)), b)
    s = g.compute("add", [at, bt], (6, 4))
    st = g.op(("transpose", (1, 0)), s)                 # a chain that starts at a compute result
    cat = g.op(("concat", 0), [st, a, b])
    u = g.compute("add", [g.op(("slice", 0, 4, 8, 1), cat), a], (4, 6))   # slice of the concat = a again
    g.output(at)
    g.output(u)
    g.output(g.op(("repeat", 1, 2), cat))
    tensors = oracle.run_graph(g.nodes, _inputs(g, 9), standin)
    dme = B.GraphDME(g.nodes, g.outputs, 2)
    rep = dme.eliminate()
    _check_loads(g, tensors, dme)
    loads = {(c, s_): (m, ids) for c, s_, m, ids in dme.loads()}
    m, ids = loads[(u, 0)]
    assert ids == [a] and B.amap_describe(m).kernel_id == B.AMAP_K_ROWS and B.amap_describe(m).n_pieces == 1
    assert rep.n_mapped_loads == 2           # at and bt into the first add; the slice-of-concat load is the identity
    assert rep.n_pairs_left == 1 + 3         # at from a; the repeated concat from s, a, b


def test_store_form_operators_are_reversed_and_eliminated():
    """Operators written as stores (where each element goes) next to operators written as loads:
    the store map is reversed on entry (Section 2.1) and from then on composes like any load."""
    g = synth.Graph(2)
    x = g.input((4, 6))
    st = g.store([("transpose", (1, 0))], x, (6, 4))              # x[i,j] -> st[j,i]
    back = g.op(("transpose", (1, 0)), st)                         # a load that undoes the store
    c = g.compute("add", [back, x], (4, 6))
    flat = g.store([("reshape", (4, 6)), ("slice", 1, 5, -1, -1)], c, (24,))   # c[i,j] -> flat[6 i + 5 - j]
    g.output(flat)
    g.output(st)
    tensors = oracle.run_graph(g.nodes, _inputs(g, 4), standin)
    assert np.array_equal(tensors[st], tensors[x].T) and np.array_equal(tensors[flat], tensors[c][:, ::-1].reshape(-1))
    dme = B.GraphDME(g.nodes, g.outputs, 2)
    rep = dme.eliminate()
    _check_loads(g, tensors, dme)
    # store + the load that undoes it: the add reads x itself, twice; both outputs still move data
    assert (rep.n_layout_ops, rep.n_pairs, rep.n_mapped_loads, rep.n_alias_outputs, rep.n_pairs_left) == (3, 3, 0, 0, 2)
    # not a bijection between input and output: refused like amap_inverse refuses it
    bad = synth.Graph(2)
    y = bad.input((4, 6))
    bad.store([("slice", 0, 0, 4, 1)], y, (5, 6))
    with pytest.raises(B.AmapError) as e:
        B.GraphDME(bad.nodes, [], 2)
    assert e.value.status == B.AMAP_E_UNSUPPORTED
    bad2 = synth.Graph(2)
    y = bad2.input((4, 6))
    bad2.store([("transpose", (1, 0))], y, (4, 6))              # the map's dst shape is not the input's
    with pytest.raises(B.AmapError) as e:
        B.GraphDME(bad2.nodes, [], 2)
    assert e.value.status == B.AMAP_E_SHAPE


def test_operator_given_as_a_composed_map():
    """amap_graph_map: a layout operator handed over as one composed map over several graph tensors."""
    a_shape, b_shape = (3, 4), (5, 4)
    m = B.amap_concat([B.amap_transpose(B.amap_source(0, a_shape, 2), (1, 0)),
                       B.amap_transpose(B.amap_source(1, b_shape, 2), (1, 0))], 1)      # [4, 8]
    nodes = [("input", a_shape), ("input", b_shape), ("map", m, [0, 1]), ("op", ("slice", 1, 3, 8, 1), [2]),
             ("compute", "add", [3, 3], (4, 5))]
    dme = B.GraphDME(nodes, [2], 2)
    rep = dme.eliminate()
    assert (rep.n_layout_ops, rep.n_pairs) == (2, 3)
    a, b = synth.random_bits(a_shape, 2, 1), synth.random_bits(b_shape, 2, 2)
    loads = {(c, s_): (mm, ids) for c, s_, mm, ids in dme.loads()}
    mm, ids = loads[(4, 0)]
    assert ids == [1]                                                                   # the slice keeps b's part only
    assert np.array_equal(B.amap_eval_host(mm, [b]), b.T)
    mm, ids = loads[(-1, 2)]
    assert np.array_equal(B.amap_eval_host(mm, [a, b]), np.concatenate([a.T, b.T], 1))
    with pytest.raises(B.AmapError) as e:                                               # shape of a graph tensor does not fit
        B.GraphDME([("input", (3, 5)), ("input", b_shape), ("map", m, [0, 1])], [], 2)
    assert e.value.status == B.AMAP_E_SHAPE


def _random_graph(seed):
    rng = np.random.default_rng(seed)
    g = synth.Graph(2 if seed % 2 else 4)
    shapes = {}
    for _ in range(int(rng.integers(1, 4))):
        s = chains.random_shape(rng, max_rank=3, max_extent=6)
        shapes[g.input(s)] = s
    for _ in range(int(rng.integers(3, 14))):
        ids = list(shapes)
        u = rng.random()
        if u < 0.12:
            # a layout operator in store form: a random bijection given by where each element goes
            t = int(rng.choice(ids))
            sin = shapes[t]
            perm = tuple(int(v) for v in rng.permutation(len(sin)))
            mid = tuple(sin[perm.index(d)] for d in range(len(sin)))
            chain, out_shape = [("transpose", perm)], mid
            if rng.random() < 0.5 and int(np.prod(mid)) > 0:
                chain, out_shape = [("reshape", mid)] + chain, (int(np.prod(mid)),)
            if rng.random() < 0.5:
                ax = int(rng.integers(len(sin)))
                if sin[ax] > 0:
                    chain = chain + [("slice", ax, sin[ax] - 1, -1, -1)]
            if int(np.prod(sin)) == 0:
                continue
            shapes[g.store(chain, t, out_shape)] = tuple(out_shape)
        elif u < 0.7:
            t = int(rng.choice(ids))
            op = chains.random_op_ext(rng, shapes[t])
            ns = chains.out_shape(shapes[t], op)
            if int(np.prod(ns)) > 4000 or int(np.prod(ns)) == 0:
                continue
            shapes[g.op(op, t)] = ns
        elif u < 0.8:
            t = int(rng.choice(ids))
            same = [i for i in ids if shapes[i][1:] == shapes[t][1:] and len(shapes[i]) == len(shapes[t])]
            pick = [int(v) for v in rng.choice(same, size=min(len(same), int(rng.integers(1, 4))))]
            ns = (sum(shapes[i][0] for i in pick),) + tuple(shapes[t][1:])
            shapes[g.op(("concat", 0), pick)] = ns
        else:
            t = int(rng.choice(ids))
            same = [i for i in ids if shapes[i] == shapes[t]]
            pick = [int(v) for v in rng.choice(same, size=min(len(same), 2), replace=False)]
            shapes[g.compute("add", pick, shapes[t])] = shapes[t]
    ids = list(shapes)
    for o in set(int(v) for v in rng.choice(ids, size=min(3, len(ids)), replace=False)):
        g.output(o)
    return g


@pytest.mark.parametrize("seed", range(120))
def test_random_graphs(seed):
    g = _random_graph(seed)
    tensors = oracle.run_graph(g.nodes, _inputs(g, 100 + seed), standin)
    dme = B.GraphDME(g.nodes, g.outputs, g.elem_size)
    rep = dme.eliminate()
    _check_loads(g, tensors, dme)
    assert rep.n_layout_ops == sum(n[0] in ("op", "store") for n in g.nodes)
    assert rep.n_pairs == sum(len(n[2]) for n in g.nodes if n[0] in ("op", "store"))


def test_graph_error_paths():
    g = synth.Graph(4)
    x = g.input((2, 3))
    with pytest.raises(B.AmapError) as e:
        B.GraphDME(g.nodes + [("op", ("transpose", (1, 0)), [5])], [], 4)
    assert e.value.status == B.AMAP_E_INVALID
    with pytest.raises(B.AmapError) as e:
        B.GraphDME(g.nodes + [("op", ("reshape", (7,)), [x])], [], 4)
    assert e.value.status == B.AMAP_E_SHAPE
    with pytest.raises(B.AmapError) as e:
        B.GraphDME(g.nodes + [("op", ("transpose", (1, 0)), [x, x])], [], 4)
    assert e.value.status == B.AMAP_E_INVALID
    with pytest.raises(B.AmapError) as e:
        B.GraphDME(g.nodes, [3], 4)
    assert e.value.status == B.AMAP_E_INVALID
    d = B.GraphDME(g.nodes, [x], 4)
    d.eliminate()
    with pytest.raises(B.AmapError):
        d.eliminate()                       # only once
