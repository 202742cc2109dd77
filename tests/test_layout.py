"""Global layout assignment (CPU only): propagation to a fixed point, copies only at conflicts,
relayout maps that really are the transposition between the two orders, and the comparison
with the per-operator assignment."""
import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth

NHWC = synth.NHWC


def _build(tensors, ops, es=2):
    g = B.LayoutGraph()
    for shape, fixed in tensors:
        g.tensor(shape, es, fixed)
    for operands, outs, reqs, same in ops:
        g.op(operands, outs, reqs, same)
    return g


def _check_plan(tensors, ops, g):
    """Every operand reaches its operator in the order it needs, through at most one listed copy,
    and every unrestricted operator sees one order per rank."""
    copies = {(op, slot): (t, m) for op, slot, t, m in g.copies()}
    for oi, (operands, outs, reqs, same) in enumerate(ops):
        # an unrestricted operator works in the order of its operands that need no copy
        seen = {len(tensors[t][0]): g.order(t) for si, t in enumerate(operands)
                if same and (reqs is None or reqs[si] is None) and (oi, si) not in copies}
        for si, t in enumerate(operands):
            have = g.order(t)
            req = None if reqs is None else reqs[si]
            if (oi, si) in copies:
                ct, m = copies[(oi, si)]
                assert ct == t
                shape = tensors[t][0]
                logical = synth.iota(shape, 4)
                need = req if req is not None else seen[len(shape)]
                src_order, dst_order = (need, have) if outs[si] else (have, need)
                m4 = B.amap_transpose(B.amap_source(0, [shape[k] for k in src_order], 4),
                                      [src_order.index(d) for d in dst_order])
                stored = oracle.transpose(logical, src_order)
                # the library's copy is the transposition between the two orders ...
                assert B.dst_shape(m) == tuple(shape[k] for k in dst_order)
                assert np.array_equal(B.amap_eval_host(m4, [stored]), oracle.transpose(logical, dst_order))
                # ... and has the same pieces as the one built here by hand
                x16 = synth.iota(shape, 2) if B.amap_describe(m).elem_size == 2 else logical
                st16 = oracle.transpose(x16, src_order)
                assert np.array_equal(B.amap_eval_host(m, [st16]), oracle.transpose(x16, dst_order))
                have = need
            if req is not None:
                assert tuple(have) == tuple(req), (oi, si)
            elif same:
                rank = len(tensors[t][0])
                assert seen.setdefault(rank, tuple(have)) == tuple(have), (oi, si)
    for t, (shape, fixed) in enumerate(tensors):
        if fixed is not None:
            assert g.order(t) == tuple(fixed)


def test_propagation_through_unrestricted_operators():
    # input (canonical) -> conv -> relu -> relu -> conv -> relu -> output (canonical)
    shp = (2, 8, 6, 6)
    tensors = [(shp, (0, 1, 2, 3))] + [(shp, None)] * 5 + [(shp, (0, 1, 2, 3))]
    ops = [([0, 1], [0, 1], [NHWC, NHWC], False), ([1, 2], [0, 1], None, True), ([2, 3], [0, 1], None, True),
           ([3, 4], [0, 1], [NHWC, NHWC], False), ([4, 5], [0, 1], None, True), ([5, 6], [0, 1], None, True)]
    g = _build(tensors, ops)
    rep = g.solve()
    _check_plan(tensors, ops, g)
    assert [g.order(t) for t in range(1, 6)] == [NHWC] * 5
    # global: one copy in front of the first convolution, one into the fixed output
    assert rep.n_copies_global == 2
    # local: every convolution converts on both sides: in (1), out->relu (1), relu->conv (1), conv out->relu (1)
    assert rep.n_copies_local == 4
    nbytes = int(np.prod(shp)) * 2
    assert rep.copy_bytes_global == 2 * 2 * nbytes and rep.copy_bytes_local == 4 * 2 * nbytes


def test_backward_propagation_and_residual_add():
    # relu(x) and relu(y) feed an add whose result goes into a convolution: the order flows backwards
    shp = (2, 4, 5, 5)
    tensors = [(shp, None)] * 6
    ops = [([0, 2], [0, 1], None, True), ([1, 3], [0, 1], None, True), ([2, 3, 4], [0, 0, 1], None, True),
           ([4, 5], [0, 1], [NHWC, NHWC], False)]
    g = _build(tensors, ops)
    rep = g.solve()
    _check_plan(tensors, ops, g)
    assert all(g.order(t) == NHWC for t in range(6))
    assert rep.n_copies_global == 0 and rep.n_copies_local == 1 and rep.n_sweeps >= 2


def test_conflicting_requirements_get_one_copy():
    # one tensor read by a convolution (channels innermost) and by an operator that wants W innermost
    shp = (2, 4, 5, 6)
    tensors = [(shp, None), (shp, None), (shp, None)]
    ops = [([0, 1], [0, 1], [NHWC, NHWC], False), ([0, 2], [0, 1], [(0, 1, 2, 3), (0, 1, 2, 3)], False)]
    g = _build(tensors, ops)
    rep = g.solve()
    _check_plan(tensors, ops, g)
    assert g.order(0) == NHWC and rep.n_copies_global == 1
    (op, slot, t, m), = g.copies()
    assert (op, slot, t) == (1, 0, 0) and B.dst_shape(m) == shp


def test_resnet_like_graph():
    tensors, ops = synth.resnet_like_layout_graph(batch=2)
    g = _build(tensors, ops)
    rep = g.solve()
    _check_plan(tensors, ops, g)
    n_conv = sum(1 for o in ops if o[2] is not None and o[2][0] == NHWC)
    assert n_conv == 36
    # global: the network input is converted once; everything up to the pooled vector stays channels-innermost
    assert rep.n_copies_global == 1
    # local: every convolution's input that was not produced by a convolution, and every consumer
    # of a convolution's output, pays a copy
    assert rep.n_copies_local > 2 * n_conv - 4
    assert rep.copy_bytes_global * 20 < rep.copy_bytes_local


def test_layout_error_paths():
    g = B.LayoutGraph()
    t = g.tensor((2, 3), 4)
    with pytest.raises(B.AmapError):
        g.tensor((2, 3), 4, (0, 0))
    with pytest.raises(B.AmapError):
        g.op([t, 7], [0, 1])
    with pytest.raises(B.AmapError):
        g.op([t], [0], [(1, 1)])
    g.op([t], [1])
    with pytest.raises(B.AmapError):
        g.op([t], [1])                      # a second producer
    g.solve()
    with pytest.raises(B.AmapError):
        g.solve()


def _random_layout_graph(seed):
    """Small graphs of rank-2 tensors (two possible orders each), so that every assignment can be tried."""
    rng = np.random.default_rng(seed)
    orders = [(0, 1), (1, 0)]
    tensors = [((int(rng.integers(2, 9)), int(rng.integers(2, 9))), orders[int(rng.integers(2))] if rng.random() < 0.7 else None)]
    ops = []
    for _ in range(int(rng.integers(3, 7))):
        n_in = int(rng.integers(1, 3))
        ins = [int(rng.integers(len(tensors))) for _ in range(n_in)]
        restricted = rng.random() < 0.5
        if not restricted:
            shape = tensors[ins[0]][0]
            ins = [t for t in ins if tensors[t][0] == shape] or ins[:1]   # element-wise: equal shapes
        else:
            shape = (int(rng.integers(2, 9)), int(rng.integers(2, 9)))
        tensors.append((shape, orders[int(rng.integers(2))] if rng.random() < 0.15 else None))
        operands = ins + [len(tensors) - 1]
        outs = [0] * len(ins) + [1]
        if restricted:
            reqs = [orders[int(rng.integers(2))] if rng.random() < 0.8 else None for _ in operands]
            ops.append((operands, outs, reqs, False))
        else:
            ops.append((operands, outs, None, True))
    return tensors, ops


def _assignment_cost(tensors, ops, order, es=2):
    cost = 0
    for operands, outs, reqs, same in ops:
        if reqs is not None:
            cost += sum(2 * es * int(np.prod(tensors[t][0])) for t, r in zip(operands, reqs) if r is not None and order[t] != r)
        elif same:
            cost += min(sum(2 * es * int(np.prod(tensors[t][0])) for t in operands if order[t] != o) for o in [(0, 1), (1, 0)])
    return cost


@pytest.mark.parametrize("seed", range(60))
def test_global_assignment_between_the_optimum_and_the_local_one(seed):
    """The propagation is a heuristic.  On graphs small enough to try every assignment its copy
    bytes can never be below the true optimum (else a needed copy is missing) and should not
    exceed what assigning every operator on its own costs."""
    import itertools
    tensors, ops = _random_layout_graph(seed)
    g = _build(tensors, ops)
    rep = g.solve()
    _check_plan(tensors, ops, g)
    free = [t for t, (_, fixed) in enumerate(tensors) if fixed is None]
    best = None
    for choice in itertools.product([(0, 1), (1, 0)], repeat=len(free)):
        order = {t: fixed for t, (_, fixed) in enumerate(tensors)}
        order.update(dict(zip(free, choice)))
        c = _assignment_cost(tensors, ops, order)
        best = c if best is None else min(best, c)
    assert best <= rep.copy_bytes_global, (best, rep.copy_bytes_global)
    assert rep.copy_bytes_global <= rep.copy_bytes_local, (rep.copy_bytes_global, rep.copy_bytes_local)
    # the solver's own figure is the cost of the assignment it reports
    assert rep.copy_bytes_global == _assignment_cost(tensors, ops, {t: g.order(t) for t in range(len(tensors))})
