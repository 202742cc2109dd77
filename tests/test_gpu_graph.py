"""GPU parity of graph-level data-movement elimination: the optimised graph (only
compute operators and the composed maps in front of them run; no layout operator
is executed on its own) against the un-optimised graph on the CPU oracle."""
import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth
from tests.test_graph_dme import _inputs, _random_graph, standin

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    from paper_2002_12798_amd import device
    device.require_gpu()
    return device


def _standin_device(kind, xs, shape):
    if kind == "add":
        acc = xs[0].clone()
        for x in xs[1:]:
            acc += x                      # integer tensors wrap like the numpy stand-in
        return acc.reshape(shape)
    if kind == "rowmix":
        return (xs[0] + xs[1][0][None, :]).reshape(shape)
    raise AssertionError(kind)


def run_optimised(dev, g, inputs):
    """Returns {tensor id: host array} for every compute result and graph output."""
    import torch
    dme = B.GraphDME(g.nodes, g.outputs, g.elem_size)
    dme.eliminate()
    by_consumer = {}
    for cons, slot, m, ids in dme.loads():
        by_consumer[(cons, slot)] = (m, ids)
    mat, it, got = {}, iter(inputs), {}
    for i, n in enumerate(g.nodes):
        if n[0] == "input":
            mat[i] = dev.to_device(next(it))
        elif n[0] == "compute":
            xs = []
            for s in range(len(n[2])):
                m, ids = by_consumer[(i, s)]
                xs.append(dev.execute(m, [mat[k] for k in ids]))
            mat[i] = _standin_device(n[1], xs, n[3]).contiguous()
            got[i] = dev.to_host(mat[i])
    for o in g.outputs:
        m, ids = by_consumer[(-1, o)]
        got[o] = dev.to_host(dev.execute(m, [mat[k] for k in ids]))
    torch.cuda.synchronize()
    return got


def test_wavenet_like_graph_on_device(dev):
    g = synth.wavenet_like_graph(layers=7, batch=2, channels=32, steps=512, skip_steps=64)
    ins = _inputs(g, 21)
    want = oracle.run_graph(g.nodes, ins, standin)
    got = run_optimised(dev, g, ins)
    assert set(g.outputs) <= set(got)
    for i, arr in got.items():
        assert np.array_equal(arr.view(want[i].dtype).reshape(want[i].shape), want[i]), i


@pytest.mark.parametrize("block", range(3))
def test_random_graphs_on_device(dev, block):
    for seed in range(block * 20, block * 20 + 20):
        print(f"[gpu] random graph seed {seed}", flush=True)
        g = _random_graph(seed)
        ins = _inputs(g, 100 + seed)
        want = oracle.run_graph(g.nodes, ins, standin)
        got = run_optimised(dev, g, ins)
        for i, arr in got.items():
            assert np.array_equal(arr.view(want[i].dtype).reshape(want[i].shape), want[i]), (seed, i)


def test_composed_maps_replay_from_a_hip_graph(dev):
    """The device entry points allocate nothing and never synchronise, so a run of them can be
    captured into a HIP graph.  Replays (with eager work and synchronisation in between) must
    all reproduce the eager result."""
    import torch
    g = synth.wavenet_like_graph(layers=3, batch=2, channels=16, steps=128, skip_steps=32)
    ins = _inputs(g, 77)
    dme = B.GraphDME(g.nodes, g.outputs, g.elem_size)
    dme.eliminate()
    shapes = {i: (n[1] if n[0] == "input" else n[3]) for i, n in enumerate(g.nodes) if n[0] != "op"}
    gen = np.random.default_rng(5)
    bufs = {i: dev.to_device(synth.random_bits(s, g.elem_size, 900 + i)) for i, s in shapes.items()}
    work = [(m, [bufs[k] for k in ids], dev.empty_dst(m)) for _, _, m, ids in dme.loads()]

    def run_all():
        for m, srcs, dst in work:
            dev.execute(m, srcs, dst)

    run_all()
    torch.cuda.synchronize()
    eager = [dev.to_host(d).copy() for _, _, d in work]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run_all()                                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run_all()
    for rep in range(4):
        for _, _, d in work:
            d.fill_(rep + 1)                        # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (_, _, d), want in zip(work, eager):
            assert np.array_equal(dev.to_host(d), want), rep
    del gen


def test_relayout_copies_of_the_global_assignment_on_device(dev):
    """The copies the global layout assignment leaves are transpose maps; run them on the GPU."""
    import torch
    from tests.test_layout import _build
    shp = (4, 24, 10, 12)
    tensors = [(shp, (0, 1, 2, 3)), (shp, None), (shp, None), (shp, None), (shp, (0, 3, 1, 2))]
    ops = [([0, 1], [0, 1], [synth.NHWC, synth.NHWC], False), ([1, 2], [0, 1], None, True),
           ([2, 3], [0, 1], [(0, 1, 2, 3), (0, 1, 2, 3)], False), ([3, 4], [0, 1], None, True)]
    g = _build(tensors, ops)
    rep = g.solve()
    assert rep.n_copies_global >= 2
    logical = synth.random_bits(shp, 2, 31)
    for op, slot, t, m in g.copies():
        have = g.order(t)
        reqs = ops[op][2]
        need = reqs[slot] if reqs is not None and reqs[slot] is not None else g.order(ops[op][0][0])
        src_order, dst_order = (need, have) if ops[op][1][slot] else (have, need)
        stored = oracle.transpose(logical, src_order)
        got = dev.to_host(dev.execute(m, [dev.to_device(stored)]))
        torch.cuda.synchronize()
        assert np.array_equal(got, oracle.transpose(logical, dst_order)), (op, slot)


def test_concat_block_feeds_the_matrix_cores_without_copies(dev):
    """Four channel-major branches -> concat -> NHWC -> rows of a pointwise convolution.  After
    elimination the product's first operand is one map over the four branch tensors; it goes
    straight into the GEMM's operand load (amap_gemm_gather), no copy kernel runs at all."""
    import torch
    n, h, w, chans, cout = 4, 16, 16, (64, 96, 128, 32), 128
    g = synth.Graph(2)
    branches = [g.input((n, c, h, w)) for c in chans]
    wt = g.input((sum(chans), cout))
    cat = g.op(("concat", 1), branches)
    nhwc = g.op(("transpose", (0, 2, 3, 1)), cat)
    rows = g.op(("reshape", (n * h * w, sum(chans))), nhwc)
    z = g.compute("matmul", [rows, wt], (n * h * w, cout))
    g.output(g.op(("reshape", (n, h, w, cout)), z))
    rng = np.random.default_rng(5)
    ins = [synth.f32_to_bf16_bits(rng.standard_normal((n, c, h, w)).astype(np.float32)) for c in chans]
    ins.append(synth.f32_to_bf16_bits((rng.standard_normal((sum(chans), cout)) * 0.05).astype(np.float32)))
    want = oracle.run_graph(g.nodes, ins, lambda kind, xs, shape: oracle.gemm_bf16(xs[0], xs[1]))

    dme = B.GraphDME(g.nodes, g.outputs, g.elem_size)
    rep = dme.eliminate()
    # the product's output, reshaped, is a view: no pair left; only the A operand carries a map
    assert rep.n_layout_ops == 4 and rep.n_pairs_left == 0 and rep.n_alias_outputs == 1 and rep.n_mapped_loads == 1
    loads = {(cons, slot): (m, ids) for cons, slot, m, ids in dme.loads()}
    mat = {i: dev.to_device(x) for i, x in zip(g.input_ids(), ins)}
    a_map, a_ids = loads[(z, 0)]
    w_map, w_ids = loads[(z, 1)]
    assert sorted(a_ids) == sorted(branches) and w_ids == [wt]
    out = torch.empty((n * h * w, cout), dtype=torch.int16, device="cuda")
    B.amap_gemm_gather([mat[k].data_ptr() for k in a_ids], a_map, mat[wt].data_ptr(), None, cout, None,
                       out.data_ptr(), 0)
    torch.cuda.synchronize()
    o_map, o_ids = loads[(-1, g.outputs[0])]
    assert o_ids == [z]                                            # the output is the product, viewed as NHWC
    got = synth.bf16_bits_to_f32(dev.to_host(out)).astype(np.float64)
    ref = synth.bf16_bits_to_f32(want[z]).astype(np.float64)
    assert np.abs(got - ref).max() <= 1e-2 * np.abs(ref).max()
    ulp = np.maximum(np.abs(ref), 2.0 ** -126) * 2.0 ** -7
    assert np.mean(np.abs(got - ref) <= ulp) > 0.999
