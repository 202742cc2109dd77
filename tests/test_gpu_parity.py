"""GPU parity: every kernel family against the CPU oracle, bit for bit, called
through the C ABI.  Needs an MI355X (-m gpu)."""
import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth
from tests import chains
from tests.test_plan_replay import ALIGNED

pytestmark = pytest.mark.gpu

FAMILIES = [None, B.AMAP_K_PROGRAM, B.AMAP_K_ELEMENT, B.AMAP_K_ROWS, B.AMAP_K_TILE, B.AMAP_K_WAVE]


@pytest.fixture(scope="module")
def dev():
    from paper_2002_12798_amd import device
    device.require_gpu()
    return device


def _run_families(dev, m, srcs, want, families=FAMILIES, min_ran=2):
    import torch
    d_srcs = [dev.to_device(s) for s in srcs]
    sentinel = 0x5A5A if want.dtype.itemsize == 2 else 0x5A5A5A5A
    ran = []
    for fam in families:
        dst = dev.empty_dst(m, fill=sentinel)
        try:
            dev.execute(m, d_srcs, dst, kernel_id=fam)
        except B.AmapError as e:
            assert e.status == B.AMAP_E_UNSUPPORTED and fam is not None, (fam, e)
            continue
        torch.cuda.synchronize()
        got = dev.to_host(dst)
        assert got.shape == want.shape
        if not np.array_equal(got, want):
            bad = np.argwhere(got != want)
            raise AssertionError(f"family {fam}: {len(bad)} mismatches, first at {bad[0]}: "
                                 f"got {got[tuple(bad[0])]:#x} want {want[tuple(bad[0])]:#x}")
        ran.append(fam)
    assert len(ran) >= min_ran, ran
    return ran


@pytest.mark.parametrize("name", synth.WORKLOAD_NAMES)
def test_workloads_all_families(dev, name):
    print(f"[gpu] workload {name}", flush=True)
    w = synth.workload(name)
    srcs = w.sources()
    oracle.set_threads(8)
    try:
        want = oracle.run_chain(srcs, w.ops)
    finally:
        oracle.set_threads(1)
    m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
    ran = _run_families(dev, m, srcs, want, min_ran=4)
    assert None in ran and B.AMAP_K_PROGRAM in ran and B.AMAP_K_ELEMENT in ran


def test_named_workloads_run_in_the_kernels_built_for_their_launch_shape(dev, monkeypatch, capfd):
    """cfg0, cfg1 and cfg3 (one tile piece or group, plus fill rows) in amap_tile16_kernel, cfg2 and the GEMM's
    materialising copy (one plain row piece) in amap_rows_kernel; a silent fall-back to the general kernel would
    keep every parity test green and lose the speed."""
    import torch
    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    for name, kernel in (("cfg0", "amap_tile16_kernel"), ("cfg1", "amap_tile16_kernel"), ("cfg3", "amap_tile16_kernel"),
                         ("cfg2_fwd", "amap_rows_kernel"), ("cfg2_rev", "amap_rows_kernel"), ("cfg4", "amap_rows_kernel"),
                         ("up3x", "amap_pieces_kernel")):
        kw = {"n": 2} if name in ("cfg1", "cfg3", "up3x") else {}
        w = synth.workload(name, **kw)
        m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
        srcs = [dev.to_device(s) for s in w.sources()]
        capfd.readouterr()
        dst = dev.execute(m, srcs)
        torch.cuda.synchronize()
        lines = [l for l in capfd.readouterr().err.splitlines() if l.startswith("amap launch:")]
        assert len(lines) == 1 and lines[0].startswith(f"amap launch: {kernel},"), (name, lines)
        assert np.array_equal(dev.to_host(dst), oracle.run_chain(w.sources(), w.ops)), name


def test_secondary_readings(dev):
    """cfg0 with exclusive slice end / symmetric pad, and one chain per Q/K/V output."""
    w = synth.workload("cfg0")
    srcs = w.sources()
    for ops in (
        [w.ops[0], w.ops[1], ("slice", 1, 128, 895, 1), w.ops[3]],
        [w.ops[0], w.ops[1], w.ops[2], ("pad", (0, 0, 2), (0, 0, 2), 0)],
    ):
        m = B.amap_compose(w.src_shapes, 4, ops)
        _run_families(dev, m, srcs, oracle.run_chain(srcs, ops))
    w2 = synth.workload("cfg2_fwd", b=2)
    s2 = w2.sources()
    for t in range(3):
        ops = synth.split_qkv_ops(t, b=2)
        m = B.amap_compose(w2.src_shapes, 2, ops)
        _run_families(dev, m, s2, oracle.run_chain(s2, ops))


def test_random_bit_payloads_survive(dev):
    """NaN payloads, -0, subnormals: data are moved as integers."""
    for name in ("cfg0", "cfg3"):
        w = synth.workload(name) if name == "cfg0" else synth.workload(name, n=2)
        srcs = [synth.random_bits(s, w.elem_size, 77 + i) for i, s in enumerate(w.src_shapes)]
        m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
        _run_families(dev, m, srcs, oracle.run_chain(srcs, w.ops))


@pytest.mark.parametrize("block", range(4))
def test_random_chains(dev, block):
    for seed in range(block * 40, block * 40 + 40):
        print(f"[gpu] random chain seed {seed}", flush=True)
        src_shapes, ops = chains.random_chain(seed)
        es = 2 if seed % 2 else 4
        srcs = [synth.random_bits(s, es, 1000 + seed + i) for i, s in enumerate(src_shapes)]
        m = B.amap_compose(src_shapes, es, ops)
        _run_families(dev, m, srcs, oracle.run_chain(srcs, ops), min_ran=2)


@pytest.mark.parametrize("block", range(4))
def test_random_chains_with_repeat_tile_and_downward_slices(dev, block):
    for seed in range(block * 40, block * 40 + 40):
        print(f"[gpu] extended random chain seed {seed}", flush=True)
        src_shapes, ops = chains.random_chain(seed, extended=True)
        es = 2 if seed % 2 else 4
        srcs = [synth.random_bits(s, es, 2000 + seed + i) for i, s in enumerate(src_shapes)]
        m = B.amap_compose(src_shapes, es, ops)
        _run_families(dev, m, srcs, oracle.run_chain(srcs, ops), min_ran=2)


def test_repeat_tile_at_bandwidth_sizes(dev):
    """Several tiles and a ragged tail per kernel family, with re-read source elements."""
    cases = [
        ((16, 200, 72), 2, [("repeat", 0, 3), ("transpose", (0, 2, 1))]),
        ((16, 200, 72), 2, [("transpose", (0, 2, 1)), ("tile", 1, 2), ("slice", 2, 199, -1, -1)]),
        ((64, 1, 520), 4, [("tile", 1, 33), ("pad", (0, 1, 0), (0, 0, 8), 0xDEADBEEF)]),
    ]
    for shape, es, ops in cases:
        print(f"[gpu] repeat/tile case {shape} {ops}", flush=True)
        srcs = [synth.random_bits(shape, es, 11)]
        m = B.amap_compose([shape], es, ops)
        _run_families(dev, m, srcs, oracle.run_chain(srcs, ops), min_ran=3)


@pytest.mark.parametrize("case", range(len(ALIGNED)))
def test_aligned_shapes(dev, case):
    shape, es, ops = ALIGNED[case]
    print(f"[gpu] aligned case {case} {shape} {ops}", flush=True)
    srcs = [synth.random_bits(shape, es, 5 + case)]
    m = B.amap_compose([shape], es, ops)
    ran = _run_families(dev, m, srcs, oracle.run_chain(srcs, ops), min_ran=3)
    assert None in ran


def test_ragged_tiles_and_tails(dev):
    """Extents that are not multiples of the tile: masked lanes on both axes."""
    for shape, es in [((3, 200, 72), 2), ((2, 100, 36), 4), ((1, 24, 1032), 2), ((5, 8, 8), 2)]:
        ops = [("transpose", (0, 2, 1))]
        srcs = [synth.random_bits(shape, es, 9)]
        m = B.amap_compose([shape], es, ops)
        _run_families(dev, m, srcs, oracle.run_chain(srcs, ops), min_ran=3)


def test_empty_and_single_element(dev):
    import torch
    m = B.amap_compose([(3, 0, 4)], 4, [("transpose", (2, 0, 1))])
    dst = dev.execute(m, [torch.empty((3, 0, 4), dtype=torch.int32, device="cuda")])
    assert dst.numel() == 0
    x = np.array([[0xBEEF]], dtype=np.uint16)
    m = B.amap_compose([(1, 1)], 2, [("transpose", (1, 0)), ("pad", (1, 0), (0, 1), 7)])
    _run_families(dev, m, [x], oracle.run_chain([x], [("transpose", (1, 0)), ("pad", (1, 0), (0, 1), 7)]))


def test_error_paths_on_device(dev):
    import torch
    m = B.amap_compose([(8, 16)], 4, [("transpose", (1, 0))])
    x = torch.zeros((8, 16), dtype=torch.int32, device="cuda")
    with pytest.raises(B.AmapError) as e:
        B.amap_execute([x.data_ptr()], x.data_ptr(), m, 0)
    assert e.value.status == B.AMAP_E_ALIAS
    with pytest.raises(B.AmapError) as e:
        B.amap_execute([x.data_ptr()], x.data_ptr() + 64, m, 0)   # partial overlap
    assert e.value.status == B.AMAP_E_ALIAS
    y = torch.zeros((16, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(B.AmapError) as e:
        B.amap_execute([0], y.data_ptr(), m, 0)
    assert e.value.status == B.AMAP_E_INVALID
    with pytest.raises(B.AmapError) as e:
        B.amap_execute([x.data_ptr() + 4], y.data_ptr(), m, 0)    # misaligned source
    assert e.value.status == B.AMAP_E_INVALID
    torch.cuda.synchronize()


def test_non_default_stream(dev):
    import torch
    w = synth.workload("cfg2_rev", b=2)
    srcs = w.sources()
    m = B.amap_compose(w.src_shapes, 2, w.ops)
    want = oracle.run_chain(srcs, w.ops)
    s = torch.cuda.Stream()
    d = [dev.to_device(x) for x in srcs]
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        dst = dev.execute(m, d)
    s.synchronize()
    assert np.array_equal(dev.to_host(dst), want)


def test_execute_multi_split_outputs(dev):
    """One source, several outputs in one call: Q, K and V as separate tensors, then a mixed bag."""
    import torch
    w = synth.workload("cfg2_fwd", b=2)
    srcs = w.sources()
    maps = [B.amap_compose(w.src_shapes, 2, synth.split_qkv_ops(t, b=2)) for t in range(3)]
    outs = dev.execute_multi(maps, [dev.to_device(srcs[0])])
    torch.cuda.synchronize()
    for t in range(3):
        assert np.array_equal(dev.to_host(outs[t]), oracle.run_chain(srcs, synth.split_qkv_ops(t, b=2))), t
    # maps of different kernel families, a fill-only one, an empty one and more pieces than one launch holds
    shape = (6, 40, 72)
    x = synth.random_bits(shape, 2, 123)
    chains_ = [
        [("transpose", (0, 2, 1))],
        [("slice", 1, 39, -1, -1)],
        [("pad", (1, 2, 3), (3, 2, 1), 0xBEEF)],
        [("repeat", 2, 2), ("transpose", (2, 0, 1))],
        [("slice", 0, 0, 1, 1), ("pad", (0, 1, 8), (0, 1, 8), 7), ("transpose", (0, 2, 1))],
        [("reshape", (240, 72)), ("slice", 0, 3, 230, 7)],
    ]
    maps = [B.amap_compose([shape], 2, ops) for ops in chains_]
    outs = dev.execute_multi(maps, [dev.to_device(x)])
    torch.cuda.synchronize()
    for ops, o in zip(chains_, outs):
        assert np.array_equal(dev.to_host(o), oracle.run_chain([x], ops)), ops
    # a channels-last tensor of 17 x 17 images split into four channel-major branches (flat tiles, in one launch
    # with a plain row copy and a blocked flat tile of another source shape)
    shape = (3, 17, 17, 256)
    x = synth.random_bits(shape, 2, 124)
    chains_ = [[("slice", 3, 64 * b, 64 * b + 64, 1), ("transpose", (0, 3, 1, 2))] for b in range(4)]
    chains_ += [[("slice", 3, 0, 8, 1)], [("reshape", (3, 289, 256)), ("transpose", (0, 2, 1)), ("slice", 2, 1, 288, 1)]]
    maps = [B.amap_compose([shape], 2, ops) for ops in chains_]
    outs = dev.execute_multi(maps, [dev.to_device(x)])
    torch.cuda.synchronize()
    for ops, o in zip(chains_, outs):
        assert np.array_equal(dev.to_host(o), oracle.run_chain([x], ops)), ops
    # overlapping outputs are refused
    d, d_x = dev.empty_dst(maps[0]), dev.to_device(x)
    with pytest.raises(B.AmapError) as e:
        B.amap_execute_multi([d_x.data_ptr()], [d.data_ptr(), d.data_ptr()], [maps[0], maps[0]], 0)
    assert e.value.status == B.AMAP_E_ALIAS


def test_rank_8_and_many_pieces(dev):
    """The rank limit, and maps with more pieces than one launch holds (several launches per call)."""
    shape = (2, 3, 2, 4, 2, 3, 2, 8)
    ops = [("transpose", (7, 0, 6, 1, 5, 2, 4, 3)), ("slice", 3, 1, 3, 1), ("pad", (0,) * 7 + (1,), (1,) + (0,) * 7, 0x1234)]
    x = synth.random_bits(shape, 2, 5)
    m = B.amap_compose([shape], 2, ops)
    assert B.amap_describe(m).rank == 8
    _run_families(dev, m, [x], oracle.run_chain([x], ops), min_ran=2)
    # 24 sources concatenated along the axis that becomes contiguous, then padded: 24 copy pieces + fills
    shapes = [(6, 8 * (1 + i % 3), 40) for i in range(24)]
    srcs = [synth.random_bits(s, 4, 50 + i) for i, s in enumerate(shapes)]
    ops = [("concat", 1), ("transpose", (0, 2, 1)), ("pad", (1, 0, 0), (0, 3, 8), 0xFEEDF00D)]
    m = B.amap_compose(shapes, 4, ops)
    info = B.amap_describe(m)
    assert info.strided and info.n_pieces > 24 and info.n_src == 24
    _run_families(dev, m, srcs, oracle.run_chain(srcs, ops), families=[None, B.AMAP_K_ELEMENT, B.AMAP_K_TILE, B.AMAP_K_WAVE],
                  min_ran=2)


def test_maps_whose_pieces_were_merged(dev):
    """Maps built from many slices and concats, whose pieces the composer merges into loops
    (also loops that walk the source backwards or stand still in it), in every kernel family."""
    rng = np.random.default_rng(0)
    xs = synth.random_bits((1000, 64), 2, 1)
    x = B.amap_source(0, (1000, 64), 2)
    perm = rng.permutation(1000)
    gathered = B.amap_concat([B.amap_slice(x, 0, int(i), int(i) + 1) for i in perm], 0)
    ys = synth.random_bits((8, 6, 40), 2, 2)
    y = B.amap_source(0, (8, 6, 40), 2)
    zs = synth.random_bits((64, 48), 4, 3)
    z = B.amap_source(0, (64, 48), 4)
    cases = [
        ("split + concat", B.amap_concat([B.amap_slice(x, 0, i, i + 1) for i in range(1000)], 0), [xs], xs, 1),
        ("rows in reverse order", B.amap_concat([B.amap_slice(x, 0, 999 - i, 1000 - i) for i in range(1000)], 0), [xs],
         xs[::-1].copy(), 1),
        ("row permutation", gathered, [xs], xs[perm], None),
        ("row permutation, transposed", B.amap_transpose(gathered, (1, 0)), [xs], np.ascontiguousarray(xs[perm].T), None),
        ("slices transposed, then concat", B.amap_concat([B.amap_transpose(B.amap_slice(y, 1, i, i + 1), (1, 0, 2))
                                                           for i in range(6)], 0), [ys],
         np.ascontiguousarray(ys.transpose(1, 0, 2)), 1),
        ("padding in two steps", B.amap_pad(B.amap_pad(z, (1, 1), (1, 1), 5), (2, 3), (1, 0), 5), [zs],
         oracle.run_chain([zs], [("pad", (3, 4), (2, 1), 5)]), None),
        ("source, its mirror image, source", B.amap_concat([z, B.amap_slice(z, 0, 63, -1, -1), z], 0), [zs],
         np.concatenate([zs, zs[::-1], zs], 0), 2),
        ("de-interleave", B.amap_concat([B.amap_slice(z, 1, 0, 48, 2), B.amap_slice(z, 1, 1, 48, 2)], 1), [zs],
         np.concatenate([zs[:, 0::2], zs[:, 1::2]], 1), 1),
    ]
    for name, m, srcs, want, n_pieces in cases:
        print(f"[gpu] merged pieces: {name}", flush=True)
        if n_pieces is not None:
            assert B.amap_describe(m).n_pieces == n_pieces, name
        assert B.amap_plan_selfcheck(m) == 0
        _run_families(dev, m, srcs, want)


def test_gathered_rows(dev):
    """dst contiguous over several loops, source without vectors (3-channel images, repeats by 3,
    a source stride of 5): gathered rows against the oracle, in every family that takes the map."""
    from tests.test_plan_replay import GATHERED, INTERLEAVED
    for i, (shape, es, ops) in enumerate(GATHERED + INTERLEAVED):
        print(f"[gpu] gathered rows case {i}", flush=True)
        x = synth.random_bits(shape, es, 40 + i)
        _run_families(dev, B.amap_compose([shape], es, ops), [x], oracle.run_chain([x], ops))
    import os
    os.environ["AMAP_INTER"] = "0"          # the same maps in the gathered form
    try:
        for i, (shape, es, ops) in enumerate(INTERLEAVED):
            print(f"[gpu] interleaved case {i} as gathered rows", flush=True)
            x = synth.random_bits(shape, es, 70 + i)
            _run_families(dev, B.amap_compose([shape], es, ops), [x], oracle.run_chain([x], ops))
    finally:
        del os.environ["AMAP_INTER"]
    for name, kw in (("rgb_nhwc", {"n": 3}), ("up3x", {"n": 2}), ("s5_nhwc_pad", {"n": 3}), ("s5_nchw_crop", {"n": 3}),
                     ("i35_nchw", {"n": 2}), ("i55_nchw", {"n": 2}), ("c8_nhwc", {"n": 5})):
        print(f"[gpu] gathered rows workload {name}", flush=True)
        w = synth.workload(name, **kw)
        srcs = w.sources()
        m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
        assert B.amap_describe(m).vec_bytes == 16
        _run_families(dev, m, srcs, oracle.run_chain(srcs, w.ops))


def test_cross_lane_rows(dev, monkeypatch, capfd):
    """Short dst rows in the cross-lane form (one vector per lane, V x V blocks exchanged between
    lanes): the small cases of the replay tests and sizes of many wavefronts with ragged tails, both
    with the form planned wherever it applies and with the default choice."""
    from tests.test_plan_replay import XLANE
    big = [
        ((37, 8, 1000), 2, [("transpose", (0, 2, 1))]),
        ((37, 16, 1000), 2, [("transpose", (0, 2, 1))]),
        ((21, 4, 1028), 4, [("transpose", (0, 2, 1))]),
        ((21, 20, 516), 4, [("transpose", (0, 2, 1))]),
        ((9, 56, 520), 2, [("transpose", (0, 2, 1))]),
        ((33, 16, 24, 32), 4, [("transpose", (0, 2, 3, 1)), ("reshape", (33, 768, 16)),
                               ("slice", 1, 96, 672, 1), ("pad", (0, 0, 0), (0, 0, 4), 0)]),
        ((64, 8, 32, 32), 2, [("transpose", (0, 2, 3, 1))]),
    ]
    for setting in ("2", None):
        if setting:
            monkeypatch.setenv("AMAP_XLANE", setting)
        else:
            monkeypatch.delenv("AMAP_XLANE")
        for i, (shape, es, ops) in enumerate(XLANE + big):
            print(f"[gpu] cross-lane case {i} AMAP_XLANE={setting}", flush=True)
            x = synth.random_bits(shape, es, 300 + i)
            monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
            capfd.readouterr()
            m = B.amap_compose([shape], es, ops)
            B.amap_describe(m)
            monkeypatch.delenv("AMAP_PLAN_TRACE")
            planned = "amap plan: xlane" in capfd.readouterr().err
            assert planned or not setting
            _run_families(dev, m, [x], oracle.run_chain([x], ops))


def test_blocked_row_order(dev, monkeypatch):
    """Short rows in the blocked order (planned from 2^21 vectors up; the floor is lowered so that the
    small cases take it too), then a head split of the planned size as it is."""
    from tests.test_plan_replay import BLOCKED_ROWS
    big = [
        ((6, 200, 3, 4, 64), 2, [("transpose", (2, 0, 3, 1, 4))]),
        ((5, 12, 333, 32), 4, [("transpose", (0, 2, 1, 3))]),
    ]
    monkeypatch.setenv("AMAP_ROWS_BLOCK_MIN_LOG2", "0")
    for i, (shape, es, ops) in enumerate(BLOCKED_ROWS + big):
        print(f"[gpu] blocked rows case {i}", flush=True)
        x = synth.random_bits(shape, es, 500 + i)
        _run_families(dev, B.amap_compose([shape], es, ops), [x], oracle.run_chain([x], ops))
    monkeypatch.delenv("AMAP_ROWS_BLOCK_MIN_LOG2")
    print("[gpu] blocked rows at the planned size", flush=True)
    shape, ops = (20, 512, 3, 4, 64), [("transpose", (2, 0, 3, 1, 4))]      # 2^21.3 vectors
    x = synth.random_bits(shape, 2, 77)
    _run_families(dev, B.amap_compose([shape], 2, ops), [x], oracle.run_chain([x], ops), families=[None, B.AMAP_K_ROWS])


def test_keep_plane_rows(dev):
    """A slice with a small step along the contiguous dimension (step 2 on 2-byte elements keeps one
    plane of an interleaved source in registers, the rest is gathered):
    every small case of the replay tests, then sizes of several blocks with a ragged last one."""
    from tests.test_plan_replay import KEEP_PLANE
    big = [
        ((37, 5, 128), 2, [("slice", 2, 0, 128, 2)]),
        ((37, 5, 128), 2, [("slice", 2, 1, 128, 2)]),
        ((1031, 264), 4, [("slice", 1, 2, 264, 3)]),
        ((1031, 264), 4, [("slice", 1, 0, 262, 3)]),
        ((513, 1024), 2, [("slice", 1, 3, 1024, 4)]),
        ((300, 520), 2, [("slice", 0, 299, -1, -1), ("slice", 1, 1, 520, 2), ("reshape", (300, 4, 65))]),
    ]
    for i, (shape, es, ops) in enumerate(KEEP_PLANE + big):
        print(f"[gpu] keep-plane rows case {i}", flush=True)
        x = synth.random_bits(shape, es, 90 + i)
        m = B.amap_compose([shape], es, ops)
        assert B.amap_plan_selfcheck(m) == 0
        _run_families(dev, m, [x], oracle.run_chain([x], ops))


def test_flat_tiles(dev):
    """Transposing pieces that are contiguous on one side with a row length that offers no vectors
    (7 x 7 positions per channel): blocks of 64 rows staged through LDS as one flat run, in both
    directions, with a ragged last block, rows at a pitch and workgroups of 1 and 4 wavefronts."""
    import os
    from tests.test_plan_replay import FLAT, FLAT_OTHER, STRADDLE
    big = [
        ((8, 2048, 7, 7), 2, [("transpose", (0, 2, 3, 1))]),
        ((8, 7, 7, 2048), 2, [("transpose", (0, 3, 1, 2))]),
        ((5, 328, 9, 9), 4, [("transpose", (0, 2, 3, 1))]),
        ((5, 9, 9, 328), 4, [("transpose", (0, 3, 1, 2))]),
        ((3, 1000, 121), 2, [("slice", 1, 8, 1000, 1), ("transpose", (0, 2, 1))]),
        ((3, 121, 1000), 2, [("slice", 2, 1, 993, 1), ("transpose", (0, 2, 1))]),
    ]
    big.append(((4, 256, 28, 28), 2, [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]))  # tile vectors across image rows
    for i, (shape, es, ops) in enumerate(FLAT + FLAT_OTHER + big + STRADDLE):
        x = synth.random_bits(shape, es, 110 + i)
        want = oracle.run_chain([x], ops)
        for waves in (None, "2"):
            print(f"[gpu] flat tiles case {i} waves_log {waves}", flush=True)
            if waves is not None:
                os.environ["AMAP_WAVES_LOG"] = waves
            try:
                m = B.amap_compose([shape], es, ops)
                assert B.amap_plan_selfcheck(m) == 0
                _run_families(dev, m, [x], want)
            finally:
                os.environ.pop("AMAP_WAVES_LOG", None)


def test_random_transposing_maps(dev):
    """Random transpositions with pads and crops around them (the generator of the replay tests):
    the planned form and the forced tile family against the oracle, after the host replay of the
    plan has found every access in bounds."""
    import torch
    from tests.test_plan_replay import _random_transposing_map
    rng = np.random.default_rng(77)
    ran = 0
    for it in range(120):
        shape, es, ops = _random_transposing_map(rng)
        x = synth.random_bits(shape, es, 500 + it)
        want = oracle.run_chain([x], ops)
        m = B.amap_compose([shape], es, ops)
        d_x = [dev.to_device(x)]
        for fam in (None, B.AMAP_K_TILE):
            try:
                assert B.amap_plan_selfcheck(m, -1 if fam is None else fam) == 0, (shape, es, ops, fam)
            except B.AmapError:
                continue
            print(f"[gpu] random transposing map {it} family {fam}: {shape} {es} {ops}", flush=True)
            dst = dev.empty_dst(m, fill=0x5A5A if es == 2 else 0x5A5A5A5A)
            dev.execute(m, d_x, dst, kernel_id=fam)
            torch.cuda.synchronize()
            assert np.array_equal(dev.to_host(dst).view(want.dtype).reshape(want.shape), want), (shape, es, ops, fam)
            ran += 1
    assert ran >= 150


def test_concat_of_odd_sized_images(dev):
    """Channel concat of channel-major branches made channels-last (and the other way round) at image
    sizes whose rows offer no vectors: every branch is a flat tile piece of its own."""
    from tests.test_plan_replay import CONCAT_ODD_IMAGES
    big = [([(4, c, 17, 17) for c in (192, 192, 192, 192)], 2, [("concat", 1), ("transpose", (0, 2, 3, 1))]),
           ([(3, c, 35, 35) for c in (64, 64, 96, 32)], 2, [("concat", 1), ("transpose", (0, 2, 3, 1))])]
    for i, (shapes, es, ops) in enumerate(CONCAT_ODD_IMAGES + big):
        print(f"[gpu] concat of odd-sized images case {i}", flush=True)
        xs = [synth.random_bits(sh, es, 200 + 10 * i + k) for k, sh in enumerate(shapes)]
        m = B.amap_compose(shapes, es, ops)
        assert B.amap_plan_selfcheck(m) == 0
        _run_families(dev, m, xs, oracle.run_chain(xs, ops))


def test_one_map_executed_from_several_host_threads(dev):
    """A map is immutable once built (its launch plan included), so host threads may execute the
    same map at the same time, each on a stream of its own."""
    import threading
    import torch
    w = synth.workload("cfg1", n=2)
    srcs = w.sources()
    m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
    want = oracle.run_chain(srcs, w.ops)
    d_srcs = [dev.to_device(s) for s in srcs]
    torch.cuda.synchronize()
    n_threads, reps = 4, 25
    dsts = [[dev.empty_dst(m, fill=0x7777) for _ in range(reps)] for _ in range(n_threads)]
    streams = [torch.cuda.Stream() for _ in range(n_threads)]
    errors = []

    def work(t):
        try:
            for r in range(reps):
                B.amap_execute([s.data_ptr() for s in d_srcs], dsts[t][r].data_ptr(), m, streams[t].cuda_stream)
            streams[t].synchronize()
        except Exception as e:  # noqa: BLE001 - reported below
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=work, args=(t,)) for t in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for t in range(n_threads):
        for r in (0, reps - 1):
            assert np.array_equal(dev.to_host(dsts[t][r]), want), (t, r)


def test_plan_of_large_tensors_on_the_workload_structures(dev):
    """From 256 MB of dst on, the planner switches to workgroups of 4 wavefronts with tiles staged in LDS
    (XOR-swizzled slots; cfg3 in the grouped form).  The switches bring that plan to sizes the oracle
    finishes in seconds: cfg1's border fills, cfg3's four-source groups, cfg2's row copies and cfg0's
    chain at 64 x its batch, each bit for bit in every kernel family that takes the map."""
    import os
    cfg0 = synth.workload("cfg0")
    cases = [
        ("cfg1 n=2", synth.workload("cfg1", n=2), None),
        ("cfg3 n=2", synth.workload("cfg3", n=2), None),
        ("cfg2_rev b=2", synth.workload("cfg2_rev", b=2), None),
        ("cfg2_fwd b=2", synth.workload("cfg2_fwd", b=2), None),
        ("cfg0 x64", None, ((512, 16, 32, 32), 4, [cfg0.ops[0], ("reshape", (512, 1024, 16)), cfg0.ops[2], cfg0.ops[3]])),
    ]
    for label, w, raw in cases:
        if w is not None:
            shapes, es, ops, srcs = w.src_shapes, w.elem_size, w.ops, w.sources()
        else:
            shape, es, ops = raw
            shapes, srcs = [shape], [synth.random_bits(shape, es, 4242)]
        oracle.set_threads(8)
        try:
            want = oracle.run_chain(srcs, ops)
        finally:
            oracle.set_threads(1)
        for env in ({"AMAP_WAVES_LOG": "2"}, {"AMAP_SMALL_BYTES_MB": "0"}):
            print(f"[gpu] large-tensor plan on {label} under {env}", flush=True)
            os.environ.update(env)
            try:
                m = B.amap_compose(shapes, es, ops)
                assert B.amap_plan_selfcheck(m) == 0
                ran = _run_families(dev, m, srcs, want, min_ran=3)
                assert None in ran
            finally:
                for k in env:
                    os.environ.pop(k, None)
