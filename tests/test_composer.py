"""Host composer vs the oracle (CPU only): the composed map, evaluated on the
host, must reproduce the un-optimised operator-by-operator program bit for bit.
Distinct source elements (iota) turn the output into the address table, so a
mismatch points at an index."""
import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth
from tests import chains


def _iota_sources(shapes, es):
    srcs, base = [], 1
    for s in shapes:
        n = int(np.prod(s))
        dt = np.uint16 if es == 2 else np.uint32
        srcs.append(((np.arange(n, dtype=np.uint64) + base) % (65521 if es == 2 else 4294967291)).astype(dt).reshape(s))
        base += n
    return srcs


def _distinct_data_elements(srcs, ops, want):
    """Distinct source elements a chain reads, from the oracle alone: positions whose value
    follows a change of every source value are data, and iota sources make values = addresses."""
    other = [(~s) for s in srcs]
    data = oracle.run_chain(other, ops) != want
    return len(np.unique(want[data]))


def _check_map(m, srcs, want, expect_strided=None, ops=None):
    info = B.amap_describe(m)
    assert B.dst_shape(m) == want.shape
    got_prog = B.amap_eval_host(m, srcs, mode=1)
    assert np.array_equal(got_prog, want), "operator program"
    if expect_strided is not None:
        assert bool(info.strided) == expect_strided
    if info.strided:
        got = B.amap_eval_host(m, srcs, mode=2)
        assert np.array_equal(got, want), "strided pieces"
        assert B.amap_check_cover(m) == (0, 0)
        assert info.write_bytes == want.nbytes
        if ops is None:
            assert info.min_read_bytes + info.fill_bytes == want.nbytes
    if ops is not None:
        assert info.min_read_bytes == _distinct_data_elements(srcs, ops, want) * want.dtype.itemsize


@pytest.mark.parametrize("name", synth.WORKLOAD_NAMES)
def test_workload_maps_small_values(name):
    w = synth.workload(name)
    srcs = w.sources()
    want = oracle.run_chain(srcs, w.ops)
    m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
    _check_map(m, srcs, want, expect_strided=True)


def test_workload_piece_counts_and_bytes():
    exp = {  # name: (pieces, fill pieces, min read bytes, write bytes, fill bytes)
        "cfg0": (2, 1, 393216, 491520, 24576 * 4),
        "cfg1": (3, 2, 51380224, 55115776, 1867776 * 2),   # top+bottom and left+right borders: one loop of two each
        "cfg2_fwd": (1, 0, 37748736, 37748736, 0),
        "cfg2_rev": (1, 0, 12582912, 12582912, 0),
        "cfg3": (4, 0, 16056320, 16056320, 0),
        "cfg4": (1, 0, 16777216, 16777216, 0),
    }
    for name, (np_, nf, rd, wr, fb) in exp.items():
        w = synth.workload(name)
        info = B.amap_describe(B.amap_compose(w.src_shapes, w.elem_size, w.ops))
        assert (info.n_pieces, info.n_fill_pieces) == (np_, nf), name
        assert (info.min_read_bytes, info.write_bytes, info.fill_bytes) == (rd, wr, fb), name


def test_builders_equal_one_shot():
    w = synth.workload("cfg3")
    ms = [B.amap_source(i, s, 2) for i, s in enumerate(w.src_shapes)]
    m = B.amap_transpose(B.amap_concat(ms, 1), (0, 2, 3, 1))
    srcs = w.sources()
    assert np.array_equal(B.amap_eval_host(m, srcs), oracle.run_chain(srcs, w.ops))


@pytest.mark.parametrize("seed", range(300))
def test_random_chains(seed):
    src_shapes, ops = chains.random_chain(seed)
    es = 2 if seed % 2 else 4
    srcs = _iota_sources(src_shapes, es)
    want = oracle.run_chain(srcs, ops)
    m = B.amap_compose(src_shapes, es, ops)
    _check_map(m, srcs, want)


@pytest.mark.parametrize("seed", range(300))
def test_random_chains_with_repeat_tile_and_downward_slices(seed):
    src_shapes, ops = chains.random_chain(seed, extended=True)
    es = 2 if seed % 2 else 4
    srcs = _iota_sources(src_shapes, es)
    want = oracle.run_chain(srcs, ops)
    m = B.amap_compose(src_shapes, es, ops)
    _check_map(m, srcs, want, ops=ops)


def test_random_chains_mostly_strided():
    n = sum(bool(B.amap_describe(B.amap_compose(s, 4, o)).strided)
            for s, o in (chains.random_chain(k) for k in range(300)))
    assert n >= 270, n


def test_tree_of_builders_with_per_branch_ops():
    rng = np.random.default_rng(5)
    for trial in range(40):
        base = chains.random_shape(rng, max_rank=3, max_extent=6)
        ax = int(rng.integers(len(base)))
        maps, outs, srcs = [], [], []
        for j in range(int(rng.integers(2, 4))):
            # each branch: its own source, one random op that keeps the rank and the off-axis extents
            s = list(base)
            s[ax] = int(rng.integers(2, 6))
            x = _iota_sources([s], 4)[0] + 1000 * j
            m = B.amap_source(j, s, 4)
            b = int(rng.integers(0, s[ax] - 1))
            m = B.amap_slice(m, ax, b, s[ax], 1)
            y = oracle.slice_(x, ax, b, s[ax], 1)
            maps.append(m)
            outs.append(y)
            srcs.append(x)
        m = B.amap_concat(maps, ax)
        want = oracle.concat(outs, ax)
        perm = tuple(int(v) for v in rng.permutation(len(base)))
        m = B.amap_transpose(m, perm)
        want = oracle.transpose(want, perm)
        _check_map(m, srcs, want, expect_strided=True)


def test_same_source_twice():
    x = _iota_sources([(3, 4)], 4)[0]
    s = B.amap_source(0, (3, 4), 4)
    m = B.amap_concat([s, B.amap_transpose(B.amap_reshape(s, (4, 3)), (1, 0))], 1)
    want = oracle.concat([x, oracle.transpose(oracle.reshape(x, (4, 3)), (1, 0))], 1)
    assert np.array_equal(B.amap_eval_host(m, [x]), want)


def test_misaligned_reshape_after_slice_splits_pieces():
    x = _iota_sources([(4, 32)], 4)[0]
    ops = [("reshape", (128,)), ("slice", 0, 5, 101, 1), ("reshape", (8, 12))]
    m = B.amap_compose([(4, 32)], 4, ops)
    _check_map(m, [x], oracle.run_chain([x], ops), expect_strided=True)
    ops = [("slice", 1, 3, 31, 1), ("reshape", (16, 7)), ("transpose", (1, 0))]
    m = B.amap_compose([(4, 32)], 4, ops)
    _check_map(m, [x], oracle.run_chain([x], ops), expect_strided=True)


@pytest.mark.parametrize("shape,to", [((2, 12), (3, 8)), ((6, 4, 10), (5, 48)), ((7, 9), (3, 21)), ((7, 9), (63,)),
                                      ((8, 8), (4, 4, 4)), ((4, 6), (2, 12)), ((3, 5, 7), (7, 15))])
def test_reshape_of_a_contiguous_tensor_is_one_piece(shape, to):
    """Loops that continue one another are merged and re-split along the new shape, so a
    reshape across the old dimension boundaries of a whole tensor stays a single piece,
    also behind a transposition that keeps the reshaped dimensions together."""
    srcs = _iota_sources([shape], 4)
    m = B.amap_compose([shape], 4, [("reshape", to)])
    assert B.amap_describe(m).n_pieces == 1
    _check_map(m, srcs, oracle.run_chain(srcs, [("reshape", to)]), expect_strided=True)
    # two leading batch dimensions swapped, the rest reshaped across its boundaries
    ops = [("transpose", (1, 0) + tuple(range(2, 2 + len(shape)))), ("reshape", (3, 2) + tuple(to))]
    big = (2, 3) + tuple(shape)
    srcs = _iota_sources([big], 4)
    m = B.amap_compose([big], 4, ops)
    assert B.amap_describe(m).n_pieces == 1
    _check_map(m, srcs, oracle.run_chain(srcs, ops), expect_strided=True)


def test_pieces_that_continue_one_another_are_merged():
    """split + concat, slices processed alike and put together again, a source repeated by concat,
    the two halves of a padding ring: pieces that are one box displaced along one dimension
    become one piece (checked element by element against the operators run one at a time)."""
    es = 4
    x = _iota_sources([(4, 10)], es)[0]
    sx = B.amap_source(0, (4, 10), es)

    def check(m, want, n_pieces, distinct=None):
        info = B.amap_describe(m)
        assert info.n_pieces == n_pieces
        if distinct is None:
            _check_map(m, [x], want, expect_strided=True)
            return
        # the same source elements read more than once
        assert np.array_equal(B.amap_eval_host(m, [x], mode=1), want) and np.array_equal(B.amap_eval_host(m, [x], mode=2), want)
        assert B.amap_check_cover(m) == (0, 0) and info.min_read_bytes == distinct * es

    check(B.amap_concat([B.amap_slice(sx, 1, 0, 4), B.amap_slice(sx, 1, 4, 10)], 1), x, 1)           # split, concat
    check(B.amap_concat([B.amap_slice(sx, 0, 0, 1), B.amap_slice(sx, 0, 1, 2), B.amap_slice(sx, 0, 2, 4)], 0), x, 1)
    check(B.amap_concat([B.amap_slice(sx, 1, 4, 10), B.amap_slice(sx, 1, 0, 4)], 1),
          np.concatenate([x[:, 4:], x[:, :4]], axis=1), 2)                                         # a rotation stays two
    check(B.amap_concat([sx, sx, sx], 0), np.concatenate([x, x, x], axis=0), 1, distinct=40)       # = tile
    check(B.amap_concat([sx, B.amap_slice(sx, 0, 3, -1, -1), sx], 0), np.concatenate([x, x[::-1], x], axis=0), 2, distinct=40)
    ring = B.amap_pad(B.amap_pad(sx, (1, 0), (1, 0), 7), (1, 0), (1, 0), 7)
    check(ring, oracle.run_chain([x], [("pad", (2, 0), (2, 0), 7)]), 3)                             # data + two border loops
    y = _iota_sources([(8, 6, 10)], es)[0]
    sy = B.amap_source(0, (8, 6, 10), es)
    m = B.amap_concat([B.amap_transpose(B.amap_slice(sy, 1, i, i + 1), (1, 0, 2)) for i in range(6)], 0)
    assert B.amap_describe(m).n_pieces == 1
    _check_map(m, [y], np.ascontiguousarray(y.transpose(1, 0, 2)), expect_strided=True)
    # a piece that already has as many loops as a launch holds is not given one more
    shape8 = (2, 3, 2, 4, 2, 3, 2, 8)
    t8 = B.amap_transpose(B.amap_source(0, shape8, es), (7, 0, 6, 1, 5, 2, 4, 3))
    twice = B.amap_concat([t8, t8], 0)
    assert B.amap_describe(twice).n_pieces == 2 and B.amap_plan_selfcheck(twice) == 0
    halves = B.amap_concat([B.amap_slice(t8, 0, 0, 4), B.amap_slice(t8, 0, 4, 8)], 0)
    assert B.amap_describe(halves).n_pieces == 1 and B.amap_plan_selfcheck(halves) == 0
    # different constants do not merge
    two = B.amap_pad(B.amap_pad(sx, (1, 0), (0, 0), 1), (0, 0), (1, 0), 2)
    assert B.amap_describe(two).n_fill_pieces == 2


def test_pad_then_flatten_and_step_slices():
    x = _iota_sources([(2, 3, 5, 6)], 2)[0]
    ops = [("pad", (0, 0, 1, 1), (0, 0, 1, 1), 7), ("reshape", (6, 56)), ("slice", 1, 3, 50, 3)]
    m = B.amap_compose([(2, 3, 5, 6)], 2, ops)
    _check_map(m, [x], oracle.run_chain([x], ops))
    ops = [("reshape", (6, 30)), ("slice", 1, 1, 29, 2), ("reshape", (6, 2, 7)), ("slice", 2, 1, 7, 4)]
    m = B.amap_compose([(2, 3, 5, 6)], 2, ops)
    _check_map(m, [x], oracle.run_chain([x], ops))


def test_inverse_closed_forms():
    for name in ["cfg2_fwd", "cfg2_rev", "cfg4"]:
        w = synth.workload(name)
        m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
        inv = B.amap_inverse(m)
        assert B.dst_shape(inv) == w.src_shapes[0]
        x = synth.random_bits(w.src_shapes[0], 2, 3)
        y = B.amap_eval_host(m, [x])
        assert np.array_equal(B.amap_eval_host(inv, [y], mode=2), x)
    # small: program and pieces of the inverse agree; inverse of inverse is the map
    x = _iota_sources([(4, 6, 10)], 4)[0]
    ops = [("transpose", (2, 0, 1)), ("reshape", (5, 8, 6)), ("transpose", (1, 2, 0))]
    m = B.amap_compose([(4, 6, 10)], 4, ops)
    y = oracle.run_chain([x], ops)
    inv = B.amap_inverse(m)
    assert np.array_equal(B.amap_eval_host(inv, [y], mode=1), x)
    assert np.array_equal(B.amap_eval_host(inv, [y], mode=2), x)
    assert np.array_equal(B.amap_eval_host(B.amap_inverse(inv), [x]), y)
    # transpose o transpose^-1 = identity, via the map algebra alone
    t = B.amap_transpose(B.amap_source(0, (3, 4, 5), 4), (2, 0, 1))
    ti = B.amap_inverse(t)
    xs = _iota_sources([(3, 4, 5)], 4)[0]
    assert np.array_equal(B.amap_eval_host(ti, [B.amap_eval_host(t, [xs])]), xs)


def test_repeat_tile_closed_forms():
    x = _iota_sources([(3, 4, 5)], 4)[0]
    s = B.amap_source(0, (3, 4, 5), 4)
    # every r-th element of a repeat is the input; the map algebra cancels the division
    m = B.amap_slice(B.amap_repeat(s, 1, 3), 1, 2, 12, 3)
    assert np.array_equal(B.amap_eval_host(m, [x], mode=2), x)
    info = B.amap_describe(m)
    assert (info.n_pieces, info.min_read_bytes) == (1, x.nbytes)
    # one block of a tile is the input
    m = B.amap_slice(B.amap_tile(s, 2, 4), 2, 10, 15, 1)
    assert np.array_equal(B.amap_eval_host(m, [x], mode=2), x)
    assert B.amap_describe(m).n_pieces == 1
    # broadcast: tile of an extent-1 axis, 7 copies read 12 elements
    b = B.amap_tile(B.amap_reshape(B.amap_slice(s, 2, 1, 2, 1), (3, 1, 4)), 1, 7)
    info = B.amap_describe(b)
    assert (info.min_read_bytes, info.write_bytes) == (12 * 4, 84 * 4)
    assert np.array_equal(B.amap_eval_host(b, [x]), np.broadcast_to(x[:, :, 1].reshape(3, 1, 4), (3, 7, 4)))
    # repeat = reshape / tile / reshape, both forms give the same table
    r1 = B.amap_repeat(s, 2, 2)
    r2 = B.amap_reshape(B.amap_tile(B.amap_reshape(s, (3, 4, 5, 1)), 3, 2), (3, 4, 10))
    assert np.array_equal(B.amap_eval_host(r1, [x], mode=2), B.amap_eval_host(r2, [x], mode=2))
    assert np.array_equal(B.amap_eval_host(r1, [x]), np.repeat(x, 2, axis=2))
    # reversing an axis twice cancels to the identity piece
    f = B.amap_slice(B.amap_slice(s, 1, 3, -1, -1), 1, 3, -1, -1)
    assert np.array_equal(B.amap_eval_host(f, [x], mode=2), x)
    assert B.amap_describe(f).kernel_id == B.AMAP_K_ROWS


def test_inverse_of_reversed_axes():
    x = _iota_sources([(4, 6, 5)], 4)[0]
    ops = [("slice", 1, 5, -1, -1), ("transpose", (2, 0, 1)), ("slice", 0, 4, -1, -1), ("reshape", (10, 12))]
    m = B.amap_compose([(4, 6, 5)], 4, ops)
    y = oracle.run_chain([x], ops)
    inv = B.amap_inverse(m)
    assert np.array_equal(B.amap_eval_host(inv, [y], mode=1), x)
    assert np.array_equal(B.amap_eval_host(inv, [y], mode=2), x)


def test_inverse_refuses_non_bijections():
    s = B.amap_source(0, (4, 6), 4)
    for m in [B.amap_slice(s, 1, 0, 3, 1), B.amap_pad(s, (0, 1), (0, 0), 0),
              B.amap_concat([s, s], 0), B.amap_repeat(s, 0, 2), B.amap_tile(s, 1, 3),
              B.amap_slice(s, 1, 5, 1, -1)]:
        with pytest.raises(B.AmapError) as e:
            B.amap_inverse(m)
        assert e.value.status == B.AMAP_E_UNSUPPORTED


def test_error_paths():
    s = B.amap_source(0, (4, 6), 4)
    cases = [
        (lambda: B.amap_source(0, (), 4), B.AMAP_E_INVALID),
        (lambda: B.amap_source(0, (1,) * 9, 4), B.AMAP_E_INVALID),
        (lambda: B.amap_source(0, (2, 3), 3), B.AMAP_E_INVALID),
        (lambda: B.amap_source(-1, (2, 3), 4), B.AMAP_E_INVALID),
        (lambda: B.amap_transpose(s, (0, 0)), B.AMAP_E_INVALID),
        (lambda: B.amap_transpose(s, (0, 2)), B.AMAP_E_INVALID),
        (lambda: B.amap_reshape(s, (5, 5)), B.AMAP_E_SHAPE),
        (lambda: B.amap_slice(s, 2, 0, 1, 1), B.AMAP_E_INVALID),
        (lambda: B.amap_slice(s, 1, 3, 3, 1), B.AMAP_E_SHAPE),
        (lambda: B.amap_slice(s, 1, 0, 7, 1), B.AMAP_E_SHAPE),
        (lambda: B.amap_slice(s, 1, 0, 6, 0), B.AMAP_E_SHAPE),
        (lambda: B.amap_slice(s, 1, 2, 2, -1), B.AMAP_E_SHAPE),
        (lambda: B.amap_slice(s, 1, 6, 0, -1), B.AMAP_E_SHAPE),
        (lambda: B.amap_slice(s, 1, 3, -2, -1), B.AMAP_E_SHAPE),
        (lambda: B.amap_repeat(s, 2, 2), B.AMAP_E_INVALID),
        (lambda: B.amap_repeat(s, 0, 0), B.AMAP_E_SHAPE),
        (lambda: B.amap_tile(s, -1, 2), B.AMAP_E_INVALID),
        (lambda: B.amap_tile(s, 0, 0), B.AMAP_E_SHAPE),
        (lambda: B.amap_pad(s, (0, -1), (0, 0)), B.AMAP_E_SHAPE),
        (lambda: B.amap_concat([s, B.amap_source(1, (5, 7), 4)], 0), B.AMAP_E_SHAPE),
        (lambda: B.amap_concat([s, B.amap_source(1, (4, 6), 2)], 0), B.AMAP_E_INVALID),
        (lambda: B.amap_concat([s, B.amap_source(0, (4, 7), 4)], 1), B.AMAP_E_SHAPE),
        (lambda: B.amap_compose([(2, 3), (2, 3)], 4, [("transpose", (1, 0))]), B.AMAP_E_INVALID),
        (lambda: B.amap_compose([(2, 3)], 4, [("transpose", (1, 0)), ("concat", 0)]), B.AMAP_E_INVALID),
    ]
    for fn, status in cases:
        with pytest.raises(B.AmapError) as e:
            fn()
        assert e.value.status == status, (fn, e.value.status)
    assert B.amap_status_str(B.AMAP_E_ALIAS) == "dst overlaps a source"


def test_empty_tensor():
    m = B.amap_compose([(3, 0, 4)], 4, [("transpose", (2, 0, 1)), ("reshape", (0, 7))])
    info = B.amap_describe(m)
    assert info.write_bytes == 0 and info.n_pieces == 0
    out = B.amap_eval_host(m, [np.zeros((3, 0, 4), np.uint32)])
    assert out.shape == (0, 7)


def test_describe_of_an_upsampling_map_needs_no_walk_over_the_source():
    """The distinct-element count of a repeat / tile over a huge source is a closed form: describing such a
    map allocates nothing of the source's size and returns at once."""
    m = B.amap_source(0, (1 << 20, 1 << 20), 2)
    m = B.amap_repeat(m, 0, 2)
    info = B.amap_describe(m)
    assert info.min_read_bytes == (1 << 40) * 2 and info.write_bytes == (1 << 41) * 2
    assert B.dst_shape(m) == (1 << 21, 1 << 20)
    # a source used twice by concat: two pieces read it, so the elements are counted one by one
    a = B.amap_source(0, (6, 8), 2)
    c = B.amap_concat([B.amap_slice(a, 0, 0, 4, 1), B.amap_slice(a, 0, 2, 6, 1)], 0)
    assert B.amap_describe(c).min_read_bytes == 6 * 8 * 2
    # ... and refused (not a crash) when the marks would not fit
    big = B.amap_source(0, (1 << 20, 1 << 20), 2)
    assert B.amap_describe(B.amap_concat([big, big], 0)).min_read_bytes == (1 << 40) * 2   # merged into one piece with a loop that stands still
    c2 = B.amap_concat([B.amap_slice(big, 0, 0, 1 << 19, 1), B.amap_slice(big, 0, 1 << 18, 1 << 19, 1)], 0)
    with pytest.raises(B.AmapError) as e:
        B.amap_describe(c2)
    assert e.value.status == B.AMAP_E_NOMEM


def test_no_program_plan_through_an_intermediate_of_2_to_31_elements():
    """small source -> tile to 2^32 elements -> reshape -> slice back to a small dst: source and dst fit 32-bit
    offsets, the intermediate does not, so the interpreter (32-bit intermediate indices) must refuse it."""
    import ctypes as C
    m = B.amap_source(0, (1 << 16,), 2)
    m = B.amap_reshape(m, (1, 1 << 16))
    m = B.amap_tile(m, 0, 1 << 16)                   # [65536, 65536]
    m = B.amap_reshape(m, (1 << 32,))
    m = B.amap_slice(m, 0, (1 << 32) - 4096, 1 << 32, 1)
    assert B.dst_shape(m) == (4096,)
    src = (C.c_uint16 * (1 << 16))()
    dst = (C.c_uint16 * 8192)()
    sp = (C.addressof(src) + 15) & ~15
    dp = (C.addressof(dst) + 15) & ~15
    with pytest.raises(B.AmapError) as e:
        B.amap_execute([sp], dp, m, 0, kernel_id=B.AMAP_K_PROGRAM)   # refused before anything is launched
    assert e.value.status == B.AMAP_E_UNSUPPORTED
    # the same chain at a size where every intermediate fits keeps its program form
    s2 = B.amap_slice(B.amap_reshape(B.amap_tile(B.amap_reshape(B.amap_source(0, (64,), 2), (1, 64)), 0, 64), (4096,)), 0, 100, 200, 1)
    assert np.array_equal(B.amap_eval_host(s2, [np.arange(64, dtype=np.uint16)], mode=1), np.arange(100, 200, dtype=np.uint16) % 64)


def test_short_source_table_is_refused_by_the_binding():
    c = B.amap_concat([B.amap_source(0, (4, 8), 2), B.amap_source(1, (4, 8), 2)], 0)
    with pytest.raises(B.AmapError) as e:
        B.amap_execute([16], 4096, c, 0)             # source 1 has no pointer: refused before the library reads the table
    assert e.value.status == B.AMAP_E_INVALID
