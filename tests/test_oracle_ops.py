"""Pins for the single-operator oracle functions (CPU only).

Each operator is checked against (i) hand-worked fixtures, (ii) the numpy
library routine it reduces to, on tensors whose elements are all distinct so
that any index mistake shows, (iii) its inverse identities, (iv) error paths.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import synth


def _parse_vals(s, dtype=np.uint32):
    return np.array([int(v) for v in s.split()], dtype=dtype)


def _golden_cases(path):
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            yield [p.strip() for p in line.split("|")]


@pytest.mark.parametrize("dtype", [np.uint16, np.uint32])
def test_handworked_fixture(golden_dir, dtype):
    n = 0
    for op, args, in_shapes, in_vals, out_shape, out_vals in _golden_cases(
            os.path.join(golden_dir, "handworked_ops.txt")):
        shapes = [tuple(int(v) for v in s.split(",")) for s in in_shapes.split(";")]
        vals = [_parse_vals(v, dtype) for v in in_vals.split(";")]
        xs = [v.reshape(s) for v, s in zip(vals, shapes)]
        want = _parse_vals(out_vals, dtype).reshape(tuple(int(v) for v in out_shape.split(",")))
        if op == "transpose":
            got = oracle.transpose(xs[0], [int(v) for v in args.split("=")[1].split(",")])
        elif op == "reshape":
            got = oracle.reshape(xs[0], [int(v) for v in args.split("=")[1].split(",")])
        elif op == "slice":
            kv = dict(a.split("=") for a in args.split(","))
            got = oracle.slice_(xs[0], int(kv["axis"]), int(kv["begin"]), int(kv["end"]),
                                int(kv["step"]))
        elif op == "pad":
            kv = dict(a.split("=") for a in args.split(";"))
            got = oracle.pad(xs[0], [int(v) for v in kv["lo"].split(",")],
                             [int(v) for v in kv["hi"].split(",")], int(kv["fill"]))
        elif op == "concat":
            got = oracle.concat(xs, int(args.split("=")[1]))
        elif op == "repeat":
            kv = dict(a.split("=") for a in args.split(","))
            got = oracle.repeat(xs[0], int(kv["axis"]), int(kv["r"]))
        elif op == "tile":
            kv = dict(a.split("=") for a in args.split(","))
            got = oracle.tile(xs[0], int(kv["axis"]), int(kv["t"]))
        else:
            raise AssertionError(op)
        assert got.shape == want.shape, (op, args)
        assert np.array_equal(got, want), (op, args)
        n += 1
    assert n == 13


SHAPES = [(1,), (5,), (3, 4), (1, 7), (2, 3, 4), (4, 1, 3), (2, 3, 2, 5), (3, 2, 1, 2, 4),
          (2, 2, 3, 2, 2, 3)]


@pytest.mark.parametrize("es", [2, 4])
@pytest.mark.parametrize("shape", SHAPES)
def test_transpose_all_perms_vs_numpy(shape, es):
    x = synth.iota(shape, es)
    perms = list(itertools.permutations(range(len(shape))))
    if len(perms) > 24:
        rng = np.random.default_rng(7)
        perms = [perms[i] for i in rng.choice(len(perms), 24, replace=False)]
    for p in perms:
        got = oracle.transpose(x, p)
        assert np.array_equal(got, np.transpose(x, p)), p
        inv = np.argsort(p)
        assert np.array_equal(oracle.transpose(got, inv), x)


def _factorisations(n, rng, count):
    out = []
    for _ in range(count):
        rem, f = n, []
        while rem > 1 and len(f) < 5:
            divs = [d for d in range(1, rem + 1) if rem % d == 0]
            d = int(rng.choice(divs))
            f.append(d)
            rem //= d
        if rem > 1:
            f.append(rem)
        if not f:
            f = [1]
        out.append(tuple(f))
    return out


@pytest.mark.parametrize("es", [2, 4])
@pytest.mark.parametrize("shape", SHAPES)
def test_reshape_vs_numpy_and_round_trip(shape, es):
    rng = np.random.default_rng(11)
    x = synth.random_bits(shape, es, 5)
    for new in _factorisations(int(np.prod(shape)), rng, 6):
        got = oracle.reshape(x, new)
        assert np.array_equal(got, np.reshape(x, new, order="C"))
        assert np.array_equal(oracle.reshape(got, shape), x)


@pytest.mark.parametrize("es", [2, 4])
def test_slice_vs_numpy(es):
    rng = np.random.default_rng(3)
    for shape in SHAPES:
        x = synth.iota(shape, es)
        for _ in range(8):
            ax = int(rng.integers(len(shape)))
            n = shape[ax]
            b = int(rng.integers(0, n))
            e = int(rng.integers(b + 1, n + 1))
            st = int(rng.integers(1, 4))
            sl = [slice(None)] * len(shape)
            sl[ax] = slice(b, e, st)
            assert np.array_equal(oracle.slice_(x, ax, b, e, st), x[tuple(sl)]), (shape, ax, b, e, st)


@pytest.mark.parametrize("es", [2, 4])
def test_negative_step_slice_vs_numpy(es):
    rng = np.random.default_rng(31)
    for shape in SHAPES:
        x = synth.iota(shape, es)
        for _ in range(8):
            ax = int(rng.integers(len(shape)))
            n = shape[ax]
            b = int(rng.integers(0, n))
            e = int(rng.integers(-1, b))
            st = -int(rng.integers(1, 4))
            sl = [slice(None)] * len(shape)
            sl[ax] = slice(b, e if e >= 0 else None, st)   # numpy spells "past index 0" as None
            assert np.array_equal(oracle.slice_(x, ax, b, e, st), x[tuple(sl)]), (shape, ax, b, e, st)
        # reversing an axis twice is the identity
        n = shape[0]
        assert np.array_equal(oracle.slice_(oracle.slice_(x, 0, n - 1, -1, -1), 0, n - 1, -1, -1), x)


@pytest.mark.parametrize("es", [2, 4])
def test_repeat_and_tile_vs_numpy_and_inverses(es):
    rng = np.random.default_rng(32)
    for shape in SHAPES:
        x = synth.iota(shape, es)
        for _ in range(4):
            ax = int(rng.integers(len(shape)))
            k = int(rng.integers(1, 5))
            r = oracle.repeat(x, ax, k)
            assert np.array_equal(r, np.repeat(x, k, axis=ax)), (shape, ax, k)
            reps = [1] * len(shape)
            reps[ax] = k
            t = oracle.tile(x, ax, k)
            assert np.array_equal(t, np.tile(x, reps)), (shape, ax, k)
            n = shape[ax]
            # every k-th element of a repeat, from any phase, is the input again
            for ph in range(k):
                assert np.array_equal(oracle.slice_(r, ax, ph, n * k, k), x)
            # every block of a tile is the input again
            for blk in range(k):
                assert np.array_equal(oracle.slice_(t, ax, blk * n, (blk + 1) * n, 1), x)
        # repeat = reshape(.., n, 1) -> tile the new axis -> reshape(.., n*k), a second definition
        ax, k = len(shape) - 1, 3
        y = oracle.reshape(x, list(shape) + [1])
        y = oracle.tile(y, len(shape), k)
        y = oracle.reshape(y, list(shape[:-1]) + [shape[-1] * k])
        assert np.array_equal(y, oracle.repeat(x, ax, k))


@pytest.mark.parametrize("es", [2, 4])
def test_pad_vs_numpy_and_slice_inverse(es):
    rng = np.random.default_rng(5)
    for shape in SHAPES:
        x = synth.iota(shape, es) + 1
        for _ in range(4):
            lo = [int(v) for v in rng.integers(0, 3, len(shape))]
            hi = [int(v) for v in rng.integers(0, 3, len(shape))]
            fill = int(rng.integers(0, 60000))
            got = oracle.pad(x, lo, hi, fill)
            want = np.pad(x, list(zip(lo, hi)), mode="constant", constant_values=fill)
            assert np.array_equal(got, want)
            # slicing the padding off again gives the input back
            y = got
            for ax in range(len(shape)):
                y = oracle.slice_(y, ax, lo[ax], lo[ax] + shape[ax], 1)
            assert np.array_equal(y, x)
            # number of fill elements
            assert int((got == fill).sum()) >= got.size - x.size


def test_pad_fill_is_truncated_to_element_width():
    x = np.array([[1, 2]], dtype=np.uint16)
    got = oracle.pad(x, (0, 1), (0, 0), 0x12345678)
    assert got.tolist() == [[0x5678, 1, 2]]
    x32 = np.array([[1, 2]], dtype=np.uint32)
    assert oracle.pad(x32, (0, 1), (0, 0), 0x12345678).tolist() == [[0x12345678, 1, 2]]


@pytest.mark.parametrize("es", [2, 4])
def test_concat_vs_numpy_and_split_inverse(es):
    rng = np.random.default_rng(9)
    for shape in SHAPES:
        for ax in range(len(shape)):
            n = int(rng.integers(1, 5))
            xs, base = [], 0
            for m in range(n):
                shp = list(shape)
                shp[ax] = int(rng.integers(1, 5))
                x = synth.iota(shp, es) + base
                base += x.size
                xs.append(x)
            got = oracle.concat(xs, ax)
            assert np.array_equal(got, np.concatenate(xs, axis=ax))
            off = 0
            for x in xs:   # each split of the concat is the original input
                assert np.array_equal(oracle.slice_(got, ax, off, off + x.shape[ax], 1), x)
                off += x.shape[ax]


def test_concat_of_split_is_identity():
    x = synth.iota((3, 10, 4), 4)
    parts = [oracle.slice_(x, 1, a, b, 1) for a, b in [(0, 3), (3, 4), (4, 10)]]
    assert np.array_equal(oracle.concat(parts, 1), x)


def test_pad_of_slice_zeroes_border():
    x = synth.iota((6, 7), 4) + 1
    inner = oracle.slice_(oracle.slice_(x, 0, 1, 5, 1), 1, 2, 6, 1)
    y = oracle.pad(inner, (1, 2), (1, 1), 0)
    want = x.copy()
    want[0, :] = 0
    want[5, :] = 0
    want[:, :2] = 0
    want[:, 6:] = 0
    assert np.array_equal(y, want)


def test_brute_force_index_enumeration_tiny():
    """Enumerate every output index in Python and apply each definition."""
    x = synth.iota((2, 3, 4), 4)
    t = oracle.transpose(x, (2, 0, 1))
    for a, b, c in itertools.product(range(4), range(2), range(3)):
        assert t[a, b, c] == x[b, c, a]
    r = oracle.reshape(x, (4, 6))
    for a, b in itertools.product(range(4), range(6)):
        L = a * 6 + b
        assert r[a, b] == x[L // 12, (L // 4) % 3, L % 4]
    s = oracle.slice_(x, 2, 1, 4, 2)
    for a, b, c in itertools.product(range(2), range(3), range(2)):
        assert s[a, b, c] == x[a, b, 1 + 2 * c]
    s = oracle.slice_(x, 2, 3, 0, -2)
    for a, b, c in itertools.product(range(2), range(3), range(2)):
        assert s[a, b, c] == x[a, b, 3 - 2 * c]
    rp = oracle.repeat(x, 1, 2)
    for a, b, c in itertools.product(range(2), range(6), range(4)):
        assert rp[a, b, c] == x[a, b // 2, c]
    tl = oracle.tile(x, 2, 3)
    for a, b, c in itertools.product(range(2), range(3), range(12)):
        assert tl[a, b, c] == x[a, b, c % 4]
    p = oracle.pad(x, (1, 0, 2), (0, 1, 0), 77)
    for a, b, c in itertools.product(range(3), range(4), range(6)):
        inside = 1 <= a < 3 and b < 3 and 2 <= c < 6
        assert p[a, b, c] == (x[a - 1, b, c - 2] if inside else 77)


def test_error_paths():
    x = synth.iota((2, 3), 4)
    with pytest.raises(oracle.OracleError):
        oracle.transpose(x, (0, 0))
    with pytest.raises(oracle.OracleError):
        oracle.reshape(x, (4, 2))
    with pytest.raises(oracle.OracleError):
        oracle.slice_(x, 1, 2, 4, 1)
    with pytest.raises(oracle.OracleError):
        oracle.slice_(x, 1, 2, 2, 1)
    with pytest.raises(oracle.OracleError):
        oracle.slice_(x, 1, 1, 1, -1)
    with pytest.raises(oracle.OracleError):
        oracle.slice_(x, 1, 3, 0, -1)
    with pytest.raises(oracle.OracleError):
        oracle.slice_(x, 1, 2, -2, -1)
    with pytest.raises(oracle.OracleError):
        oracle.slice_(x, 1, 0, 2, 0)
    with pytest.raises(oracle.OracleError):
        oracle.repeat(x, 2, 2)
    with pytest.raises(oracle.OracleError):
        oracle.tile(x, 0, 0)
    with pytest.raises(oracle.OracleError):
        oracle.pad(x, (0, -1), (0, 0))
    with pytest.raises(oracle.OracleError):
        oracle.concat([x, synth.iota((3, 3), 4)], 1)
    with pytest.raises(oracle.OracleError):
        oracle.run_chain([x, x], [("transpose", (1, 0))])


def test_threads_do_not_change_results():
    x = synth.random_bits((5, 6, 7, 3), 2, 1)
    ops = [("transpose", (3, 1, 0, 2)), ("reshape", (18, 35)), ("slice", 1, 3, 30, 2),
           ("pad", (1, 2), (0, 3), 5)]
    a = oracle.run_chain([x], ops)
    oracle.set_threads(4)
    try:
        b = oracle.run_chain([x], ops)
    finally:
        oracle.set_threads(1)
    assert np.array_equal(a, b)


def test_store_form_hand_worked_closed_forms_and_errors():
    """The store t_s[f_s(i)] = v of Section 2 executed as written.  Pins: a hand-worked 2 x 3 example,
    numpy's inverse permutation / flip / reshape as closed forms, gather-after-store = identity."""
    x = np.array([[10, 20, 30], [40, 50, 60]], dtype=np.uint16)
    # f_s = transposition of the [3,2] output's index space: element (i,j) of x goes to out[j,i]
    out = oracle.store_form(x, [("transpose", (1, 0))], (3, 2))
    assert out.tolist() == [[10, 40], [20, 50], [30, 60]]
    # reversed rows of the output: x[i] goes to out[1 - i]
    assert oracle.store_form(x, [("slice", 0, 1, -1, -1)], (2, 3)).tolist() == [[40, 50, 60], [10, 20, 30]]
    rng = np.random.default_rng(0)
    for shape in [(3, 4, 5), (2, 3, 2, 5), (7, 6)]:
        y = synth.random_bits(shape, 4, 9)
        for _ in range(6):
            perm = tuple(int(p) for p in rng.permutation(len(shape)))
            # the chain turns out_shape into y's shape, so out_shape is y's shape pulled back through perm
            out_shape = tuple(shape[perm.index(d)] for d in range(len(shape)))
            got = oracle.store_form(y, [("transpose", perm)], out_shape)
            assert np.array_equal(got, np.transpose(y, np.argsort(perm)))
            # reading the stored tensor back through the same chain gives the input again
            assert np.array_equal(oracle.run_chain([got], [("transpose", perm)]), y)
        flat = int(np.prod(shape))
        got = oracle.store_form(y, [("reshape", shape)], (flat,))
        assert np.array_equal(got, y.reshape(-1))
        chain = [("reshape", shape), ("slice", 0, shape[0] - 1, -1, -1)]
        got = oracle.store_form(y, chain, (flat,))
        assert np.array_equal(got, y[::-1].reshape(-1)) and np.array_equal(oracle.run_chain([got], chain), y)
    with pytest.raises(oracle.OracleError):
        oracle.store_form(x, [("slice", 0, 0, 2, 1)], (3, 3))          # rows of the output never written
    with pytest.raises(oracle.OracleError):
        oracle.store_form(np.zeros((4, 3), np.uint16), [("repeat", 0, 2)], (2, 3))   # written twice
    with pytest.raises(oracle.OracleError):
        oracle.store_form(x, [("transpose", (1, 0))], (2, 3))          # wrong shape
