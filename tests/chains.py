"""Seeded random operator chains for property tests (data only: which
operators, which arguments).  Shapes stay small so the oracle runs instantly."""
import numpy as np


def _factorisation(n, rng, max_rank=5):
    f, rem = [], n
    while rem > 1 and len(f) < max_rank - 1:
        divs = [d for d in range(1, rem + 1) if rem % d == 0]
        d = int(rng.choice(divs))
        if d == 1 and rng.random() < 0.7:
            continue
        f.append(d)
        rem //= d
    f.append(rem)
    pos = int(rng.integers(0, len(f) + 1))
    if rng.random() < 0.2 and len(f) < max_rank:
        f.insert(pos, 1)
    return tuple(f)


def random_shape(rng, max_rank=4, max_extent=7):
    r = int(rng.integers(1, max_rank + 1))
    return tuple(int(v) for v in rng.integers(1, max_extent + 1, r))


def random_op(rng, shape, allow_step=True):
    kind = rng.choice(["transpose", "reshape", "slice", "pad"], p=[0.3, 0.3, 0.25, 0.15])
    r = len(shape)
    if kind == "transpose":
        return ("transpose", tuple(int(v) for v in rng.permutation(r)))
    if kind == "reshape":
        return ("reshape", _factorisation(int(np.prod(shape)), rng))
    if kind == "slice":
        ax = int(rng.integers(r))
        n = shape[ax]
        b = int(rng.integers(0, n))
        e = int(rng.integers(b + 1, n + 1))
        st = int(rng.integers(1, 4)) if allow_step and rng.random() < 0.4 else 1
        return ("slice", ax, b, e, st)
    lo = tuple(int(v) for v in rng.integers(0, 3, r))
    hi = tuple(int(v) for v in rng.integers(0, 3, r))
    return ("pad", lo, hi, int(rng.integers(1, 60000)))


def random_op_ext(rng, shape):
    """Like random_op, plus the non-injective gathers and downward slices."""
    u = rng.random()
    r = len(shape)
    if u < 0.18:
        return ("repeat", int(rng.integers(r)), int(rng.integers(1, 5)))
    if u < 0.36:
        return ("tile", int(rng.integers(r)), int(rng.integers(1, 5)))
    if u < 0.54:
        ax = int(rng.integers(r))
        n = shape[ax]
        b = int(rng.integers(0, n))
        e = int(rng.integers(-1, b)) if b > 0 else -1
        return ("slice", ax, b, e, -int(rng.integers(1, 4)))
    return random_op(rng, shape)


def out_shape(shape, op):
    k = op[0]
    if k == "transpose":
        return tuple(shape[p] for p in op[1])
    if k == "reshape":
        return tuple(op[1])
    if k == "slice":
        s = list(shape)
        s[op[1]] = -((op[2] - op[3]) // op[4])   # ceil((end - begin) / step), either sign of step
        return tuple(s)
    if k in ("repeat", "tile"):
        s = list(shape)
        s[op[1]] *= op[2]
        return tuple(s)
    if k == "pad":
        return tuple(l + s + h for l, s, h in zip(op[1], shape, op[2]))
    raise ValueError(k)


def random_chain(seed, max_ops=5, n_src_max=3, max_volume=20000, extended=False):
    """Returns (src_shapes, ops).  extended: also repeat, tile and negative-step slices."""
    rng = np.random.default_rng(seed if not extended else [seed, 77])
    shape = random_shape(rng)
    ops, src_shapes = [], [shape]
    if rng.random() < 0.3:
        n = int(rng.integers(2, n_src_max + 1))
        ax = int(rng.integers(len(shape)))
        src_shapes = []
        for _ in range(n):
            s = list(shape)
            s[ax] = int(rng.integers(1, 6))
            src_shapes.append(tuple(s))
        ops.append(("concat", ax))
        s = list(shape)
        s[ax] = sum(t[ax] for t in src_shapes)
        shape = tuple(s)
    for _ in range(int(rng.integers(1, max_ops + 1))):
        op = random_op_ext(rng, shape) if extended else random_op(rng, shape)
        ns = out_shape(shape, op)
        if int(np.prod(ns)) > max_volume or len(ns) > 8:
            continue
        ops.append(op)
        shape = ns
    return src_shapes, ops
