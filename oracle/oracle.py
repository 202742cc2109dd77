"""Python face of the CPU oracle (oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the CPU
baseline leg of the benchmark; never by the product path.  Shares no code with
the HIP library.

`run_chain` executes a chain of layout operators one operator at a time, each
into a freshly allocated, fully materialised row-major intermediate, i.e. the
program *before* data-movement elimination (paper Section 2.1): every operator
is its own load/store pair and every intermediate tensor exists.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
# ORACLE_LIB_PATH: a build of oracle.c made elsewhere (the sanitizer test loads an instrumented one)
_SO = os.environ.get("ORACLE_LIB_PATH") or os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc into liboracle.so (next to the source)."""
    if os.environ.get("ORACLE_LIB_PATH"):
        return _SO
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC",
                               _SRC, "-o", _SO, "-lm"])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        i64p = C.POINTER(C.c_int64)
        i32p = C.POINTER(C.c_int32)
        L.oracle_set_threads.argtypes = [C.c_int]
        L.oracle_get_threads.restype = C.c_int
        L.oracle_transpose.argtypes = [C.c_void_p, C.c_void_p, C.c_int, i64p, i32p, C.c_int]
        L.oracle_reshape.argtypes = [C.c_void_p, C.c_void_p, C.c_int, i64p, C.c_int, i64p, C.c_int]
        L.oracle_slice.argtypes = [C.c_void_p, C.c_void_p, C.c_int, i64p, C.c_int, C.c_int64,
                                   C.c_int64, C.c_int64, C.c_int]
        L.oracle_repeat.argtypes = [C.c_void_p, C.c_void_p, C.c_int, i64p, C.c_int, C.c_int64, C.c_int]
        L.oracle_tile.argtypes = [C.c_void_p, C.c_void_p, C.c_int, i64p, C.c_int, C.c_int64, C.c_int]
        L.oracle_pad.argtypes = [C.c_void_p, C.c_void_p, C.c_int, i64p, i64p, i64p, C.c_uint32,
                                 C.c_int]
        L.oracle_concat.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_void_p, C.c_int, i64p,
                                    C.c_int, C.c_int]
        L.oracle_gemm_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                       C.c_int64]
        L.oracle_gemm_bf16_point.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                             C.c_int64, C.c_int64]
        L.oracle_gemm_bf16_point.restype = C.c_double
        L.oracle_double_to_bf16.argtypes = [C.c_double]
        L.oracle_double_to_bf16.restype = C.c_uint16
        L.oracle_bf16_to_double.argtypes = [C.c_uint16]
        L.oracle_bf16_to_double.restype = C.c_double
        _lib = L
    return _lib


class OracleError(ValueError):
    pass


def set_threads(n: int) -> None:
    lib().oracle_set_threads(int(n))


def get_threads() -> int:
    return lib().oracle_get_threads()


def _i64(v):
    return (C.c_int64 * len(v))(*[int(x) for x in v])


def _i32(v):
    return (C.c_int32 * len(v))(*[int(x) for x in v])


def _check(rc, what):
    if rc != 0:
        raise OracleError(f"{what}: bad argument (code {rc})")


def _prep(x):
    x = np.ascontiguousarray(x)
    if x.dtype.itemsize not in (2, 4):
        raise OracleError("element size must be 2 or 4 bytes")
    return x


def transpose(x, perm):
    x = _prep(x)
    perm = [int(p) for p in perm]
    if len(perm) != x.ndim or sorted(perm) != list(range(x.ndim)):
        raise OracleError("transpose: perm is not a permutation of the axes")
    out = np.empty([x.shape[p] for p in perm], dtype=x.dtype)
    _check(lib().oracle_transpose(x.ctypes.data, out.ctypes.data, x.ndim, _i64(x.shape),
                                  _i32(perm), x.dtype.itemsize), "transpose")
    return out


def reshape(x, shape):
    x = _prep(x)
    shape = [int(s) for s in shape]
    out = np.empty(shape, dtype=x.dtype) if int(np.prod(shape)) == x.size else None
    if out is None:
        raise OracleError("reshape: element counts differ")
    _check(lib().oracle_reshape(x.ctypes.data, out.ctypes.data, x.ndim, _i64(x.shape),
                                len(shape), _i64(shape), x.dtype.itemsize), "reshape")
    return out


def slice_(x, axis, begin, end, step=1):
    """step >= 1: indices begin, begin+step, .. < end.  step <= -1: begin, begin+step, .. > end
    (end = -1 reaches index 0)."""
    x = _prep(x)
    if not 0 <= axis < x.ndim:
        raise OracleError("slice: bad axis")
    n = x.shape[axis]
    if step >= 1 and 0 <= begin < end <= n:
        count = -((begin - end) // step)
    elif step <= -1 and -1 <= end < begin <= n - 1:
        count = -((end - begin) // -step)
    else:
        raise OracleError("slice: out of range")
    shp = list(x.shape)
    shp[axis] = count
    out = np.empty(shp, dtype=x.dtype)
    _check(lib().oracle_slice(x.ctypes.data, out.ctypes.data, x.ndim, _i64(x.shape), axis,
                              begin, end, step, x.dtype.itemsize), "slice")
    return out


def repeat(x, axis, r):
    x = _prep(x)
    if not (0 <= axis < x.ndim and r >= 1):
        raise OracleError("repeat: bad axis or count")
    shp = list(x.shape)
    shp[axis] *= int(r)
    out = np.empty(shp, dtype=x.dtype)
    _check(lib().oracle_repeat(x.ctypes.data, out.ctypes.data, x.ndim, _i64(x.shape), axis,
                               int(r), x.dtype.itemsize), "repeat")
    return out


def tile(x, axis, t):
    x = _prep(x)
    if not (0 <= axis < x.ndim and t >= 1):
        raise OracleError("tile: bad axis or count")
    shp = list(x.shape)
    shp[axis] *= int(t)
    out = np.empty(shp, dtype=x.dtype)
    _check(lib().oracle_tile(x.ctypes.data, out.ctypes.data, x.ndim, _i64(x.shape), axis,
                             int(t), x.dtype.itemsize), "tile")
    return out


def pad(x, lo, hi, fill_bits=0):
    x = _prep(x)
    if len(lo) != x.ndim or len(hi) != x.ndim or min(list(lo) + list(hi)) < 0:
        raise OracleError("pad: bad widths")
    shp = [int(l) + s + int(h) for l, s, h in zip(lo, x.shape, hi)]
    out = np.empty(shp, dtype=x.dtype)
    _check(lib().oracle_pad(x.ctypes.data, out.ctypes.data, x.ndim, _i64(x.shape), _i64(lo),
                            _i64(hi), int(fill_bits) & 0xFFFFFFFF, x.dtype.itemsize), "pad")
    return out


def concat(xs, axis):
    xs = [_prep(x) for x in xs]
    r = xs[0].ndim
    if not 0 <= axis < r:
        raise OracleError("concat: bad axis")
    for x in xs:
        if x.ndim != r or x.dtype != xs[0].dtype:
            raise OracleError("concat: rank/dtype mismatch")
        if any(x.shape[k] != xs[0].shape[k] for k in range(r) if k != axis):
            raise OracleError("concat: extents differ off the axis")
    shp = list(xs[0].shape)
    shp[axis] = sum(x.shape[axis] for x in xs)
    out = np.empty(shp, dtype=xs[0].dtype)
    ptrs = (C.c_void_p * len(xs))(*[x.ctypes.data for x in xs])
    flat = [d for x in xs for d in x.shape]
    _check(lib().oracle_concat(ptrs, len(xs), out.ctypes.data, r, _i64(flat), axis,
                               xs[0].dtype.itemsize), "concat")
    return out


def apply_op(xs, op):
    """Apply one operator to the list of current tensors; returns the new list."""
    kind = op[0]
    if kind == "concat":
        return [concat(xs, op[1])]
    if len(xs) != 1:
        raise OracleError(f"{kind} needs exactly one input tensor")
    x = xs[0]
    if kind == "transpose":
        return [transpose(x, op[1])]
    if kind == "reshape":
        return [reshape(x, op[1])]
    if kind == "slice":
        return [slice_(x, op[1], op[2], op[3], op[4] if len(op) > 4 else 1)]
    if kind == "pad":
        return [pad(x, op[1], op[2], op[3] if len(op) > 3 else 0)]
    if kind == "repeat":
        return [repeat(x, op[1], op[2])]
    if kind == "tile":
        return [tile(x, op[1], op[2])]
    raise OracleError(f"unknown operator {kind}")


def run_chain(srcs, ops, keep_intermediates=False):
    """Run the un-optimised program: one materialising operator after another."""
    xs = [np.ascontiguousarray(s) for s in srcs]
    inter = []
    for op in ops:
        xs = apply_op(xs, op)
        if keep_intermediates:
            inter.append(xs[0])
    if len(xs) != 1:
        raise OracleError("chain must end in a single tensor")
    return (xs[0], inter) if keep_intermediates else xs[0]


def store_form(x, chain, out_shape):
    """A layout operator written as a store (Section 2, the store t_s[f_s(i)] = v): element i of x
    goes to position f_s(i) of the output.  f_s is given as the operator chain that, applied to the
    index space of the output, yields the shape of x; running the chain on the output's linear
    indices gives f_s(i) for every i, and the store is executed as written, one element at a time."""
    x = np.ascontiguousarray(x)
    n = int(np.prod(out_shape))
    where = run_chain([np.arange(n, dtype=np.uint32).reshape(out_shape)], list(chain))
    if where.shape != x.shape:
        raise OracleError("store map does not have the shape of the stored tensor")
    out = np.empty(n, dtype=x.dtype)
    written = np.zeros(n, dtype=bool)
    for pos, v in zip(where.reshape(-1).tolist(), x.reshape(-1)):
        if written[pos]:
            raise OracleError("store map writes an element twice")
        written[pos] = True
        out[pos] = v
    if not written.all():
        raise OracleError("store map leaves elements of the output unwritten")
    return out.reshape(out_shape)


def run_graph(nodes, inputs, compute):
    """Run an operator graph the un-optimised way: every node one at a time, every
    tensor materialised.  nodes: ("input", shape) | ("op", op, [ids]) |
    ("compute", kind, [ids], shape), node i defines tensor i; inputs: arrays for the
    "input" nodes in order; compute(kind, arrays, shape) stands in for the opaque
    compute operators.  Returns the list of all tensors."""
    it = iter(inputs)
    t = []
    for n in nodes:
        if n[0] == "input":
            x = np.ascontiguousarray(next(it))
            if x.shape != tuple(n[1]):
                raise OracleError("graph input has the wrong shape")
            t.append(x)
        elif n[0] == "op":
            t.append(apply_op([t[i] for i in n[2]], n[1])[0])
        elif n[0] == "store":
            t.append(store_form(t[n[2][0]], n[1], tuple(n[3])))
        elif n[0] == "compute":
            y = np.ascontiguousarray(compute(n[1], [t[i] for i in n[2]], tuple(n[3])))
            if y.shape != tuple(n[3]):
                raise OracleError("compute stand-in returned the wrong shape")
            t.append(y)
        else:
            raise OracleError(f"unknown node {n[0]}")
    return t


def gemm_bf16(a_bits, w_bits):
    a = np.ascontiguousarray(a_bits, dtype=np.uint16)
    w = np.ascontiguousarray(w_bits, dtype=np.uint16)
    if a.ndim != 2 or w.ndim != 2 or a.shape[1] != w.shape[0]:
        raise OracleError("gemm: shapes do not contract")
    out = np.empty((a.shape[0], w.shape[1]), dtype=np.uint16)
    _check(lib().oracle_gemm_bf16(a.ctypes.data, w.ctypes.data, out.ctypes.data, a.shape[0],
                                  a.shape[1], w.shape[1]), "gemm")
    return out


def gemm_bf16_point(a_bits, w_bits, m, n):
    a = np.ascontiguousarray(a_bits, dtype=np.uint16)
    w = np.ascontiguousarray(w_bits, dtype=np.uint16)
    return lib().oracle_gemm_bf16_point(a.ctypes.data, w.ctypes.data, a.shape[1], w.shape[1],
                                        int(m), int(n))


def double_to_bf16(x: float) -> int:
    return int(lib().oracle_double_to_bf16(float(x)))


def bf16_to_double(b: int) -> float:
    return float(lib().oracle_bf16_to_double(int(b)))
