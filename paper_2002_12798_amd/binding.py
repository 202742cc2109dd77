"""ctypes binding to libamap.so: argument marshalling only.

Every function here has the name of the C entry point it wraps (include/amap.h)
and does no index arithmetic and no data movement of its own.  If the shared
library is missing the import of this module fails: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

# PyTorch allocates the device memory and owns the streams this library is
# handed, so both must sit on ONE HIP runtime: torch ships its own
# libamdhip64 (same soname as the system one) and has to be loaded first, so
# that libamap.so binds to that copy instead of bringing in a second runtime.
import torch  # noqa: F401  (import order matters)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("AMAP_LIB_PATH") or os.path.join(_HERE, "libamap.so")

AMAP_OK, AMAP_E_INVALID, AMAP_E_SHAPE, AMAP_E_UNSUPPORTED, AMAP_E_NOMEM, AMAP_E_ALIAS, AMAP_E_HIP = range(7)
AMAP_TRANSPOSE, AMAP_RESHAPE, AMAP_SLICE, AMAP_PAD, AMAP_CONCAT, AMAP_REPEAT, AMAP_TILE = range(7)
AMAP_K_PROGRAM, AMAP_K_ELEMENT, AMAP_K_ROWS, AMAP_K_TILE, AMAP_K_WAVE = range(5)
KERNEL_NAMES = {0: "program", 1: "element", 2: "rows", 3: "tile", 4: "wave"}
AMAP_MAX_RANK = 8

EXPORTS = [
    "amap_source", "amap_transpose", "amap_reshape", "amap_slice", "amap_repeat", "amap_tile", "amap_pad",
    "amap_concat",
    "amap_inverse", "amap_compose", "amap_free", "amap_describe", "amap_source_shape",
    "amap_eval_host", "amap_check_cover", "amap_plan_selfcheck", "amap_gemm_selfcheck", "amap_execute", "amap_execute_multi", "amap_execute_kernel",
    "amap_gemm_fused", "amap_gemm_fused_store", "amap_gemm_mapped", "amap_gemm_gather", "amap_status_str", "amap_last_error",
    "amap_graph_create", "amap_graph_free", "amap_graph_input", "amap_graph_op", "amap_graph_map", "amap_graph_store",
    "amap_graph_compute",
    "amap_graph_output", "amap_graph_eliminate", "amap_graph_load",
    "amap_layout_create", "amap_layout_free", "amap_layout_tensor", "amap_layout_op", "amap_layout_solve",
    "amap_layout_order", "amap_layout_copy",
]


class AmapError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        detail = ""
        if status == AMAP_E_HIP or (status == AMAP_E_UNSUPPORTED and what.startswith(("amap_gemm", "amap_execute"))):
            detail = f" [{_L.amap_last_error().decode()}]"
        super().__init__(f"{what}: {_status_str(status)} (status {status}){detail}")


class amap_src_desc(C.Structure):
    _fields_ = [("rank", C.c_int), ("shape", C.POINTER(C.c_int64)), ("es", C.c_int)]


class amap_op(C.Structure):
    _fields_ = [("kind", C.c_int), ("axis", C.c_int), ("n", C.c_int),
                ("a", C.POINTER(C.c_int64)), ("b", C.POINTER(C.c_int64)), ("fill_bits", C.c_uint32)]


class amap_info(C.Structure):
    _fields_ = [("rank", C.c_int), ("shape", C.c_int64 * AMAP_MAX_RANK), ("elem_size", C.c_int),
                ("n_src", C.c_int), ("strided", C.c_int), ("n_pieces", C.c_int),
                ("n_fill_pieces", C.c_int), ("kernel_id", C.c_int), ("vec_bytes", C.c_int),
                ("min_read_bytes", C.c_int64), ("write_bytes", C.c_int64), ("fill_bytes", C.c_int64)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")

_L = C.CDLL(LIB_PATH)
_vp = C.c_void_p
_pp = C.POINTER(C.c_void_p)
_i64p = C.POINTER(C.c_int64)
_i32p = C.POINTER(C.c_int32)

_L.amap_source.argtypes = [C.c_int, C.c_int, _i64p, C.c_int, _pp]
_L.amap_transpose.argtypes = [_vp, _i32p, _pp]
_L.amap_reshape.argtypes = [_vp, C.c_int, _i64p, _pp]
_L.amap_slice.argtypes = [_vp, C.c_int, C.c_int64, C.c_int64, C.c_int64, _pp]
_L.amap_repeat.argtypes = [_vp, C.c_int, C.c_int64, _pp]
_L.amap_tile.argtypes = [_vp, C.c_int, C.c_int64, _pp]
_L.amap_pad.argtypes = [_vp, _i64p, _i64p, C.c_uint32, _pp]
_L.amap_concat.argtypes = [_pp, C.c_int, C.c_int, _pp]
_L.amap_inverse.argtypes = [_vp, _pp]
_L.amap_compose.argtypes = [C.POINTER(amap_src_desc), C.c_int, C.POINTER(amap_op), C.c_int, _pp]
_L.amap_free.argtypes = [_vp]
_L.amap_free.restype = None
_L.amap_describe.argtypes = [_vp, C.POINTER(amap_info)]
_L.amap_source_shape.argtypes = [_vp, C.c_int, C.POINTER(C.c_int), _i64p]
_L.amap_eval_host.argtypes = [_vp, _pp, _vp, C.c_int]
_L.amap_check_cover.argtypes = [_vp, _i64p, _i64p]
_L.amap_plan_selfcheck.argtypes = [_vp, C.c_int, _i64p]
_L.amap_gemm_selfcheck.argtypes = [_vp, _vp, C.c_int64, _vp, C.c_int, _i64p]
_L.amap_execute.argtypes = [_pp, _vp, _vp, _vp]
_L.amap_execute_kernel.argtypes = [_pp, _vp, _vp, _vp, C.c_int]
_L.amap_execute_multi.argtypes = [_pp, _pp, _pp, C.c_int, _vp]
_L.amap_gemm_fused.argtypes = [_vp, _vp, _vp, C.c_int64, _vp, _vp]
_L.amap_gemm_fused_store.argtypes = [_vp, _vp, _vp, C.c_int64, _vp, _vp, _vp]
_L.amap_gemm_mapped.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp]
_L.amap_gemm_gather.argtypes = [_pp, _vp, _vp, _vp, C.c_int64, _vp, _vp, _vp]
_L.amap_status_str.argtypes = [C.c_int]
_L.amap_status_str.restype = C.c_char_p

_L.amap_last_error.restype = C.c_char_p



class amap_graph_report(C.Structure):
    _fields_ = [("n_layout_ops", C.c_int), ("n_pairs", C.c_int), ("n_pairs_left", C.c_int), ("n_loads", C.c_int),
                ("n_rewrites", C.c_int), ("n_alias_outputs", C.c_int), ("moved_bytes_before", C.c_int64),
                ("moved_bytes_after", C.c_int64), ("intermediate_bytes", C.c_int64), ("n_mapped_loads", C.c_int),
                ("mapped_load_bytes", C.c_int64)]


_ip = C.POINTER(C.c_int)
_L.amap_graph_create.argtypes = [_pp]
_L.amap_graph_free.argtypes = [_vp]
_L.amap_graph_free.restype = None
_L.amap_graph_input.argtypes = [_vp, C.c_int, _i64p, C.c_int, _ip]
_L.amap_graph_op.argtypes = [_vp, C.POINTER(amap_op), _ip, C.c_int, _ip]
_L.amap_graph_map.argtypes = [_vp, _vp, _ip, C.c_int, _ip]
_L.amap_graph_store.argtypes = [_vp, _vp, C.c_int, _ip]
_L.amap_graph_compute.argtypes = [_vp, _ip, C.c_int, C.c_int, _i64p, C.c_int, _ip]
_L.amap_graph_output.argtypes = [_vp, C.c_int]
_L.amap_graph_eliminate.argtypes = [_vp, C.POINTER(amap_graph_report)]
_L.amap_graph_load.argtypes = [_vp, C.c_int, _ip, _ip, _pp, _ip, _ip]



class amap_layout_report(C.Structure):
    _fields_ = [("n_copies_local", C.c_int), ("copy_bytes_local", C.c_int64), ("n_copies_global", C.c_int),
                ("copy_bytes_global", C.c_int64), ("n_sweeps", C.c_int)]


_L.amap_layout_create.argtypes = [_pp]
_L.amap_layout_free.argtypes = [_vp]
_L.amap_layout_free.restype = None
_L.amap_layout_tensor.argtypes = [_vp, C.c_int, _i64p, C.c_int, _i32p, _ip]
_L.amap_layout_op.argtypes = [_vp, _ip, _ip, C.POINTER(_i32p), C.c_int, C.c_int, _ip]
_L.amap_layout_solve.argtypes = [_vp, C.POINTER(amap_layout_report)]
_L.amap_layout_order.argtypes = [_vp, C.c_int, _i32p]
_L.amap_layout_copy.argtypes = [_vp, C.c_int, _ip, _ip, _ip, _pp]

raw = _L  # the raw CDLL, for callers that pre-marshal their arguments


def _status_str(s):
    return _L.amap_status_str(int(s)).decode()


def amap_status_str(s):
    return _status_str(s)


def _i64(v):
    return (C.c_int64 * len(v))(*[int(x) for x in v])


def _check(st, what):
    if st != AMAP_OK:
        raise AmapError(st, what)


class Map:
    """Owner of one amap_t*; frees it when collected."""

    def __init__(self, handle):
        self._h = C.c_void_p(handle)

    @property
    def handle(self):
        return self._h

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _L is not None:  # _L is gone when the interpreter shuts down
            _L.amap_free(h)


def _new(fn, what, *args):
    out = C.c_void_p()
    _check(fn(*args, C.byref(out)), what)
    return Map(out.value)


def amap_source(src_id, shape, es):
    return _new(_L.amap_source, "amap_source", int(src_id), len(shape), _i64(shape), int(es))


def amap_transpose(m, perm):
    if len(perm) != amap_describe(m).rank:
        raise AmapError(AMAP_E_INVALID, "amap_transpose")
    return _new(_L.amap_transpose, "amap_transpose", m.handle, (C.c_int32 * len(perm))(*[int(p) for p in perm]))


def amap_reshape(m, shape):
    return _new(_L.amap_reshape, "amap_reshape", m.handle, len(shape), _i64(shape))


def amap_slice(m, axis, begin, end, step=1):
    return _new(_L.amap_slice, "amap_slice", m.handle, int(axis), int(begin), int(end), int(step))


def amap_repeat(m, axis, count):
    return _new(_L.amap_repeat, "amap_repeat", m.handle, int(axis), int(count))


def amap_tile(m, axis, count):
    return _new(_L.amap_tile, "amap_tile", m.handle, int(axis), int(count))


def amap_pad(m, lo, hi, fill_bits=0):
    r = amap_describe(m).rank
    if len(lo) != r or len(hi) != r:
        raise AmapError(AMAP_E_INVALID, "amap_pad")
    return _new(_L.amap_pad, "amap_pad", m.handle, _i64(lo), _i64(hi), int(fill_bits) & 0xFFFFFFFF)


def amap_concat(ms, axis):
    arr = (C.c_void_p * len(ms))(*[m.handle for m in ms])
    return _new(_L.amap_concat, "amap_concat", arr, len(ms), int(axis))


def amap_inverse(m):
    return _new(_L.amap_inverse, "amap_inverse", m.handle)


def marshal_chain(src_shapes, es, ops):
    """Build the ctypes arguments of amap_compose for an operator list
    (tuples as in synth.py).  Returned tuple keeps every buffer alive."""
    keep = []
    srcs = (amap_src_desc * len(src_shapes))()
    for i, s in enumerate(src_shapes):
        buf = _i64(s)
        keep.append(buf)
        srcs[i].rank, srcs[i].shape, srcs[i].es = len(s), buf, int(es)
    cops = (amap_op * max(1, len(ops)))()
    for k, op in enumerate(ops):
        o = cops[k]
        kind = op[0]
        if kind == "transpose":
            a = _i64(op[1])
            o.kind, o.n, o.a = AMAP_TRANSPOSE, len(op[1]), a
        elif kind == "reshape":
            a = _i64(op[1])
            o.kind, o.n, o.a = AMAP_RESHAPE, len(op[1]), a
        elif kind == "slice":
            a = _i64([op[2], op[3], op[4] if len(op) > 4 else 1])
            o.kind, o.axis, o.n, o.a = AMAP_SLICE, int(op[1]), 3, a
        elif kind == "pad":
            a, b = _i64(op[1]), _i64(op[2])
            keep.append(b)
            o.kind, o.n, o.a, o.b = AMAP_PAD, len(op[1]), a, b
            o.fill_bits = (int(op[3]) if len(op) > 3 else 0) & 0xFFFFFFFF
        elif kind in ("repeat", "tile"):
            a = _i64([op[2]])
            o.kind, o.axis, o.n, o.a = (AMAP_REPEAT if kind == "repeat" else AMAP_TILE), int(op[1]), 1, a
        elif kind == "concat":
            a = None
            o.kind, o.axis = AMAP_CONCAT, int(op[1])
        else:
            raise AmapError(AMAP_E_INVALID, f"unknown operator {kind}")
        keep.append(a)
    return srcs, len(src_shapes), cops, len(ops), keep


def amap_compose(src_shapes, es, ops):
    srcs, n_src, cops, n_ops, keep = marshal_chain(src_shapes, es, ops)
    m = _new(_L.amap_compose, "amap_compose", srcs, n_src, cops, n_ops)
    del keep
    return m


def amap_describe(m):
    info = amap_info()
    _check(_L.amap_describe(m.handle, C.byref(info)), "amap_describe")
    return info


def dst_shape(m):
    info = amap_describe(m)
    return tuple(info.shape[k] for k in range(info.rank))


def amap_source_shape(m, src_id):
    rank = C.c_int()
    shape = (C.c_int64 * AMAP_MAX_RANK)()
    _check(_L.amap_source_shape(m.handle, int(src_id), C.byref(rank), shape), "amap_source_shape")
    return tuple(shape[k] for k in range(rank.value))


def amap_check_cover(m):
    un, ov = C.c_int64(), C.c_int64()
    _check(_L.amap_check_cover(m.handle, C.byref(un), C.byref(ov)), "amap_check_cover")
    return un.value, ov.value


def amap_plan_selfcheck(m, kernel_id=-1):
    n = C.c_int64()
    _check(_L.amap_plan_selfcheck(m.handle, int(kernel_id), C.byref(n)), "amap_plan_selfcheck")
    return n.value


def amap_gemm_selfcheck(a_map, n, out_map=None, n_workgroups=256, w_map=None):
    """Errors found by the host replay of the 256 x 256-tile GEMM kernel's loads and stores."""
    e = C.c_int64()
    _check(_L.amap_gemm_selfcheck(a_map.handle, w_map.handle if w_map is not None else None, int(n),
                                  out_map.handle if out_map is not None else None, int(n_workgroups),
                                  C.byref(e)), "amap_gemm_selfcheck")
    return e.value


def amap_eval_host(m, srcs, mode=0):
    """Host evaluator on numpy arrays (composer tests without a GPU)."""
    import numpy as np
    info = amap_describe(m)
    dt = {2: np.uint16, 4: np.uint32}[info.elem_size]
    arrs = [None if s is None else np.ascontiguousarray(s).view(dt) for s in srcs]
    for i, a in enumerate(arrs):
        if a is None or i >= info.n_src:
            continue
        try:
            want = int(np.prod(amap_source_shape(m, i)))
        except AmapError:
            continue  # an id the map no longer reads
        if a.size != want:
            raise AmapError(AMAP_E_SHAPE, "amap_eval_host: source size")
    ptrs = (C.c_void_p * max(1, info.n_src, len(arrs)))(*[None if a is None else a.ctypes.data for a in arrs])
    out = np.empty(dst_shape(m), dtype=dt)
    _check(_L.amap_eval_host(m.handle, ptrs, out.ctypes.data, int(mode)), "amap_eval_host")
    return out


def _ptr_array(ptrs, n_min=0):
    """Pointer table for the C side, padded with NULL up to n_min entries: the library reads one
    entry per source id of the map and the ABI carries no count, so a short table must never be handed over."""
    vals = [int(p) if p else None for p in ptrs]
    vals += [None] * (max(1, n_min) - len(vals))
    return (C.c_void_p * len(vals))(*vals)


def _src_array(src_ptrs, maps, what):
    """Source table sized to the maps it serves; a table too short for a source id a map reads is an error
    here, before the library sees it (NULL entries are the library's to judge: an empty map reads none)."""
    n_src = 0
    for m in maps:
        info = amap_describe(m)
        n_src = max(n_src, info.n_src)
        for i in range(info.n_src):
            try:
                amap_source_shape(m, i)
            except AmapError:
                continue  # an id the map no longer reads
            if i >= len(src_ptrs):
                raise AmapError(AMAP_E_INVALID, f"{what}: no pointer for source {i}")
    return _ptr_array(src_ptrs, n_src)


def amap_execute(src_ptrs, dst_ptr, m, stream=0, kernel_id=None):
    """src_ptrs: device addresses (ints) indexed by source id; dst_ptr: device address."""
    arr = _src_array(src_ptrs, [m], "amap_execute")
    if kernel_id is None:
        _check(_L.amap_execute(arr, C.c_void_p(dst_ptr), m.handle, C.c_void_p(stream)), "amap_execute")
    else:
        _check(_L.amap_execute_kernel(arr, C.c_void_p(dst_ptr), m.handle, C.c_void_p(stream), int(kernel_id)),
               "amap_execute_kernel")


def amap_execute_kernel(src_ptrs, dst_ptr, m, stream, kernel_id):
    amap_execute(src_ptrs, dst_ptr, m, stream, kernel_id)


def amap_execute_multi(src_ptrs, dst_ptrs, maps, stream=0):
    """One source table, several (map, dst) pairs, packed into shared launches."""
    handles = (C.c_void_p * len(maps))(*[m.handle for m in maps])
    _check(_L.amap_execute_multi(_src_array(src_ptrs, maps, "amap_execute_multi"), _ptr_array(dst_ptrs), handles, len(maps), C.c_void_p(stream)),
           "amap_execute_multi")


def amap_gemm_fused(a_src_ptr, a_map, w_ptr, n, out_ptr, stream=0):
    _check(_L.amap_gemm_fused(C.c_void_p(a_src_ptr), a_map.handle, C.c_void_p(w_ptr), int(n),
                              C.c_void_p(out_ptr), C.c_void_p(stream)), "amap_gemm_fused")


def amap_gemm_fused_store(a_src_ptr, a_map, w_ptr, n, out_map, out_ptr, stream=0):
    _check(_L.amap_gemm_fused_store(C.c_void_p(a_src_ptr), a_map.handle, C.c_void_p(w_ptr), int(n), out_map.handle,
                                    C.c_void_p(out_ptr), C.c_void_p(stream)), "amap_gemm_fused_store")


def amap_gemm_mapped(a_src_ptr, a_map, w_src_ptr, w_map, out_map, out_ptr, stream=0):
    _check(_L.amap_gemm_mapped(C.c_void_p(a_src_ptr), a_map.handle, C.c_void_p(w_src_ptr), w_map.handle,
                               out_map.handle if out_map is not None else None, C.c_void_p(out_ptr),
                               C.c_void_p(stream)), "amap_gemm_mapped")


def amap_gemm_gather(a_src_ptrs, a_map, w_src_ptr, w_map, n, out_map, out_ptr, stream=0):
    """a_src_ptrs: device pointers by source id of a_map (None for ids the map does not use)."""
    _check(_L.amap_gemm_gather(_ptr_array(a_src_ptrs, amap_describe(a_map).n_src), a_map.handle, C.c_void_p(w_src_ptr),
                               w_map.handle if w_map is not None else None, int(n),
                               out_map.handle if out_map is not None else None, C.c_void_p(out_ptr),
                               C.c_void_p(stream)), "amap_gemm_gather")


class GraphDME:
    """Owner of one amap_graph_t*.  Build from a synth.Graph-style node list, run
    data-movement elimination, then read the rewritten loads."""

    def __init__(self, nodes, outputs, es):
        h = C.c_void_p()
        _check(_L.amap_graph_create(C.byref(h)), "amap_graph_create")
        self._h = h
        self.report = None
        for n in nodes:
            tid = C.c_int(-1)
            if n[0] == "input":
                _check(_L.amap_graph_input(h, len(n[1]), _i64(n[1]), int(es), C.byref(tid)), "amap_graph_input")
            elif n[0] == "op":
                _, _, cops, _, keep = marshal_chain([(1,)], es, [n[1]])
                ins = (C.c_int * len(n[2]))(*n[2])
                _check(_L.amap_graph_op(h, cops, ins, len(n[2]), C.byref(tid)), "amap_graph_op")
                del keep
            elif n[0] == "store":
                # ("store", chain, [input], out_shape): out[f_s(i)] = in[i], f_s = the chain applied to
                # the index space of the OUTPUT, which must give the input's shape
                sm = amap_compose([tuple(n[3])], es, list(n[1]))
                _check(_L.amap_graph_store(h, sm.handle, int(n[2][0]), C.byref(tid)), "amap_graph_store")
            elif n[0] == "map":
                # ("map", Map, [inputs]): a layout operator given as a composed map in gather form
                ins = (C.c_int * len(n[2]))(*n[2])
                _check(_L.amap_graph_map(h, n[1].handle, ins, len(n[2]), C.byref(tid)), "amap_graph_map")
            elif n[0] == "compute":
                ins = (C.c_int * max(1, len(n[2])))(*n[2])
                _check(_L.amap_graph_compute(h, ins, len(n[2]), len(n[3]), _i64(n[3]), int(es), C.byref(tid)),
                       "amap_graph_compute")
            else:
                raise AmapError(AMAP_E_INVALID, f"unknown node {n[0]}")
        for o in outputs:
            _check(_L.amap_graph_output(h, int(o)), "amap_graph_output")

    def eliminate(self):
        rep = amap_graph_report()
        _check(_L.amap_graph_eliminate(self._h, C.byref(rep)), "amap_graph_eliminate")
        self.report = rep
        return rep

    def loads(self):
        """[(consumer tensor or -1, slot, Map, [source tensor ids])] after eliminate()."""
        out = []
        for i in range(self.report.n_loads):
            cons, slot, n_src = C.c_int(), C.c_int(), C.c_int()
            m = C.c_void_p()
            ids = (C.c_int * 16)()
            _check(_L.amap_graph_load(self._h, i, C.byref(cons), C.byref(slot), C.byref(m), ids, C.byref(n_src)),
                   "amap_graph_load")
            out.append((cons.value, slot.value, Map(m.value), [ids[k] for k in range(n_src.value)]))
        return out

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _L is not None:
            _L.amap_graph_free(h)


class LayoutGraph:
    """Owner of one amap_layout_graph_t* (global layout assignment)."""

    def __init__(self):
        h = C.c_void_p()
        _check(_L.amap_layout_create(C.byref(h)), "amap_layout_create")
        self._h = h
        self.ranks = []
        self.report = None

    def tensor(self, shape, es, fixed_order=None):
        tid = C.c_int(-1)
        fo = None if fixed_order is None else (C.c_int32 * len(fixed_order))(*[int(v) for v in fixed_order])
        _check(_L.amap_layout_tensor(self._h, len(shape), _i64(shape), int(es), fo, C.byref(tid)), "amap_layout_tensor")
        self.ranks.append(len(shape))
        return tid.value

    def op(self, operands, is_output, req_orders=None, same_layout=False):
        """operands: tensor ids; is_output: flags; req_orders: per operand None or a permutation."""
        n = len(operands)
        req_orders = req_orders or [None] * n
        keep = [None if r is None else (C.c_int32 * len(r))(*[int(v) for v in r]) for r in req_orders]
        arr = (_i32p * n)(*[None if k is None else C.cast(k, _i32p) for k in keep])
        oid = C.c_int(-1)
        _check(_L.amap_layout_op(self._h, (C.c_int * n)(*operands), (C.c_int * n)(*[int(bool(v)) for v in is_output]),
                                 arr, n, int(bool(same_layout)), C.byref(oid)), "amap_layout_op")
        return oid.value

    def solve(self):
        rep = amap_layout_report()
        _check(_L.amap_layout_solve(self._h, C.byref(rep)), "amap_layout_solve")
        self.report = rep
        return rep

    def order(self, tensor):
        o = (C.c_int32 * AMAP_MAX_RANK)()
        _check(_L.amap_layout_order(self._h, int(tensor), o), "amap_layout_order")
        return tuple(o[k] for k in range(self.ranks[tensor]))

    def copies(self):
        """[(op, slot, tensor, Map)] of the global assignment."""
        out = []
        for i in range(self.report.n_copies_global):
            op, slot, t = C.c_int(), C.c_int(), C.c_int()
            m = C.c_void_p()
            _check(_L.amap_layout_copy(self._h, i, C.byref(op), C.byref(slot), C.byref(t), C.byref(m)), "amap_layout_copy")
            out.append((op.value, slot.value, t.value, Map(m.value)))
        return out

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _L is not None:
            _L.amap_layout_free(h)
