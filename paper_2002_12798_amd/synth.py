"""Seeded synthetic inputs and the layout-operator chains of the workloads.

This module holds data only: tensor shapes, value distributions, seeds and the
operator lists (which operator, with which arguments, in which order).  It does
no index arithmetic of the method itself, so both the CPU oracle and the HIP
library can take their inputs from it without sharing any of their logic.

Tensors are returned as numpy arrays of *opaque element bits* (uint16 for
bf16/fp16, uint32 for fp32): layout operators move bits, they never interpret
them.

A chain is a list of operator tuples applied left to right:
    ("transpose", perm)                      numpy/torch permute convention
    ("reshape", shape)
    ("slice", axis, begin, end, step)        half-open [begin, end)
    ("pad", lo, hi, fill_bits)               per-dimension low/high padding
    ("concat", axis)                         joins all sources; only first
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 200212798


def _rng(cfg_index: int, tensor_index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + cfg_index + 100 * tensor_index))


def f32_bits(x: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 storage bits, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def uniform_f32(shape, cfg_index, tensor_index=0) -> np.ndarray:
    return _rng(cfg_index, tensor_index).uniform(-1.0, 1.0, size=shape).astype(np.float32)


def normal_f32(shape, cfg_index, tensor_index=0, std=1.0) -> np.ndarray:
    g = _rng(cfg_index, tensor_index).standard_normal(size=shape, dtype=np.float32)
    return (g * np.float32(std)).astype(np.float32)


def random_bits(shape, elem_size: int, seed: int) -> np.ndarray:
    """Arbitrary bit patterns (NaN payloads, -0, subnormals included)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    dt = {2: np.uint16, 4: np.uint32}[elem_size]
    return rng.integers(0, np.iinfo(dt).max, size=shape, dtype=dt, endpoint=True)


def iota(shape, elem_size: int) -> np.ndarray:
    """0,1,2,... in row-major order (needs prod(shape) to fit the element)."""
    dt = {2: np.uint16, 4: np.uint32}[elem_size]
    n = int(np.prod(shape))
    return np.arange(n, dtype=np.uint64).astype(dt).reshape(shape)


class Workload:
    """One workload: its sources, its operator chain and (for the fused GEMM)
    the weight operand."""

    def __init__(self, name, elem_size, src_shapes, ops, make_sources, gemm_n=None, make_w=None,
                 batch_axis=None):
        self.name = name
        self.elem_size = elem_size
        self.src_shapes = [tuple(s) for s in src_shapes]
        self.ops = ops
        self._make_sources = make_sources
        self.gemm_n = gemm_n
        self._make_w = make_w
        self.batch_axis = batch_axis

    def sources(self):
        return self._make_sources()

    def weight(self):
        return self._make_w() if self._make_w else None


def _cfg0(n=8):
    shp = (n, 16, 32, 32)
    ops = [("transpose", (0, 2, 3, 1)), ("reshape", (n, 1024, 16)),
           ("slice", 1, 128, 896, 1), ("pad", (0, 0, 0), (0, 0, 4), 0)]
    return Workload("cfg0" if n == 8 else f"cfg0_n{n}", 4, [shp], ops, lambda: [f32_bits(uniform_f32(shp, 0))])


def _cfg1(n=32):
    shp = (n, 256, 56, 56)
    ops = [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]
    return Workload("cfg1" if n == 32 else f"cfg1_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 1))])


def _cfg2_fwd(b=16):
    shp = (b, 512, 2304)
    ops = [("reshape", (b, 512, 3, 12, 64)), ("transpose", (2, 0, 3, 1, 4))]
    return Workload("cfg2_fwd" if b == 16 else f"cfg2_fwd_b{b}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 2))])


def _cfg2_rev(b=16):
    shp = (b, 12, 512, 64)
    ops = [("transpose", (0, 2, 1, 3)), ("reshape", (b, 512, 768))]
    return Workload("cfg2_rev" if b == 16 else f"cfg2_rev_b{b}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 2, 1))])


def _cfg3(n=32):
    chans = (64, 96, 128, 32)
    shps = [(n, c, 28, 28) for c in chans]
    ops = [("concat", 1), ("transpose", (0, 2, 3, 1))]
    return Workload("cfg3" if n == 32 else f"cfg3_n{n}", 2, shps, ops,
                    lambda: [f32_to_f16_bits(uniform_f32(s, 3, j)) for j, s in enumerate(shps)])


def _cfg4():
    shp = (16, 16, 512, 64)
    ops = [("transpose", (0, 2, 1, 3)), ("reshape", (8192, 1024))]
    return Workload("cfg4", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 4))],
                    gemm_n=4096,
                    make_w=lambda: f32_to_bf16_bits(normal_f32((1024, 4096), 4, 1, std=0.02)))


# ---- workloads for the non-injective gathers and reversed axes (repeat, tile, negative step) ----
def _up2x(n=32):
    """Nearest-neighbour 2x up-sampling of an NCHW activation: repeat on H and on W."""
    shp = (n, 256, 28, 28)
    ops = [("repeat", 2, 2), ("repeat", 3, 2)]
    return Workload("up2x" if n == 32 else f"up2x_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 5))])


def _up2x_nhwc(n=32):
    """The same up-sampling in NHWC: the repeated axes are outer, channel rows stay contiguous."""
    shp = (n, 28, 28, 256)
    ops = [("repeat", 1, 2), ("repeat", 2, 2)]
    return Workload("up2x_nhwc" if n == 32 else f"up2x_nhwc_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 5, 1))])


def _bcast(n=32):
    """A per-channel vector broadcast to a whole NHWC activation (tile of extent-1 axes)."""
    shp = (1, 1, 1, 256)
    ops = [("tile", 0, n), ("tile", 1, 56), ("tile", 2, 56)]
    return Workload("bcast" if n == 32 else f"bcast_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 6))])


def _flip_seq(b=16):
    """Sequence reversal of [b, 512, 768] (a slice with step -1 on the sequence axis)."""
    shp = (b, 512, 768)
    ops = [("slice", 1, 511, -1, -1)]
    return Workload("flip_seq" if b == 16 else f"flip_seq_b{b}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 7))])


def _rgb_nhwc(n=64):
    """A batch of 3-channel images from planar (NCHW) to interleaved (NHWC): the innermost dst
    extent is 3, so no side of the transposition offers vectors."""
    shp = (n, 3, 224, 224)
    ops = [("transpose", (0, 2, 3, 1))]
    return Workload("rgb_nhwc" if n == 64 else f"rgb_nhwc_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 8))])


def _up3x(n=32):
    """Nearest-neighbour up-sampling by 3 of [n,128,28,28] on H and W (repeats by a factor that
    is no power of two, along the contiguous dimension too)."""
    shp = (n, 128, 28, 28)
    ops = [("repeat", 2, 3), ("repeat", 3, 3)]
    return Workload("up3x" if n == 32 else f"up3x_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 9))])


def _s5_nhwc_pad(n=128):
    """The chain of cfg1 at the last stage of the same network: [n,2048,7,7] channel-major to
    channels-last with one pixel of zero padding.  49 positions per channel: no vectors along
    the image on the source side."""
    shp = (n, 2048, 7, 7)
    ops = [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]
    return Workload("s5_nhwc_pad" if n == 128 else f"s5_nhwc_pad_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 9))])


def _s5_nchw_crop(n=128):
    """The way back: the interior of a padded channels-last [n,9,9,2048] made channel-major."""
    shp = (n, 9, 9, 2048)
    ops = [("slice", 1, 1, 8, 1), ("slice", 2, 1, 8, 1), ("transpose", (0, 3, 1, 2))]
    return Workload("s5_nchw_crop" if n == 128 else f"s5_nchw_crop_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 10))])


def _i35_nchw(n=64):
    """Channels-last [n,35,35,288] made channel-major: dst rows of 1225 elements, an odd number."""
    shp = (n, 35, 35, 288)
    ops = [("transpose", (0, 3, 1, 2))]
    return Workload("i35_nchw" if n == 64 else f"i35_nchw_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 11))])


def _i55_nchw(n=64):
    """Channels-last [n,55,55,96] made channel-major: dst rows of 3025 elements, too long for LDS."""
    shp = (n, 55, 55, 96)
    ops = [("transpose", (0, 3, 1, 2))]
    return Workload("i55_nchw" if n == 64 else f"i55_nchw_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 12))])


def _c8_nhwc(n=1024):
    """A narrow activation [n,8,64,64] made channels-last: dst rows of 8 elements, one 16-byte vector."""
    shp = (n, 8, 64, 64)
    ops = [("transpose", (0, 2, 3, 1))]
    return Workload("c8_nhwc" if n == 1024 else f"c8_nhwc_n{n}", 2, [shp], ops,
                    lambda: [f32_to_bf16_bits(normal_f32(shp, 13))])


NEXT_FACTORIES = {"up2x": _up2x, "up2x_nhwc": _up2x_nhwc, "bcast": _bcast, "flip_seq": _flip_seq,
                  "rgb_nhwc": _rgb_nhwc, "up3x": _up3x,
                  "s5_nhwc_pad": _s5_nhwc_pad, "s5_nchw_crop": _s5_nchw_crop, "i35_nchw": _i35_nchw, "i55_nchw": _i55_nchw,
                  "c8_nhwc": _c8_nhwc}

_FACTORIES = {
    "cfg0": _cfg0, "cfg1": _cfg1, "cfg2_fwd": _cfg2_fwd, "cfg2_rev": _cfg2_rev,
    "cfg3": _cfg3, "cfg4": _cfg4,
}

WORKLOAD_NAMES = tuple(_FACTORIES)


NEXT_WORKLOAD_NAMES = tuple(NEXT_FACTORIES)


def workload(name: str, **kw) -> Workload:
    return (_FACTORIES.get(name) or NEXT_FACTORIES[name])(**kw)


def split_qkv_ops(t: int, b: int = 16):
    """Secondary reading of the head split: one chain per Q/K/V output, ending
    in a slice of the leading axis and a reshape that drops it."""
    return [("reshape", (b, 512, 3, 12, 64)), ("transpose", (2, 0, 3, 1, 4)),
            ("slice", 0, t, t + 1, 1), ("reshape", (b, 12, 512, 64))]


# ---- operator graphs for graph-level data-movement elimination (Section 2.1) ----
# A graph is plain data: a list of nodes in topological order, node i defines tensor i.
#   ("input", shape)                      a tensor that exists in memory
#   ("op", op_tuple, [input tensor ids])  a layout operator (concat takes several inputs)
#   ("compute", kind, [input ids], shape) an opaque compute operator producing `shape`
# plus the list of graph outputs.  The compute kinds are stand-ins executed by the test
# harness only: "add" (wrapping integer sum of same-shaped inputs) and "rowmix"
# (A[M,K], W[K,K] -> out[m,n] = A[m,n] + W[0,n], wrapping): the library treats them as opaque.

class Graph:
    def __init__(self, elem_size=2):
        self.elem_size = elem_size
        self.nodes = []
        self.outputs = []

    def input(self, shape):
        self.nodes.append(("input", tuple(shape)))
        return len(self.nodes) - 1

    def op(self, op, inputs):
        self.nodes.append(("op", tuple(op), [int(i) for i in (inputs if isinstance(inputs, (list, tuple)) else [inputs])]))
        return len(self.nodes) - 1

    def store(self, chain, inp, out_shape):
        """A layout operator in store form: out[f_s(i)] = in[i], where f_s is `chain` applied to the
        index space of the output (the chain must turn out_shape into the input's shape)."""
        self.nodes.append(("store", [tuple(o) for o in chain], [int(inp)], tuple(out_shape)))
        return len(self.nodes) - 1

    def compute(self, kind, inputs, shape):
        self.nodes.append(("compute", kind, [int(i) for i in inputs], tuple(shape)))
        return len(self.nodes) - 1

    def output(self, t):
        self.outputs.append(int(t))

    def input_ids(self):
        return [i for i, n in enumerate(self.nodes) if n[0] == "input"]


def wavenet_like_graph(layers=10, batch=1, channels=32, steps=256, skip_steps=64, elem_size=2):
    """A stack of dilated causal gated layers written the way a framework lowers them:
    the shifted taps, the channel concat, the layout change in front of the 1x1
    convolution (a matrix product here), the gate split and the skip slices are all
    separate copy operators between the compute operators.  Stand-in for the paper's
    Parallel WaveNet graph (whose load/store pair count the paper reports); shapes
    [batch, channels, steps]."""
    B, Cc, T = batch, channels, steps
    g = Graph(elem_size)
    x = g.input((B, Cc, T))
    skips = []
    for l in range(layers):
        d = 1 << (l % 6)
        w = g.input((2 * Cc, 2 * Cc))
        p = g.op(("pad", (0, 0, d), (0, 0, 0), 0), x)                 # causal padding
        tap0 = g.op(("slice", 2, 0, T, 1), p)                         # x[t - d]
        tap1 = g.op(("slice", 2, d, T + d, 1), p)                     # x[t]
        cat = g.op(("concat", 1), [tap0, tap1])                       # [B, 2C, T]
        tr = g.op(("transpose", (0, 2, 1)), cat)                      # [B, T, 2C]
        a = g.op(("reshape", (B * T, 2 * Cc)), tr)                    # rows of the matrix product
        z = g.compute("rowmix", [a, w], (B * T, 2 * Cc))
        zr = g.op(("reshape", (B, T, 2 * Cc)), z)
        zt = g.op(("transpose", (0, 2, 1)), zr)                       # back to [B, 2C, T]
        f = g.op(("slice", 1, 0, Cc, 1), zt)                          # filter half
        gt = g.op(("slice", 1, Cc, 2 * Cc, 1), zt)                    # gate half
        gated = g.compute("add", [f, gt], (B, Cc, T))
        skips.append(g.op(("slice", 2, T - skip_steps, T, 1), gated))  # last steps feed the skip path
        x = g.compute("add", [x, gated], (B, Cc, T))                  # residual
    s = g.op(("concat", 1), skips)                                    # [B, layers*C, skip_steps]
    out = g.op(("transpose", (0, 2, 1)), s)
    g.output(out)
    g.output(x)
    return g


# ---- operator graphs for the global layout assignment (Section 2.2) ----
# Plain data again: tensors = [(shape, fixed order or None)], ops = [(operands, is_output flags,
# required orders (None = free), same_layout)].  Logical activations are [N, C, H, W]; a
# convolution asks for channels innermost (order 0,2,3,1) on its input and output, a matrix
# product for row-major operands; normalisation / activation / residual add / pooling take
# any order as long as their operands agree.

NHWC = (0, 2, 3, 1)


def resnet_like_layout_graph(batch=32, stages=((64, 56, 3), (128, 28, 4), (256, 14, 6), (512, 7, 3)), classes=1000):
    """Basic residual blocks (two convolutions, normalisation and activation after each, a
    residual add) in four stages, global pooling and a classifier.  The network input is
    given in the canonical [N, C, H, W] order.  Stand-in for the paper's ResNet-50 run."""
    tensors, ops = [], []

    def tensor(shape, fixed=None):
        tensors.append((tuple(shape), fixed))
        return len(tensors) - 1

    def conv(x, cout, hw):
        y = tensor((batch, cout, hw, hw))
        ops.append(([x, y], [0, 1], [NHWC, NHWC], False))
        return y

    def same(ins, shape):
        y = tensor(shape)
        ops.append((list(ins) + [y], [0] * len(ins) + [1], None, True))
        return y

    x = tensor((batch, 3, 224, 224), fixed=(0, 1, 2, 3))
    x = conv(x, 64, 112)                                    # stem
    x = same([x], (batch, 64, 112, 112))                    # normalisation + activation
    x = same([x], (batch, 64, 56, 56))                      # pooling
    cin = 64
    for cout, hw, blocks in stages:
        for b in range(blocks):
            shp = (batch, cout, hw, hw)
            skip = x if cin == cout else conv(x, cout, hw)  # projection on the skip path when the width changes
            y = conv(x, cout, hw)
            y = same([y], shp)
            y = conv(y, cout, hw)
            y = same([y], shp)
            x = same([y, skip], shp)                        # residual add
            x = same([x], shp)
            cin = cout
    p = same([x], (batch, cin, 1, 1))                       # global average pooling
    flat = tensor((batch, cin))
    ops.append(([p, flat], [0, 1], None, False))            # flatten (free on both sides)
    w = tensor((cin, classes), fixed=(0, 1))
    logits = tensor((batch, classes), fixed=(0, 1))
    ops.append(([flat, w, logits], [0, 0, 1], [(0, 1), (0, 1), (0, 1)], False))
    return tensors, ops
