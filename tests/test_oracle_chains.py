"""Pins for oracle chains: the hand-derived closed-form address function of
each workload's composed chain (full size, iota sources so that the output *is*
the address table), permutation / fill-count invariants, and chain identities.
"""
import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import synth


def _iota_sources(w):
    # 4-byte iota regardless of the workload's element size: the oracle moves
    # opaque elements, and 32 bits keep every source position distinct.
    srcs, base = [], 0
    for s in w.src_shapes:
        srcs.append((np.arange(int(np.prod(s)), dtype=np.uint32) + np.uint32(base)).reshape(s))
        base += int(np.prod(s))
    return srcs


FILL = 0xFFFFFFFF


def _ops_with_fill(ops):
    return [(o[0], o[1], o[2], FILL) if o[0] == "pad" else o for o in ops]


def test_cfg0_closed_form():
    w = synth.workload("cfg0")
    out = oracle.run_chain(_iota_sources(w), _ops_with_fill(w.ops))
    assert out.shape == (8, 768, 20)
    n, r, c = np.meshgrid(np.arange(8), np.arange(768), np.arange(20), indexing="ij")
    want = np.where(c < 16, n * 16384 + c * 1024 + r + 128, FILL).astype(np.uint32)
    assert np.array_equal(out, want)
    assert int((out == FILL).sum()) == 24576
    data = out[out != FILL]
    assert np.unique(data).size == data.size == 98304  # 393,216 source bytes are needed


def test_cfg1_closed_form():
    w = synth.workload("cfg1")
    out = oracle.run_chain(_iota_sources(w), _ops_with_fill(w.ops))
    assert out.shape == (32, 58, 58, 256)
    n = np.arange(32).reshape(32, 1, 1, 1)
    y = np.arange(58).reshape(1, 58, 1, 1)
    x = np.arange(58).reshape(1, 1, 58, 1)
    c = np.arange(256).reshape(1, 1, 1, 256)
    inside = (y >= 1) & (y <= 56) & (x >= 1) & (x <= 56)
    addr = n * 802816 + c * 3136 + (y - 1) * 56 + (x - 1)
    want = np.where(inside, addr, FILL).astype(np.uint32)
    assert np.array_equal(out, want)
    assert int((out == FILL).sum()) == 1867776
    data = out[out != FILL]
    assert np.array_equal(np.sort(data), np.arange(32 * 256 * 56 * 56, dtype=np.uint32))


def test_cfg2_fwd_closed_form():
    w = synth.workload("cfg2_fwd")
    out = oracle.run_chain(_iota_sources(w), w.ops)
    assert out.shape == (3, 16, 12, 512, 64)
    t = np.arange(3).reshape(3, 1, 1, 1, 1)
    b = np.arange(16).reshape(1, 16, 1, 1, 1)
    h = np.arange(12).reshape(1, 1, 12, 1, 1)
    s = np.arange(512).reshape(1, 1, 1, 512, 1)
    d = np.arange(64).reshape(1, 1, 1, 1, 64)
    want = (b * 1179648 + s * 2304 + t * 768 + h * 64 + d).astype(np.uint32)
    assert np.array_equal(out, want)
    assert np.array_equal(np.sort(out.ravel()), np.arange(out.size, dtype=np.uint32))
    # secondary reading: one chain per Q/K/V output gives the three leading blocks
    for tt in range(3):
        q = oracle.run_chain(_iota_sources(w), synth.split_qkv_ops(tt))
        assert np.array_equal(q, out[tt])


def test_cfg2_rev_closed_form():
    w = synth.workload("cfg2_rev")
    out = oracle.run_chain(_iota_sources(w), w.ops)
    assert out.shape == (16, 512, 768)
    b = np.arange(16).reshape(16, 1, 1)
    s = np.arange(512).reshape(1, 512, 1)
    e = np.arange(768).reshape(1, 1, 768)
    want = (b * 393216 + (e // 64) * 32768 + s * 64 + (e % 64)).astype(np.uint32)
    assert np.array_equal(out, want)
    assert np.array_equal(np.sort(out.ravel()), np.arange(out.size, dtype=np.uint32))


def test_cfg2_rev_inverts_fwd_block():
    """Merging the heads of the Q block undoes the split of a [B,S,768] tensor."""
    x = synth.random_bits((4, 32, 768), 2, 21)
    split = oracle.run_chain([x], [("reshape", (4, 32, 12, 64)), ("transpose", (0, 2, 1, 3))])
    merged = oracle.run_chain([split], [("transpose", (0, 2, 1, 3)), ("reshape", (4, 32, 768))])
    assert np.array_equal(merged, x)


def test_cfg3_closed_form():
    w = synth.workload("cfg3")
    srcs = _iota_sources(w)
    out = oracle.run_chain(srcs, w.ops)
    assert out.shape == (32, 28, 28, 320)
    chans, offs = (64, 96, 128, 32), (0, 64, 160, 288)
    n = np.arange(32).reshape(32, 1, 1, 1)
    y = np.arange(28).reshape(1, 28, 1, 1)
    x = np.arange(28).reshape(1, 1, 28, 1)
    base = 0
    for cm, off in zip(chans, offs):
        c = np.arange(cm).reshape(1, 1, 1, cm)
        want = (base + n * cm * 784 + c * 784 + y * 28 + x).astype(np.uint32)
        assert np.array_equal(out[..., off:off + cm], want)
        base += 32 * cm * 784
    assert np.array_equal(np.sort(out.ravel()), np.arange(out.size, dtype=np.uint32))


def test_cfg4_closed_form():
    w = synth.workload("cfg4")
    out = oracle.run_chain(_iota_sources(w), w.ops)
    assert out.shape == (8192, 1024)
    m = np.arange(8192).reshape(8192, 1)
    k = np.arange(1024).reshape(1, 1024)
    want = ((m // 512) * 524288 + (k // 64) * 32768 + (m % 512) * 64 + (k % 64)).astype(np.uint32)
    assert np.array_equal(out, want)


@pytest.mark.parametrize("name", ["cfg0", "cfg2_rev", "cfg3"])
def test_real_inputs_match_numpy_pipeline(name):
    """Same chains through numpy's own routines on the real seeded inputs."""
    w = synth.workload(name)
    srcs = w.sources()
    got = oracle.run_chain(srcs, w.ops)
    xs = srcs
    for op in w.ops:
        if op[0] == "concat":
            xs = [np.concatenate(xs, axis=op[1])]
        elif op[0] == "transpose":
            xs = [np.transpose(xs[0], op[1])]
        elif op[0] == "reshape":
            xs = [np.reshape(np.ascontiguousarray(xs[0]), op[1])]
        elif op[0] == "slice":
            sl = [slice(None)] * xs[0].ndim
            sl[op[1]] = slice(op[2], op[3], op[4])
            xs = [xs[0][tuple(sl)]]
        elif op[0] == "pad":
            xs = [np.pad(xs[0], list(zip(op[1], op[2])), constant_values=op[3])]
    assert np.array_equal(got, np.ascontiguousarray(xs[0]))


def test_transpose_inverse_and_reshape_round_trip_chain():
    x = synth.random_bits((3, 4, 5, 6), 4, 2)
    p = (2, 0, 3, 1)
    ops = [("transpose", p), ("transpose", tuple(int(v) for v in np.argsort(p))),
           ("reshape", (12, 30)), ("reshape", (3, 4, 5, 6))]
    assert np.array_equal(oracle.run_chain([x], ops), x)


def test_intermediates_are_materialised():
    w = synth.workload("cfg0")
    out, inter = oracle.run_chain(w.sources(), w.ops, keep_intermediates=True)
    assert [t.shape for t in inter] == [(8, 32, 32, 16), (8, 1024, 16), (8, 768, 16), (8, 768, 20)]
    # bytes written by the un-optimised program: every intermediate once
    assert sum(t.nbytes for t in inter) == 524288 + 524288 + 393216 + 491520
    assert out is inter[-1]
