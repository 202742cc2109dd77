"""Host replay of the 256 x 256-tile GEMM kernel's global accesses (CPU only): every workgroup's load
cursor and every store of every tile, walked with the kernel's own address functions.  All loads must
stay inside A's source and W, every k-step must fetch exactly its own block of both operands, in the
order of use, and every element of out must be written once."""
import numpy as np
import pytest

from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth

SHAPES = [
    # (A source shape, chain -> [M,K]), N, chain on the product or None
    (((512, 128), []), 256, None),                                                                  # two k-steps
    (((256, 192), []), 256, None),
    (((2, 4, 256, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (512, 256))]), 512, None),
    (((2, 2, 512, 64), [("transpose", (1, 2, 0, 3)), ("reshape", (1024, 128))]), 512, None),         # K = 128 over two digits of k
    (((2, 1024, 2, 64), [("transpose", (0, 2, 1, 3)), ("slice", 2, 256, 768, 1), ("transpose", (0, 2, 1, 3)),
                         ("reshape", (1024, 128))]), 256, None),                                    # base offset
    (((512, 128), []), 768, [("reshape", (2, 256, 3, 4, 64)), ("transpose", (2, 0, 3, 1, 4))]),     # mapped store
    (((4352, 128), []), 4096, None),                                                                # more tiles than workgroups
    (((4352, 192), []), 4096, [("reshape", (4352, 64, 64)), ("transpose", (1, 0, 2))]),
]


@pytest.mark.parametrize("case", range(len(SHAPES)))
def test_replay_of_fixed_shapes(case):
    (shape, ops), n, c_ops = SHAPES[case]
    a = B.amap_compose([shape], 2, ops)
    m, _ = B.dst_shape(a)
    out_map = B.amap_compose([(m, n)], 2, c_ops) if c_ops else None
    for nwg in (256, 3, 1):          # 3 and 1: every workgroup walks many tiles
        assert B.amap_gemm_selfcheck(a, n, out_map, nwg) == 0, nwg


def test_replay_of_the_headline_product():
    w = synth.workload("cfg4")
    a = B.amap_compose(w.src_shapes, 2, w.ops)
    assert B.amap_gemm_selfcheck(a, w.gemm_n, None, 256) == 0
    # the QKV projection stored in the head-split layout
    a2 = B.amap_compose([(8192, 768)], 2, [])
    store = B.amap_compose([(8192, 2304)], 2, synth.workload("cfg2_fwd").ops)
    assert B.amap_gemm_selfcheck(a2, 2304, store, 256) == 0


def test_replay_of_random_aligned_shapes():
    rng = np.random.default_rng(5)
    ran = 0
    for _ in range(60):
        b, h = int(rng.integers(1, 3)), int(rng.integers(1, 5))
        s, d = 256 * int(rng.integers(1, 3)), 64 * int(rng.integers(1, 3))
        if h * d < 128:
            h = 2
        n = 256 * int(rng.integers(1, 4))
        form = int(rng.integers(3))
        if form == 0:
            shape, ops = (b, h, s, d), [("transpose", (0, 2, 1, 3)), ("reshape", (b * s, h * d))]
        elif form == 1:
            shape, ops = (b * s, h * d), []
        else:
            shape, ops = (h, b, s, d), [("transpose", (1, 2, 0, 3)), ("reshape", (b * s, h * d))]
        a = B.amap_compose([shape], 2, ops)
        m = b * s
        out_map = B.amap_compose([(m, n)], 2, [("reshape", (m, n // 64, 64)), ("transpose", (1, 0, 2))]) if rng.random() < 0.5 else None
        assert B.amap_gemm_selfcheck(a, n, out_map, int(rng.choice([1, 2, 5, 256]))) == 0, (shape, ops, n)
        ran += 1
    assert ran == 60


def test_products_of_the_general_kernel_have_no_replay():
    for shape, ops, n in [((200, 72), [], 128),                                   # K is no multiple of 64
                          ((512, 64), [], 256),                                   # one k-step
                          ((2, 4, 250, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (500, 256))], 512),   # tiles would straddle the two digits of m
                          ((256, 136), [("pad", (0, 0), (0, 56), 0)], 256),       # padded
                          ((128, 512), [("transpose", (1, 0))], 256)]:            # runs along m
        a = B.amap_compose([shape], 2, ops)
        with pytest.raises(B.AmapError) as e:
            B.amap_gemm_selfcheck(a, n)
        assert e.value.status == B.AMAP_E_UNSUPPORTED


def test_replay_of_an_operand_of_more_than_2_31_elements():
    """Tile and k-step bases are 64-bit: A[1048832, 2048] (4.3 GB) read plainly and through a head merge."""
    m, k, n = 4097 * 256, 2048, 256
    assert B.amap_gemm_selfcheck(B.amap_compose([(m, k)], 2, []), n, None, 256) == 0
    merged = B.amap_compose([(4097, 16, 256, 128)], 2, [("transpose", (0, 2, 1, 3)), ("reshape", (m, k))])
    assert B.amap_gemm_selfcheck(merged, n, None, 64) == 0
    # not for the general kernel, and not with a mapped store
    assert B.amap_gemm_selfcheck(B.amap_compose([(m + 8, k)], 2, []), n, None, 256) == 0        # a partial last tile
    for a, out_map in [(B.amap_compose([(m, k + 8)], 2, []), None),                             # K is no multiple of 64
                       (B.amap_compose([(m, k)], 2, []), B.amap_compose([(m, n)], 2, [("reshape", (m, 4, 64)), ("transpose", (1, 0, 2))]))]:
        with pytest.raises(B.AmapError) as e:
            B.amap_gemm_selfcheck(a, n, out_map, 256)
        assert e.value.status == B.AMAP_E_UNSUPPORTED


WT_SHAPES = [
    # (A source shape, chain), (W source shape, chain -> [K,N]), chain on the product or None
    (((512, 128), []), ((256, 128), [("transpose", (1, 0))]), None),
    (((512, 256), []), ((768, 320), [("slice", 1, 64, 320, 1), ("transpose", (1, 0))]), [("reshape", (512, 12, 64)), ("transpose", (1, 0, 2))]),
    (((4352, 128), []), ((4096, 128), [("transpose", (1, 0))]), None),
    (((512, 192), []), ((2, 256, 192), [("transpose", (2, 0, 1)), ("reshape", (192, 512))]), None),
    (((16, 16, 512, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (8192, 1024))]), ((4096, 1024), [("transpose", (1, 0))]), None),
]


@pytest.mark.parametrize("case", range(len(WT_SHAPES)))
def test_replay_with_the_weight_kept_transposed(case):
    (shape, ops), (w_shape, w_ops), c_ops = WT_SHAPES[case]
    a, w = B.amap_compose([shape], 2, ops), B.amap_compose([w_shape], 2, w_ops)
    (m, _), (_, n) = B.dst_shape(a), B.dst_shape(w)
    out_map = B.amap_compose([(m, n)], 2, c_ops) if c_ops else None
    for nwg in (256, 2):
        assert B.amap_gemm_selfcheck(a, n, out_map, nwg, w) == 0, nwg


def test_a_weight_with_runs_along_n_through_a_map_has_no_replay():
    a, w = B.amap_compose([(512, 128)], 2, []), B.amap_compose([(128, 256)], 2, [])
    with pytest.raises(B.AmapError) as e:
        B.amap_gemm_selfcheck(a, 256, None, 256, w)
    assert e.value.status == B.AMAP_E_UNSUPPORTED


EDGE_SHAPES = [
    # M, K, N, workgroups: partial last tiles in M and / or N
    (200, 128, 136, 256), (300, 192, 264, 256), (1000, 256, 1000, 3), (8, 128, 8, 256), (257, 128, 8, 1), (256, 128, 264, 2),
]


@pytest.mark.parametrize("case", range(len(EDGE_SHAPES)))
def test_replay_of_partial_last_tiles(case):
    m, k, n, nwg = EDGE_SHAPES[case]
    a = B.amap_compose([(m, k)], 2, [])
    assert B.amap_gemm_selfcheck(a, n, None, nwg) == 0
    wt = B.amap_compose([(n, k)], 2, [("transpose", (1, 0))])          # the weight kept as [N,K]
    assert B.amap_gemm_selfcheck(a, n, None, nwg, wt) == 0
    if n % 8 == 0 and n >= 16:
        store = B.amap_compose([(m, n)], 2, [("reshape", (m, n // 8, 8)), ("transpose", (1, 0, 2))])
        assert B.amap_gemm_selfcheck(a, n, store, nwg) == 0


def test_replay_of_random_partial_shapes():
    rng = np.random.default_rng(17)
    for _ in range(60):
        m, k, n = int(rng.integers(1, 1200)), 64 * int(rng.integers(2, 6)), 8 * int(rng.integers(1, 150))
        a = B.amap_compose([(m + 3, k + 64)], 2, [("slice", 0, 3, m + 3, 1), ("slice", 1, 64, k + 64, 1)])   # base offset, longer rows
        assert B.amap_gemm_selfcheck(a, n, None, int(rng.choice([1, 4, 256]))) == 0, (m, k, n)
