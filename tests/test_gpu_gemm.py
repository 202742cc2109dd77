"""GPU parity of the fused-prologue GEMM against the CPU oracle (which
materialises A with the operator chain, then multiplies in float64)."""
import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-2  # max|err| <= TOL * max|ref|  (bf16 inputs, fp32 accumulation, bf16 output)


@pytest.fixture(scope="module")
def dev():
    from paper_2002_12798_amd import device
    device.require_gpu()
    return device


def _gemm(dev, src_bits, shape, ops, w_bits):
    import torch
    m = B.amap_compose([shape], 2, ops)
    out = dev.gemm_fused(dev.to_device(src_bits), m, dev.to_device(w_bits))
    torch.cuda.synchronize()
    return dev.to_host(out)


def _check(got_bits, a_bits, w_bits, exact=False):
    oracle.set_threads(8)
    try:
        want_bits = oracle.gemm_bf16(a_bits, w_bits)
    finally:
        oracle.set_threads(1)
    if exact:
        assert np.array_equal(got_bits, want_bits)
        return
    got, want = synth.bf16_bits_to_f32(got_bits).astype(np.float64), synth.bf16_bits_to_f32(want_bits).astype(np.float64)
    err = np.abs(got - want).max()
    ref = np.abs(want).max()
    assert err <= TOL * ref, (err, ref)
    # much tighter in practice: both sides round an almost identical sum to bf16
    ulp = np.maximum(np.abs(want), 2.0 ** -126) * 2.0 ** -7
    assert np.mean(np.abs(got - want) <= ulp) > 0.999


def test_cfg4_full_size(dev):
    print("[gpu] gemm cfg4", flush=True)
    w = synth.workload("cfg4")
    src = w.sources()[0]
    wt = w.weight()
    got = _gemm(dev, src, w.src_shapes[0], w.ops, wt)
    a = oracle.run_chain([src], w.ops)
    assert got.shape == (8192, 4096)
    _check(got, a, wt)
    # sampled outputs recomputed one by one
    rng = np.random.default_rng(1)
    gf = synth.bf16_bits_to_f32(got)
    for m, n in zip(rng.integers(0, 8192, 64), rng.integers(0, 4096, 64)):
        ref = oracle.gemm_bf16_point(a, wt, m, n)
        assert abs(gf[m, n] - ref) <= 2.0 ** -7 * abs(ref) + 1e-6


def test_identity_weight_isolates_the_prologue(dev):
    """W = shifted identity: every output is one A element times 1.0, exact in
    any summation order, so C must reproduce A bit for bit."""
    shape, ops = (2, 4, 128, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (256, 256))]
    src = synth.f32_to_bf16_bits(np.random.default_rng(3).standard_normal(shape).astype(np.float32))
    wf = np.zeros((256, 512), dtype=np.float32)
    wf[np.arange(256), (np.arange(256) * 7 + 5) % 512] = 1.0
    got = _gemm(dev, src, shape, ops, synth.f32_to_bf16_bits(wf))
    a = oracle.run_chain([src], ops)
    want = np.zeros((256, 512), dtype=np.uint16)
    want[:, (np.arange(256) * 7 + 5) % 512] = a
    # -0.0 * 1 + 0 sums to +0.0 in both; compare values of zeros, bits elsewhere
    nz = (a & 0x7FFF) != 0
    assert np.array_equal(got[:, (np.arange(256) * 7 + 5) % 512][nz], a[nz])
    assert not (got & 0x7FFF)[want == 0].any()


def test_small_integers_are_exact(dev):
    rng = np.random.default_rng(4)
    shape = (256, 192)
    a = rng.integers(-3, 4, shape).astype(np.float32)
    wf = rng.integers(-3, 4, (192, 256)).astype(np.float32)   # |sum| <= 192*9 = 1728 < 2^11: exact in fp32
    got = _gemm(dev, synth.f32_to_bf16_bits(a), shape, [], synth.f32_to_bf16_bits(wf))
    _check(got, synth.f32_to_bf16_bits(a), synth.f32_to_bf16_bits(wf), exact=True)


CASES = [
    # source shape, chain producing A[M,K]
    ((256, 64), []),                                                            # smallest, identity map
    ((512, 192), []),
    ((8, 64, 64), [("transpose", (1, 0, 2)), ("reshape", (64, 512)), ("transpose", (1, 0)), ("reshape", (8, 64, 64)),
                   ("transpose", (0, 2, 1)), ("reshape", (512, 64))]),          # several ops, k = former row index
    ((4, 2, 128, 32), [("transpose", (0, 2, 1, 3)), ("reshape", (512, 64))]),    # head merge, 32-element runs
    ((3, 256, 8, 8), [("transpose", (1, 0, 2, 3)), ("reshape", (256, 192))]),    # 64-element runs, 3 k digits
    ((2, 8, 128, 8), [("transpose", (0, 2, 1, 3)), ("reshape", (256, 64))]),     # 8-element runs (one vector)
    ((300, 128), [("slice", 0, 22, 278, 1)]),                                    # base offset in the source
    ((2, 256, 2, 64), [("transpose", (0, 1, 3, 2)), ("transpose", (0, 1, 3, 2)), ("reshape", (512, 128))]),
    ((64, 128), [("repeat", 0, 4)]),                                             # every A row read by 4 output rows
    ((2, 128, 64), [("slice", 1, 127, -1, -1), ("tile", 0, 2), ("reshape", (512, 64))]),  # rows walked backwards, tiled
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_maps_vs_oracle(dev, case):
    shape, ops = CASES[case]
    print(f"[gpu] gemm case {case} {shape} {ops}", flush=True)
    rng = np.random.default_rng(10 + case)
    src = synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    a = oracle.run_chain([src], ops) if ops else src
    K = a.shape[1]
    N = 128 * (1 + case % 4)
    wt = synth.f32_to_bf16_bits((rng.standard_normal((K, N)) * 0.05).astype(np.float32))
    got = _gemm(dev, src, shape, ops, wt)
    _check(got, a, wt)


def test_unsupported_and_error_paths(dev):
    import torch
    x = torch.zeros(1 << 20, dtype=torch.int16, device="cuda")
    y = torch.zeros(1 << 20, dtype=torch.int16, device="cuda")
    w = torch.zeros(1 << 20, dtype=torch.int16, device="cuda")

    def call(m, n=256, a=None, wp=None, o=None):
        B.amap_gemm_fused((x if a is None else a).data_ptr(), m, (w if wp is None else wp).data_ptr(), n,
                          (y if o is None else o).data_ptr(), 0)

    for m, n, status in [
        (B.amap_compose([(256, 68)], 2, []), 256, B.AMAP_E_UNSUPPORTED),                    # K % 8
        (B.amap_compose([(256, 64)], 2, []), 196, B.AMAP_E_UNSUPPORTED),                    # N % 8
        (B.amap_compose([(256, 64)], 4, []), 256, B.AMAP_E_INVALID),                        # not 2-byte
        (B.amap_compose([(4, 256, 64)], 2, []), 256, B.AMAP_E_INVALID),                     # not a matrix
        (B.amap_compose([(256, 60)], 2, [("pad", (0, 0), (0, 4), 0)]), 256, B.AMAP_E_UNSUPPORTED),  # padding that cuts a 16-byte vector
        (B.amap_compose([(256, 64)], 2, [("pad", (0, 0), (0, 8), 0), ("pad", (0, 0), (0, 8), 5)]), 256, B.AMAP_E_UNSUPPORTED),  # two pad constants
        (B.amap_compose([(64, 252)], 2, [("transpose", (1, 0))]), 256, B.AMAP_E_UNSUPPORTED),       # runs along m, M % 8
        (B.amap_compose([(64, 512)], 2, [("transpose", (1, 0)), ("slice", 0, 0, 512, 2)]), 256, B.AMAP_E_UNSUPPORTED),  # no runs at all
        (B.amap_compose([(256, 128)], 2, [("slice", 1, 0, 128, 2)]), 256, B.AMAP_E_UNSUPPORTED),    # strided k
    ]:
        with pytest.raises(B.AmapError) as e:
            call(m, n)
        assert e.value.status == status, (e.value.status, status)
    m = B.amap_compose([(256, 64)], 2, [])
    with pytest.raises(B.AmapError) as e:
        call(m, o=x)
    assert e.value.status == B.AMAP_E_ALIAS
    with pytest.raises(B.AmapError) as e:
        B.amap_gemm_fused(x.data_ptr() + 2, m, w.data_ptr(), 256, y.data_ptr(), 0)
    assert e.value.status == B.AMAP_E_INVALID
    torch.cuda.synchronize()


EDGE_CASES = [
    # M, K, N not whole numbers of 256 x 64 x 128 tiles; (A source shape, chain -> [M,K]), N
    (((200, 64), []), 128),                                                    # M edge only
    (((256, 72), []), 128),                                                    # K edge only
    (((256, 64), []), 200),                                                    # N edge only
    (((8, 8), []), 8),                                                         # everything smaller than one tile
    (((3, 100, 40), [("transpose", (1, 0, 2)), ("reshape", (100, 120))]), 136),  # mapped A, all three edges
    (((700, 200), [("slice", 0, 699, -1, -1)]), 264),                          # several tiles and an edge each way
]


@pytest.mark.parametrize("case", range(len(EDGE_CASES)))
def test_edge_tiles(dev, case):
    (shape, ops), N = EDGE_CASES[case]
    print(f"[gpu] gemm edge case {case}", flush=True)
    src = synth.f32_to_bf16_bits(np.random.default_rng(700 + case).standard_normal(shape).astype(np.float32))
    a = oracle.run_chain([src], ops)
    K = a.shape[1]
    w = synth.f32_to_bf16_bits((np.random.default_rng(800 + case).standard_normal((K, N)) * 0.05).astype(np.float32))
    _check(_gemm(dev, src, shape, ops, w), a, w)
    # transposed weight and a mapped store on the same shapes
    import torch
    a_map = B.amap_compose([shape], 2, ops)
    w_map = B.amap_compose([(N, K)], 2, [("transpose", (1, 0))])
    out_map = B.amap_compose([(a.shape[0], N)], 2, [("slice", 0, a.shape[0] - 1, -1, -1)])
    d_src, d_wt = dev.to_device(src), dev.to_device(np.ascontiguousarray(w.T))
    out = dev.empty_dst(out_map)
    B.amap_gemm_mapped(d_src.data_ptr(), a_map, d_wt.data_ptr(), w_map, out_map, out.data_ptr(), 0)
    torch.cuda.synchronize()
    _check(dev.to_host(out)[::-1], a, w)


# ---- store side: the product written through a layout chain (the paper's store map f_s)

STORE_CASES = [
    # (A source shape, A chain -> [M,K]), N, chain applied to the [M,N] product
    (((512, 64), []), 384, [("reshape", (2, 256, 3, 2, 64)), ("transpose", (2, 0, 3, 1, 4))]),     # QKV head split
    (((256, 128), []), 256, [("reshape", (4, 64, 4, 64)), ("transpose", (0, 2, 1, 3)), ("reshape", (16, 64, 64))]),
    (((2, 4, 128, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (256, 256))]), 128,
     [("reshape", (2, 128, 2, 64)), ("transpose", (2, 0, 1, 3))]),                                  # both sides mapped
    (((256, 64), []), 128, [("slice", 0, 255, -1, -1)]),                                            # rows stored backwards
]


@pytest.mark.parametrize("case", range(len(STORE_CASES)))
def test_store_mapped_product_vs_oracle(dev, case):
    import torch
    (shape, a_ops), N, c_ops = STORE_CASES[case]
    print(f"[gpu] store-mapped gemm case {case}", flush=True)
    src = synth.f32_to_bf16_bits(np.random.default_rng(300 + case).standard_normal(shape).astype(np.float32))
    a_map = B.amap_compose([shape], 2, a_ops)
    M, K = B.dst_shape(a_map)
    w = synth.f32_to_bf16_bits((np.random.default_rng(400 + case).standard_normal((K, N)) * 0.05).astype(np.float32))
    out_map = B.amap_compose([(M, N)], 2, c_ops)
    out = dev.gemm_fused(dev.to_device(src), a_map, dev.to_device(w), out_map=out_map)
    torch.cuda.synchronize()
    got = dev.to_host(out)
    a_bits = oracle.run_chain([src], a_ops)
    want = oracle.run_chain([oracle.gemm_bf16(a_bits, w)], c_ops)     # un-fused: product, then the chain on it
    assert got.shape == want.shape
    # the same numbers as the plain fused product, only stored elsewhere: compare bit for bit with it
    plain = dev.to_host(dev.gemm_fused(dev.to_device(src), a_map, dev.to_device(w)))
    assert np.array_equal(got, oracle.run_chain([plain], c_ops))
    g, r = synth.bf16_bits_to_f32(got).astype(np.float64), synth.bf16_bits_to_f32(want).astype(np.float64)
    assert np.abs(g - r).max() <= TOL * np.abs(r).max()


def test_store_map_error_paths(dev):
    import torch
    a_map = B.amap_compose([(256, 64)], 2, [])
    a = torch.zeros((256, 64), dtype=torch.int16, device="cuda")
    w = torch.zeros((64, 128), dtype=torch.int16, device="cuda")
    out = torch.zeros((256, 128), dtype=torch.int16, device="cuda")
    bad = [
        (B.amap_compose([(256, 128)], 2, [("slice", 1, 0, 64, 1)]), B.AMAP_E_UNSUPPORTED),     # drops half: no bijection
        (B.amap_compose([(256, 128)], 2, [("transpose", (1, 0))]), B.AMAP_E_UNSUPPORTED),      # n not contiguous in out
        (B.amap_compose([(128, 128)], 2, []), B.AMAP_E_INVALID),                               # not the product's shape
        (B.amap_compose([(256, 128)], 4, []), B.AMAP_E_INVALID),                               # wrong element size
        (B.amap_compose([(256, 128)], 2, [("repeat", 0, 2)]), B.AMAP_E_UNSUPPORTED),           # written twice
    ]
    for om, status in bad:
        with pytest.raises(B.AmapError) as e:
            B.amap_gemm_fused_store(a.data_ptr(), a_map, w.data_ptr(), 128, om, out.data_ptr(), 0)
        assert e.value.status == status, status


# ---- W read through a map too

W_CASES = [
    # (W source shape, chain -> [K,N]); A is the identity of [256,K]
    ((384, 128), [("transpose", (1, 0))]),                                         # transposed weight: runs along k
    ((2, 64, 128), [("transpose", (1, 0, 2)), ("reshape", (64, 256))]),            # runs along n, two blocks per row
    ((4, 128, 64), [("transpose", (1, 0, 2)), ("reshape", (128, 256)), ("transpose", (1, 0))]),  # [256,128]: runs of 64 along k
    ((130, 128), [("slice", 0, 2, 130, 1)]),                                       # row-major weight at an offset
    ((128, 256), [("transpose", (1, 0)), ("slice", 0, 255, -1, -1)]),              # runs along k, k walked backwards in blocks
]


@pytest.mark.parametrize("case", range(len(W_CASES)))
def test_w_operand_through_a_map(dev, case):
    import torch
    w_shape, w_ops = W_CASES[case]
    print(f"[gpu] mapped-W gemm case {case}", flush=True)
    w_src = synth.f32_to_bf16_bits((np.random.default_rng(500 + case).standard_normal(w_shape) * 0.05).astype(np.float32))
    w_map = B.amap_compose([w_shape], 2, w_ops)
    K, N = B.dst_shape(w_map)
    a = synth.f32_to_bf16_bits(np.random.default_rng(600 + case).standard_normal((256, K)).astype(np.float32))
    a_map = B.amap_compose([(256, K)], 2, [])
    out = torch.empty((256, N), dtype=torch.int16, device="cuda")
    d_a, d_w = dev.to_device(a), dev.to_device(w_src)          # kept alive until the product has been read back
    try:
        B.amap_gemm_mapped(d_a.data_ptr(), a_map, d_w.data_ptr(), w_map, None, out.data_ptr(), 0)
    except B.AmapError as e:
        # the last case reverses k element by element: runs of one element along k, refused
        assert case == len(W_CASES) - 1 and e.status == B.AMAP_E_UNSUPPORTED
        return
    torch.cuda.synchronize()
    assert case != len(W_CASES) - 1
    _check(dev.to_host(out), a, oracle.run_chain([w_src], w_ops))


def test_all_three_accesses_mapped(dev):
    """A, W and the store each through their own chain; against product-then-chain on the oracle."""
    import torch
    a_shape, a_ops = (2, 4, 128, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (256, 256))]
    w_shape, w_ops = (256, 256), [("transpose", (1, 0))]
    c_ops = [("reshape", (2, 128, 4, 64)), ("transpose", (2, 0, 1, 3))]
    a_src = synth.f32_to_bf16_bits(np.random.default_rng(71).standard_normal(a_shape).astype(np.float32))
    w_src = synth.f32_to_bf16_bits((np.random.default_rng(72).standard_normal(w_shape) * 0.05).astype(np.float32))
    a_map, w_map = B.amap_compose([a_shape], 2, a_ops), B.amap_compose([w_shape], 2, w_ops)
    out_map = B.amap_compose([(256, 256)], 2, c_ops)
    out = dev.empty_dst(out_map)
    d_a, d_w = dev.to_device(a_src), dev.to_device(w_src)
    B.amap_gemm_mapped(d_a.data_ptr(), a_map, d_w.data_ptr(), w_map, out_map, out.data_ptr(), 0)
    torch.cuda.synchronize()
    prod = oracle.gemm_bf16(oracle.run_chain([a_src], a_ops), oracle.run_chain([w_src], w_ops))
    want = oracle.run_chain([prod], c_ops)
    got = dev.to_host(out)
    g, r = synth.bf16_bits_to_f32(got).astype(np.float64), synth.bf16_bits_to_f32(want).astype(np.float64)
    assert got.shape == want.shape and np.abs(g - r).max() <= TOL * np.abs(r).max()
    ulp = np.maximum(np.abs(r), 2.0 ** -126) * 2.0 ** -7
    assert np.mean(np.abs(g - r) <= ulp) > 0.999


# ---- A whose contiguous runs lie along m: a transposed operand, a channel-major activation

A_M_CASES = [
    # (A source shape, chain -> [M,K]), N
    (((64, 256), [("transpose", (1, 0))]), 128),                                              # A kept as [K,M]
    (((2, 64, 16, 16), [("transpose", (0, 2, 3, 1)), ("reshape", (512, 64))]), 256),          # NCHW into a pointwise convolution
    (((3, 40, 10, 12), [("transpose", (0, 2, 3, 1)), ("reshape", (360, 40))]), 136),          # the same with an edge in M, K and N
    (((128, 304), [("slice", 1, 24, 280, 1), ("transpose", (1, 0))]), 128),                   # runs start at an offset
    (((192, 8), [("transpose", (1, 0))]), 8),                                                 # smaller than one tile
    (((2, 72, 264), [("transpose", (0, 2, 1)), ("reshape", (528, 72))]), 384),                # several tiles each way
]


@pytest.mark.parametrize("case", range(len(A_M_CASES)))
def test_a_operand_with_runs_along_m(dev, case):
    import torch
    (shape, ops), N = A_M_CASES[case]
    print(f"[gpu] m-major A gemm case {case}", flush=True)
    src = synth.f32_to_bf16_bits(np.random.default_rng(900 + case).standard_normal(shape).astype(np.float32))
    a = oracle.run_chain([src], ops)
    M, K = a.shape
    w = synth.f32_to_bf16_bits((np.random.default_rng(950 + case).standard_normal((K, N)) * 0.05).astype(np.float32))
    _check(_gemm(dev, src, shape, ops, w), a, w)
    # with the weight kept transposed and the product stored through a chain as well
    a_map = B.amap_compose([shape], 2, ops)
    w_map = B.amap_compose([(N, K)], 2, [("transpose", (1, 0))])
    out_map = B.amap_compose([(M, N)], 2, [("slice", 0, M - 1, -1, -1)])
    d_src, d_wt = dev.to_device(src), dev.to_device(np.ascontiguousarray(w.T))
    out = dev.empty_dst(out_map)
    B.amap_gemm_mapped(d_src.data_ptr(), a_map, d_wt.data_ptr(), w_map, out_map, out.data_ptr(), 0)
    torch.cuda.synchronize()
    _check(dev.to_host(out)[::-1], a, w)


def test_m_major_identity_weight_is_exact(dev):
    """W = permutation matrix: every output is one A element, so the transposing prologue
    must reproduce A bit for bit (values of zeros aside)."""
    shape, ops = (2, 128, 8, 32), [("transpose", (0, 2, 3, 1)), ("reshape", (512, 128))]
    src = synth.f32_to_bf16_bits(np.random.default_rng(31).standard_normal(shape).astype(np.float32))
    cols = (np.arange(128) * 5 + 3) % 128
    wf = np.zeros((128, 128), dtype=np.float32)
    wf[np.arange(128), cols] = 1.0
    got = _gemm(dev, src, shape, ops, synth.f32_to_bf16_bits(wf))
    a = oracle.run_chain([src], ops)
    nz = (a & 0x7FFF) != 0
    assert np.array_equal(got[:, cols][nz], a[nz])


# ---- A gathered from several sources: a concat along k that is never materialised

GATHER_CASES = [
    # source shapes, chain -> [M,K], N
    ([(256, 64), (256, 128), (256, 64)], [("concat", 1)], 128),                                        # runs along k, ends at 64, 192
    ([(2, 8, 16, 64), (2, 8, 16, 128)], [("concat", 3), ("reshape", (256, 192))], 256),                # NHWC branches
    ([(2, 64, 16, 16), (2, 96, 16, 16), (2, 128, 16, 16), (2, 32, 16, 16)],
     [("concat", 1), ("transpose", (0, 2, 3, 1)), ("reshape", (512, 320))], 128),                      # NCHW branches: runs along m
    ([(3, 32, 10, 12), (3, 40, 10, 12)], [("concat", 1), ("transpose", (0, 2, 3, 1)), ("reshape", (360, 72))], 136),  # + edges
    ([(200, 64), (200, 40)], [("concat", 1)], 72),                                                     # runs along k, edges
    ([(520, 128)] * 8, [("concat", 1)], 384),                                                          # eight sources, several tiles
]


@pytest.mark.parametrize("case", range(len(GATHER_CASES)))
def test_a_gathered_from_several_sources(dev, case):
    import torch
    shapes, ops, N = GATHER_CASES[case]
    print(f"[gpu] gather gemm case {case}", flush=True)
    rng = np.random.default_rng(1200 + case)
    srcs = [synth.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32)) for s in shapes]
    a = oracle.run_chain(srcs, ops)
    M, K = a.shape
    w = synth.f32_to_bf16_bits((rng.standard_normal((K, N)) * 0.05).astype(np.float32))
    a_map = B.amap_compose(shapes, 2, ops)
    d_srcs, d_w = [dev.to_device(s) for s in srcs], dev.to_device(w)
    out = torch.empty((M, N), dtype=torch.int16, device="cuda")
    B.amap_gemm_gather([t.data_ptr() for t in d_srcs], a_map, d_w.data_ptr(), None, N, None, out.data_ptr(), 0)
    torch.cuda.synchronize()
    _check(dev.to_host(out), a, w)
    # transposed weight and mapped store on top
    w_map = B.amap_compose([(N, K)], 2, [("transpose", (1, 0))])
    out_map = B.amap_compose([(M, N)], 2, [("slice", 0, M - 1, -1, -1)])
    d_wt = dev.to_device(np.ascontiguousarray(w.T))
    out2 = dev.empty_dst(out_map)
    B.amap_gemm_gather([t.data_ptr() for t in d_srcs], a_map, d_wt.data_ptr(), w_map, 0, out_map, out2.data_ptr(), 0)
    torch.cuda.synchronize()
    assert np.array_equal(dev.to_host(out2)[::-1], dev.to_host(out))


def test_gather_one_source_twice_and_error_paths(dev):
    import torch
    rng = np.random.default_rng(77)
    x = synth.f32_to_bf16_bits(rng.standard_normal((256, 64)).astype(np.float32))
    y = synth.f32_to_bf16_bits(rng.standard_normal((256, 64)).astype(np.float32))
    sx, sy = B.amap_source(0, (256, 64), 2), B.amap_source(1, (256, 64), 2)
    a_map = B.amap_concat([sx, sy, sx], 1)                      # [X | Y | X]: source 0 feeds two ranges of k
    w = synth.f32_to_bf16_bits((rng.standard_normal((192, 128)) * 0.05).astype(np.float32))
    d_x, d_y, d_w = dev.to_device(x), dev.to_device(y), dev.to_device(w)
    out = torch.empty((256, 128), dtype=torch.int16, device="cuda")
    B.amap_gemm_gather([d_x.data_ptr(), d_y.data_ptr()], a_map, d_w.data_ptr(), None, 128, None, out.data_ptr(), 0)
    torch.cuda.synchronize()
    _check(dev.to_host(out), np.concatenate([x, y, x], axis=1), w)

    def refused(shapes, ops, status, ptrs=None):
        m = B.amap_compose(shapes, 2, ops)
        with pytest.raises(B.AmapError) as e:
            B.amap_gemm_gather(ptrs or [d_x.data_ptr()] * len(shapes), m, d_w.data_ptr(), None, 128, None, out.data_ptr(), 0)
        assert e.value.status == status, (e.value.status, status)

    refused([(256, 32), (256, 96)], [("concat", 1)], B.AMAP_E_UNSUPPORTED)                  # range ends inside a k-step
    refused([(128, 64), (128, 64)], [("concat", 0)], B.AMAP_E_UNSUPPORTED)                  # concat along m
    refused([(256, 64), (256, 64)], [("concat", 1)], B.AMAP_E_INVALID, [d_x.data_ptr(), 0])  # a source pointer missing
    refused([(256, 64)] * 9, [("concat", 1)], B.AMAP_E_UNSUPPORTED)                         # more than 8 ranges
    # one source along k, the other along m
    mixed = B.amap_concat([B.amap_source(0, (256, 64), 2), B.amap_transpose(B.amap_source(1, (64, 256), 2), (1, 0))], 1)
    with pytest.raises(B.AmapError) as e:
        B.amap_gemm_gather([d_x.data_ptr(), d_y.data_ptr()], mixed, d_w.data_ptr(), None, 128, None, out.data_ptr(), 0)
    assert e.value.status == B.AMAP_E_UNSUPPORTED
    # the single-source entry point refuses a gathered A
    two = B.amap_compose([(256, 64), (256, 64)], 2, [("concat", 1)])
    with pytest.raises(B.AmapError) as e:
        B.amap_gemm_fused(d_x.data_ptr(), two, d_w.data_ptr(), 128, out.data_ptr(), 0)
    assert e.value.status == B.AMAP_E_UNSUPPORTED
    torch.cuda.synchronize()


# ---- 256 x 256 tiles, operands loaded straight into LDS (a kernel of its own)

T256_CASES = [
    # (A source shape, A chain -> [M,K]), N, chain on the product or None
    (((512, 128), []), 256, None),                                                                 # two k-steps, 2 x 1 tiles
    (((256, 192), []), 256, None),                                                                 # odd number of k-steps, one tile
    (((2, 4, 256, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (512, 256))]), 512, None),        # head merge: 64-element runs
    (((1024, 128), []), 1024, None),                                                               # 16 tiles
    (((2, 1024, 2, 64), [("transpose", (0, 2, 1, 3)), ("slice", 2, 256, 768, 1), ("transpose", (0, 2, 1, 3)),
                         ("reshape", (1024, 128))]), 256, None),                                   # base offset, rows 128 elements apart
    (((512, 128), []), 768, [("reshape", (2, 256, 3, 4, 64)), ("transpose", (2, 0, 3, 1, 4))]),    # QKV head split on the store side
    (((2, 2, 256, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (512, 128))]), 256,
     [("reshape", (2, 256, 4, 64)), ("transpose", (2, 0, 1, 3))]),                                 # both sides mapped
    # two k-steps and more tiles than workgroups (272 tiles): once both k-steps of its first tile are fetched, a
    # workgroup's load cursor must stand on its NEXT tile (it once stayed at k = K: weight rows past the end of W
    # were fetched, and the second tile of a workgroup was computed on the wrong stage)
    (((4352, 128), []), 4096, None),
    (((2, 2, 512, 64), [("transpose", (1, 2, 0, 3)), ("reshape", (1024, 128))]), 512, None),       # K = 128 over two digits of k
    (((4352, 192), []), 4096, [("reshape", (4352, 64, 64)), ("transpose", (1, 0, 2))]),            # three k-steps, two tiles per workgroup, mapped store
]


@pytest.mark.parametrize("case", range(len(T256_CASES)))
def test_tile256_kernel_vs_oracle_and_general_kernel(dev, case, monkeypatch, capfd):
    import torch
    (shape, a_ops), N, c_ops = T256_CASES[case]
    print(f"[gpu] tile256 gemm case {case} {shape} N={N}", flush=True)
    rng = np.random.default_rng(700 + case)
    src = synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    a_map = B.amap_compose([shape], 2, a_ops)
    M, K = B.dst_shape(a_map)
    w = synth.f32_to_bf16_bits((rng.standard_normal((K, N)) * 0.05).astype(np.float32))
    out_map = B.amap_compose([(M, N)], 2, c_ops) if c_ops else None
    d_src, d_w = dev.to_device(src), dev.to_device(w)

    def run():
        out = dev.gemm_fused(d_src, a_map, d_w, out_map=out_map) if out_map else dev.gemm_fused(d_src, a_map, d_w)
        torch.cuda.synchronize()
        return dev.to_host(out)

    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    got = run()
    assert "256 x 256 tiles" in capfd.readouterr().err           # the kernel under test is the one that ran
    monkeypatch.setenv("AMAP_GEMM_TILE256", "0")
    general = run()
    assert "256 x 128 tiles" in capfd.readouterr().err
    monkeypatch.delenv("AMAP_GEMM_TILE256")
    monkeypatch.delenv("AMAP_PLAN_TRACE")
    a_bits = oracle.run_chain([src], a_ops) if a_ops else src
    want = oracle.gemm_bf16(a_bits, w)
    if c_ops:
        want = oracle.run_chain([want], c_ops)
    assert got.shape == want.shape
    g, r = synth.bf16_bits_to_f32(got).astype(np.float64), synth.bf16_bits_to_f32(want).astype(np.float64)
    assert np.abs(g - r).max() <= TOL * np.abs(r).max()
    ulp = np.maximum(np.abs(r), 2.0 ** -126) * 2.0 ** -7
    assert np.mean(np.abs(g - r) <= ulp) > 0.999
    # both kernels add the same products in the same order (k ascending, 16 at a time in the same MFMA)
    assert np.array_equal(got, general)


def test_tile256_identity_weight_is_exact(dev, monkeypatch, capfd):
    """W = shifted identity on the 256 x 256 kernel: C reproduces the mapped A bit for bit, so a wrong
    lane -> address permutation of the LDS loads or of the transposing reads cannot hide in rounding."""
    shape, ops = (2, 2, 256, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (512, 128))]
    src = synth.f32_to_bf16_bits(np.random.default_rng(31).standard_normal(shape).astype(np.float32))
    cols = (np.arange(128) * 5 + 3) % 256
    wf = np.zeros((128, 256), dtype=np.float32)
    wf[np.arange(128), cols] = 1.0
    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    got = _gemm(dev, src, shape, ops, synth.f32_to_bf16_bits(wf))
    assert "256 x 256 tiles" in capfd.readouterr().err
    a = oracle.run_chain([src], ops)
    nz = (a & 0x7FFF) != 0
    assert np.array_equal(got[:, cols][nz], a[nz])
    rest = np.ones(256, dtype=bool)
    rest[cols] = False
    assert not (got[:, rest] & 0x7FFF).any()


T256_WT_CASES = [
    # (A source shape, A chain -> [M,K]), (W source shape, W chain -> [K,N]), chain on the product or None
    (((512, 128), []), ((256, 128), [("transpose", (1, 0))]), None),                                # a weight kept as [N,K]
    (((2, 4, 256, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (512, 256))]), ((512, 256), [("transpose", (1, 0))]), None),
    (((512, 256), []), ((768, 320), [("slice", 1, 64, 320, 1), ("transpose", (1, 0))]),
     [("reshape", (512, 12, 64)), ("transpose", (1, 0, 2))]),                                       # rows 320 apart, base offset, mapped store
    (((4352, 128), []), ((4096, 128), [("transpose", (1, 0))]), None),                              # two k-steps, two tiles per workgroup
    (((512, 192), []), ((2, 256, 192), [("transpose", (2, 0, 1)), ("reshape", (192, 512))]), None),  # n over two digits
]


@pytest.mark.parametrize("case", range(len(T256_WT_CASES)))
def test_tile256_kernel_with_the_weight_kept_transposed(dev, case, monkeypatch, capfd):
    """W with its runs along k (nn.Linear's [out_features, in_features]) on the 256 x 256 kernel: its stage is laid out
    like A's.  Against the oracle and, bit for bit, against the general kernel."""
    import torch
    (shape, a_ops), (w_shape, w_ops), c_ops = T256_WT_CASES[case]
    print(f"[gpu] tile256 gemm, W along k, case {case} {shape} {w_shape}", flush=True)
    rng = np.random.default_rng(900 + case)
    src = synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    w_src = synth.f32_to_bf16_bits((rng.standard_normal(w_shape) * 0.05).astype(np.float32))
    a_map, w_map = B.amap_compose([shape], 2, a_ops), B.amap_compose([w_shape], 2, w_ops)
    (M, K), (K2, N) = B.dst_shape(a_map), B.dst_shape(w_map)
    assert K == K2
    out_map = B.amap_compose([(M, N)], 2, c_ops) if c_ops else None
    d_src, d_w = dev.to_device(src), dev.to_device(w_src)

    def run():
        out = torch.empty(B.dst_shape(out_map) if out_map else (M, N), dtype=torch.int16, device="cuda")
        B.amap_gemm_mapped(d_src.data_ptr(), a_map, d_w.data_ptr(), w_map, out_map, out.data_ptr(), 0)
        torch.cuda.synchronize()
        return dev.to_host(out)

    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    got = run()
    assert "256 x 256 tiles (W runs along k)" in capfd.readouterr().err
    monkeypatch.setenv("AMAP_GEMM_TILE256", "0")
    general = run()
    assert "256 x 128 tiles" in capfd.readouterr().err
    monkeypatch.delenv("AMAP_GEMM_TILE256")
    monkeypatch.delenv("AMAP_PLAN_TRACE")
    a_bits = oracle.run_chain([src], a_ops) if a_ops else src
    w_bits = oracle.run_chain([w_src], w_ops)
    oracle.set_threads(8)
    try:
        want = oracle.gemm_bf16(a_bits, w_bits)
    finally:
        oracle.set_threads(1)
    if c_ops:
        want = oracle.run_chain([want], c_ops)
    assert got.shape == want.shape
    g, r = synth.bf16_bits_to_f32(got).astype(np.float64), synth.bf16_bits_to_f32(want).astype(np.float64)
    assert np.abs(g - r).max() <= TOL * np.abs(r).max()
    ulp = np.maximum(np.abs(r), 2.0 ** -126) * 2.0 ** -7
    assert np.mean(np.abs(g - r) <= ulp) > 0.999
    assert np.array_equal(got, general)


def test_tile256_transposed_identity_weight_is_exact(dev, monkeypatch, capfd):
    """W^T = shifted identity, kept as [N,K]: C reproduces A bit for bit (a wrong chunk or row in W's stage shows)."""
    import torch
    shape = (512, 128)
    src = synth.f32_to_bf16_bits(np.random.default_rng(33).standard_normal(shape).astype(np.float32))
    cols = (np.arange(128) * 5 + 3) % 256
    wt = np.zeros((256, 128), dtype=np.float32)
    wt[cols, np.arange(128)] = 1.0
    a_map, w_map = B.amap_compose([shape], 2, []), B.amap_compose([(256, 128)], 2, [("transpose", (1, 0))])
    out = torch.empty((512, 256), dtype=torch.int16, device="cuda")
    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    d_src, d_wt = dev.to_device(src), dev.to_device(synth.f32_to_bf16_bits(wt))    # (kept alive until the product has run)
    B.amap_gemm_mapped(d_src.data_ptr(), a_map, d_wt.data_ptr(), w_map, None, out.data_ptr(), 0)
    torch.cuda.synchronize()
    assert "256 x 256 tiles (W runs along k)" in capfd.readouterr().err
    got = dev.to_host(out)
    nz = (src & 0x7FFF) != 0
    assert np.array_equal(got[:, cols][nz], src[nz])
    rest = np.ones(256, dtype=bool)
    rest[cols] = False
    assert not (got[:, rest] & 0x7FFF).any()


T256_EDGE_CASES = [
    # M, K, N, weight kept as [N,K]?, chain on the product or None: partial last tiles of 256 in M and / or N
    (200, 128, 136, False, None),
    (300, 192, 264, False, None),
    (1000, 256, 1000, False, None),
    (8, 128, 8, False, None),
    (1000, 256, 1000, True, None),
    (257, 128, 520, True, None),
    (520, 256, 200, False, [("reshape", (520, 25, 8)), ("transpose", (1, 0, 2))]),
    (4352 + 40, 128, 4096 + 8, False, None),                  # partial tiles, two k-steps, two tiles per workgroup
]


@pytest.mark.parametrize("case", range(len(T256_EDGE_CASES)))
def test_tile256_kernel_with_partial_last_tiles(dev, case, monkeypatch, capfd):
    """M and N that are no multiples of 256 on the 256 x 256 kernel (lanes past the last row / column load the last
    existing one, stores are masked): against the oracle and, bit for bit, against the general kernel."""
    import torch
    M, K, N, w_t, c_ops = T256_EDGE_CASES[case]
    print(f"[gpu] tile256 gemm, partial tiles, case {case}: {M} x {K} x {N}", flush=True)
    rng = np.random.default_rng(1100 + case)
    src = synth.f32_to_bf16_bits(rng.standard_normal((M + 3, K + 64)).astype(np.float32))
    a_ops = [("slice", 0, 3, M + 3, 1), ("slice", 1, 64, K + 64, 1)]          # base offset, rows longer than K
    w = synth.f32_to_bf16_bits((rng.standard_normal((K, N)) * 0.05).astype(np.float32))
    a_map = B.amap_compose([(M + 3, K + 64)], 2, a_ops)
    w_map = B.amap_compose([(N, K)], 2, [("transpose", (1, 0))]) if w_t else None
    out_map = B.amap_compose([(M, N)], 2, c_ops) if c_ops else None
    d_src = dev.to_device(src)
    d_w = dev.to_device(np.ascontiguousarray(w.T) if w_t else w)

    def run():
        out = torch.full(B.dst_shape(out_map) if out_map else (M, N), 0x5A5A, dtype=torch.int16, device="cuda")
        B.amap_gemm_gather([d_src.data_ptr()], a_map, d_w.data_ptr(), w_map, N, out_map, out.data_ptr(), 0)
        torch.cuda.synchronize()
        return dev.to_host(out)

    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    got = run()
    err = capfd.readouterr().err
    assert "256 x 256 tiles" in err and "(partial last tiles)" in err
    monkeypatch.setenv("AMAP_GEMM_TILE256", "0")
    general = run()
    assert "256 x 128 tiles" in capfd.readouterr().err
    monkeypatch.delenv("AMAP_GEMM_TILE256")
    monkeypatch.delenv("AMAP_PLAN_TRACE")
    oracle.set_threads(8)
    try:
        want = oracle.gemm_bf16(oracle.run_chain([src], a_ops), w)
    finally:
        oracle.set_threads(1)
    if c_ops:
        want = oracle.run_chain([want], c_ops)
    assert got.shape == want.shape
    g, r = synth.bf16_bits_to_f32(got).astype(np.float64), synth.bf16_bits_to_f32(want).astype(np.float64)
    assert np.abs(g - r).max() <= TOL * np.abs(r).max()
    ulp = np.maximum(np.abs(r), 2.0 ** -126) * 2.0 ** -7
    assert np.mean(np.abs(g - r) <= ulp) > 0.999
    assert np.array_equal(got, general)


def _random_product(rng):
    """A random product the 256 x 256 kernel takes: (A source shape, chain), N, weight kept [N,K]?, chain on the product."""
    k = 64 * int(rng.integers(2, 6))
    form = int(rng.integers(3))
    if form == 0:                                            # plain rows, any M
        m = 8 * int(rng.integers(1, 100))
        shape, ops = (m, k), []
    elif form == 1:                                          # rows longer than K, behind an offset
        m = 8 * int(rng.integers(1, 100))
        shape, ops = (m + 5, k + 64), [("slice", 0, 5, m + 5, 1), ("slice", 1, 64, k + 64, 1)]
    else:                                                    # head merge: blocks of 256 rows, k over two digits
        b, h = int(rng.integers(1, 3)), int(rng.integers(2, 4))
        m, k = b * 256, h * 64
        shape, ops = (b, h, 256, 64), [("transpose", (0, 2, 1, 3)), ("reshape", (m, k))]
    n = 8 * int(rng.integers(1, 100))
    c_ops = [("reshape", (m, n // 8, 8)), ("transpose", (1, 0, 2))] if rng.random() < 0.4 else None
    return (shape, ops), n, bool(rng.random() < 0.5), c_ops


@pytest.mark.parametrize("seed", range(12))
def test_random_products_on_the_tile256_kernel(dev, seed, monkeypatch, capfd):
    """Random shapes (partial tiles, offsets, a mapped store, the weight either way round): the kernel's addressing is
    replayed on the host first, then the product is compared with the oracle."""
    import torch
    rng = np.random.default_rng(4200 + seed)
    (shape, a_ops), N, w_t, c_ops = _random_product(rng)
    print(f"[gpu] random tile256 product, seed {seed}: {shape} {a_ops} N={N} w_t={w_t} store={c_ops}", flush=True)
    a_map = B.amap_compose([shape], 2, a_ops)
    M, K = B.dst_shape(a_map)
    w_map = B.amap_compose([(N, K)], 2, [("transpose", (1, 0))]) if w_t else None
    out_map = B.amap_compose([(M, N)], 2, c_ops) if c_ops else None
    assert B.amap_gemm_selfcheck(a_map, N, out_map, 256, w_map) == 0
    assert B.amap_gemm_selfcheck(a_map, N, out_map, 3, w_map) == 0
    src = synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    w = synth.f32_to_bf16_bits((rng.standard_normal((K, N)) * 0.05).astype(np.float32))
    d_src = dev.to_device(src)
    d_w = dev.to_device(np.ascontiguousarray(w.T) if w_t else w)
    out = torch.full(B.dst_shape(out_map) if out_map else (M, N), 0x5A5A, dtype=torch.int16, device="cuda")
    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    B.amap_gemm_gather([d_src.data_ptr()], a_map, d_w.data_ptr(), w_map, N, out_map, out.data_ptr(), 0)
    torch.cuda.synchronize()
    assert "256 x 256 tiles" in capfd.readouterr().err
    monkeypatch.delenv("AMAP_PLAN_TRACE")
    got = dev.to_host(out)
    want = oracle.gemm_bf16(oracle.run_chain([src], a_ops) if a_ops else src, w)
    if c_ops:
        want = oracle.run_chain([want], c_ops)
    assert got.shape == want.shape
    g, r = synth.bf16_bits_to_f32(got).astype(np.float64), synth.bf16_bits_to_f32(want).astype(np.float64)
    assert np.abs(g - r).max() <= TOL * np.abs(r).max()
    ulp = np.maximum(np.abs(r), 2.0 ** -126) * 2.0 ** -7
    assert np.mean(np.abs(g - r) <= ulp) > 0.999


# ---- padding in front of the product: the pad operator's load composed into the operand load (Section 2.1, eq. 4)

PAD_CASES = [
    # A source shape, chain -> [M,K] (with fill pieces), N
    ((200, 120), [("pad", (3, 8), (5, 16), 0)], 128),                                               # rows and columns padded: [208,144]
    ((2, 6, 6, 32), [("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0), ("reshape", (128, 32))], 72),           # padded image, then flattened: rows inside and outside alternate
    ((64, 4, 24), [("pad", (0, 0, 0), (0, 0, 8), 0), ("reshape", (64, 128))], 64),                   # padding inside k: 24 of every 32
    ((100, 64), [("pad", (28, 0), (128, 0), 0x3FC0)], 136),                                          # pad constant 1.5, several row tiles
    ((3, 40, 64), [("transpose", (1, 0, 2)), ("pad", (4, 0, 0), (4, 0, 8), 0), ("reshape", (48, 216))], 40),  # mapped source under the padding
]


@pytest.mark.parametrize("case", range(len(PAD_CASES)))
def test_padded_a_operand_vs_oracle(dev, case):
    shape, ops, N = PAD_CASES[case]
    print(f"[gpu] padded gemm case {case} {shape} {ops}", flush=True)
    rng = np.random.default_rng(900 + case)
    src = synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    a = oracle.run_chain([src], ops)                      # pad materialised by the oracle
    K = a.shape[1]
    wt = synth.f32_to_bf16_bits((rng.standard_normal((K, N)) * 0.05).astype(np.float32))
    m = B.amap_compose([shape], 2, ops)
    assert B.amap_describe(m).n_fill_pieces >= 1
    got = _gemm(dev, src, shape, ops, wt)
    _check(got, a, wt)


def test_padded_a_identity_weight_is_exact(dev):
    """W = identity: the product reproduces the padded A bit for bit, pad constant included."""
    shape, ops = (2, 6, 6, 32), [("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0x4049), ("reshape", (128, 32))]
    src = synth.f32_to_bf16_bits(np.random.default_rng(5).standard_normal(shape).astype(np.float32))
    got = _gemm(dev, src, shape, ops, synth.f32_to_bf16_bits(np.eye(32, dtype=np.float32)))
    a = oracle.run_chain([src], ops)
    nz = (a & 0x7FFF) != 0
    assert np.array_equal(got[nz], a[nz]) and not (got[~nz] & 0x7FFF).any()
