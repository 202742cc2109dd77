"""GPU parity beyond 32-bit offsets: tensors of more than 2^31 elements (pieces run in 64-bit
windows), and the same code path forced on small tensors by lowering the span limit."""
import os

import numpy as np
import pytest

from oracle import oracle
from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth
from tests import chains
from tests.test_plan_replay import ALIGNED

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    from paper_2002_12798_amd import device
    device.require_gpu()
    return device


def _run(dev, m, srcs, want):
    import torch
    dst = dev.empty_dst(m, fill=0x5A5A if want.dtype.itemsize == 2 else 0x5A5A5A5A)
    dev.execute(m, [dev.to_device(s) for s in srcs], dst)
    torch.cuda.synchronize()
    got = dev.to_host(dst)
    assert got.shape == want.shape
    assert np.array_equal(got, want)


def test_small_tensors_through_the_window_path(dev, monkeypatch):
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "10")
    for case, (shape, es, ops) in enumerate(ALIGNED):
        print(f"[gpu] windowed aligned case {case}", flush=True)
        srcs = [synth.random_bits(shape, es, 40 + case)]
        _run(dev, B.amap_compose([shape], es, ops), srcs, oracle.run_chain(srcs, ops))
    for seed in range(60):
        print(f"[gpu] windowed random chain {seed}", flush=True)
        src_shapes, ops = chains.random_chain(seed, extended=seed % 2 == 0, max_volume=60000)
        es = 2 if seed % 3 else 4
        srcs = [synth.random_bits(s, es, 3000 + seed + i) for i, s in enumerate(src_shapes)]
        m = B.amap_compose(src_shapes, es, ops)
        if B.amap_describe(m).strided:
            _run(dev, m, srcs, oracle.run_chain(srcs, ops))
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "14")
    w = synth.workload("cfg1", n=1)
    srcs = w.sources()
    _run(dev, B.amap_compose(w.src_shapes, w.elem_size, w.ops), srcs, oracle.run_chain(srcs, w.ops))


def _host_gib():
    try:
        return os.sysconf("SC_PHYS_PAGES") * os.sysconf("SC_PAGE_SIZE") / 2 ** 30
    except (ValueError, OSError):
        return 0.0


_BIG = {}


def _big_input(shape):
    """x[r, c] = a 16-bit mix of r and c (wrapping uint16 arithmetic; built once, in slabs of rows):
    neighbouring rows and columns differ, so a shifted or transposed index shows."""
    if shape not in _BIG:
        x = np.empty(shape, dtype=np.uint16)
        col = (np.arange(shape[1], dtype=np.uint32) * 25173).astype(np.uint16)[None, :]
        for r in range(0, shape[0], 4000):
            rows = np.arange(r, min(r + 4000, shape[0]), dtype=np.uint32)
            rmix = ((rows * 40503) ^ (rows >> 5)).astype(np.uint16)[:, None]
            np.add(rmix, col, out=x[r:r + 4000])
        _BIG[shape] = x
    return _BIG[shape]


@pytest.mark.parametrize("ops", [
    [("slice", 1, 0, 32992, 1), ("slice", 0, 65999, -1, -1)],     # row copy, rows walked backwards
    [("transpose", (1, 0))],                                      # tile transpose
])
def test_more_than_2_31_elements(dev, ops):
    import torch
    shape = (66000, 33000)                                         # 2.178e9 two-byte elements, 4.36 GB
    free, _ = torch.cuda.mem_get_info()
    if free < 12 * 2 ** 30 or _host_gib() < 40:
        pytest.skip("needs 12 GiB of device memory and 40 GiB of host memory")
    print(f"[gpu] large tensor {shape} {ops}", flush=True)
    x = _big_input(shape)
    m = B.amap_compose([shape], 2, ops)
    info = B.amap_describe(m)
    assert info.strided and info.write_bytes > 2 ** 32
    oracle.set_threads(16)
    try:
        want = oracle.run_chain([x], ops)
    finally:
        oracle.set_threads(1)
    d_src = dev.to_device(x)
    dst = dev.execute(m, [d_src])
    torch.cuda.synchronize()
    got = dev.to_host(dst)
    del d_src, dst
    torch.cuda.empty_cache()
    assert got.shape == want.shape
    # compare in slabs to keep the temporaries small
    for r in range(0, want.shape[0], 4096):
        assert np.array_equal(got[r:r + 4096], want[r:r + 4096]), r


def test_gemm_operand_of_more_than_2_31_elements(dev, monkeypatch, capfd):
    """A[1048832, 2048] (2.15e9 elements, 4.3 GB) x W[2048, 256] on the 256 x 256-tile kernel, whose tile and k-step
    bases are 64-bit: whole 512-row blocks at the start, in the middle and at the end (the last one holds element
    2^31 of A) against the oracle's product of those rows, and sampled outputs recomputed one by one."""
    import torch
    M, K, N = 4097 * 256, 2048, 256
    free, _ = torch.cuda.mem_get_info()
    if free < 16 * 2 ** 30:
        pytest.skip("needs 16 GiB of device memory")
    print(f"[gpu] wide gemm operand {M} x {K}", flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2024)
    a = torch.empty((M, K), dtype=torch.int16, device="cuda")
    for r in range(0, M, 65536):
        rows = min(65536, M - r)
        a[r:r + rows] = torch.randn((rows, K), generator=gen, device="cuda").bfloat16().view(torch.int16)
    w = synth.f32_to_bf16_bits((np.random.default_rng(9).standard_normal((K, N)) * 0.02).astype(np.float32))
    d_w = dev.to_device(w)
    out = torch.empty((M, N), dtype=torch.int16, device="cuda")
    a_map = B.amap_compose([(M, K)], 2, [])
    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    B.amap_gemm_fused(a.data_ptr(), a_map, d_w.data_ptr(), N, out.data_ptr(), 0)
    torch.cuda.synchronize()
    assert "256 x 256 tiles" in capfd.readouterr().err
    monkeypatch.delenv("AMAP_PLAN_TRACE")
    oracle.set_threads(8)
    try:
        for r0 in (0, 524288, M - 512):
            a_rows = a[r0:r0 + 512].cpu().numpy().view(np.uint16)
            got = out[r0:r0 + 512].cpu().numpy().view(np.uint16)
            want = oracle.gemm_bf16(a_rows, w)
            g, r = synth.bf16_bits_to_f32(got).astype(np.float64), synth.bf16_bits_to_f32(want).astype(np.float64)
            assert np.abs(g - r).max() <= 1e-2 * np.abs(r).max(), r0
            ulp = np.maximum(np.abs(r), 2.0 ** -126) * 2.0 ** -7
            assert np.mean(np.abs(g - r) <= ulp) > 0.999, r0
    finally:
        oracle.set_threads(1)
    rng = np.random.default_rng(3)
    for m, n in zip(rng.integers(0, M, 48), rng.integers(0, N, 48)):
        row = a[int(m):int(m) + 1].cpu().numpy().view(np.uint16)
        ref = oracle.gemm_bf16_point(row, w, 0, int(n))
        gv = float(synth.bf16_bits_to_f32(out[int(m), int(n)].cpu().numpy().view(np.uint16).reshape(1))[0])
        assert abs(gv - ref) <= 2.0 ** -7 * abs(ref) + 1e-6, (m, n)
    del a, out
    torch.cuda.empty_cache()
    # what only the 256 x 256-tile kernel reaches is refused elsewhere, not run with wrapped offsets
    x = torch.zeros(1 << 20, dtype=torch.int16, device="cuda")
    wide_general = B.amap_compose([(M, K + 8)], 2, [])          # K is no multiple of 64: the general kernel's
    with pytest.raises(B.AmapError) as e:
        B.amap_gemm_fused(x.data_ptr(), wide_general, d_w.data_ptr(), N, x.data_ptr() + 2 * (1 << 19), 0)
    assert e.value.status in (B.AMAP_E_UNSUPPORTED, B.AMAP_E_ALIAS)
