"""Pins for the oracle GEMM and its bf16 rounding."""
import numpy as np
import torch

from oracle import oracle
from paper_2002_12798_amd import synth


def test_bf16_rounding_hand_cases():
    # 1.0 = 0x3F80; one ulp at 1.0 is 2^-7
    assert oracle.double_to_bf16(1.0) == 0x3F80
    assert oracle.double_to_bf16(-2.0) == 0xC000
    assert oracle.double_to_bf16(1.0 + 2.0 ** -8) == 0x3F80          # tie -> even (down)
    assert oracle.double_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82      # tie -> even (up)
    assert oracle.double_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81  # just above the tie
    assert oracle.double_to_bf16(2.0 - 2.0 ** -9) == 0x4000           # carries into next binade
    assert oracle.double_to_bf16(0.0) == 0 and oracle.double_to_bf16(-0.0) == 0x8000
    assert oracle.double_to_bf16(2.0 ** -133) == 0x0001               # smallest subnormal
    assert oracle.double_to_bf16(2.0 ** -134) == 0x0000               # tie to even (zero)
    assert oracle.double_to_bf16(2.0 ** -126) == 0x0080               # smallest normal
    assert oracle.double_to_bf16(1e40) == 0x7F80
    assert oracle.bf16_to_double(0x3FC0) == 1.5


def test_bf16_rounding_vs_torch():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * s
                        for s in (1e-3, 1.0, 37.0, 1e20, 1e-39)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.double_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
    # and it agrees with the input generator's own rounding
    assert np.array_equal(synth.f32_to_bf16_bits(x), want)


def test_gemm_identity_weight_is_exact():
    a = synth.f32_to_bf16_bits(np.random.default_rng(2).standard_normal((37, 24)).astype(np.float32))
    w = np.zeros((24, 40), dtype=np.float32)
    w[np.arange(24), np.arange(24) + 5] = 1.0
    c = oracle.gemm_bf16(a, synth.f32_to_bf16_bits(w))
    assert np.array_equal(c[:, 5:29], a)
    assert not c[:, :5].any() and not c[:, 29:].any()


def test_gemm_small_integers_exact():
    rng = np.random.default_rng(3)
    a = rng.integers(-4, 5, (19, 33)).astype(np.float32)
    w = rng.integers(-4, 5, (33, 21)).astype(np.float32)
    c = oracle.gemm_bf16(synth.f32_to_bf16_bits(a), synth.f32_to_bf16_bits(w))
    want = (a.astype(np.int64) @ w.astype(np.int64)).astype(np.float32)
    # |sum| <= 33*16 = 528 needs 10 bits: not all exact in bf16, so round the exact integer
    assert np.array_equal(c, synth.f32_to_bf16_bits(want))


def test_gemm_is_not_transposed_and_uses_every_k():
    # A = e_m e_k^T picks one entry of W: C[m,:] = W[k,:]
    w = synth.f32_to_bf16_bits(np.random.default_rng(4).standard_normal((7, 9)).astype(np.float32))
    for m, k in [(0, 0), (2, 6), (4, 3)]:
        a = np.zeros((5, 7), dtype=np.float32)
        a[m, k] = 1.0
        c = oracle.gemm_bf16(synth.f32_to_bf16_bits(a), w)
        assert np.array_equal(c[m], w[k])
        assert not np.delete(c, m, axis=0).any()


def test_gemm_vs_float64_matmul():
    rng = np.random.default_rng(5)
    a = synth.f32_to_bf16_bits(rng.standard_normal((64, 300)).astype(np.float32))
    w = synth.f32_to_bf16_bits((rng.standard_normal((300, 48)) * 0.02).astype(np.float32))
    c = synth.bf16_bits_to_f32(oracle.gemm_bf16(a, w)).astype(np.float64)
    ref = (torch.from_numpy(synth.bf16_bits_to_f32(a)).double()
           @ torch.from_numpy(synth.bf16_bits_to_f32(w)).double()).numpy()
    # the only error left is the final bf16 rounding: half an ulp, 2^-9 relative
    assert np.all(np.abs(c - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-30)
    for m, n in [(0, 0), (63, 47), (10, 20)]:
        assert abs(oracle.gemm_bf16_point(a, w, m, n) - ref[m, n]) <= 1e-12 * max(1.0, abs(ref[m, n]))
