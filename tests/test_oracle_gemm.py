"""Pins for the oracle's block-scaled FP8 GEMM (Sec. 3.1, Fig. 3b): exact rational
dot products on tiny shapes, reduction to a library matmul when every level-2
scale is 1, and agreement of the whole quantize -> GEMM -> dequantize chain with
the unquantized product to within the quantization noise."""
from fractions import Fraction

import numpy as np
import torch

import moss_inputs as mi

TABLE = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def finite_codes(rng, shape):
    c = rng.integers(0, 256, size=shape, dtype=np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x38
    return c


def test_tiny_shapes_against_exact_rational_arithmetic(oracle):
    rng = np.random.default_rng(0)
    for (M, N, K) in [(1, 1, 32), (3, 2, 64), (2, 5, 96)]:
        a, b = finite_codes(rng, (M, K)), finite_codes(rng, (N, K))
        ae = rng.integers(110, 128, size=(M, K // 32), dtype=np.uint8)
        be = rng.integers(120, 131, size=(N, K // 32), dtype=np.uint8)
        a_s, b_s = np.float32(0.37), np.float32(1.0 / 3.0)
        got = oracle.gemm(a, ae, a_s, b, be, b_s)
        for m in range(M):
            for n in range(N):
                acc = Fraction(0)
                for k in range(K):
                    # codes as integers times 2^-9, exponents summed: no floating point
                    ia = Fraction(float(TABLE[a[m, k]])) * 512
                    ib = Fraction(float(TABLE[b[n, k]])) * 512
                    assert ia.denominator == 1 and ib.denominator == 1
                    sh = int(ae[m, k // 32]) - 127 + int(be[n, k // 32]) - 127 - 18
                    acc += ia * ib * (Fraction(2) ** sh)
                exact = acc * Fraction(float(a_s)) * Fraction(float(b_s))
                assert abs(Fraction(float(got[m, n])) - exact) <= abs(exact) * Fraction(1, 10 ** 13) + Fraction(1, 10 ** 300)


def test_unit_exponents_reduce_to_library_matmul(oracle):
    rng = np.random.default_rng(1)
    M, N, K = 17, 9, 128
    a, b = finite_codes(rng, (M, K)), finite_codes(rng, (N, K))
    ref = (TABLE[a] @ TABLE[b].T) * float(np.float32(0.5)) * float(np.float32(0.125))
    for ae, be in [(None, None), (np.full((M, K // 32), 127, np.uint8), None),
                   (None, np.full((N, K // 32), 127, np.uint8))]:
        got = oracle.gemm(a, ae, 0.5, b, be, 0.125)
        assert np.allclose(got, ref, rtol=1e-13, atol=0)


def test_general_exponents_against_library_matmul_of_dequantized_operands(oracle):
    rng = np.random.default_rng(2)
    M, N, K = 8, 12, 160
    a, b = finite_codes(rng, (M, K)), finite_codes(rng, (N, K))
    ae = rng.integers(100, 128, size=(M, K // 32), dtype=np.uint8)
    be = rng.integers(100, 128, size=(N, K // 32), dtype=np.uint8)
    da = TABLE[a] * np.repeat(2.0 ** (ae.astype(np.int64) - 127), 32, axis=1)
    db = TABLE[b] * np.repeat(2.0 ** (be.astype(np.int64) - 127), 32, axis=1)
    got = oracle.gemm(a, ae, 2.0, b, be, 3.0)
    assert np.allclose(got, 6.0 * da @ db.T, rtol=1e-12, atol=1e-300)
    assert np.allclose(oracle.dequant(a, ae, 2.0), 2.0 * da, rtol=0, atol=0)
    assert np.allclose(oracle.row_norms(a, ae, 2.0), np.linalg.norm(2.0 * da, axis=1), rtol=1e-14)
    ms = np.array([0, 7, 3, 3]); ns = np.array([11, 0, 5, 5])
    assert np.array_equal(oracle.gemm_sampled(a, ae, 2.0, b, be, 3.0, ms, ns), got[ms, ns])


def test_quantized_linear_tracks_the_unquantized_product(oracle):
    # a transposed operand, a dropped exponent or a wrong global scale would wreck this
    xb, wb = mi.config1(seed=1)
    xb, wb = xb[:64, :256], wb[:48, :256]
    x = mi.bf16_bits_to_f32(xb).astype(np.float64)
    w = mi.bf16_bits_to_f32(wb).astype(np.float64)
    for mode in (0, 1):
        q, e, s = oracle.quant_act_2level(xb, 0, mode)
        st, wq, _ = oracle.weight_init(mi.bf16_bits_to_f32(wb))
        y = oracle.gemm(q, e, s, wq, None, st.s_cur)
        ref = x @ w.T
        snr = 10 * np.log10((ref ** 2).sum() / ((y - ref) ** 2).sum())
        assert snr > (25.0 if mode == 1 else 15.0)
    # backward operand plan: dW = dY^T X contracts over tokens, so both operands are
    # quantized with groups along the token axis and stored transposed
    _, _, dyb = mi.config3_linear(0, tokens=64, k=256, n=48)
    dy = mi.bf16_bits_to_f32(dyb).astype(np.float64)
    qa, ea, sa = oracle.quant_act_2level(dyb, 1, 1)      # [N x T]
    qb, eb, sb = oracle.quant_act_2level(xb, 1, 1)       # [K x T]
    dw = oracle.gemm(qa, ea, sa, qb, eb, sb)             # [N x K]
    ref = dy.T @ x
    snr = 10 * np.log10((ref ** 2).sum() / ((dw - ref) ** 2).sum())
    assert snr > 25.0
