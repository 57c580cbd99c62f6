"""Pins of the oracle's RMSNorm (the BF16 producer in front of the QKV and gate / up projections' quantizers;
the paper keeps the non-linear layers in BF16, Sec. 4.1): the library routine in FP64, autograd, closed forms,
invariances, central differences."""
import numpy as np
import torch

import moss_inputs as mi


def bits(x):
    return mi.f32_to_bf16_bits(np.asarray(x, np.float32))


def vals(b):
    return mi.bf16_bits_to_f32(b).astype(np.float64)


def test_forward_against_the_library_rms_norm(oracle):
    rng = np.random.default_rng(1)
    h = bits(rng.standard_normal((37, 96)) * 3.0); g = bits(1.0 + 0.1 * rng.standard_normal(96))
    for eps in (1e-5, 0.0, 0.5):
        y = oracle.rmsnorm(h, g, eps)
        ref = torch.nn.functional.rms_norm(torch.from_numpy(vals(h)), (96,), torch.from_numpy(vals(g)), eps).numpy()
        assert np.allclose(y, ref, rtol=1e-13, atol=1e-300), eps


def test_forward_closed_forms(oracle):
    # a constant row c: y = gamma c / sqrt(c^2 + eps)
    g = bits([1.0, 2.0, -0.5, 4.0])
    y = oracle.rmsnorm(bits([[3.0] * 4]), g, 0.25)
    assert np.allclose(y[0], vals(g) * 3.0 / np.sqrt(9.25), rtol=1e-15)
    # a single nonzero entry v among n: mean square v^2 / n, so y = gamma sign(v) sqrt(n) without eps
    y = oracle.rmsnorm(bits([[0.0, -7.0, 0.0, 0.0]]), g, 0.0)
    assert np.allclose(y[0], [0.0, -2.0 * 2.0, 0.0, 0.0], rtol=1e-15)
    # scale invariance without eps (exact for powers of two), and the unit mean square of y / gamma
    rng = np.random.default_rng(2)
    h = bits(rng.standard_normal((5, 64)))
    ones = bits(np.ones(64))
    y1 = oracle.rmsnorm(h, ones, 0.0)
    y2 = oracle.rmsnorm(bits(vals(h) * 8.0), ones, 0.0)
    assert np.array_equal(y1, y2)
    assert np.allclose((y1 ** 2).mean(axis=1), 1.0, rtol=1e-14)
    # rows do not mix
    assert np.array_equal(oracle.rmsnorm(h[2:3], ones, 1e-5), oracle.rmsnorm(h, ones, 1e-5)[2:3])


def test_backward_against_autograd_and_differences(oracle):
    rng = np.random.default_rng(3)
    rows, cols, eps = 9, 48, 1e-5
    h = bits(rng.standard_normal((rows, cols)) * 2.0); g = bits(1.0 + 0.2 * rng.standard_normal(cols))
    dy = bits(rng.standard_normal((rows, cols))); dr = bits(rng.standard_normal((rows, cols)) * 0.3)
    th = torch.from_numpy(vals(h)).requires_grad_(True)
    y = torch.nn.functional.rms_norm(th, (cols,), torch.from_numpy(vals(g)), eps)
    (y * torch.from_numpy(vals(dy))).sum().backward()
    d_norm = oracle.rmsnorm_backward(h, g, dy, None, eps)
    assert np.allclose(d_norm, th.grad.numpy(), rtol=1e-11, atol=1e-14)
    # the residual-path gradient is simply added
    assert np.allclose(oracle.rmsnorm_backward(h, g, dy, dr, eps), d_norm + vals(dr), rtol=1e-14, atol=1e-16)
    # central differences of the forward formula written out here
    hv, gv, dv = vals(h), vals(g), vals(dy)
    f = lambda a: a / np.sqrt((a ** 2).mean(axis=1, keepdims=True) + eps) * gv
    num = np.zeros_like(hv)
    step = 1e-6
    for c in range(cols):
        e = np.zeros_like(hv); e[:, c] = step
        num[:, c] = ((f(hv + e) - f(hv - e)) * dv).sum(axis=1) / (2 * step)
    assert np.allclose(d_norm, num, rtol=1e-6, atol=1e-8)
    # without eps the norm is scale invariant, so the gradient is orthogonal to h
    d0 = oracle.rmsnorm_backward(h, g, dy, None, 0.0)
    assert np.abs((d0 * hv).sum(axis=1)).max() < 1e-12
