"""Pins of the oracle's SwiGLU (the BF16 producer in front of the down projection's quantizer;
the paper keeps the non-linear layers in BF16, Sec. 4.1): library routines in FP64, closed forms,
the derivative against central differences."""
import numpy as np
import pytest
import torch

import moss_inputs as mi


def bits(x):
    return mi.f32_to_bf16_bits(np.asarray(x, np.float32))


def vals(b):
    return mi.bf16_bits_to_f32(b).astype(np.float64)


def test_forward_against_the_library_silu(oracle):
    rng = np.random.default_rng(1)
    g = bits(rng.standard_normal((64, 96)) * 4.0); u = bits(rng.standard_normal((64, 96)) * 3.0)
    h = oracle.swiglu(g, u)
    ref = (torch.nn.functional.silu(torch.from_numpy(vals(g))) * torch.from_numpy(vals(u))).numpy()
    assert np.allclose(h, ref, rtol=1e-14, atol=1e-300)


def test_forward_closed_forms(oracle):
    one = bits([1.0])
    assert oracle.swiglu(bits([0.0]), one)[0] == 0.0
    # silu(x) - silu(-x) = x, silu(x) + silu(-x) = x tanh(x / 2)
    x = np.array([0.125, 0.5, 1.0, 3.0, 7.5, 20.0])
    p = oracle.swiglu(bits(x), bits(np.ones_like(x))); n = oracle.swiglu(bits(-x), bits(np.ones_like(x)))
    assert np.allclose(p - n, x, rtol=1e-15)
    assert np.allclose(p + n, x * np.tanh(x / 2), rtol=1e-13)
    # far out: the identity and zero
    assert oracle.swiglu(bits([64.0]), one)[0] == pytest.approx(64.0, rel=1e-15)
    assert abs(oracle.swiglu(bits([-64.0]), one)[0]) < 1e-25
    # linear in the up projection, sign included
    assert oracle.swiglu(bits([2.0]), bits([-3.0]))[0] == pytest.approx(-3.0 * oracle.swiglu(bits([2.0]), one)[0], rel=1e-15)


def test_backward_against_autograd_and_differences(oracle):
    rng = np.random.default_rng(2)
    g = bits(rng.standard_normal(512) * 3.0); u = bits(rng.standard_normal(512) * 2.0); d = bits(rng.standard_normal(512))
    dg, du = oracle.swiglu_backward(g, u, d)
    tg = torch.from_numpy(vals(g)).requires_grad_(True); tu = torch.from_numpy(vals(u)).requires_grad_(True)
    (torch.nn.functional.silu(tg) * tu).backward(torch.from_numpy(vals(d)))
    assert np.allclose(dg, tg.grad.numpy(), rtol=1e-12, atol=1e-300)
    assert np.allclose(du, tu.grad.numpy(), rtol=1e-12, atol=1e-300)
    # central differences of the forward formula written out here
    f = lambda a, b: a / (1.0 + np.exp(-a)) * b
    gv, uv, dv, eps = vals(g), vals(u), vals(d), 1e-6
    assert np.allclose(dg, dv * (f(gv + eps, uv) - f(gv - eps, uv)) / (2 * eps), rtol=1e-6, atol=1e-8)
    assert np.allclose(du, dv * (f(gv, uv + eps) - f(gv, uv - eps)) / (2 * eps), rtol=1e-6, atol=1e-8)
    # special points: sig'(0) gives d_gate = dh u / 2, d_up = 0
    dg0, du0 = oracle.swiglu_backward(bits([0.0]), bits([3.0]), bits([2.0]))
    assert dg0[0] == 3.0 and du0[0] == 0.0
