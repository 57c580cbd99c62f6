"""GPU parity of moss_add_rmsnorm_bf16 and moss_rmsnorm_bf16_backward (the BF16 producers in front of the
quantizers of the QKV, gate / up projections and of the O projection's dY) against the CPU oracle's FP64 RMSNorm.

Tolerance: the kernels evaluate in FP32 (sums over a row of a few thousand terms, one correctly rounded
reciprocal square root) and round once to BF16, so an output is the correctly rounded BF16 value of the exact
result except when the exact result lies closer to a rounding boundary than the FP32 evaluation error.
Forward: |gpu - exact| <= (1/2 + 2^-9) BF16 ulp everywhere.  Backward: the result is a difference of terms that
may cancel, so the FP32 error scales with the terms, not with the result: |gpu - exact| <= 1/2 BF16 ulp of the
result + 2^-18 (|d_res| + (|g| + |n mean(g n)|) / rms).  The residual sum h = x + delta is an FP32 sum rounded to
BF16: within (1/2 + 2^-15) BF16 ulp of the exact sum.  y is compared with the oracle's norm of the h the GPU
stored; every maximum word must be exactly the largest magnitude bit pattern written."""
import numpy as np
import pytest
import torch

import moss_inputs as mi
import paper_2511_05811_amd as moss
from gpu_util import bf16_to_gpu, scalar, u8

pytestmark = pytest.mark.gpu
EPS = 1e-5


def bits_of(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def vals(b):
    return mi.bf16_bits_to_f32(b).astype(np.float64)


def ulp_bf16(v):
    return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -126))) - 7)


def make(rows, cols, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, cols)) * 1.5
    x[:, rng.choice(cols, max(1, cols // 64), replace=False)] *= 20.0            # a few large channels
    delta = rng.standard_normal((rows, cols)) * 0.3
    gamma = 1.0 + 0.2 * rng.standard_normal(cols)
    dy = rng.standard_normal((rows, cols)) * 1e-3
    dres = rng.standard_normal((rows, cols)) * 1e-3
    f = lambda a: mi.f32_to_bf16_bits(a.astype(np.float32))
    return f(x), f(delta), f(gamma), f(dy), f(dres)


@pytest.mark.parametrize("shape", [(1, 8), (5, 40), (33, 2048), (64, 4096), (300, 4096 + 64), (16, 11008), (8, 16384)])
def test_rmsnorm_forward_and_backward(oracle, shape):
    rows, cols = shape
    print(f"[rmsnorm parity] {shape}", flush=True)
    xb, db, gb, dyb, drb = make(rows, cols, rows * 13 + cols)
    x, d, g, dy, dr = (bf16_to_gpu(a) for a in (xb, db, gb, dyb, drb))
    # plain norm of x
    _, y, ymax = moss.add_rmsnorm_bf16(x, g, EPS)
    # residual add + norm
    h, y2, y2max = moss.add_rmsnorm_bf16(x, g, EPS, delta=d)
    torch.cuda.synchronize()
    yb, hb, y2b = bits_of(y), bits_of(h), bits_of(y2)
    exact = oracle.rmsnorm(xb, gb, EPS)
    assert (np.abs(vals(yb) - exact) <= (0.5 + 2.0 ** -9) * ulp_bf16(exact)).all()
    assert int(ymax.item()) == int((yb & 0x7FFF).max())
    hsum = vals(xb) + vals(db)
    assert (np.abs(vals(hb) - hsum) <= (0.5 + 2.0 ** -15) * ulp_bf16(hsum)).all()
    exact2 = oracle.rmsnorm(hb, gb, EPS)                       # the norm of what was stored
    assert (np.abs(vals(y2b) - exact2) <= (0.5 + 2.0 ** -9) * ulp_bf16(exact2)).all()
    assert int(y2max.item()) == int((y2b & 0x7FFF).max())
    # backward, with and without the residual-path gradient
    for res_bits, res in ((None, None), (drb, dr)):
        dh, dhmax = moss.rmsnorm_bf16_backward(h, g, dy, EPS, d_res=res)
        torch.cuda.synchronize()
        dhb = bits_of(dh)
        ex = oracle.rmsnorm_backward(hb, gb, dyb, res_bits, EPS)
        hv = vals(hb)
        rms = np.sqrt((hv ** 2).mean(axis=1, keepdims=True) + EPS)
        gterm = np.abs(vals(dyb) * vals(gb))
        n = hv / rms
        mean_gn = (vals(dyb) * vals(gb) * n).mean(axis=1, keepdims=True)
        scale = (gterm + np.abs(n * mean_gn)) / rms + (0.0 if res_bits is None else np.abs(vals(res_bits)))
        assert (np.abs(vals(dhb) - ex) <= 0.5 * ulp_bf16(ex) + 2.0 ** -18 * scale).all(), res_bits is None
        assert int(dhmax.item()) == int((dhb & 0x7FFF).max())


def test_rmsnorm_on_a_strided_view_and_word_is_overwritten(oracle):
    rows, cols, ld = 40, 96, 128
    xb, db, gb, _, _ = make(rows, ld, 5)
    x_full, d_full = bf16_to_gpu(xb), bf16_to_gpu(db)
    g = bf16_to_gpu(gb[:cols].copy())
    y_full = torch.full((rows, ld), 3.0, dtype=torch.bfloat16, device=x_full.device)
    h_full = torch.full((rows, ld), 5.0, dtype=torch.bfloat16, device=x_full.device)
    word = torch.full((1,), 12345, dtype=torch.int32, device=x_full.device)
    h, y, ymax = moss.add_rmsnorm_bf16(x_full[:, :cols], g, EPS, delta=d_full[:, :cols], h=h_full[:, :cols], y=y_full[:, :cols],
                                       absmax_bits=word)
    torch.cuda.synchronize()
    assert (y_full[:, cols:] == 3.0).all() and (h_full[:, cols:] == 5.0).all()        # padding columns untouched
    hb = bits_of(h)
    exact = oracle.rmsnorm(hb, gb[:cols], EPS)
    assert (np.abs(vals(bits_of(y)) - exact) <= (0.5 + 2.0 ** -9) * ulp_bf16(exact)).all()
    assert int(ymax.item()) == int((bits_of(y) & 0x7FFF).max())
    z = torch.zeros((8, 64), dtype=torch.bfloat16, device=x_full.device)
    _, yz, zmax = moss.add_rmsnorm_bf16(z, bf16_to_gpu(gb[:64].copy()), EPS, absmax_bits=word)
    torch.cuda.synchronize()
    assert int(zmax.item()) == 0 and (bits_of(yz) & 0x7FFF).max() == 0


def test_rmsnorm_feeds_the_quantizer_in_one_pass(oracle):
    """Residual add + RMSNorm writes y and its maximum; the quantizer reads y once.  The codes are those the oracle's
    quantizer gives for the y the GPU wrote (both groupings)."""
    rows, cols = 2048, 4096
    xb, db, gb, _, _ = make(rows, cols, 77)
    x, d, g = bf16_to_gpu(xb), bf16_to_gpu(db), bf16_to_gpu(gb)
    _, y, ymax = moss.add_rmsnorm_bf16(x, g, EPS, delta=d)
    got = moss.quant_act_2level_given_max(y, ymax, moss.MOSS_Q_ROW | moss.MOSS_Q_COL)
    torch.cuda.synchronize()
    yb = bits_of(y)
    qr, er, s = oracle.quant_act_2level(yb, 0, 0)
    qc, ec, _ = oracle.quant_act_2level(yb, 1, 0)
    assert scalar(got["s"]) == s
    assert np.array_equal(u8(got["q_row"]), qr) and np.array_equal(u8(got["e_row"]), er)
    assert np.array_equal(u8(got["q_col"]), qc) and np.array_equal(u8(got["e_col"]), ec)
