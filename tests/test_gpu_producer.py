"""GPU parity of the producer side of the quantizer: moss_swiglu_bf16 (+ backward) against the CPU
oracle's FP64 SwiGLU, and moss_quant_act_2level_given_max (the quantizer of Sec. 3.1, Eq. 2-3 with
the tensor maximum handed in) bit for bit against the oracle.

SwiGLU tolerance: the kernel evaluates in FP32 with hardware exp2 / reciprocal approximations and
rounds once to BF16, so an output is the correctly rounded BF16 value of the exact result except when
the exact result lies closer to a rounding boundary than the FP32 evaluation error (a few times 2^-20
relative): then it is the BF16 neighbour.  The test asserts |gpu - exact| <= (1/2 + 2^-9) BF16 ulp for
every element and that at most 0.5 % of the elements differ from the correctly rounded value.  The
maximum word must be exactly the largest magnitude bit pattern the kernel wrote."""
import numpy as np
import pytest
import torch

import moss_inputs as mi
import paper_2511_05811_amd as moss
from gpu_util import bf16_to_gpu, scalar, u8

pytestmark = pytest.mark.gpu
ROW, COL, CEIL = moss.MOSS_Q_ROW, moss.MOSS_Q_COL, moss.MOSS_EXP_CEIL


def bits_of(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def check_rounded(got_bits, exact, tag):
    got = mi.bf16_bits_to_f32(got_bits).astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(exact), 2.0 ** -126))) - 7)      # BF16: 8 significant bits
    err = np.abs(got - exact)
    worst = float((err / ulp).max())
    want_bits = mi.f32_to_bf16_bits(exact.astype(np.float32))     # exact is far from FP32 resolution: good enough a stand-in
    off = float(np.mean(got_bits != want_bits))
    print(f"[swiglu parity] {tag}: max |err| = {worst:.4f} ulp, {off * 100:.4f} % not the nearest BF16", flush=True)
    assert worst <= 0.5 + 2.0 ** -9, tag
    assert off <= 5e-3, tag


def make_inputs(rows, cols, seed):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((rows, cols)) * 2.5
    g[rng.random((rows, cols)) < 0.01] *= 8.0                # a few far-out gates (sigmoid saturated either way)
    u = rng.standard_normal((rows, cols)) * 1.5
    d = rng.standard_normal((rows, cols)) * 1e-3
    return mi.f32_to_bf16_bits(g.astype(np.float32)), mi.f32_to_bf16_bits(u.astype(np.float32)), mi.f32_to_bf16_bits(d.astype(np.float32))


@pytest.mark.parametrize("shape", [(1, 8), (3, 40), (32, 64), (257, 1000), (1024, 2048 + 8)])
def test_swiglu_forward_and_backward(oracle, shape):
    rows, cols = shape
    gb, ub, db = make_inputs(rows, cols, rows * 31 + cols)
    g, u, d = bf16_to_gpu(gb), bf16_to_gpu(ub), bf16_to_gpu(db)
    h, hmax = moss.swiglu_bf16(g, u)
    dg, du, dgmax, dumax = moss.swiglu_bf16_backward(g, u, d)
    torch.cuda.synchronize()
    hb, dgb, dub = bits_of(h), bits_of(dg), bits_of(du)
    check_rounded(hb, oracle.swiglu(gb, ub), f"h {shape}")
    eg, eu = oracle.swiglu_backward(gb, ub, db)
    check_rounded(dgb, eg, f"d_gate {shape}")
    check_rounded(dub, eu, f"d_up {shape}")
    assert int(hmax.item()) == int((hb & 0x7FFF).max())
    assert int(dgmax.item()) == int((dgb & 0x7FFF).max())
    assert int(dumax.item()) == int((dub & 0x7FFF).max())


def test_swiglu_on_a_strided_view_and_zero_tensor(oracle):
    rows, cols, ld = 64, 96, 128
    gb, ub, _ = make_inputs(rows, ld, 7)
    g_full, u_full = bf16_to_gpu(gb), bf16_to_gpu(ub)
    g, u = g_full[:, :cols], u_full[:, :cols]
    h_full = torch.full((rows, ld), 3.0, dtype=torch.bfloat16, device=g.device)
    h, hmax = moss.swiglu_bf16(g, u, h=h_full[:, :cols])
    torch.cuda.synchronize()
    check_rounded(bits_of(h), oracle.swiglu(gb[:, :cols], ub[:, :cols]), "strided")
    assert (h_full[:, cols:] == 3.0).all()                   # the padding columns are not touched
    assert int(hmax.item()) == int((bits_of(h) & 0x7FFF).max())
    z = torch.zeros((32, 64), dtype=torch.bfloat16, device=g.device)
    hmax.fill_(12345)                                        # the word is written, not accumulated
    h, hmax = moss.swiglu_bf16(z, u_full[:32, :64].contiguous(), absmax_bits=hmax)
    torch.cuda.synchronize()
    assert int(hmax.item()) == 0 and (bits_of(h) & 0x7FFF).max() == 0


@pytest.mark.parametrize("flag", [0, CEIL])
@pytest.mark.parametrize("shape", [(32, 64), (96, 160), (1056, 2080), (4128, 3104)])
def test_quantizer_with_the_maximum_handed_in(oracle, shape, flag):
    rows, cols = shape
    mode = 1 if flag else 0
    xb = mi.heavy_tailed_activation(rows, cols, seed=rows + cols + mode)
    x = bf16_to_gpu(xb)
    true_bits = int((xb & 0x7FFF).max())
    for given in (true_bits, true_bits + 1, true_bits + 200):
        word = torch.tensor([given], dtype=torch.int32, device=x.device)
        qr, er, s = oracle.quant_act_2level_given_max(xb, given, 0, mode)
        qc, ec, _ = oracle.quant_act_2level_given_max(xb, given, 1, mode)
        for f in (ROW, COL, ROW | COL):
            got = moss.quant_act_2level_given_max(x, word, f | flag)
            torch.cuda.synchronize()
            assert scalar(got["s"]) == s, (shape, given, f)
            if f & ROW:
                assert np.array_equal(u8(got["q_row"]), qr) and np.array_equal(u8(got["e_row"]), er), (shape, given, f)
            if f & COL:
                assert np.array_equal(u8(got["q_col"]), qc) and np.array_equal(u8(got["e_col"]), ec), (shape, given, f)
    # with the true maximum: the searching entry point's outputs, bit for bit
    ref = moss.quant_act_2level(x, ROW | COL | flag)
    got = moss.quant_act_2level_given_max(x, torch.tensor([true_bits], dtype=torch.int32, device=x.device), ROW | COL | flag)
    torch.cuda.synchronize()
    for k in ("q_row", "e_row", "q_col", "e_col", "s"):
        assert torch.equal(ref[k], got[k]), k


def test_quantizer_with_the_maximum_handed_in_on_a_strided_view(oracle):
    rows, cols, ld = 1056, 2080, 2304
    full = mi.heavy_tailed_activation(rows, ld, seed=17)
    xb = np.ascontiguousarray(full[:, :cols])
    x = bf16_to_gpu(full)[:, :cols]
    given = int((xb & 0x7FFF).max())
    got = moss.quant_act_2level_given_max(x, torch.tensor([given], dtype=torch.int32, device=x.device), ROW | COL)
    torch.cuda.synchronize()
    qr, er, s = oracle.quant_act_2level(xb, 0, 0)
    qc, ec, _ = oracle.quant_act_2level(xb, 1, 0)
    assert scalar(got["s"]) == s
    assert np.array_equal(u8(got["q_row"]), qr) and np.array_equal(u8(got["e_row"]), er)
    assert np.array_equal(u8(got["q_col"]), qc) and np.array_equal(u8(got["e_col"]), ec)


def test_swiglu_feeds_the_quantizer_in_one_pass(oracle):
    """The chain the two entry points are for: SwiGLU writes h and its maximum, the quantizer reads h once.
    The codes are those the oracle's quantizer gives for the h the GPU wrote."""
    rows, cols = 2048, 2752
    gb, ub, _ = make_inputs(rows, cols, 99)
    g, u = bf16_to_gpu(gb), bf16_to_gpu(ub)
    h, hmax = moss.swiglu_bf16(g, u)
    got = moss.quant_act_2level_given_max(h, hmax, ROW | COL)
    torch.cuda.synchronize()
    hb = bits_of(h)
    qr, er, s = oracle.quant_act_2level(hb, 0, 0)
    qc, ec, _ = oracle.quant_act_2level(hb, 1, 0)
    assert scalar(got["s"]) == s
    assert np.array_equal(u8(got["q_row"]), qr) and np.array_equal(u8(got["e_row"]), er)
    assert np.array_equal(u8(got["q_col"]), qc) and np.array_equal(u8(got["e_col"]), ec)
