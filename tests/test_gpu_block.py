"""Config 5 (one LLaMA-7B-shaped decoder block, batch 2 x seq 4096): the operands that reach the
library inside a real forward + backward pass -- attention outputs, SwiGLU products, the
gradients that flow back through them -- quantize bit-exactly against the oracle, and the
GEMM outputs they produce match it on sampled entries (Sec. 3.1; tolerance as for config 3)."""
import numpy as np
import pytest
import torch

import paper_2511_05811_amd as moss
from gpu_util import scalar, u8
from paper_2511_05811_amd import block as blk
from test_gpu_gemm import check_sampled

pytestmark = pytest.mark.gpu


def bf16_bits(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


SAMPLE = dict(n_rows=4, n_cols=4, n_rand=8192)     # per GEMM; config 3 carries the large sample on the same shapes


def test_config5_block_linears_match_the_oracle(oracle):
    """All five linears of the block, forward and backward: the BF16 tensors that reach the library (normalised
    hidden states, attention output, SwiGLU product, and the gradients flowing back) quantize bit-exactly in both
    groupings, and Y, dX and dW match the oracle's sums over those codes on sampled outputs."""
    b = blk.DecoderBlock(moss, torch, "moss", **blk.sizes_7b())
    xin, yout, dy, dx = {}, {}, {}, {}
    inner = b.fn

    class Tap:
        """records, per linear, the BF16 input, the output, and the gradients of both"""
        @staticmethod
        def apply(x, layer):
            name = next(n for n, l in b.lin.items() if l is layer)
            xi = x.view(x.shape)                    # a node of its own: its gradient is this linear's dX alone
            if xi.requires_grad:
                xi.register_hook(lambda g, name=name: dx.__setitem__(name, g.detach().clone()))
            y = inner.apply(xi, layer)
            xin[name], yout[name] = x.detach(), y.detach()
            y.register_hook(lambda g, name=name: dy.__setitem__(name, g.detach().clone()))
            return y
    b.fn = Tap
    x = b.x.detach().requires_grad_(True)
    out = b.forward(x)
    out.backward(b.upstream)
    torch.cuda.synchronize()
    rng = np.random.default_rng(55)
    for name, layer in b.lin.items():
        print(f"[config5] {name}: X {tuple(xin[name].shape)} dY {tuple(dy[name].shape)}", flush=True)
        st, owq, owq_t = oracle.weight_init(layer.w.cpu().numpy(), want_transpose=True)     # (no optimizer step has run)
        assert scalar(layer.s_w) == st.s_cur and np.array_equal(u8(layer.wq), owq) and np.array_equal(u8(layer.wq_t), owq_t)
        w, wt = (owq, None, st.s_cur), (owq_t, None, st.s_cur)
        got = {}
        for key, t, buf in (("x", xin[name], layer.qx), ("dy", dy[name], layer.qdy)):
            bits = bf16_bits(t)
            qr, er, s = oracle.quant_act_2level(bits, 0, 0)
            qc, ec, _ = oracle.quant_act_2level(bits, 1, 0)
            assert scalar(buf["s"]) == s, (name, key)
            for k2, want in (("q_row", qr), ("e_row", er), ("q_col", qc), ("e_col", ec)):
                assert np.array_equal(u8(buf[k2]), want), (name, key, k2)
            got[key] = ((qr, er, s), (qc, ec, s))
        check_sampled(oracle, f"config5 {name} Y", yout[name], got["x"][0], w, rng, **SAMPLE)
        check_sampled(oracle, f"config5 {name} dX", dx[name], got["dy"][0], wt, rng, **SAMPLE)
        check_sampled(oracle, f"config5 {name} dW", layer.dw, got["dy"][1], got["x"][1], rng, **SAMPLE)
    assert torch.isfinite(x.grad.float()).all()
