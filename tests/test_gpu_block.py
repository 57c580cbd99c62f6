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


def test_config5_block_linears_match_the_oracle(oracle):
    b = blk.DecoderBlock(moss, torch, "moss", **blk.sizes_7b())
    taps, grads = {}, {}
    inner = b.fn

    class Tap:
        """records the BF16 input and output of every linear on the way through"""
        @staticmethod
        def apply(x, layer):
            y = inner.apply(x, layer)
            name = next(n for n, l in b.lin.items() if l is layer)
            taps[name] = (x.detach(), y.detach())
            y.register_hook(lambda g, name=name: grads.__setitem__(name, g.detach().clone()))
            return y
    b.fn = Tap
    x = b.x.detach().requires_grad_(True)
    out = b.forward(x)
    # forward operands of the two linears fed by non-linear layers: attention output -> o, SwiGLU -> down
    rng = np.random.default_rng(55)
    for name in ("o", "down"):
        layer = b.lin[name]
        xin, y = taps[name]
        print(f"[config5] forward {name}: X {tuple(xin.shape)}", flush=True)
        q, e, s = oracle.quant_act_2level(bf16_bits(xin), 0, 0)
        assert scalar(layer.qx["s"]) == s
        assert np.array_equal(u8(layer.qx["e_row"]), e) and np.array_equal(u8(layer.qx["q_row"]), q)
        check_sampled(oracle, f"config5 {name} Y", y, (q, e, s), (u8(layer.wq), None, scalar(layer.s_w)), rng)
    # backward: the gradient that reaches the down projection is the upstream gradient itself; the one
    # that reaches gate has passed through the SwiGLU backward
    out.backward(b.upstream)
    torch.cuda.synchronize()
    for name in ("down", "gate"):
        layer = b.lin[name]
        print(f"[config5] backward {name}: dW {tuple(layer.dw.shape)}", flush=True)
        # dW = dY^T X from the column-grouped codes the library kept for this layer
        qdy = (u8(layer.qdy["q_col"]), u8(layer.qdy["e_col"]), scalar(layer.qdy["s"]))
        qx = (u8(layer.qx["q_col"]), u8(layer.qx["e_col"]), scalar(layer.qx["s"]))
        gq, ge, gs = oracle.quant_act_2level(bf16_bits(grads[name]), 1, 0)
        assert gs == qdy[2] and np.array_equal(qdy[0], gq) and np.array_equal(qdy[1], ge)
        xin = taps[name][0]
        qc, ec, sc = oracle.quant_act_2level(bf16_bits(xin), 1, 0)
        assert sc == qx[2] and np.array_equal(qx[0], qc) and np.array_equal(qx[1], ec)
        check_sampled(oracle, f"config5 {name} dW", layer.dw, qdy, qx, rng)
    assert torch.isfinite(x.grad.float()).all()
