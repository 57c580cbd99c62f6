"""The side tables of paper_2511_05811_amd.microbench run end to end on small shapes and
their outputs have the properties the paper states (Sec. 3.2: automatic scaling never
lets a cast overflow and costs no max-reduction pass)."""
import pytest
import torch

import paper_2511_05811_amd as moss
from paper_2511_05811_amd import microbench

pytestmark = pytest.mark.gpu


def test_scaling_table_small():
    res = microbench.scaling(moss, torch, small=True)
    row = res["sizes"][0]
    assert row["fused_step_auto_ms"] > 0 and row["step_with_max_reduction_ms"] > 0
    for s in res["interval_sweep"]:
        assert s["clipped_count"] == 0
        assert s["min_predicted_over_exact_scale"] >= 1.0   # the predicted scale never falls below the exact one


def test_gemm_table_small():
    res = microbench.gemm(moss, torch, small=True)
    assert res["rows"][0]["fp8_mx_ms"] > 0 and res["rows"][0]["bf16_hand_gemm_ms"] > 0


def test_producer_table_small():
    t = microbench.producer(moss, torch, small=True)["times"]
    assert t["swiglu_with_max_ms"] > 0 and t["quant_given_max_ms"] > 0 and t["chain_fused_ms"] > 0


def test_quant_table_small():
    rows = microbench.quant(moss, torch, small=True)["rows"]
    assert len(rows) == 3 and all(r["searching_ms"] > 0 and r["given_max_ms"] > 0 and r["device_copy_ms"] > 0 for r in rows)


def test_limits_table_small():
    res = microbench.limits(moss, torch, small=True)
    assert len(res["gemm_by_operand_content"]) == 3 and all(r["tflops"] > 0 for r in res["gemm_by_operand_content"])
    assert res["device_copy"][0]["gbs_read_plus_write"] > 0


def test_decoder_block_arms_agree_on_a_small_block():
    """The FP8 arm of the decoder-block step stays close to the BF16 arm (same seeds, same scaffolding):
    outputs, input gradients and weight gradients differ only by quantization noise."""
    from paper_2511_05811_amd import block as blk
    sz = blk.sizes_small()
    a = blk.DecoderBlock(moss, torch, "moss", **sz)
    b = blk.DecoderBlock(moss, torch, "bf16", **sz)
    for name in a.lin:      # same initial weights by construction (same generator seed and order)
        assert torch.allclose(a.lin[name].w, b.lin[name].master.data)
    oa, ga = a.train_step()
    ob, gb = b.train_step()
    torch.cuda.synchronize()

    def rel(x, y):
        x, y = x.detach().double(), y.detach().double()
        return float((x - y).norm() / y.norm())
    assert rel(oa, ob) < 0.02
    assert rel(ga, gb) < 0.03
    # dW sums only 64 token products of two FP8-quantized factors here (E4M3 keeps 3 mantissa bits and the
    # printed round-to-nearest exponent clips group maxima): about 15 % relative noise on this tiny block
    for name in a.lin:
        assert rel(a.lin[name].dw, b.lin[name].dw) < 0.25, name
    # the library's SwiGLU (which also hands the tensor maxima to the quantizers) against torch's silu and mul:
    # the same step up to BF16 rounding of the SwiGLU outputs
    # ... and its RMSNorm kernels against torch's rms_norm and add
    c = blk.DecoderBlock(moss, torch, "moss", swiglu="torch", norm="torch", **sz)
    oc, gc = c.train_step()
    torch.cuda.synchronize()
    assert rel(oa, oc) < 0.01 and rel(ga, gc) < 0.02
    # the maxima handed over were used: X of qkv, gate, up, down and dY of o, gate, up
    assert a.words is not None and a.words.used == 7 and c.words is None
    res = microbench.block(moss, torch, small=True)
    assert res["arms"]["moss"]["tokens_per_s"] > 0 and res["arms"]["bf16"]["tokens_per_s"] > 0
    assert res["arms"]["moss_torch_norm"]["tokens_per_s"] > 0 and res["arms"]["moss_torch_norm_torch_swiglu"]["tokens_per_s"] > 0
