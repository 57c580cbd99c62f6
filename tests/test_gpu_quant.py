"""GPU parity of moss_quant_act_2level against the CPU oracle: bit-exact codes,
exponent bytes and global scale (paper Sec. 3.1, Eq. 2-3)."""
import numpy as np
import pytest
import torch

import moss_inputs as mi
import paper_2511_05811_amd as moss
from gpu_util import bf16_to_gpu, scalar, u8

pytestmark = pytest.mark.gpu

ROW, COL, CEIL = moss.MOSS_Q_ROW, moss.MOSS_Q_COL, moss.MOSS_EXP_CEIL


def check_against_oracle(oracle, xb, mode_flag, tag, x_dev=None):
    print(f"[quant parity] {tag} shape={xb.shape} mode={'ceil' if mode_flag else 'nearest'}", flush=True)
    x = bf16_to_gpu(xb) if x_dev is None else x_dev
    mode = 1 if mode_flag else 0
    qr, er, sr = oracle.quant_act_2level(xb, 0, mode)
    got = moss.quant_act_2level(x, ROW | mode_flag)
    torch.cuda.synchronize()
    assert scalar(got["s"]) == sr, tag
    assert np.array_equal(u8(got["e_row"]), er), tag
    assert np.array_equal(u8(got["q_row"]), qr), tag
    if xb.shape[0] % 32 == 0:
        qc, ec, sc = oracle.quant_act_2level(xb, 1, mode)
        got = moss.quant_act_2level(x, COL | mode_flag)
        torch.cuda.synchronize()
        assert scalar(got["s"]) == sc == sr, tag
        assert np.array_equal(u8(got["e_col"]), ec), tag
        assert np.array_equal(u8(got["q_col"]), qc), tag
        both = moss.quant_act_2level(x, ROW | COL | mode_flag)
        torch.cuda.synchronize()
        assert scalar(both["s"]) == sr
        assert np.array_equal(u8(both["q_row"]), qr) and np.array_equal(u8(both["e_row"]), er)
        assert np.array_equal(u8(both["q_col"]), qc) and np.array_equal(u8(both["e_col"]), ec)


def test_every_bf16_value_through_the_converter(oracle):
    # all finite BF16 bit patterns up to 2^20 in magnitude (including subnormals and both
    # zeros), laid out so that groups mix magnitudes; larger patterns are replaced by zero
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ex = (bits >> 7) & 0xFF
    bits[ex > 127 + 20] = 0
    rng = np.random.default_rng(3)
    xb = rng.permutation(bits).reshape(64, 1024)
    for flag in (0, CEIL):
        check_against_oracle(oracle, xb, flag, "all-bf16 shuffled")
    # sorted layout: neighbouring values share a group, so every code of the E4M3 grid and
    # many exact rounding ties are hit
    check_against_oracle(oracle, np.sort(bits).reshape(64, 1024), 0, "all-bf16 sorted")


def test_config1_activation(oracle):
    xb, _ = mi.config1()
    for flag in (0, CEIL):
        check_against_oracle(oracle, xb, flag, "config1 X")


@pytest.mark.parametrize("name", ["zeros", "zero_groups", "one_outlier", "signed_zeros", "tiny", "tiny_zero_groups",
                                  "subnormal", "tiny_groups_under_large_max", "big", "sqrt2_boundary", "wide_range"])
def test_adversarial_tensors(oracle, name):
    xb = mi.adversarial_activations(64, 128)[name]
    for flag in (0, CEIL):
        check_against_oracle(oracle, xb, flag, name)


@pytest.mark.parametrize("shape", [(32, 32), (1, 32), (7, 96), (96, 160), (33, 4096), (1056, 1184), (2080, 32)])
def test_ragged_shapes(oracle, shape):
    xb = mi.heavy_tailed_activation(shape[0], shape[1], seed=20 + shape[0])
    check_against_oracle(oracle, xb, 0, f"ragged {shape}")


# Tensors with at least two 128 x 128 tiles per compute unit take the one-launch kernel (a bounded
# grid that meets once for the global maximum and keeps its first tiles in registers).
@pytest.mark.parametrize("shape,flag", [((4128, 2080), 0),      # ragged edges, every tile kept
                                        ((4133, 2080), CEIL),   # rows not a multiple of 8: row grouping only
                                        ((1056, 8352), 0),      # (fewer tiles: the two-launch path)
                                        ((4128, 8352), 0),      # a few workgroups fetch a fifth tile again
                                        ((8224, 7200), CEIL)])  # several tiles per workgroup beyond the kept ones
def test_many_tiles_with_ragged_edges(oracle, shape, flag):
    xb = mi.heavy_tailed_activation(shape[0], shape[1], seed=40 + shape[1])
    check_against_oracle(oracle, xb, flag, f"many tiles {shape}")


def with_adversarial_blocks(rows, cols, seed, scale=1.0):
    """N(0, scale) with the adversarial 64 x 128 blocks of moss_inputs pasted into different tiles: whole tiles
    that the fast form covers, tiles with zero groups, and tiles that need the general form (subnormal group
    maxima, groups so tiny under the tensor maximum that 2^-e / s leaves the finite range)."""
    rng = np.random.default_rng(seed)
    x = mi.f32_to_bf16_bits((rng.standard_normal((rows, cols)) * scale).astype(np.float32))
    blocks = mi.adversarial_activations(64, 128)
    names = ["zeros", "zero_groups", "signed_zeros", "tiny", "tiny_zero_groups", "subnormal", "tiny_groups_under_large_max",
             "sqrt2_boundary", "wide_range"]
    places = [(r, c) for r in range(0, rows - 63, 192) for c in range(0, cols - 127, 384)]
    for i, (r, c) in enumerate(places):
        blk = blocks[names[i % len(names)]].copy()
        if names[i % len(names)] in ("wide_range", "sqrt2_boundary", "tiny_groups_under_large_max"):
            blk = mi.f32_to_bf16_bits(np.minimum(np.abs(mi.bf16_bits_to_f32(blk)), 2.0) * np.sign(mi.bf16_bits_to_f32(blk)))
        x[r:r + 64, c:c + 128] = blk
    return x


@pytest.mark.parametrize("flag", [0, CEIL])
def test_adversarial_blocks_inside_full_tiles_two_launch_path(oracle, flag):
    check_against_oracle(oracle, with_adversarial_blocks(384, 768, 51), flag, "adversarial blocks, tile kernel")
    check_against_oracle(oracle, with_adversarial_blocks(384, 800, 52, scale=300.0), flag, "adversarial blocks, large maximum")


def test_tensor_with_a_subnormal_maximum_in_full_tiles(oracle):
    rng = np.random.default_rng(53)
    xb = mi.f32_to_bf16_bits((rng.standard_normal((256, 384)) * 2.0 ** -129).astype(np.float32))
    for flag in (0, CEIL):
        check_against_oracle(oracle, xb, flag, "subnormal maximum")


@pytest.mark.parametrize("flag", [0, CEIL])
def test_adversarial_blocks_on_the_one_launch_path(oracle, flag):
    # 32 x 24 = 768 tiles: the one-launch kernel; a fifth of its tiles needs the general form
    check_against_oracle(oracle, with_adversarial_blocks(4096, 3072, 54), flag, "adversarial blocks, one-launch kernel")


def test_one_launch_path_when_the_meeting_times_out(oracle):
    # poll limit 0: every workgroup that finds the maximum not yet published computes it by itself
    xb = mi.heavy_tailed_activation(4128, 2080, seed=47)
    moss.quant_set_poll_limit(0)
    try:
        check_against_oracle(oracle, xb, 0, "one-launch, no polling")
    finally:
        moss.quant_set_poll_limit(32768)


def test_one_launch_path_reuses_a_dirty_workspace(oracle):
    xb = mi.heavy_tailed_activation(4128, 2080, seed=48)
    x = bf16_to_gpu(xb)
    ws = torch.full((1 << 15,), 0xFF, dtype=torch.uint8, device=x.device)
    qr, er, s = oracle.quant_act_2level(xb, 0, 0)
    for _ in range(2):
        got = moss.quant_act_2level(x, ROW | COL, workspace=ws)
        torch.cuda.synchronize()
        assert scalar(got["s"]) == s
        assert np.array_equal(u8(got["q_row"]), qr) and np.array_equal(u8(got["e_row"]), er)


def test_kept_workspace_needs_no_clearing_launch(oracle):
    """MOSS_WS_KEPT: a zero-filled workspace that only these calls write to.  The one-launch kernel leaves its
    meeting words at zero, on the meeting path and on the timed-out path, so calls in a row (different shapes, the
    last ones with polling switched off) give the oracle's outputs and the words read zero after every call."""
    dev = torch.device("cuda:0")
    ws = torch.zeros(moss.load().moss_quant_workspace_bytes(8192, 4096, 3), dtype=torch.uint8, device=dev)
    calls = [((4096, 4096), 32768), ((2048, 4096), 32768), ((4000, 4128), 32768), ((8192, 4096), 32768),
             ((4128, 2080), 0), ((2048, 4096), 0), ((4096, 4096), 32768)]
    try:
        for i, ((rows, cols), polls) in enumerate(calls):
            print(f"[kept workspace] call {i}: {rows}x{cols} polls={polls}", flush=True)
            xb = mi.heavy_tailed_activation(rows, cols, seed=70 + i)
            moss.quant_set_poll_limit(polls)
            got = moss.quant_act_2level(bf16_to_gpu(xb), ROW | COL | moss.MOSS_WS_KEPT, workspace=ws)
            torch.cuda.synchronize()
            assert int(ws[8192:].to(torch.int32).sum()) == 0, (i, "meeting words not back at zero")
            qr, er, s = oracle.quant_act_2level(xb, 0, 0)
            qc, ec, _ = oracle.quant_act_2level(xb, 1, 0)
            assert scalar(got["s"]) == s, i
            assert np.array_equal(u8(got["q_row"]), qr) and np.array_equal(u8(got["e_row"]), er), i
            assert np.array_equal(u8(got["q_col"]), qc) and np.array_equal(u8(got["e_col"]), ec), i
    finally:
        moss.quant_set_poll_limit(32768)


def test_row_stride_larger_than_cols(oracle):
    xb_full = mi.heavy_tailed_activation(96, 256, seed=31)
    x_full = bf16_to_gpu(xb_full)
    x_view = x_full[:, 64:224]                     # ld = 256, cols = 160, 16-byte aligned start
    xb = np.ascontiguousarray(xb_full[:, 64:224])
    check_against_oracle(oracle, xb, 0, "strided view", x_dev=x_view)


@pytest.mark.parametrize("flag", [0, CEIL])
def test_config2_full_size(oracle, flag):
    xb = mi.config2()
    assert xb.shape == (8192, 4096)
    check_against_oracle(oracle, xb, flag, "config2 full")


def test_one_launch_path_on_a_strided_view(oracle):
    xb_full = mi.heavy_tailed_activation(4128, 2304, seed=49)
    x_full = bf16_to_gpu(xb_full)
    x_view = x_full[:, 128:2208]                   # ld = 2304, cols = 2080
    xb = np.ascontiguousarray(xb_full[:, 128:2208])
    check_against_oracle(oracle, xb, 0, "one-launch strided view", x_dev=x_view)


def test_outputs_are_written_exactly_once_into_caller_buffers(oracle):
    # poison the output buffers: every byte must be overwritten, nothing beyond them touched
    xb = mi.heavy_tailed_activation(96, 160, seed=33)
    x = bf16_to_gpu(xb)
    d = x.device
    pad = 64
    bufs = {k: torch.full((n + 2 * pad,), 0xAB, dtype=torch.uint8, device=d)
            for k, n in dict(q_row=96 * 160, e_row=96 * 5, q_col=96 * 160, e_col=160 * 3).items()}
    out = dict(q_row=bufs["q_row"][pad:-pad].view(96, 160), e_row=bufs["e_row"][pad:-pad].view(96, 5),
               q_col=bufs["q_col"][pad:-pad].view(160, 96), e_col=bufs["e_col"][pad:-pad].view(160, 3))
    got = moss.quant_act_2level(x, ROW | COL, out=out)
    torch.cuda.synchronize()
    qr, er, s = oracle.quant_act_2level(xb, 0, 0)
    qc, ec, _ = oracle.quant_act_2level(xb, 1, 0)
    assert np.array_equal(u8(got["q_row"]), qr) and np.array_equal(u8(got["e_row"]), er)
    assert np.array_equal(u8(got["q_col"]), qc) and np.array_equal(u8(got["e_col"]), ec)
    for b in bufs.values():
        assert (b[:pad] == 0xAB).all() and (b[-pad:] == 0xAB).all()
