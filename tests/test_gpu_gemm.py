"""GPU parity of moss_gemm_fp8_mx (and of the whole quantize -> cast -> GEMM chain)
against the CPU oracle's dequantize-then-FP64 GEMM (paper Sec. 3.1, Fig. 3b).
Tolerance: |gpu - oracle| <= 1e-3 * |a_row|_2 * |b_row|_2 per output for FP32 outputs;
BF16 outputs get the same bound plus one rounding step of the BF16 output format."""
import numpy as np
import pytest
import torch

import moss_inputs as mi
import paper_2511_05811_amd as moss
from gpu_util import bf16_out_to_f64, bf16_to_gpu, to_gpu, u8

pytestmark = pytest.mark.gpu
REL = 1e-3


def finite_codes(rng, shape):
    c = rng.integers(0, 256, size=shape, dtype=np.uint8)
    c[(c & 0x7F) == 0x7F] = 0x38
    return c


def gpu_gemm(a_q, a_e, a_s, b_q, b_e, b_s, **kw):
    d = lambda x: None if x is None else to_gpu(x)
    sa = to_gpu(np.array([a_s], np.float32)); sb = to_gpu(np.array([b_s], np.float32))
    out = moss.gemm_fp8_mx(d(a_q), d(a_e), sa, d(b_q), d(b_e), sb, **kw)
    torch.cuda.synchronize()
    return out


def assert_close(got, ref, na, nb, bf16, tag):
    tol = REL * np.outer(na, nb) if ref.ndim == 2 else REL * na * nb
    err = np.abs(got - ref)
    worst = float((err / np.maximum(tol / REL, 1e-300)).max())
    print(f"[gemm parity] {tag}: max |err| / (|a||b|) = {worst:.3e}", flush=True)
    if bf16:
        # the bar applies to the FP32-accumulated result; storing it as BF16 adds one rounding of
        # the output format (at most 2^-8 |y|), which alone can exceed 1e-3 |a||b| when a and b
        # are nearly parallel
        assert (err <= tol + 2.0 ** -8 * np.abs(ref) + 1e-30).all(), tag
        assert (err <= 2.0 ** -8 * np.abs(ref) + 3e-4 * tol / REL + 1e-30).all(), tag
    else:
        assert (err <= tol + 1e-30).all(), tag
        # tighter than the bar, to notice regressions: the matrix instruction sums each run of
        # 16 products in a fixed-point window about 14 bits below the largest of them
        # (measured), so wide-range random codes reach about 1e-4 at K = 512, quantized data 1e-6
        assert (err <= 3e-4 * tol / REL + 1e-30).all(), tag


@pytest.mark.parametrize("shape", [(16, 16, 32), (1, 1, 32), (5, 3, 64), (128, 128, 128), (200, 136, 96),
                                   (257, 129, 416), (130, 260, 1024), (64, 512, 160),
                                   # >= 8 tiles of 256 x 256 with K % 128 == 0: the large-tile kernel
                                   (520, 776, 640), (1024, 2048, 512), (2049, 257, 1152), (512, 1024, 2176)])
@pytest.mark.parametrize("exps", ["both", "a_only", "none"])
def test_random_codes_all_tile_edges(oracle, shape, exps):
    M, N, K = shape
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    a, b = finite_codes(rng, (M, K)), finite_codes(rng, (N, K))
    ae = rng.integers(100, 128, size=(M, K // 32), dtype=np.uint8) if exps != "none" else None
    be = rng.integers(100, 128, size=(N, K // 32), dtype=np.uint8) if exps == "both" else None
    a_s, b_s = np.float32(0.013), np.float32(1.7)
    ref = oracle.gemm(a, ae, a_s, b, be, b_s)
    na, nb = oracle.row_norms(a, ae, a_s), oracle.row_norms(b, be, b_s)
    out = gpu_gemm(a, ae, a_s, b, be, b_s, out_dtype=torch.float32)
    assert_close(out.cpu().numpy().astype(np.float64), ref, na, nb, False, f"{shape} {exps} f32")
    out = gpu_gemm(a, ae, a_s, b, be, b_s, out_dtype=torch.bfloat16)
    assert_close(bf16_out_to_f64(out), ref, na, nb, True, f"{shape} {exps} bf16")


@pytest.mark.parametrize("K", [512, 640])
def test_more_tiles_than_compute_units_full_compare(oracle, K):
    """17 x 16 = 272 tiles of 256 x 256 on 256 compute units: every workgroup of the persistent grid
    hands over from one tile to the next (with K = 512 after the shortest possible main loop of four
    stages, with K = 640 after an odd number of stages, so the LDS slots swap roles between tiles),
    and the grid is trimmed to the 136 workgroups two rounds need.  Every output is compared."""
    M, N = 4352 - 3, 4096
    rng = np.random.default_rng(K)
    a, b = finite_codes(rng, (M, K)), finite_codes(rng, (N, K))
    ae = rng.integers(110, 128, size=(M, K // 32), dtype=np.uint8)
    be = rng.integers(110, 128, size=(N, K // 32), dtype=np.uint8) if K == 640 else None
    a_s, b_s = np.float32(0.5), np.float32(0.25)
    ref = oracle.gemm(a, ae, a_s, b, be, b_s)
    na, nb = oracle.row_norms(a, ae, a_s), oracle.row_norms(b, be, b_s)
    out = gpu_gemm(a, ae, a_s, b, be, b_s, out_dtype=torch.float32)
    assert_close(out.cpu().numpy().astype(np.float64), ref, na, nb, False, f"272 tiles K={K} f32")
    out = gpu_gemm(a, ae, a_s, b, be, b_s, out_dtype=torch.bfloat16)
    assert_close(bf16_out_to_f64(out), ref, na, nb, True, f"272 tiles K={K} bf16")


def test_one_hot_operands_pin_the_lane_and_scale_mapping(oracle):
    # a single nonzero code in a and in b at the same k: exactly one output is nonzero and
    # equals the product of the two decoded values and their two level-2 scales
    M, N, K = 48, 40, 256
    rng = np.random.default_rng(5)
    ae = rng.integers(110, 128, size=(M, K // 32), dtype=np.uint8)
    be = rng.integers(110, 128, size=(N, K // 32), dtype=np.uint8)
    for (m, n, k) in [(0, 0, 0), (17, 5, 33), (47, 39, 255), (16, 20, 100), (31, 3, 64 + 17), (5, 33, 128 + 95)]:
        a = np.zeros((M, K), np.uint8); b = np.zeros((N, K), np.uint8)
        a[m, k] = 0x3A; b[n, k] = 0xC5
        ref = oracle.gemm(a, ae, 1.0, b, be, 1.0)
        out = gpu_gemm(a, ae, 1.0, b, be, 1.0, out_dtype=torch.float32).cpu().numpy().astype(np.float64)
        assert np.count_nonzero(ref) == 1 and ref[m, n] != 0
        assert np.array_equal(out, ref), (m, n, k)


@pytest.mark.parametrize("shape,ld", [((70, 52, 192), 64),          # general kernel
                                      ((600, 1000, 512), 1004),     # ld_out % 8 != 0: the general kernel (the large-tile epilogue stores whole 16-byte pieces)
                                      ((1024, 776, 640), 784)])     # large-tile kernel, vector stores, ragged N
def test_fp32_accumulate_and_padded_output(oracle, shape, ld):
    M, N, K = shape
    rng = np.random.default_rng(9)
    a, b = finite_codes(rng, (M, K)), finite_codes(rng, (N, K))
    ae = rng.integers(115, 128, size=(M, K // 32), dtype=np.uint8)
    ref = oracle.gemm(a, ae, 0.5, b, None, 0.25)
    na, nb = oracle.row_norms(a, ae, 0.5), oracle.row_norms(b, None, 0.25)
    base = rng.standard_normal((M, ld)).astype(np.float32)
    buf = to_gpu(base.copy())
    out = buf[:, :N]                                   # ld_out = ld > N
    sa = to_gpu(np.array([0.5], np.float32)); sb = to_gpu(np.array([0.25], np.float32))
    moss.gemm_fp8_mx(to_gpu(a), to_gpu(ae), sa, to_gpu(b), None, sb, out=out, accumulate=True)
    torch.cuda.synchronize()
    res = buf.cpu().numpy()
    assert np.array_equal(res[:, N:], base[:, N:])     # padding columns untouched
    assert_close(res[:, :N].astype(np.float64) - base[:, :N].astype(np.float64), ref, na, nb, False, "accumulate")
    moss.gemm_fp8_mx(to_gpu(a), to_gpu(ae), sa, to_gpu(b), None, sb, out=out, accumulate=False)
    torch.cuda.synchronize()
    assert_close(buf.cpu().numpy()[:, :N].astype(np.float64), ref, na, nb, False, "overwrite")


def test_config1_linear_forward_chain(oracle):
    # quantize X (two-level), cast W (per tensor), GEMM, dequantize in the epilogue
    xb, wb = mi.config1()
    x, w = bf16_to_gpu(xb), bf16_to_gpu(wb)
    for flag, mode in ((0, 0), (moss.MOSS_EXP_CEIL, 1)):
        qx = moss.quant_act_2level(x, moss.MOSS_Q_ROW | flag)
        state = moss.new_wscale_state(w.device)
        wq, _ = moss.weight_autoscale_init(w, state)
        s_w = state[4:8].view(torch.float32)           # s_cur field of the device-resident state
        y = moss.gemm_fp8_mx(qx["q_row"], qx["e_row"], qx["s"], wq, None, s_w)
        torch.cuda.synchronize()
        q, e, s = oracle.quant_act_2level(xb, 0, mode)
        st, owq, _ = oracle.weight_init(mi.bf16_bits_to_f32(wb))
        assert np.array_equal(u8(qx["q_row"]), q) and np.array_equal(u8(qx["e_row"]), e) and np.array_equal(u8(wq), owq)
        ref = oracle.gemm(q, e, s, owq, None, st.s_cur)
        assert_close(bf16_out_to_f64(y), ref, oracle.row_norms(q, e, s), oracle.row_norms(owq, None, st.s_cur), True,
                     f"config1 chain mode {mode}")
        # and the quantized product tracks the BF16 one (end-to-end sanity, not a parity bar)
        xf = mi.bf16_bits_to_f32(xb).astype(np.float64); wf = mi.bf16_bits_to_f32(wb).astype(np.float64)
        exact = xf @ wf.T
        snr = 10 * np.log10((exact ** 2).sum() / ((bf16_out_to_f64(y) - exact) ** 2).sum())
        assert snr > (24.0 if mode else 15.0)


def sampled_pairs(rng, M, N, n_rows=32, n_cols=32, n_rand=65536):
    ms, ns = [], []
    for r in rng.choice(M, n_rows, replace=False):
        ms.append(np.full(N, r)); ns.append(np.arange(N))
    for c in rng.choice(N, n_cols, replace=False):
        ms.append(np.arange(M)); ns.append(np.full(M, c))
    ms.append(rng.integers(0, M, n_rand)); ns.append(rng.integers(0, N, n_rand))
    # the four corners and the last tile edge
    ms.append(np.array([0, 0, M - 1, M - 1])); ns.append(np.array([0, N - 1, 0, N - 1]))
    return np.concatenate(ms).astype(np.int64), np.concatenate(ns).astype(np.int64)


def check_sampled(oracle, tag, out, oa, ob, rng, **sample):
    """Outputs on 32 random full rows, 32 random full columns, 65 536 random entries and the four corners (or the
    smaller sample given) against the oracle's FP64 sums over the same codes."""
    (aq, ae, a_s), (bq, be, b_s) = oa, ob
    M, N = aq.shape[0], bq.shape[0]
    ms, ns = sampled_pairs(rng, M, N, **sample)
    ref = oracle.gemm_sampled(aq, ae, a_s, bq, be, b_s, ms, ns)
    na = oracle.row_norms(aq, ae, a_s)[ms]
    nb = oracle.row_norms(bq, be, b_s)[ns]
    got = out[torch.from_numpy(ms).to(out.device), torch.from_numpy(ns).to(out.device)]
    got = got.float().cpu().numpy().astype(np.float64)
    assert_close(got, ref, na, nb, out.dtype == torch.bfloat16, tag)


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_config3_llama7b_linears_fwd_bwd_sampled(oracle, index):
    """Y = X W^T, dX = dY W, dW = dY^T X at tokens = 8192 on the five 7B shapes, in the launch configuration the
    benchmark times; codes and exponents bit-exact, every GEMM output checked on 32 rows, 32 columns and
    65 536 entries."""
    name, K, N = mi.LLAMA7B_LINEARS[index]
    print(f"[config3] linear {name}: tokens=8192 K={K} N={N}", flush=True)
    xb, wb, dyb = mi.config3_linear(index)
    rng = np.random.default_rng(100 + index)
    x, w, dy = bf16_to_gpu(xb), bf16_to_gpu(wb), bf16_to_gpu(dyb)
    qx = moss.quant_act_2level(x, moss.MOSS_Q_ROW | moss.MOSS_Q_COL)
    qdy = moss.quant_act_2level(dy, moss.MOSS_Q_ROW | moss.MOSS_Q_COL)
    state = moss.new_wscale_state(w.device)
    wq, wq_t = moss.weight_autoscale_init(w, state, want_transpose=True)
    s_w = state[4:8].view(torch.float32)
    y = moss.gemm_fp8_mx(qx["q_row"], qx["e_row"], qx["s"], wq, None, s_w)                       # [T x N]
    dx = moss.gemm_fp8_mx(qdy["q_row"], qdy["e_row"], qdy["s"], wq_t, None, s_w)                 # [T x K]
    dw = moss.gemm_fp8_mx(qdy["q_col"], qdy["e_col"], qdy["s"], qx["q_col"], qx["e_col"], qx["s"],
                          out_dtype=torch.float32)                                               # [N x K]
    torch.cuda.synchronize()

    oxr = oracle.quant_act_2level(xb, 0, 0); oxc = oracle.quant_act_2level(xb, 1, 0)
    assert np.array_equal(u8(qx["q_row"]), oxr[0]) and np.array_equal(u8(qx["e_row"]), oxr[1])
    assert np.array_equal(u8(qx["q_col"]), oxc[0]) and np.array_equal(u8(qx["e_col"]), oxc[1])
    del xb
    odr = oracle.quant_act_2level(dyb, 0, 0); odc = oracle.quant_act_2level(dyb, 1, 0)
    assert np.array_equal(u8(qdy["q_row"]), odr[0]) and np.array_equal(u8(qdy["e_row"]), odr[1])
    assert np.array_equal(u8(qdy["q_col"]), odc[0]) and np.array_equal(u8(qdy["e_col"]), odc[1])
    del dyb
    st, owq, owq_t = oracle.weight_init(mi.bf16_bits_to_f32(wb), want_transpose=True)
    assert np.array_equal(u8(wq), owq) and np.array_equal(u8(wq_t), owq_t)
    ow, owt = (owq, None, st.s_cur), (owq_t, None, st.s_cur)
    check_sampled(oracle, f"{name} Y", y, oxr, ow, rng)
    check_sampled(oracle, f"{name} dX", dx, odr, owt, rng)
    check_sampled(oracle, f"{name} dW", dw, odc, oxc, rng)


# The (M, N, K) of the paper's table "Runtime of quantized FP8 GEMM" (Sec. 4.5.1).
PAPER_GEMM_SHAPES = [(2048, 7168, 4096), (2048, 7168, 11008), (4096, 2048, 7168), (4096, 4096, 8192),
                     (4096, 4096, 12288), (5120, 5120, 10240), (8192, 8192, 8192)]


@pytest.mark.parametrize("shape", PAPER_GEMM_SHAPES)
def test_paper_gemm_table_shapes_sampled(oracle, shape):
    """The second GEMM workload: activations with level-2 exponents against per-tensor weights (a_e given, b_e
    absent, as in the paper's kernel), random finite codes, BF16 output; 8 rows, 8 columns and 16 384 entries."""
    M, N, K = shape
    print(f"[gemm table] M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng(M + N + K)
    a, b = finite_codes(rng, (M, K)), finite_codes(rng, (N, K))
    ae = rng.integers(112, 128, size=(M, K // 32), dtype=np.uint8)
    a_s, b_s = np.float32(0.02), np.float32(3.0e-4)
    out = gpu_gemm(a, ae, a_s, b, None, b_s, out_dtype=torch.bfloat16)
    check_sampled(oracle, f"table {shape}", out, (a, ae, a_s), (b, None, b_s), rng, n_rows=8, n_cols=8, n_rand=16384)


def test_bf16_baseline_gemm_matches_fp64_product():
    rng = np.random.default_rng(11)
    for (M, N, K) in [(200, 136, 96), (256, 384, 512), (130, 70, 1056)]:
        a = mi.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
        b = mi.f32_to_bf16_bits(rng.standard_normal((N, K)).astype(np.float32) * 0.02)
        out = moss.gemm_bf16_baseline(bf16_to_gpu(a), bf16_to_gpu(b))
        torch.cuda.synchronize()
        af = mi.bf16_bits_to_f32(a).astype(np.float64); bf = mi.bf16_bits_to_f32(b).astype(np.float64)
        ref = af @ bf.T
        tol = np.outer(np.linalg.norm(af, axis=1), np.linalg.norm(bf, axis=1))
        err = np.abs(bf16_out_to_f64(out) - ref)
        assert (err <= 2.0 ** -8 * np.abs(ref) + 1e-5 * tol).all()
