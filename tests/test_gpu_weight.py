"""GPU parity of moss_weight_autoscale_init / moss_weight_autoscale_cast against the
CPU oracle: bit-exact W, m, v, codes, transposed codes and every state field
(paper Sec. 3.2, Eq. 6; AdamW of Sec. 2.2)."""
import numpy as np
import pytest
import torch

import moss_inputs as mi
import paper_2511_05811_amd as moss
from gpu_util import assert_same_bits, bf16_to_gpu, to_gpu, u8

pytestmark = pytest.mark.gpu


def make_args(oracle, t, **kw):
    hp = mi.adamw_hparams(t, **kw)
    return oracle.adamw_args(**hp), moss.AdamWArgs(hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"],
                                                   hp["one_minus_beta1"], hp["one_minus_beta2"], hp["bias_corr1"],
                                                   hp["bias_corr2"], hp["margin"], hp["interval"], t)


def assert_state_equal(gs, os_, tag):
    for f in ("s_base", "s_cur", "cum_lr", "step", "last_rebase", "amax_seen", "overflow_count"):
        assert getattr(gs, f) == getattr(os_, f), (tag, f, getattr(gs, f), getattr(os_, f))


def run_parity(oracle, rows, cols, steps, seed, interval=500, bf16_grad=False, sparse=False, transpose=True,
               lr=3e-4, margin=1.0, check_every=1):
    w = mi.config4_weights(rows, cols, seed=seed).copy()
    m = np.zeros_like(w); v = np.zeros_like(w)
    wd, md, vd = to_gpu(w), to_gpu(m), to_gpu(v)
    state = moss.new_wscale_state(wd.device)
    wq_d, wqt_d = moss.weight_autoscale_init(wd, state, want_transpose=transpose)
    st, wq, wq_t = oracle.weight_init(w, want_transpose=transpose)
    torch.cuda.synchronize()
    assert np.array_equal(u8(wq_d), wq)
    if transpose:
        assert np.array_equal(u8(wqt_d), wq_t)
    assert_state_equal(moss.read_wscale_state(state), st, "init")
    for t in range(1, steps + 1):
        g = mi.config4_grad(t, rows, cols, seed=seed, sparse_spikes=sparse)
        if bf16_grad:
            gb = mi.f32_to_bf16_bits(g)
            g_dev, g_cpu = bf16_to_gpu(gb), gb
        else:
            g_dev, g_cpu = to_gpu(g), g
        oargs, gargs = make_args(oracle, t, interval=interval, lr=lr, margin=margin)
        wq, wq_t = oracle.weight_step(w, m, v, g_cpu, oargs, st, want_transpose=transpose)
        wq_d, wqt_d = moss.weight_autoscale_cast(wd, md, vd, g_dev, gargs, state, want_transpose=transpose)
        if t % check_every == 0 or t == steps:
            torch.cuda.synchronize()
            tag = f"step {t}"
            assert_same_bits(md.cpu().numpy(), m, tag + " m")
            assert_same_bits(vd.cpu().numpy(), v, tag + " v")
            assert_same_bits(wd.cpu().numpy(), w, tag + " w")
            assert_same_bits(u8(wq_d), wq, tag + " wq")
            if transpose:
                assert_same_bits(u8(wqt_d), wq_t, tag + " wq_t")
            assert_state_equal(moss.read_wscale_state(state), st, tag)
    return st


def test_small_run_with_interval_rescaling(oracle):
    print("[weight parity] 48x96, 60 steps, interval 20", flush=True)
    st = run_parity(oracle, 48, 96, 60, seed=4, interval=20)
    assert st.last_rebase == 60 and st.overflow_count == 0


def test_bf16_gradients_and_sparse_spikes(oracle):
    print("[weight parity] 40x72 bf16 grads, sparse spikes", flush=True)
    run_parity(oracle, 40, 72, 25, seed=5, bf16_grad=True, sparse=True, interval=500)


def test_ragged_size_not_a_multiple_of_the_block(oracle):
    print("[weight parity] 333x52 (n % 1024 != 0)", flush=True)
    run_parity(oracle, 333, 52, 6, seed=6, interval=4)


def test_broken_bound_saturates_and_counts(oracle):
    print("[weight parity] overflow path", flush=True)
    st = run_parity(oracle, 64, 64, 6, seed=7, lr=1e-2, margin=1e-4)
    assert st.overflow_count > 0


def test_bf16_weights_at_init(oracle):
    _, wb = mi.config1()
    w32 = mi.bf16_bits_to_f32(wb)
    wd = bf16_to_gpu(wb)
    state = moss.new_wscale_state(wd.device)
    wq_d, wqt_d = moss.weight_autoscale_init(wd, state, want_transpose=True)
    st, wq, wq_t = oracle.weight_init(w32, want_transpose=True)
    torch.cuda.synchronize()
    assert np.array_equal(u8(wq_d), wq) and np.array_equal(u8(wqt_d), wq_t)
    assert_state_equal(moss.read_wscale_state(state), st, "bf16 init")


def test_config4_reduced_size_200_steps(oracle):
    print("[weight parity] config 4 at 512x1376, 200 steps", flush=True)
    st = run_parity(oracle, 512, 1376, 200, seed=4, interval=500, transpose=False, check_every=20)
    assert st.overflow_count == 0 and st.step == 200


def test_config4_full_size_first_steps(oracle):
    print("[weight parity] config 4 at 4096x11008, 6 steps, re-scaling at step 5", flush=True)
    st = run_parity(oracle, 4096, 11008, 6, seed=4, interval=5, check_every=1)
    assert st.overflow_count == 0 and st.last_rebase == 5


def test_config4_full_size_200_steps_never_overflow():
    """All 200 steps of config 4 at 4096 x 11008 on the GPU (gradients drawn on the device, x20 on the
    deterministic spike steps): the predicted scale never falls below the exact one, no element is
    clipped, the by-product amax is the exact maximum of the new weights, and the scale is re-based
    exactly at the interval (Sec. 3.2, Eq. 6 and its last paragraph)."""
    rows, cols, interval = 4096, 11008, 50
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(4)
    w = torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32) * 0.02
    m = torch.zeros_like(w); v = torch.zeros_like(w)
    state = moss.new_wscale_state(dev)
    wq = torch.empty((rows, cols), dtype=torch.uint8, device=dev)
    wq_t = torch.empty((cols, rows), dtype=torch.uint8, device=dev)
    moss.weight_autoscale_init(w, state, wq=wq, wq_t=wq_t)
    rebases = []
    for t in range(1, 201):
        g = torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32) * 1e-3
        if mi.config4_is_spike_step(t):
            g *= 20.0
        hp = mi.adamw_hparams(t, interval=interval)
        args = moss.AdamWArgs(hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"], hp["one_minus_beta1"],
                              hp["one_minus_beta2"], hp["bias_corr1"], hp["bias_corr2"], hp["margin"], hp["interval"], t)
        moss.weight_autoscale_cast(w, m, v, g, args, state, wq=wq, wq_t=wq_t)
        if t % 10 == 0 or t % interval == 1:
            st = moss.read_wscale_state(state)
            assert st.overflow_count == 0, t
            assert st.s_cur >= st.amax_seen / 448.0 * (1.0 - 1e-6), (t, st.s_cur, st.amax_seen)
            assert abs(st.amax_seen - float(w.abs().max())) == 0.0
            if st.last_rebase not in rebases:
                rebases.append(st.last_rebase)
    assert rebases == [0, 50, 100, 150, 200]
    st = moss.read_wscale_state(state)
    assert st.step == 200 and st.s_cur == np.float32(st.amax_seen) / np.float32(448.0)     # step 200 re-based
    # transposed codes are the byte transpose of the codes
    assert torch.equal(wq_t, wq.t().contiguous())
