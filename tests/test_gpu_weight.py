"""GPU parity of moss_weight_autoscale_init / moss_weight_autoscale_cast against the
CPU oracle: bit-exact W, m, v, codes, transposed codes and every state field
(paper Sec. 3.2, Eq. 10; AdamW of Sec. 2.2)."""
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
    for f in ("s_base", "s_cur", "cum_lr", "step", "last_rebase", "amax_seen", "overflow_count", "clipped_count"):
        assert getattr(gs, f) == getattr(os_, f), (tag, f, getattr(gs, f), getattr(os_, f))
    assert gs.flags == 0, (tag, gs.flags)


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
    assert st.last_rebase == 60 and st.clipped_count == 0


def test_bf16_gradients_and_sparse_spikes(oracle):
    print("[weight parity] 40x72 bf16 grads, sparse spikes", flush=True)
    run_parity(oracle, 40, 72, 25, seed=5, bf16_grad=True, sparse=True, interval=500)


def test_ragged_size_not_a_multiple_of_the_block(oracle):
    print("[weight parity] 333x52 (n % 1024 != 0)", flush=True)
    run_parity(oracle, 333, 52, 6, seed=6, interval=4)


def test_broken_bound_saturates_and_counts(oracle):
    print("[weight parity] overflow path", flush=True)
    st = run_parity(oracle, 64, 64, 6, seed=7, lr=1e-2, margin=1e-4)
    assert st.overflow_count >= st.clipped_count > 0


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
    assert st.clipped_count == 0 and st.step == 200


def test_config4_full_size_first_steps(oracle):
    print("[weight parity] config 4 at 4096x11008, 6 steps, re-scaling at step 5", flush=True)
    st = run_parity(oracle, 4096, 11008, 6, seed=4, interval=5, check_every=1)
    assert st.clipped_count == 0 and st.last_rebase == 5


def gpu_args(t, **kw):
    hp = mi.adamw_hparams(t, **kw)
    return moss.AdamWArgs(hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"], hp["one_minus_beta1"],
                          hp["one_minus_beta2"], hp["bias_corr1"], hp["bias_corr2"], hp["margin"], hp["interval"], t)


@pytest.mark.parametrize("sparse", [False, True], ids=["spike_steps", "sparse_spikes"])
def test_config4_full_size_200_steps_band_against_oracle(oracle, sparse):
    """Config 4 at its full size, 4096 x 11008, 200 steps, interval 500 (no re-scaling inside the run), in the launch
    configuration the benchmark times (fused step that also writes the transposed codes).  AdamW and the cast are
    element-wise and the predicted scale depends only on s_0 and the step count (Sec. 3.2, Eq. 10), so the oracle
    is initialised on the whole host-drawn tensor and then follows a band of 192 rows that crosses tile boundaries,
    fed with host-drawn gradients; the other rows get device-drawn gradients of the same recipe.  Every 50 steps the
    band's W, m, v, codes and transposed codes and the scale state are compared bit for bit; over the whole tensor
    no predicted scale may let an element out of range, and the by-product maximum must be the tensor's."""
    rows, cols, steps, band0, band = 4096, 11008, 200, 1000, 192
    print(f"[weight parity] config 4 full size, band rows {band0}..{band0 + band}, sparse={sparse}", flush=True)
    dev = torch.device("cuda:0")
    w_host = mi.config4_weights(rows, cols, seed=4)
    ost, owq, _ = oracle.weight_init(w_host)
    wb = w_host[band0:band0 + band].copy(); mb = np.zeros_like(wb); vb = np.zeros_like(wb)
    w = to_gpu(w_host); m = torch.zeros_like(w); v = torch.zeros_like(w)
    state = moss.new_wscale_state(dev)
    wq = torch.empty((rows, cols), dtype=torch.uint8, device=dev)
    wq_t = torch.empty((cols, rows), dtype=torch.uint8, device=dev)
    moss.weight_autoscale_init(w, state, wq=wq, wq_t=wq_t)
    torch.cuda.synchronize()
    assert_same_bits(u8(wq), owq, "init wq")
    assert_state_equal(moss.read_wscale_state(state), ost, "init")
    init_out_of_range = ost.overflow_count      # the exact scale may sit one rounding below amax/448
    gen = torch.Generator(device=dev)
    gen.manual_seed(44 + int(sparse))
    for t in range(1, steps + 1):
        g = torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32) * 1e-3
        if sparse:
            g = torch.where(torch.rand((rows, cols), generator=gen, device=dev) < 1e-3, g * 20.0, g)
        elif mi.config4_is_spike_step(t):
            g *= 20.0
        gb = mi.config4_grad(t, band, cols, seed=4, sparse_spikes=sparse)
        g[band0:band0 + band] = to_gpu(gb)
        oargs, gargs = make_args(oracle, t, interval=500)
        oq, _ = oracle.weight_step(wb, mb, vb, gb, oargs, ost)
        moss.weight_autoscale_cast(w, m, v, g, gargs, state, wq=wq, wq_t=wq_t)
        if t % 50 == 0:
            torch.cuda.synchronize()
            tag = f"step {t}"
            sl = slice(band0, band0 + band)
            assert_same_bits(w[sl].cpu().numpy(), wb, tag + " w")
            assert_same_bits(m[sl].cpu().numpy(), mb, tag + " m")
            assert_same_bits(v[sl].cpu().numpy(), vb, tag + " v")
            assert_same_bits(u8(wq[sl]), oq, tag + " wq")
            assert_same_bits(u8(wq_t[:, sl]), oq.T, tag + " wq_t")
            gs = moss.read_wscale_state(state)
            for f in ("s_base", "s_cur", "cum_lr", "step", "last_rebase"):
                assert getattr(gs, f) == getattr(ost, f), (tag, f)
            assert gs.flags == 0 and gs.clipped_count == 0 and ost.clipped_count == 0
            assert gs.overflow_count == init_out_of_range, (tag, gs.overflow_count, init_out_of_range)
            amax = float(w.abs().max())
            assert gs.amax_seen == amax and gs.s_cur >= np.float32(amax) / np.float32(448.0)
            assert torch.equal(wq_t, wq.t().contiguous())


@pytest.mark.parametrize("sparse", [False, True], ids=["spike_steps", "sparse_spikes"])
def test_config4_full_size_200_steps_with_rescaling_against_oracle(oracle, sparse):
    """The same launch configuration with interval 50 (re-scaling at steps 50, 100, 150, 200: Sec. 3.2, last
    paragraph).  The exact scale needs the maximum of the whole tensor, so here the 4096 x 11008 tensor and its
    gradients are 16 vertical copies of a host-drawn 256-row band: the oracle run on the band then predicts every
    element, the maximum and therefore the re-based scales of the full tensor, and the counters times 16."""
    rows, cols, steps, band, interval = 4096, 11008, 200, 256, 50
    reps = rows // band
    print(f"[weight parity] config 4 full size, periodic band, interval {interval}, sparse={sparse}", flush=True)
    dev = torch.device("cuda:0")
    wb = mi.config4_weights(band, cols, seed=41).copy(); mb = np.zeros_like(wb); vb = np.zeros_like(wb)
    w = to_gpu(wb).repeat(reps, 1).contiguous(); m = torch.zeros_like(w); v = torch.zeros_like(w)
    state = moss.new_wscale_state(dev)
    wq = torch.empty((rows, cols), dtype=torch.uint8, device=dev)
    wq_t = torch.empty((cols, rows), dtype=torch.uint8, device=dev)
    moss.weight_autoscale_init(w, state, wq=wq, wq_t=wq_t)
    ost, oq, _ = oracle.weight_init(wb)

    def check(tag):
        torch.cuda.synchronize()
        for name, got, want in (("w", w, wb), ("m", m, mb), ("v", v, vb), ("wq", wq, oq)):
            want_d = to_gpu(want)
            assert torch.equal(got.view(reps, band, cols), want_d.unsqueeze(0).expand(reps, band, cols)), (tag, name)
        assert torch.equal(wq_t, wq.t().contiguous()), tag
        gs = moss.read_wscale_state(state)
        for f in ("s_base", "s_cur", "cum_lr", "step", "last_rebase", "amax_seen"):
            assert getattr(gs, f) == getattr(ost, f), (tag, f, getattr(gs, f), getattr(ost, f))
        assert gs.overflow_count == reps * ost.overflow_count and gs.clipped_count == reps * ost.clipped_count == 0
        assert gs.flags == 0
    check("init")
    for t in range(1, steps + 1):
        gb = mi.config4_grad(t, band, cols, seed=41, sparse_spikes=sparse)
        g = to_gpu(gb).repeat(reps, 1).contiguous()
        oargs, gargs = make_args(oracle, t, interval=interval)
        oq, _ = oracle.weight_step(wb, mb, vb, gb, oargs, ost)
        moss.weight_autoscale_cast(w, m, v, g, gargs, state, wq=wq, wq_t=wq_t)
        if t % 50 in (0, 1, 49):
            check(f"step {t}")
    assert ost.last_rebase == 200 and ost.s_cur == np.float32(ost.amax_seen) / np.float32(448.0)


def test_checkpoint_of_the_device_state_resumes_bit_identically():
    """Run 120 steps; run 60, copy W, m, v and the 48-byte scale state to the host and into fresh device tensors,
    run the other 60 there: every tensor and the state must agree bit for bit (the state struct is all the path
    keeps between steps).  Interval 25, so re-scaling steps fall on both sides of the checkpoint."""
    rows, cols, steps, half = 256, 384, 120, 60
    print("[weight] checkpoint / resume", flush=True)

    def fresh():
        w = to_gpu(mi.config4_weights(rows, cols, seed=9)); m = torch.zeros_like(w); v = torch.zeros_like(w)
        st = moss.new_wscale_state(w.device)
        moss.weight_autoscale_init(w, st, want_transpose=True)
        return w, m, v, st

    def advance(w, m, v, st, t0, t1):
        out = None
        for t in range(t0, t1 + 1):
            g = to_gpu(mi.config4_grad(t, rows, cols, seed=9))
            out = moss.weight_autoscale_cast(w, m, v, g, gpu_args(t, interval=25), st, want_transpose=True)
        torch.cuda.synchronize()
        return out
    w1, m1, v1, st1 = fresh()
    q1, qt1 = advance(w1, m1, v1, st1, 1, steps)
    w2, m2, v2, st2 = fresh()
    advance(w2, m2, v2, st2, 1, half)
    saved = [t.cpu().numpy().copy() for t in (w2, m2, v2, st2)]
    del w2, m2, v2, st2
    w3, m3, v3, st3 = (to_gpu(a) for a in saved)
    q3, qt3 = advance(w3, m3, v3, st3, half + 1, steps)
    for a, b, tag in ((w1, w3, "w"), (m1, m3, "m"), (v1, v3, "v"), (q1, q3, "wq"), (qt1, qt3, "wq_t"), (st1, st3, "state")):
        assert torch.equal(a, b), tag
    gs = moss.read_wscale_state(st3)
    assert gs.step == steps and gs.last_rebase == 100 and gs.flags == 0


def test_step_number_that_disagrees_with_the_state_is_flagged():
    rows, cols = 64, 96
    w = to_gpu(mi.config4_weights(rows, cols, seed=10)); m = torch.zeros_like(w); v = torch.zeros_like(w)
    st = moss.new_wscale_state(w.device)
    moss.weight_autoscale_init(w, st)
    g = to_gpu(mi.config4_grad(1, rows, cols, seed=10))
    moss.weight_autoscale_cast(w, m, v, g, gpu_args(1), st)
    assert moss.read_wscale_state(st).flags == 0
    moss.weight_autoscale_cast(w, m, v, g, gpu_args(5), st)          # the state is at step 1: 5 is not the next step
    gs = moss.read_wscale_state(st)
    assert gs.flags & moss.MOSS_WSTATE_STEP_MISMATCH and gs.step == 2
    moss.weight_autoscale_cast(w, m, v, g, gpu_args(3), st)          # sticky
    assert moss.read_wscale_state(st).flags & moss.MOSS_WSTATE_STEP_MISMATCH
    moss.weight_autoscale_init(w, st)                                # a new initialisation clears it
    assert moss.read_wscale_state(st).flags == 0
