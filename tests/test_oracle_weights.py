"""Pins for the oracle's weight path: AdamW (Sec. 2.2, Eq. 1) against a library
optimizer, the closed form of the automatic scaling rule (Sec. 3.2, Eq. 10), the
bound it rests on, interval re-scaling, restart equivalence and the cast."""
import copy
from fractions import Fraction

import numpy as np
import pytest
import torch

import moss_inputs as mi

HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def args_for(oracle, step, **kw):
    hp = mi.adamw_hparams(step, **{**HP, **kw})
    return oracle.adamw_args(**hp)


def exact_out_of_range(w, s):
    """#{|w| > 448 s} in exact rational arithmetic (every float is a rational)."""
    limit = 448 * Fraction(float(s))
    return sum(1 for x in np.abs(w).ravel().tolist() if Fraction(x) > limit)


def small_run(oracle, steps, rows=48, cols=96, interval=500, margin=1.0, sparse=False, on_step=None, lr=3e-4):
    w = mi.config4_weights(rows, cols, seed=4).copy()
    m = np.zeros_like(w)
    v = np.zeros_like(w)
    st, wq, _ = oracle.weight_init(w)
    for t in range(1, steps + 1):
        g = mi.config4_grad(t, rows, cols, seed=4, sparse_spikes=sparse)
        wq, wq_t = oracle.weight_step(w, m, v, g, args_for(oracle, t, interval=interval, margin=margin, lr=lr), st,
                                      want_transpose=True)
        if on_step:
            on_step(t, w, st, wq, wq_t)
    return w, m, v, st, wq


def test_adamw_matches_library_optimizer(oracle):
    rows, cols, steps = 8, 64, 60
    w = mi.config4_weights(rows, cols, seed=21).copy()
    m = np.zeros_like(w); v = np.zeros_like(w)
    p = torch.nn.Parameter(torch.from_numpy(w.astype(np.float64)))
    opt = torch.optim.AdamW([p], lr=HP["lr"], betas=(float(np.float32(0.9)), float(np.float32(0.95))),
                            eps=HP["eps"], weight_decay=HP["weight_decay"])
    st, _, _ = oracle.weight_init(w)
    for t in range(1, steps + 1):
        g = mi.config4_grad(t, rows, cols, seed=21)
        oracle.weight_step(w, m, v, g, args_for(oracle, t), st)
        p.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
        ref = p.detach().numpy()
        # float32 arithmetic against the float64 library trajectory
        assert np.abs(w - ref).max() <= 2e-6 * np.abs(ref).max() + 1e-9, t
    state = opt.state[p]
    assert np.allclose(m, state["exp_avg"].numpy(), rtol=1e-5, atol=1e-12)
    assert np.allclose(v, state["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-16)


def test_single_spike_update_closed_form(oracle):
    # gradient zero at every earlier step and nonzero only now (the extreme case in the
    # proof of Thm 2): m = (1-b1) g, v = (1-b2) g^2, so with eps negligible and no decay
    # |delta| = eta * (1-b1)/sqrt(1-b2) * sqrt(1-b2^t)/(1-b1^t).
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.95))
    for t_spike in (1, 5, 20, 60):
        w = np.full((1, 32), 0.5, np.float32); m = np.zeros_like(w); v = np.zeros_like(w)
        st, _, _ = oracle.weight_init(w)
        for t in range(1, t_spike + 1):
            g = np.zeros_like(w) if t < t_spike else np.full_like(w, 0.37)
            w_before = w.copy()
            oracle.weight_step(w, m, v, g, args_for(oracle, t, weight_decay=0.0), st)
        delta = float(np.abs(w - w_before).max())
        closed = HP["lr"] * (1 - b1) / np.sqrt(1 - b2) * np.sqrt(1 - b2 ** t_spike) / (1 - b1 ** t_spike)
        assert abs(delta - closed) <= 2e-6 * 0.5 + 1e-6 * closed   # limited by float32 spacing at w = 0.5
    # a constant gradient gives exactly |delta| = eta (the typical case of Thm 2)
    w = np.full((1, 32), 0.5, np.float32); m = np.zeros_like(w); v = np.zeros_like(w)
    st, _, _ = oracle.weight_init(w)
    for t in range(1, 30):
        w_before = w.copy()
        oracle.weight_step(w, m, v, np.full_like(w, -2e-3), args_for(oracle, t, weight_decay=0.0), st)
        assert abs(float((w - w_before).max()) - HP["lr"]) <= 1e-7


def test_scale_prediction_closed_form(oracle):
    # Eq. 10: s_t = s_0 + eta * t / 448
    seen = []

    def on_step(t, w, st, wq, wq_t):
        seen.append((t, st.s_base, st.s_cur, st.cum_lr))
    small_run(oracle, 40, on_step=on_step)
    s0 = seen[0][1]
    eta = HP["lr"]
    for t, s_base, s_cur, cum in seen:
        assert s_base == s0
        closed = float(s0) + float(np.float32(eta)) * t / 448.0
        assert abs(float(s_cur) - closed) <= 1.2e-7 * closed
        assert abs(cum - float(np.float32(eta)) * t) <= 1e-12


@pytest.mark.parametrize("sparse", [False, True])
def test_predicted_scale_dominates_exact_scale_and_never_overflows(oracle, sparse):
    # Sec. 3.2: max|W_t| <= max|W_0| + eta*t, so the automatic curve lies above the
    # just-in-time curve and the cast never saturates (observed on the seeded data).
    ratios = []

    def on_step(t, w, st, wq, wq_t):
        s_jit = np.float32(np.abs(w).max()) / np.float32(448.0)
        assert st.s_cur >= s_jit
        assert st.amax_seen == np.abs(w).max()
        assert (wq & 0x7F).max() <= 0x7E
        assert np.array_equal(wq_t, wq.T)
        ratios.append(float(st.s_cur) / float(s_jit))
    w, m, v, st, wq = small_run(oracle, 120, sparse=sparse, on_step=on_step)
    # no predicted scale let an element out of range; what the counter holds comes from the exact scale of
    # the initialisation, which may sit one rounding of amax/448 below the largest element
    assert st.overflow_count == exact_out_of_range(mi.config4_weights(48, 96, seed=4), st.s_base)
    assert st.clipped_count == 0
    assert st.step == 120 and st.last_rebase == 0
    assert 1.0 <= min(ratios) and max(ratios) < 2.0   # curves stay close (Fig. 4)


def test_interval_rescaling_resets_to_exact_scale(oracle):
    def on_step(t, w, st, wq, wq_t):
        if t % 25 == 0:
            exact = np.float32(np.abs(w).max()) / np.float32(448.0)
            assert st.s_base == exact and st.s_cur == exact and st.cum_lr == 0.0 and st.last_rebase == t
        else:
            k = t % 25
            closed = float(st.s_base) + float(np.float32(HP["lr"])) * k / 448.0
            assert abs(float(st.s_cur) - closed) <= 1.2e-7 * closed
    small_run(oracle, 80, interval=25, on_step=on_step)


def test_cast_matches_library_cast_and_dequant_error(oracle):
    def on_step(t, w, st, wq, wq_t):
        inv = np.float32(1.0) / np.float32(st.s_cur)
        ref = torch.from_numpy(w * inv).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(wq, ref)
        if t == 7:
            dq = oracle.dequant(wq, None, st.s_cur)
            y = np.abs(w.astype(np.float64)) / float(st.s_cur)
            half_ulp = 0.5 * 2.0 ** (np.floor(np.log2(np.maximum(y, 2.0 ** -6))) - 3)
            assert (np.abs(dq - w) <= (half_ulp + y * 2.0 ** -21) * float(st.s_cur)).all()
    small_run(oracle, 10, on_step=on_step)


def test_overflow_is_counted_and_saturated_when_the_bound_is_broken(oracle):
    # predictor told a far smaller step size than the optimizer uses: the bound fails,
    # the cast must clip to +-448 and say how often.
    rows, cols = 16, 64
    w = mi.config4_weights(rows, cols, seed=5).copy() * np.float32(0.01)
    m = np.zeros_like(w); v = np.zeros_like(w)
    st, _, _ = oracle.weight_init(w)
    total = 0
    out_of_range = exact_out_of_range(w, st.s_cur)
    for t in range(1, 6):
        g = mi.config4_grad(t, rows, cols, seed=5)
        a = args_for(oracle, t, lr=1e-2, margin=1e-4)
        wq, _ = oracle.weight_step(w, m, v, g, a, st)
        y = w * (np.float32(1.0) / np.float32(st.s_cur))
        total += int((np.abs(y) > 464.0).sum())
        out_of_range += exact_out_of_range(w, st.s_cur)
        assert ((wq & 0x7F) == 0x7E).sum() >= (np.abs(y) > 464.0).sum()
        # everything the count leaves out is what the library's unsaturated cast also maps to 448
        keep = np.abs(y) <= 464.0
        assert np.array_equal(wq[keep], torch.from_numpy(y[keep]).to(torch.float8_e4m3fn).view(torch.uint8).numpy())
        assert (wq & 0x7F).max() <= 0x7E
    assert total > 0 and st.clipped_count == total
    # the range test itself, |w| > 448 s_t, counted in exact rational arithmetic
    assert st.overflow_count == out_of_range and out_of_range >= total


def test_range_counter_at_the_exact_scale(oracle):
    # s_0 = fl(amax / 448) can round below amax / 448: the largest elements are then (by less than one
    # part in 2^24) outside 448 s_0 and are counted, although their codes are +-448 without any clipping.
    below = above = 0
    for k in range(400):
        amax = np.float32(0.02 + k * 1.37e-5)
        s = amax / np.float32(448.0)
        w = np.full((2, 32), 0.25, np.float32) * amax
        w[0, 3] = amax; w[1, 7] = -amax; w[1, 9] = np.nextafter(amax, np.float32(0))
        st, wq, _ = oracle.weight_init(w)
        assert st.s_base == s and st.clipped_count == 0
        assert wq[0, 3] == 0x7E and wq[1, 7] == 0xFE
        rounded_down = 448 * Fraction(float(s)) < Fraction(float(amax))
        assert st.overflow_count == (2 if rounded_down else 0) == exact_out_of_range(w, s)
        below += rounded_down; above += not rounded_down
    assert below > 50 and above > 50          # both roundings occur in the sweep


def test_restart_equivalence(oracle):
    snap = {}

    def grab(t, w, st, wq, wq_t):
        if t == 30:
            snap["w"] = w.copy()
            snap["st"] = copy.deepcopy(st)
    w_full, m_full, v_full, st_full, wq_full = small_run(oracle, 60, interval=20, on_step=grab)
    # run 30, copy everything, continue in fresh arrays
    rows, cols = 48, 96
    w = mi.config4_weights(rows, cols, seed=4).copy(); m = np.zeros_like(w); v = np.zeros_like(w)
    st, _, _ = oracle.weight_init(w)
    for t in range(1, 31):
        oracle.weight_step(w, m, v, mi.config4_grad(t, rows, cols, seed=4), args_for(oracle, t, interval=20), st)
    assert np.array_equal(w, snap["w"])
    w2, m2, v2 = w.copy(), m.copy(), v.copy()
    st2 = type(st).from_buffer_copy(bytes(st))
    for t in range(31, 61):
        wq2, _ = oracle.weight_step(w2, m2, v2, mi.config4_grad(t, rows, cols, seed=4),
                                    args_for(oracle, t, interval=20), st2)
    assert np.array_equal(w2, w_full) and np.array_equal(m2, m_full) and np.array_equal(v2, v_full)
    assert np.array_equal(wq2, wq_full)
    assert bytes(st2) == bytes(st_full)


def test_bf16_gradients_equal_expanded_fp32_gradients(oracle):
    rows, cols = 8, 64
    w = mi.config4_weights(rows, cols, seed=6).copy(); m = np.zeros_like(w); v = np.zeros_like(w)
    w2, m2, v2 = w.copy(), m.copy(), v.copy()
    st, _, _ = oracle.weight_init(w); st2, _, _ = oracle.weight_init(w2)
    for t in range(1, 6):
        gb = mi.f32_to_bf16_bits(mi.config4_grad(t, rows, cols, seed=6))
        q1, _ = oracle.weight_step(w, m, v, gb, args_for(oracle, t), st)
        q2, _ = oracle.weight_step(w2, m2, v2, mi.bf16_bits_to_f32(gb), args_for(oracle, t), st2)
        assert np.array_equal(w, w2) and np.array_equal(q1, q2)


def test_zero_weight_tensor(oracle):
    w = np.zeros((4, 32), np.float32)
    st, wq, _ = oracle.weight_init(w)
    assert st.s_base == 0.0 and not wq.any()
