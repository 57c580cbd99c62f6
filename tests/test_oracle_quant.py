"""Pins for the oracle's two-level microscaling quantizer (Sec. 3.1, Eq. 2-3):
an exact-rational brute force written independently in Python, the error bound
the rounding implies, metamorphic relations and a special case that reduces to
a plain per-tensor library cast."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import moss_inputs as mi

E4M3_TABLE = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
POS_CODES = [(Fraction(float(E4M3_TABLE[c])), c) for c in range(0x7F)]   # finite, non-negative


def nearest_code_bruteforce(y):
    """Search the whole table for the representable value nearest to the rational y;
    ties -> even code; beyond the largest finite value -> that value."""
    sign = 0x80 if y < 0 else 0
    a = abs(y)
    best, best_d = None, None
    for v, c in POS_CODES:
        d = abs(v - a)
        if best is None or d < best_d or (d == best_d and c % 2 == 0):
            best, best_d = c, d
    return best | sign


def round_fraction_to_bits(p, bits):
    """Round a rational to `bits` significant bits, ties to even, no exponent limit."""
    if p == 0:
        return p
    a = abs(p)
    ex = 0
    while a >= 2:
        a /= 2; ex += 1
    while a < 1:
        a *= 2; ex -= 1
    scaled = a * (1 << (bits - 1))
    fl = scaled.numerator // scaled.denominator
    rem = scaled - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    r = Fraction(fl, 1 << (bits - 1)) * (Fraction(2) ** ex)
    return r if p > 0 else -r


def log2_round_exact(ratio, mode):
    """round(log2(ratio)) (mode 0) or ceil (mode 1) for a rational 0 < ratio <= 1."""
    k = 0
    while Fraction(2) ** k > ratio:          # largest k with 2^k <= ratio
        k -= 1
    if mode == 0:
        # nearest in the log domain: go up when ratio >= sqrt(2) * 2^k
        return k + 1 if ratio * ratio >= Fraction(2) ** (2 * k + 1) else k
    return k if Fraction(2) ** k == ratio else k + 1


def brute_quant(xbits, axis, mode, given_max=None):
    x = mi.bf16_bits_to_f32(xbits).astype(np.float64)
    if axis == 1:
        x = x.T
    outer, inner = x.shape
    amax = np.abs(x).max() if given_max is None else float(given_max)
    s = np.float32(amax) / np.float32(448.0) if amax > 0 else np.float32(1.0)
    with np.errstate(over="ignore"):
        inv_s = np.float32(1.0) / s
    if not np.isfinite(inv_s):                     # reciprocal beyond FP32: largest finite value, zeros stay zero
        inv_s = np.finfo(np.float32).max
    q = np.zeros((outer, inner), np.uint8)
    e = np.zeros((outer, inner // 32), np.uint8)
    for o in range(outer):
        for g in range(inner // 32):
            grp = x[o, g * 32:(g + 1) * 32]
            amax_i = np.abs(grp).max()
            if amax_i == 0:
                k = -127
            else:
                k = max(-127, log2_round_exact(Fraction(float(amax_i)) / Fraction(float(amax)), mode))
            e[o, g] = k + 127
            for j in range(32):
                p = round_fraction_to_bits(Fraction(float(grp[j])) * Fraction(float(inv_s)), 24)
                y = p / (Fraction(2) ** k)
                code = nearest_code_bruteforce(y)
                if grp[j] == 0 and np.signbit(grp[j]):
                    code = 0x80
                q[o, g * 32 + j] = code
    return q, e, s


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("mode", [0, 1])
def test_bruteforce_rational_tiny(oracle, axis, mode):
    rng = np.random.default_rng(10 + axis + 2 * mode)
    x = rng.standard_normal((32, 64)).astype(np.float32) * np.exp(rng.uniform(-6, 3, (32, 1))).astype(np.float32)
    x[:, 40] *= 30
    xb = mi.f32_to_bf16_bits(x)
    q, e, s = oracle.quant_act_2level(xb, axis, mode)
    qb, eb, sb = brute_quant(xb, axis, mode)
    assert s == sb
    assert np.array_equal(e, eb)
    assert np.array_equal(q, qb)


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("mode", [0, 1])
def test_given_maximum(oracle, axis, mode):
    """The tensor maximum handed in by the producer: with the true maximum the result is that of the
    searching quantizer; with a larger bound it is Eq. 2-3 with that bound (exact-rational brute force);
    a value below max|x| is refused."""
    rng = np.random.default_rng(90 + axis + 2 * mode)
    x = rng.standard_normal((32, 64)).astype(np.float32) * np.exp(rng.uniform(-5, 2, (32, 1))).astype(np.float32)
    xb = mi.f32_to_bf16_bits(x)
    true_bits = int((xb & 0x7FFF).max())
    q, e, s = oracle.quant_act_2level(xb, axis, mode)
    q1, e1, s1 = oracle.quant_act_2level_given_max(xb, true_bits, axis, mode)
    assert s1 == s and np.array_equal(q1, q) and np.array_equal(e1, e)
    for bigger in (true_bits + 1, true_bits + 37, true_bits + 3 * 128):      # next value, same binade, three binades up
        bound = float(mi.bf16_bits_to_f32(np.array([bigger], np.uint16))[0])
        q2, e2, s2 = oracle.quant_act_2level_given_max(xb, bigger, axis, mode)
        qb, eb, sb = brute_quant(xb, axis, mode, given_max=bound)
        assert s2 == sb and s2 > s
        assert np.array_equal(e2, eb) and np.array_equal(q2, qb)
    with pytest.raises(Exception):
        oracle.quant_act_2level_given_max(xb, true_bits - 1, axis, mode)


@pytest.mark.parametrize("name", ["zeros", "zero_groups", "one_outlier", "signed_zeros", "tiny", "tiny_zero_groups",
                                  "subnormal", "tiny_groups_under_large_max", "big", "sqrt2_boundary", "wide_range"])
def test_bruteforce_rational_adversarial(oracle, name):
    xb = mi.adversarial_activations(32, 64)[name]
    for axis in (0, 1):
        q, e, s = oracle.quant_act_2level(xb, axis, 0)
        qb, eb, sb = brute_quant(xb, axis, 0)
        assert s == sb, name
        assert np.array_equal(e, eb), name
        assert np.array_equal(q, qb), name


def test_zero_tensor_and_zero_group_conventions(oracle):
    adv = mi.adversarial_activations(32, 64)
    q, e, s = oracle.quant_act_2level(adv["zeros"], 0, 0)
    assert s == np.float32(1.0) and not e.any() and not (q & 0x7F).any()
    q, e, s = oracle.quant_act_2level(adv["zero_groups"], 0, 0)
    assert (e[:, 1] == 0).all() and (e[5] == 0).all()
    assert not (q[:, 32:64] & 0x7F).any()


def test_scales_are_powers_of_two_in_unit_interval(oracle):
    xb = mi.heavy_tailed_activation(64, 256, seed=5)
    for mode in (0, 1):
        q, e, s = oracle.quant_act_2level(xb, 0, mode)
        assert e.max() == 127                       # the group holding the tensor maximum has ss = 1
        assert e.max() <= 127                       # ss_i in (0, 1]  (Sec. 3.1, proof of Thm 1)
        x = mi.bf16_bits_to_f32(xb).astype(np.float64)
        r, c = np.unravel_index(np.abs(x).argmax(), x.shape)
        assert e[r, c // 32] == 127
        assert s == np.float32(np.float32(np.abs(x).max()) / np.float32(448.0))


def _ulp_half_gap(y_abs):
    """Half the spacing of the E4M3 grid at |y| (grid cell that contains it)."""
    y_abs = np.minimum(y_abs, 448.0)
    ex = np.floor(np.log2(np.maximum(y_abs, 2.0 ** -6)))
    return 0.5 * 2.0 ** (ex - 3)


@pytest.mark.parametrize("axis", [0, 1])
def test_half_ulp_error_bound(oracle, axis):
    xb = mi.heavy_tailed_activation(96, 256, seed=6)
    x = mi.bf16_bits_to_f32(xb).astype(np.float64)
    if axis == 1:
        x = x.T
    for mode in (0, 1):
        q, e, s = oracle.quant_act_2level(xb, axis, mode)
        scale = float(s) * 2.0 ** (e.astype(np.int64) - 127)
        scale = np.repeat(scale, 32, axis=1)
        y = x / scale
        dq = oracle.dequant(q, e, s)
        err = np.abs(dq - x) / scale
        bound = _ulp_half_gap(np.abs(y)) + 2.0 ** -21 * np.abs(y)
        ok = np.abs(y) <= 448.0
        assert (err[ok] <= bound[ok]).all()
        if mode == 1:
            assert ok.all()                          # ceil exponents never saturate
        else:
            assert np.abs(y).max() < 448.0 * 1.4143  # nearest: at most sqrt(2) over range
            assert (np.abs(dq[~ok] / scale[~ok]) == 448.0).all()


def test_metamorphic_power_of_two_scaling(oracle):
    xb = mi.heavy_tailed_activation(64, 128, seed=8)
    x = mi.bf16_bits_to_f32(xb)
    q0, e0, s0 = oracle.quant_act_2level(xb, 0, 0)
    for j in (-20, -3, 5, 17):
        q, e, s = oracle.quant_act_2level(mi.f32_to_bf16_bits(x * np.float32(2.0 ** j)), 0, 0)
        assert np.array_equal(q, q0) and np.array_equal(e, e0)
        assert s == np.float32(s0 * np.float32(2.0 ** j))


def test_sign_symmetry_and_group_permutation(oracle):
    xb = mi.heavy_tailed_activation(64, 128, seed=9)
    q0, e0, s0 = oracle.quant_act_2level(xb, 0, 0)
    q, e, s = oracle.quant_act_2level(xb ^ np.uint16(0x8000), 0, 0)
    assert s == s0 and np.array_equal(e, e0) and np.array_equal(q, q0 ^ 0x80)
    perm = np.random.default_rng(0).permutation(4)
    xp = xb.reshape(64, 4, 32)[:, perm].reshape(64, 128)
    q, e, s = oracle.quant_act_2level(xp, 0, 0)
    assert s == s0
    assert np.array_equal(e, e0[:, perm])
    assert np.array_equal(q, q0.reshape(64, 4, 32)[:, perm].reshape(64, 128))


def test_column_grouping_is_row_grouping_of_the_transpose(oracle):
    xb = mi.heavy_tailed_activation(96, 160, seed=11)
    for mode in (0, 1):
        qc, ec, sc = oracle.quant_act_2level(xb, 1, mode)
        qr, er, sr = oracle.quant_act_2level(np.ascontiguousarray(xb.T), 0, mode)
        assert sc == sr and np.array_equal(qc, qr) and np.array_equal(ec, er)
        _, _, s_row = oracle.quant_act_2level(xb, 0, mode)
        assert s_row == sc                           # one global scale per tensor


def test_monotone_within_group(oracle):
    xb = mi.heavy_tailed_activation(32, 64, seed=12)
    x = mi.bf16_bits_to_f32(xb).astype(np.float64)
    q, e, s = oracle.quant_act_2level(xb, 0, 0)
    dq = oracle.dequant(q, e, s)
    for r in range(32):
        for g in range(2):
            xs, ds = x[r, g * 32:(g + 1) * 32], dq[r, g * 32:(g + 1) * 32]
            order = np.argsort(xs, kind="stable")
            assert (np.diff(ds[order]) >= 0).all()


def test_uniform_group_maxima_reduce_to_per_tensor_cast(oracle):
    # if every group reaches the tensor maximum, every ss_i is 1 and the codes are the
    # library's plain cast of fl(x * fl(1/s)).
    rng = np.random.default_rng(13)
    x = rng.uniform(-1, 1, (16, 128)).astype(np.float32)
    x[:, ::32] = 3.0
    xb = mi.f32_to_bf16_bits(x)
    q, e, s = oracle.quant_act_2level(xb, 0, 0)
    assert (e == 127).all()
    xf = mi.bf16_bits_to_f32(xb)
    inv = np.float32(1.0) / s
    ref = torch.from_numpy(xf * inv).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(q, ref)


def test_moss_snr_vs_per_tensor_cast(oracle):
    # soft, synthetic only (Thm 1 is qualitative).  A power-of-two local scale cannot
    # improve the relative precision of a floating-point code, so the gain shows only
    # where a single per-tensor scale pushes small values into E4M3's subnormal /
    # underflow range: never worse, and clearly better once the outliers are large.
    def both(gain):
        xb = mi.heavy_tailed_activation(256, 512, seed=14, outlier_gain=gain)
        x = mi.bf16_bits_to_f32(xb).astype(np.float64)
        q, e, s = oracle.quant_act_2level(xb, 0, 1)
        snr_moss = oracle.snr_db(x, oracle.dequant(q, e, s))
        inv = np.float32(1.0) / s
        qt = torch.from_numpy(mi.bf16_bits_to_f32(xb) * inv).to(torch.float8_e4m3fn).to(torch.float64).numpy()
        return snr_moss, oracle.snr_db(x, qt * float(s))
    moss, tensor = both(100.0)
    assert moss >= tensor - 1e-3 and moss > 25.0
    # restrict the comparison to the non-outlier channels: that is where underflow bites
    xb = mi.heavy_tailed_activation(256, 512, seed=14, outlier_gain=1.0e4)
    x = mi.bf16_bits_to_f32(xb).astype(np.float64)
    small = np.abs(x).max(axis=0) < 1.0e3
    q, e, s = oracle.quant_act_2level(xb, 0, 1)
    dq = oracle.dequant(q, e, s)
    inv = np.float32(1.0) / s
    qt = torch.from_numpy(mi.bf16_bits_to_f32(xb) * inv).to(torch.float8_e4m3fn).to(torch.float64).numpy() * float(s)
    snr_moss = oracle.snr_db(x[:, small], dq[:, small])
    snr_tensor = oracle.snr_db(x[:, small], qt[:, small])
    assert snr_moss > snr_tensor + 3.0


def test_snr_db_closed_forms(oracle):
    """Sec. 3.1, Eq. 4: SNR = 10 log10(E|x|^2 / E|dq - x|^2), pinned to values the mathematics fixes."""
    import math
    # signal 3^2 + 4^2 = 25, noise 1^2: 10 log10 25 (20 log10 would give 27.96, the swapped ratio -13.98)
    assert abs(oracle.snr_db(np.array([3.0, 4.0, 0.0]), np.array([3.0, 4.0, 1.0])) - 13.979400086720377) < 1e-12
    # not symmetric in its arguments: signal 4, noise 1 is 10 log10 4; with the arguments swapped 0 dB
    assert abs(oracle.snr_db(np.array([2.0, 0.0]), np.array([1.0, 0.0])) - 6.020599913279624) < 1e-12
    assert abs(oracle.snr_db(np.array([1.0, 0.0]), np.array([2.0, 0.0]))) < 1e-12
    # a uniform relative error delta on any signal gives -20 log10 delta, whatever the signal
    rng = np.random.default_rng(5)
    x = rng.standard_normal(4096) * 7.0
    for k in (1, 4, 10, 20):
        delta = 2.0 ** -k
        assert abs(oracle.snr_db(x, x * (1.0 + delta)) - 20.0 * k * math.log10(2.0)) < 1e-9
        assert abs(oracle.snr_db(np.ones(33), np.ones(33) * (1.0 - delta)) - 20.0 * k * math.log10(2.0)) < 1e-9
    # the definition with expectations written out (numpy), on unrelated signal and noise
    dq = x + rng.standard_normal(4096) * 0.03
    ref = 10.0 * np.log10(np.mean(x ** 2) / np.mean((dq - x) ** 2))
    assert abs(oracle.snr_db(x, dq) - ref) < 1e-9
    # scaling both by a constant changes nothing; doubling the noise amplitude costs 20 log10 2 dB
    assert abs(oracle.snr_db(3.0 * x, 3.0 * dq) - ref) < 1e-9
    assert abs(oracle.snr_db(x, x + 2.0 * (dq - x)) - (ref - 20.0 * math.log10(2.0))) < 1e-9


def test_groupwise_comparators_against_exact_rationals(oracle):
    """Per-tensor and per-group FP8 (Sec. 3.1, Eq. 5-6 context): scales, codes and dequantized values against a
    brute force over the E4M3 grid in exact rational arithmetic, plus what the definitions imply."""
    from fractions import Fraction
    grid = [(c, Fraction(oracle.e4m3_decode(c))) for c in range(0x7F)]          # non-negative finite codes, ascending values

    def nearest_code(y):                    # y: Fraction; ties to the even code, beyond 448 saturates
        a = abs(y)
        best = min(grid, key=lambda cv: (abs(cv[1] - a), cv[0] & 1))
        return best[0] | (0x80 if y < 0 else 0)
    rng = np.random.default_rng(61)
    x = (rng.standard_t(3.0, size=(6, 64)) * 0.7).astype(np.float32)
    x[2, 5] = 90.0; x[4, :32] = 0.0; x[0, 0] = -0.0
    xb = mi.f32_to_bf16_bits(x)
    xf = mi.bf16_bits_to_f32(xb)
    for group in (0, 64, 32, 16):
        q, scales, dq = oracle.groupwise_fp8(xb, group)
        g = group or xf.size
        blocks = xf.reshape(-1, g)
        assert scales.shape == (blocks.shape[0],)
        for b in range(blocks.shape[0]):
            amax = np.abs(blocks[b]).max()
            s = np.float32(amax) / np.float32(448.0) if amax > 0 else np.float32(1.0)
            assert scales[b] == s
            for j, v in enumerate(blocks[b]):
                code = int(q.reshape(-1, g)[b, j])
                if v == 0:
                    assert code in (0x00, 0x80)
                else:
                    assert code == nearest_code(Fraction(float(v)) / Fraction(float(s))), (group, b, j)
                assert dq.reshape(-1, g)[b, j] == oracle.e4m3_decode(code) * float(s)
            if amax > 0:                    # the largest element of a group sits on the top code
                assert (q.reshape(-1, g)[b] & 0x7F).max() == 0x7E
    # the relative error of a value that is not in the subnormal range of its scale is at most 2^-4 (three mantissa
    # bits, round to nearest), whatever the group size
    for g in (0, 64, 32, 16):
        q, scales, dq = oracle.groupwise_fp8(xb, g)
        s_el = np.repeat(scales, g or xf.size).reshape(xf.shape).astype(np.float64)
        normal = np.abs(xf) >= 2.0 ** -6 * s_el
        assert (np.abs(dq - xf)[normal] <= 2.0 ** -4 * np.abs(xf)[normal] * (1 + 1e-6)).all()
    # a group size that does not divide the row is refused
    with pytest.raises(ValueError):
        oracle.groupwise_fp8(xb, 48)
