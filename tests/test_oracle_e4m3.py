"""Pins for the oracle's E4M3 codec: a library cast (torch.float8_e4m3fn on CPU),
exact midpoints, saturation and sign rules, and the paper's Delta_max."""
import math
import os
from fractions import Fraction

import numpy as np
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def paper_constants():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def torch_table():
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def test_decode_matches_library_table(oracle):
    ref = torch_table()
    for c in range(256):
        v = oracle.e4m3_decode(c)
        if math.isnan(ref[c]):
            assert math.isnan(v) and c in (0x7F, 0xFF)
        else:
            assert v == ref[c], c
            assert math.copysign(1.0, v) == math.copysign(1.0, ref[c])


def test_max_finite_is_paper_delta_max(oracle):
    k = paper_constants()
    finite = [oracle.e4m3_decode(c) for c in range(256) if c not in (0x7F, 0xFF)]
    assert max(finite) == k["e4m3_max"] == 448.0
    assert oracle.e4m3_decode(0x7E) == 448.0


def test_round_trip_all_codes(oracle):
    for c in range(256):
        if c in (0x7F, 0xFF):
            continue
        assert oracle.e4m3_encode(oracle.e4m3_decode(c)) == c


def test_monotone_and_ties_to_even(oracle):
    # every midpoint between neighbouring positive codes goes to the code with an even
    # mantissa bit; one float64 ulp either side goes to the nearer neighbour
    for c in range(0, 0x7E):
        lo, hi = oracle.e4m3_decode(c), oracle.e4m3_decode(c + 1)
        assert hi > lo
        mid = float((Fraction(lo) + Fraction(hi)) / 2)
        even = c if c % 2 == 0 else c + 1
        assert oracle.e4m3_encode(mid) == even, (c, mid)
        assert oracle.e4m3_encode(-mid) == (even | 0x80)
        assert oracle.e4m3_encode(np.nextafter(mid, hi)) == c + 1
        assert oracle.e4m3_encode(np.nextafter(mid, lo)) == c


def test_saturation_and_signs(oracle):
    for y in (448.0, 448.0000001, 449.0, 463.9, 464.0, 465.0, 480.0, 1e4, 1e30, float(np.finfo(np.float32).max)):
        assert oracle.e4m3_encode(y) == 0x7E, y
        assert oracle.e4m3_encode(-y) == 0xFE, y
    assert oracle.e4m3_encode(0.0) == 0x00
    assert oracle.e4m3_encode(-0.0) == 0x80
    assert oracle.e4m3_encode(-1e-12) == 0x80
    assert oracle.e4m3_encode(2.0 ** -10) == 0x00          # tie between 0 and 2^-9 -> even (0)
    assert oracle.e4m3_encode(np.nextafter(2.0 ** -10, 1.0)) == 0x01
    assert oracle.e4m3_encode(3 * 2.0 ** -10) == 0x02      # tie between codes 1 and 2 -> even
    # NaN codes are never produced from finite input
    rng = np.random.default_rng(0)
    ys = np.concatenate([rng.standard_normal(2000) * 300, rng.standard_normal(2000) * 1e6])
    for y in ys:
        assert oracle.e4m3_encode(float(y)) not in (0x7F, 0xFF)


def test_encode_matches_library_cast_dense_sweep(oracle):
    # torch's CPU cast is round-to-nearest-even without saturation: identical to the
    # oracle wherever |y| <= 464 (above that the library returns NaN, the oracle 448).
    vals = []
    for ex in range(-13, 9):
        m = np.arange(0, 1 << 9, dtype=np.float64) / (1 << 9)
        vals.append((1.0 + m) * 2.0 ** ex)
    vals = np.concatenate(vals)
    rng = np.random.default_rng(1)
    rnd = np.exp(rng.uniform(np.log(1e-5), np.log(464.0), 20000))
    vals = np.concatenate([vals, rnd, [0.0, 448.0, 464.0, 2.0 ** -9, 2.0 ** -10, 1.5 * 2.0 ** -9]])
    vals = vals[vals <= 464.0].astype(np.float32)
    vals = np.concatenate([vals, -vals])
    ref = torch.from_numpy(vals).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(float(v)) for v in vals], np.uint8)
    assert np.array_equal(ref, got)
