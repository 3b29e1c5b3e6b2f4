"""Pins of the INT8 KV-cache oracle (per-head, per-token symmetric quantization)."""
import numpy as np
import pytest

import workloads as wl
from oracle.kv_int8 import dequantize_rows, quantize_rows


def test_row_whose_largest_magnitude_is_127_keeps_integers():
    # amax = 127 -> inv = 1, s = 1: integers are their own codes, halves round to even
    x = np.array([[127.0, -3.0, 0.5, 1.5, 2.5, -0.5, -1.5, 64.25]], np.float32)
    codes, s = quantize_rows(x)
    assert s[0] == 1.0
    assert codes[0].tolist() == [127, -3, 0, 2, 2, 0, -2, 64]


def test_largest_element_maps_to_plus_or_minus_127_and_scale_is_amax_over_127():
    rng = np.random.default_rng(0)
    x = wl.bf16_bits_to_f32(wl.to_bf16_bits(rng.standard_normal((50, 128)).astype(np.float32)))
    codes, s = quantize_rows(x)
    amax = np.abs(x).max(-1)
    np.testing.assert_array_equal(s, (amax / np.float32(127)).astype(np.float32))
    assert (np.abs(codes).max(-1) == 127).all()
    j = np.abs(x).argmax(-1)
    assert (np.sign(codes[np.arange(50), j]) == np.sign(x[np.arange(50), j])).all()


def test_error_is_at_most_half_a_step_and_zero_rows_stay_zero():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((20, 64)) * rng.uniform(0.01, 30, size=(20, 1))).astype(np.float32)
    x[3] = 0
    codes, s = quantize_rows(x)
    xh = dequantize_rows(codes, s)
    assert (np.abs(xh - x) <= 0.5 * s[:, None] * (1 + 1e-5)).all()
    assert (codes[3] == 0).all() and s[3] == 0 and (xh[3] == 0).all()


def test_symmetry_scaling_by_powers_of_two_and_idempotence():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((10, 128)).astype(np.float32)
    c1, s1 = quantize_rows(x)
    c2, s2 = quantize_rows(-x)
    assert (c2 == -c1).all() and (s2 == s1).all()                     # symmetric quantizer
    c3, s3 = quantize_rows(x * np.float32(8))                         # exact scaling: same codes, 8x the scale
    assert (c3 == c1).all() and (s3 == s1 * 8).all()
    c4, s4 = quantize_rows(dequantize_rows(c1, s1))                   # represented values quantize to themselves
    assert (c4 == c1).all()
    np.testing.assert_allclose(s4, s1, rtol=1e-6)


def test_against_exact_rational_arithmetic_away_from_ties():
    # the codes are round(127 x / amax) in exact arithmetic wherever that is not within fp32 error of a tie
    from fractions import Fraction
    rng = np.random.default_rng(3)
    x = wl.bf16_bits_to_f32(wl.to_bf16_bits(rng.standard_normal((4, 32)).astype(np.float32)))
    codes, _ = quantize_rows(x)
    for r in range(4):
        amax = max(abs(Fraction(float(v))) for v in x[r])
        for d in range(32):
            t = Fraction(float(x[r, d])) * 127 / amax
            frac = abs(t - round(t))
            if abs(frac - Fraction(1, 2)) > Fraction(1, 10000):
                assert codes[r, d] == round(t)


def test_planted_mistakes_are_caught():
    x = np.array([[127.0, 0.6, 1.5, -2.7]], np.float32)
    codes, _ = quantize_rows(x)
    assert codes[0].tolist() == [127, 1, 2, -3]
    assert np.trunc(x[0]).astype(int).tolist() != codes[0].tolist()          # truncation
    assert np.floor(x[0] + 0.5).astype(int).tolist() == [127, 1, 2, -3]       # half-up agrees here ...
    y = np.array([[127.0, 0.5, 2.5]], np.float32)
    assert quantize_rows(y)[0][0].tolist() == [127, 0, 2]                     # ... but not at ties: half to even
