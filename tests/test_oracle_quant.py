"""Pins for the INT8 KV quantiser oracle (CPU only).

Paper section 2.2: K and V are cached as INT8 with one scale per token per head.  The
definition used here: symmetric, scale = fl32(amax/127), code = RNE(fl32(x/scale)),
clamped to +-127.  The oracle's fp32 arithmetic is pinned against exact rational
arithmetic, hand cases with power-of-two scales, constructed ties, and exhaustive sweeps
of both divisions over bf16 inputs.
"""
from fractions import Fraction

import numpy as np
import pytest

from paper_2407_07304_amd.inputs import f32_to_bf16_bits, bf16_bits_to_f32, normal_bf16


def _bits(vals):
    b = f32_to_bf16_bits(np.asarray(vals, dtype=np.float32))
    assert np.array_equal(bf16_bits_to_f32(b), np.asarray(vals, dtype=np.float32)), "not bf16-representable"
    return b


def _round_half_even(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def _fl32(fr: Fraction) -> Fraction:
    """Exact round-to-nearest-even of a rational to the fp32 grid (subnormals included)."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    quantum = Fraction(2) ** (max(e, -126) - 23)
    return sign * _round_half_even(a / quantum) * quantum


def exact_quant_row(x_f32_row):
    xs = [Fraction(float(x)) for x in x_f32_row]
    amax = max(abs(x) for x in xs)
    if amax == 0:
        return [0] * len(xs), Fraction(0)
    scale = _fl32(amax / 127)
    codes = []
    for x in xs:
        c = _round_half_even(_fl32(x / scale))
        codes.append(max(-127, min(127, c)))
    return codes, scale


def test_quantiser_matches_exact_rational_arithmetic(oracle):
    rng = np.random.default_rng(21)
    rows = normal_bf16(rng, (40, 16))
    # a few rows at other magnitudes, including bf16 subnormals
    rows[30] = f32_to_bf16_bits((rng.standard_normal(16) * 1e-3).astype(np.float32))
    rows[31] = f32_to_bf16_bits((rng.standard_normal(16) * 1e4).astype(np.float32))
    rows[32] = np.array([0x0001, 0x0002, 0x8003, 0x0010, 0x007f, 0x0080, 0x8081, 0, 0, 0, 0, 0, 0, 0, 0, 0x0040],
                        dtype=np.uint16)
    codes, scales = oracle.kv_quant_int8(rows)
    xf = bf16_bits_to_f32(rows)
    for r in range(rows.shape[0]):
        want_codes, want_scale = exact_quant_row(xf[r])
        assert Fraction(float(scales[r])) == want_scale, r
        assert codes[r].tolist() == want_codes, r


def test_power_of_two_scales_and_exact_codes(oracle):
    for kexp in (-20, -3, 0, 5):
        s = 2.0 ** kexp
        ints = np.array([127, -127, 0, 1, -1, 64, -100, 3], dtype=np.float32)
        codes, scales = oracle.kv_quant_int8(_bits(ints * s)[None, :])
        assert scales[0] == np.float32(s)
        assert codes[0].tolist() == ints.astype(int).tolist()


def test_single_nonzero_gets_full_range_and_zero_row_is_all_zero(oracle):
    x = np.zeros((3, 8), dtype=np.float32)
    x[0, 2] = 0.3710937500  # bf16-representable
    x[1, 5] = -12.5
    codes, scales = oracle.kv_quant_int8(_bits(x))
    assert codes[0].tolist() == [0, 0, 127, 0, 0, 0, 0, 0]
    assert codes[1].tolist() == [0, 0, 0, 0, 0, -127, 0, 0]
    assert scales[0] == np.float32(0.37109375) / np.float32(127) and scales[1] == np.float32(12.5) / np.float32(127)
    assert scales[2] == 0 and not codes[2].any()


def test_ties_round_to_even(oracle):
    # amax = 127 -> scale = 1 exactly, so x/scale = x; n + 0.5 is bf16-representable for n <= 127.
    halves = np.array([0.5, 1.5, 2.5, 3.5, 4.5, 125.5, 126.5, -0.5, -1.5, -2.5, -126.5, 127.0], dtype=np.float32)
    codes, scales = oracle.kv_quant_int8(_bits(halves)[None, :])
    assert scales[0] == 1.0
    assert codes[0].tolist() == [0, 2, 2, 4, 4, 126, 126, 0, -2, -2, -126, 127]
    # same at scale 2^-4
    codes, scales = oracle.kv_quant_int8(_bits(halves / 16)[None, :])
    assert scales[0] == np.float32(1 / 16)
    assert codes[0].tolist() == [0, 2, 2, 4, 4, 126, 126, 0, -2, -2, -126, 127]


def test_invariants_on_normal_data(oracle):
    rng = np.random.default_rng(22)
    rows = normal_bf16(rng, (4096, 128))
    codes, scales = oracle.kv_quant_int8(rows)
    x = bf16_bits_to_f32(rows).astype(np.float64)
    assert codes.min() >= -127 and codes.max() <= 127
    assert (np.abs(codes.astype(np.int32)).max(axis=1) == 127).all()
    # the position of the +-127 is the position of amax, with its sign
    am = np.argmax(np.abs(x), axis=1)
    picked = codes[np.arange(len(am)), am].astype(np.int32)
    assert np.array_equal(picked, 127 * np.sign(x[np.arange(len(am)), am]).astype(np.int32))
    err = np.abs(x - codes.astype(np.float64) * scales.astype(np.float64)[:, None])
    bound = scales.astype(np.float64)[:, None] * (0.5 + 2.0 ** -17)
    assert (err <= bound).all()
    assert np.array_equal(scales, (np.abs(bf16_bits_to_f32(rows)).max(axis=1) / np.float32(127)).astype(np.float32))


def test_c_and_numpy_quantisers_agree_bit_for_bit(oracle):
    rng = np.random.default_rng(23)
    rows = normal_bf16(rng, (2000, 64))
    rows[:50] = rng.integers(0, 0x7f80, (50, 64)).astype(np.uint16) | (rng.integers(0, 2, (50, 64)).astype(np.uint16) << 15)
    rows[50:60] = rng.integers(0, 0x0100, (10, 64)).astype(np.uint16)  # subnormal and tiny
    rows[60] = 0
    c1, s1 = oracle.kv_quant_int8(rows)
    c2, s2 = oracle.kv_quant_int8_np(rows)
    assert np.array_equal(s1.view(np.uint32), s2.view(np.uint32))
    assert np.array_equal(c1, c2)


def test_exhaustive_scale_division_sweep_numpy():
    # every positive finite bf16 amax: fp32 division == fp64 quotient narrowed once
    bits = np.arange(1, 0x7f80, dtype=np.uint16)
    amax = bf16_bits_to_f32(bits)
    s32 = (amax / np.float32(127)).astype(np.float32)
    s64 = (amax.astype(np.float64) / 127.0).astype(np.float32)
    assert np.array_equal(s32.view(np.uint32), s64.view(np.uint32))
    assert (s32 > 0).all()


def test_exhaustive_division_sweeps_c(oracle):
    # all ~5.3e8 (x, amax) bf16 pairs with |x| <= amax, and all amax; a few seconds in C
    bad_scale, bad_quo, pairs = oracle.quant_division_sweep(1)
    assert pairs == sum(range(2, 0x7f7f + 2))
    assert bad_scale == 0 and bad_quo == 0


def test_shapes_and_layout(oracle):
    rng = np.random.default_rng(24)
    x = normal_bf16(rng, (2, 3, 5, 64))
    codes, scales = oracle.kv_quant_int8(x)
    assert codes.shape == (2, 3, 5, 64) and scales.shape == (2, 3, 5)
    c_row, s_row = oracle.kv_quant_int8(x[1, 2, 4][None, :])
    assert np.array_equal(codes[1, 2, 4], c_row[0]) and scales[1, 2, 4] == s_row[0]
