"""Pins of the half-precision-storage oracle (Table 1, "DWM FP16" column) against things that
are not the oracle: numpy's own binary16 conversion, closed forms worked out by hand from the
2-tap and 1-tap Winograd forms, and the FP64 definition of the convolution on inputs whose
transforms are exactly representable."""
import numpy as np
import pytest

import oracle


# ---------------------------------------------------------------------------------------
# round_binary16 against numpy's float64 -> float16 conversion
# ---------------------------------------------------------------------------------------
def _np_round(a):
    with np.errstate(over="ignore"):
        return np.asarray(a, np.float64).astype(np.float16).astype(np.float64)


def test_round_fixed_points_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    finite = np.isfinite(vals)
    out = oracle.round_binary16(vals[finite])
    assert np.array_equal(out, vals[finite])
    assert np.array_equal(np.signbit(out), np.signbit(vals[finite]))


def test_round_midpoints_go_to_even():
    # every pair of adjacent non-negative finite binary16 values: the midpoint is a tie
    bits = np.arange(0, 0x7BFF, dtype=np.uint16)
    lo = bits.view(np.float16).astype(np.float64)
    hi = (bits + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = 0.5 * (lo + hi)  # exact in double
    want = np.where(bits % 2 == 0, lo, hi)  # the one whose last significand bit is 0
    assert np.array_equal(oracle.round_binary16(mid), want)
    assert np.array_equal(oracle.round_binary16(-mid), -want)
    # a hair off the tie goes to the nearer one
    assert np.array_equal(oracle.round_binary16(np.nextafter(mid, np.inf)), hi)
    assert np.array_equal(oracle.round_binary16(np.nextafter(mid, -np.inf)), lo)


def test_round_random_against_numpy():
    rng = np.random.default_rng(5)
    for scale in (1e-8, 1e-6, 1e-4, 1e-2, 1.0, 1e2, 3e4, 7e4):
        a = rng.standard_normal(20000) * scale
        assert np.array_equal(oracle.round_binary16(a), _np_round(a))


def test_round_limits():
    a = np.array([65504.0, 65519.999, 65520.0, 1e9, -65520.0, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.001,
                  1.5 * 2.0 ** -24, 0.0, -0.0, np.inf, -np.inf])
    out = oracle.round_binary16(a)
    assert np.array_equal(out, _np_round(a))
    assert out[2] == np.inf and out[4] == -np.inf and out[6] == 0.0 and out[7] == 2.0 ** -24
    assert out[8] == 2.0 ** -23  # tie between 1 and 2 steps of 2^-24 -> even
    assert np.isnan(oracle.round_binary16(np.array([np.nan]))[0])


# ---------------------------------------------------------------------------------------
# where the rounding sits: closed forms from the 2-tap form
#   y0 = (d0-d1) g0 + d1 (g0+g1),   y1 = d1 (g0+g1) + (d2-d1) g1
# ---------------------------------------------------------------------------------------
def _conv_1x2(d, g):
    x = np.array(d, np.float32).reshape(1, 1, 1, 3)
    w = np.array(g, np.float32).reshape(1, 1, 1, 2)
    return oracle.dwm_half_f64(x, w, 1, 0).reshape(-1), oracle.direct_f64(x, w, 1, 0).reshape(-1)


def test_filter_side_rounded_before_product():
    h = 2.0 ** -11
    # g0+g1 = 1+2^-11 is a tie between 1 and 1+2^-10 -> 1 (even): y0 = (d0-d1) + d1 = d0
    yh, yd = _conv_1x2([0.5, 1.0, 0.25], [1.0, h])
    assert yd[0] == 0.5 + h and yd[1] == 1.0 + 0.25 * h
    assert yh[0] == 0.5
    assert yh[1] == 1.0 * 1.0 + (0.25 - 1.0) * h  # d1*round(g0+g1) + (d2-d1)*g1
    # 1+3*2^-11 is a tie between 1+2^-10 and 1+2^-9 -> the even one, 1+2^-9
    yh, _ = _conv_1x2([0.0, 1.0, 1.0], [1.0, 3 * h])
    assert yh[0] == -1.0 + (1.0 + 4 * h)


def test_input_side_rounded_before_product():
    h = 2.0 ** -11
    # d0-d1 = 1+2^-11 -> 1: y0 = 1*g0 + d1*(g0+g1)
    yh, yd = _conv_1x2([1.0, -h, 0.0], [1.0, 0.0])
    assert yd[0] == 1.0
    assert yh[0] == 1.0 - h
    # d2-d1 = 1+2^-11 -> 1 on the other output
    yh, yd = _conv_1x2([0.0, -h, 1.0], [0.0, 1.0])
    assert yd[1] == 1.0
    assert yh[1] == 1.0 - h


def test_three_tap_filter_rounding():
    # printed F(2,3): U = [g0, (g0+g1+g2)/2, (g0-g1+g2)/2, g2], V = [d0-d2, d1+d2, d2-d1, d1-d3],
    # y0 = m1+m2+m3, y1 = m2-m3-m4.  g = (1, 2^-11, 0): U1 = (1+2^-11)/2 is a tie -> 1/2,
    # U2 = 1/2 - 2^-12 is exact.  d = (0,1,0,0): V = [0, 1, -1, 1].
    h = 2.0 ** -11
    x = np.array([0.0, 1.0, 0.0, 0.0], np.float32).reshape(1, 1, 1, 4)
    w = np.array([1.0, h, 0.0], np.float32).reshape(1, 1, 1, 3)
    yh = oracle.dwm_half_f64(x, w, 1, 0).reshape(-1)
    yd = oracle.direct_f64(x, w, 1, 0).reshape(-1)
    assert yd[0] == h and yd[1] == 1.0
    assert yh[0] == 0.5 - (0.5 - h / 2)
    assert yh[1] == 0.5 + (0.5 - h / 2)


def test_input_transform_is_evaluated_in_binary32_before_its_rounding():
    """The reading's precision for V (the paper fixes none): B^T d B in binary32, columns first, then ONE
    rounding to binary16.  It differs from rounding the exact value only where a sum spans more than 13
    binades.  3x3 filter with the single tap g00 = 1 on a 4x4 input: U = G e0 (G e0)^T with G e0 =
    (1, 1/2, 1/2, 0), and with d00 = a, d20 = b, d02 = c the transform is
    V = [[a-b-c, c, c, 0], [b, 0, 0, 0], [b, 0, 0, 0], 0], so y00 = V00 + (c + c)/2 + (b + b)/2.
    a = 1 + 2^-9, b = 2^-11, c = 2^-24: a - b = 1 + 2^-10 + 2^-11 is the midpoint of 1 + 2^-10 and 1 + 2^-9;
    the exact a - b - c lies below it (-> 1 + 2^-10), in binary32 it is a tie at 2^-24 that goes to the even
    neighbour a - b, and the binary16 tie there goes to the even 1 + 2^-9."""
    a, b, c = 1 + 2.0 ** -9, 2.0 ** -11, 2.0 ** -24
    x = np.zeros((1, 1, 4, 4), np.float32)
    x[0, 0, 0, 0], x[0, 0, 2, 0], x[0, 0, 0, 2] = a, b, c
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 0, 0] = 1.0
    assert np.float32(np.float32(a) - np.float32(b)) - np.float32(c) == np.float32(a - b)  # the binary32 tie
    yh = oracle.dwm_half_f64(x, w, 1, 0)
    assert oracle.direct_f64(x, w, 1, 0)[0, 0, 0, 0] == a
    assert yh[0, 0, 0, 0] == (1 + 2.0 ** -9) + c + b
    assert yh[0, 0, 0, 0] != (1 + 2.0 ** -10) + c + b  # what rounding the exact a - b - c would give
    # where every sum is exact in binary32 the two evaluations agree: the same case with c = 2^-20
    x[0, 0, 0, 2] = 2.0 ** -20
    assert oracle.dwm_half_f64(x, w, 1, 0)[0, 0, 0, 0] == (1 + 2.0 ** -10) + 2.0 ** -20 + b


def test_sums_are_not_rounded():
    # 1x1 kernel: no transform, y = sum_c d_c g_c; 1 + 2^-30 needs 31 bits
    x = np.array([1.0, 2.0 ** -15], np.float32).reshape(1, 2, 1, 1)
    w = np.array([1.0, 2.0 ** -15], np.float32).reshape(1, 2, 1, 1)
    y = oracle.dwm_half_f64(x, w, 1, 0)
    assert y[0, 0, 0, 0] == 1.0 + 2.0 ** -30


def test_inputs_must_be_binary16():
    x = np.full((1, 1, 4, 4), 0.1, np.float32)
    w = np.ones((1, 1, 3, 3), np.float32)
    with pytest.raises(ValueError):
        oracle.dwm_half_f64(x, w, 1, 1)
    oracle.dwm_half_f64(x.astype(np.float16), w, 1, 1)


# ---------------------------------------------------------------------------------------
# exactly representable transforms: the rounding is the identity, result = definition
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("R,S,stride,pad", [(3, 3, 1, 1), (5, 5, 1, 2), (7, 7, 2, 3), (3, 3, 2, 1), (11, 11, 4, 0),
                                            (4, 6, 3, 2), (1, 1, 1, 0), (2, 2, 1, 0)])
def test_small_integers_equal_definition(R, S, stride, pad):
    rng = np.random.default_rng(R * 100 + S * 10 + stride)
    H = max(R + 5, 12)
    x = rng.integers(-4, 5, size=(2, 3, H, H + 1)).astype(np.float32)
    w = (4 * rng.integers(-3, 4, size=(4, 3, R, S))).astype(np.float32)  # G's 1/2 * 1/2 stays integral
    yh = oracle.dwm_half_f64(x, w, stride, pad)
    assert np.array_equal(yh, oracle.direct_f64(x, w, stride, pad))


# ---------------------------------------------------------------------------------------
# generic data: the error has the size binary16 storage gives, and no more
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("R,stride,pad", [(3, 1, 1), (5, 1, 2), (7, 2, 3)])
def test_error_scale(R, stride, pad):
    rng = np.random.default_rng(R)
    C = 16
    x = rng.uniform(-1, 1, size=(2, C, 20, 20)).astype(np.float16)
    w = (rng.standard_normal((8, C, R, R)) * np.sqrt(2.0 / (C * R * R))).astype(np.float16)
    yh = oracle.dwm_half_f64(x, w, stride, pad)
    yd = oracle.direct_f64(x.astype(np.float32), w.astype(np.float32), stride, pad)
    y2 = oracle.dwm_f64(x.astype(np.float32), w.astype(np.float32), stride, pad)
    assert np.max(np.abs(y2 - yd)) < 1e-12
    err = np.max(np.abs(yh - yd)) / np.max(np.abs(yd))
    # every product carries two relative roundings of at most 2^-11 each, of Winograd-domain values
    # that are sums of up to four inputs / nine taps: a small multiple of 2^-11 overall
    assert 1e-6 < err < 8 * 2.0 ** -11
    rms = np.sqrt(np.mean((yh - yd) ** 2)) / np.sqrt(np.mean(yd ** 2))
    assert 2.0 ** -14 < rms < 2 * 2.0 ** -11
