"""Pins of the bfloat16-storage oracle against things that are not the oracle: PyTorch's CPU
float32 -> bfloat16 conversion, the integer carry trick on the float32 bit pattern, closed forms
worked out by hand from the 2- and 3-tap Winograd forms, and the FP64 definition of the convolution
on inputs whose transforms are exactly representable."""
import numpy as np
import pytest
import torch

import oracle

H8 = 2.0 ** -8  # half a step of the 8-bit significand at 1.0


def _bits_to_f64(bits16):
    """bfloat16 bit patterns -> their values (a bfloat16 is the upper half of a float32)."""
    with np.errstate(invalid="ignore"):  # signalling-NaN patterns
        return (np.asarray(bits16, np.uint32) << 16).view(np.float32).astype(np.float64)


def _torch_round(a32):
    return torch.from_numpy(np.ascontiguousarray(a32, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def _carry_round(a32):
    """Round-to-nearest-even by integer arithmetic on the float32 pattern (finite inputs)."""
    b = np.ascontiguousarray(a32, np.float32).view(np.uint32).astype(np.uint64)
    r = (b + 0x7FFF + ((b >> 16) & 1)) >> 16
    return _bits_to_f64(r.astype(np.uint32))


def test_round_fixed_points_all_bit_patterns():
    vals = _bits_to_f64(np.arange(65536, dtype=np.uint32))
    finite = np.isfinite(vals)
    out = oracle.round_bfloat16(vals[finite])
    assert np.array_equal(out, vals[finite])
    assert np.array_equal(np.signbit(out), np.signbit(vals[finite]))


def test_round_midpoints_go_to_even():
    # every pair of adjacent non-negative finite bfloat16 values: the midpoint is a tie
    bits = np.arange(0, 0x7F7F, dtype=np.uint32)
    lo, hi = _bits_to_f64(bits), _bits_to_f64(bits + 1)
    mid = 0.5 * (lo + hi)  # exact in double
    want = np.where(bits % 2 == 0, lo, hi)
    assert np.array_equal(oracle.round_bfloat16(mid), want)
    assert np.array_equal(oracle.round_bfloat16(-mid), -want)
    assert np.array_equal(oracle.round_bfloat16(np.nextafter(mid, np.inf)), hi)
    assert np.array_equal(oracle.round_bfloat16(np.nextafter(mid, -np.inf)), lo)
    # the midpoints are float32 values, so the library conversion is a single rounding there too
    assert np.array_equal(_torch_round(mid.astype(np.float32)), want)


def test_round_random_against_torch_and_the_carry_trick():
    rng = np.random.default_rng(5)
    for scale in (1e-40, 1e-38, 1e-30, 1e-8, 1e-2, 1.0, 1e2, 3e4, 1e20, 1e38):
        with np.errstate(over="ignore"):
            a = (rng.standard_normal(20000) * scale).astype(np.float32)  # float32 values: one rounding in the library
        got = oracle.round_bfloat16(a.astype(np.float64))
        assert np.array_equal(got, _torch_round(a)), scale
        fin = np.isfinite(_carry_round(a))
        assert np.array_equal(got[fin], _carry_round(a)[fin]), scale


def test_round_directly_from_double():
    # values that a detour through float32 would round twice: just above a bfloat16 tie by less than
    # half a float32 step -> the tie-break must not happen
    x = (1.0 + H8) + 2.0 ** -40
    assert oracle.round_bfloat16(np.array([x]))[0] == 1.0 + 2 * H8
    assert float(np.float32(x)) == 1.0 + H8  # the detour lands on the tie ...
    assert _torch_round(np.array([np.float32(x)]))[0] == 1.0  # ... and then goes to even
    x = (1.0 + 3 * H8) - 2.0 ** -40
    assert oracle.round_bfloat16(np.array([x]))[0] == 1.0 + 2 * H8


def test_round_limits():
    big = (2.0 - 2.0 ** -7) * 2.0 ** 127   # largest finite bfloat16
    edge = (2.0 - 2.0 ** -8) * 2.0 ** 127  # half a step above it
    tiny = 2.0 ** -133                     # smallest subnormal
    a = np.array([big, np.nextafter(edge, 0), edge, 1e300, -edge, tiny, tiny / 2, tiny / 2 * 1.001, 1.5 * tiny,
                  0.0, -0.0, np.inf, -np.inf])
    out = oracle.round_bfloat16(a)
    assert out[0] == big and out[1] == big and out[2] == np.inf and out[3] == np.inf and out[4] == -np.inf
    assert out[5] == tiny and out[6] == 0.0 and out[7] == tiny and out[8] == 2 * tiny
    assert out[9] == 0.0 and np.signbit(out[10]) and out[11] == np.inf and out[12] == -np.inf
    assert np.isnan(oracle.round_bfloat16(np.array([np.nan]))[0])


# ---------------------------------------------------------------------------------------
# where the rounding sits: closed forms from the 2-tap form
#   y0 = (d0-d1) g0 + d1 (g0+g1),   y1 = d1 (g0+g1) + (d2-d1) g1
# ---------------------------------------------------------------------------------------
def _conv_1x2(d, g):
    x = np.array(d, np.float32).reshape(1, 1, 1, 3)
    w = np.array(g, np.float32).reshape(1, 1, 1, 2)
    return oracle.dwm_bf16_f64(x, w, 1, 0).reshape(-1), oracle.direct_f64(x, w, 1, 0).reshape(-1)


def test_filter_side_rounded_before_product():
    h = H8
    # g0+g1 = 1+2^-8 is a tie between 1 and 1+2^-7 -> 1 (even): y0 = (d0-d1) + d1 = d0
    yh, yd = _conv_1x2([0.5, 1.0, 0.25], [1.0, h])
    assert yd[0] == 0.5 + h and yd[1] == 1.0 + 0.25 * h
    assert yh[0] == 0.5
    assert yh[1] == 1.0 * 1.0 + (0.25 - 1.0) * h  # d1*round(g0+g1) + (d2-d1)*g1
    # 1+3*2^-8 is a tie between 1+2^-7 and 1+2^-6 -> the even one, 1+2^-6
    yh, _ = _conv_1x2([0.0, 1.0, 1.0], [1.0, 3 * h])
    assert yh[0] == -1.0 + (1.0 + 4 * h)


def test_input_side_rounded_before_product():
    h = H8
    yh, yd = _conv_1x2([1.0, -h, 0.0], [1.0, 0.0])  # d0-d1 = 1+2^-8 -> 1
    assert yd[0] == 1.0
    assert yh[0] == 1.0 - h
    yh, yd = _conv_1x2([0.0, -h, 1.0], [0.0, 1.0])  # d2-d1 = 1+2^-8 -> 1 on the other output
    assert yd[1] == 1.0
    assert yh[1] == 1.0 - h


def test_three_tap_filter_rounding():
    # printed F(2,3): U = [g0, (g0+g1+g2)/2, (g0-g1+g2)/2, g2], V = [d0-d2, d1+d2, d2-d1, d1-d3],
    # y0 = m1+m2+m3, y1 = m2-m3-m4.  g = (1, 2^-8, 0): U1 = (1+2^-8)/2 is a tie -> 1/2,
    # U2 = 1/2 - 2^-9 is exact.  d = (0,1,0,0): V = [0, 1, -1, 1].
    h = H8
    x = np.array([0.0, 1.0, 0.0, 0.0], np.float32).reshape(1, 1, 1, 4)
    w = np.array([1.0, h, 0.0], np.float32).reshape(1, 1, 1, 3)
    yh = oracle.dwm_bf16_f64(x, w, 1, 0).reshape(-1)
    yd = oracle.direct_f64(x, w, 1, 0).reshape(-1)
    assert yd[0] == h and yd[1] == 1.0
    assert yh[0] == 0.5 - (0.5 - h / 2)
    assert yh[1] == 0.5 + (0.5 - h / 2)


def test_it_is_not_the_binary16_rounding():
    # 1 + 2^-9 survives binary16 (11 bits) but not bfloat16 (8 bits): g0+g1 -> 1
    x = np.array([0.0, 1.0, 0.0], np.float32).reshape(1, 1, 1, 3)
    w = np.array([1.0, 2.0 ** -9], np.float32).reshape(1, 1, 1, 2)
    # (w[1] = 2^-9 is a bfloat16 value; only the SUM g0+g1 needs more bits)
    yb = oracle.dwm_bf16_f64(x, w, 1, 0).reshape(-1)
    yh = oracle.dwm_half_f64(x, w, 1, 0).reshape(-1)
    assert yb[0] == -1.0 + 1.0          # (d0-d1) g0 + d1 round(g0+g1) with the sum rounded to 1
    assert yh[0] == -1.0 + (1.0 + 2.0 ** -9)


def test_input_transform_is_evaluated_in_binary32_before_its_rounding():
    """As for binary16 (same layer, same derivation: y00 = V00 + c + b with V00 the rounded a - b - c), with
    bfloat16's 8 significant bits: a = 1 + 2^-6, b = 2^-8, c = 2^-24.  a - b = 1 + 2^-7 + 2^-8 is the midpoint of
    1 + 2^-7 and 1 + 2^-6; exactly, a - b - c rounds down to 1 + 2^-7; in binary32 it ties to a - b, whose
    bfloat16 tie goes to the even 1 + 2^-6."""
    a, b, c = 1 + 2.0 ** -6, 2.0 ** -8, 2.0 ** -24
    x = np.zeros((1, 1, 4, 4), np.float32)
    x[0, 0, 0, 0], x[0, 0, 2, 0], x[0, 0, 0, 2] = a, b, c
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 0, 0] = 1.0
    yb = oracle.dwm_bf16_f64(x, w, 1, 0)
    assert oracle.direct_f64(x, w, 1, 0)[0, 0, 0, 0] == a
    assert yb[0, 0, 0, 0] == (1 + 2.0 ** -6) + c + b
    assert yb[0, 0, 0, 0] != (1 + 2.0 ** -7) + c + b
    x[0, 0, 0, 2] = 2.0 ** -16  # every sum exact in binary32: the exact value's rounding
    assert oracle.dwm_bf16_f64(x, w, 1, 0)[0, 0, 0, 0] == (1 + 2.0 ** -7) + 2.0 ** -16 + b


def test_sums_are_not_rounded():
    x = np.array([1.0, 2.0 ** -15], np.float32).reshape(1, 2, 1, 1)
    w = np.array([1.0, 2.0 ** -15], np.float32).reshape(1, 2, 1, 1)
    assert oracle.dwm_bf16_f64(x, w, 1, 0)[0, 0, 0, 0] == 1.0 + 2.0 ** -30


def test_inputs_must_be_bfloat16():
    x = np.full((1, 1, 4, 4), 0.1, np.float32)
    w = np.ones((1, 1, 3, 3), np.float32)
    with pytest.raises(ValueError):
        oracle.dwm_bf16_f64(x, w, 1, 1)
    oracle.dwm_bf16_f64(_torch_round(x).astype(np.float32), w, 1, 1)


@pytest.mark.parametrize("R,S,stride,pad", [(3, 3, 1, 1), (5, 5, 1, 2), (7, 7, 2, 3), (3, 3, 2, 1), (11, 11, 4, 0),
                                            (4, 6, 3, 2), (1, 1, 1, 0), (2, 2, 1, 0)])
def test_small_integers_equal_definition(R, S, stride, pad):
    # transforms of small integers stay below 2^8: the rounding is the identity, the result the definition
    rng = np.random.default_rng(R * 100 + S * 10 + stride)
    H = max(R + 5, 12)
    x = rng.integers(-4, 5, size=(2, 3, H, H + 1)).astype(np.float32)
    w = (4 * rng.integers(-3, 4, size=(4, 3, R, S))).astype(np.float32)  # G's 1/2 * 1/2 stays integral
    assert np.array_equal(oracle.dwm_bf16_f64(x, w, stride, pad), oracle.direct_f64(x, w, stride, pad))


@pytest.mark.parametrize("R,stride,pad", [(3, 1, 1), (5, 1, 2), (7, 2, 3)])
def test_error_scale(R, stride, pad):
    rng = np.random.default_rng(R)
    C = 16
    x = _torch_round(rng.uniform(-1, 1, size=(2, C, 20, 20)).astype(np.float32)).astype(np.float32)
    w = _torch_round((rng.standard_normal((8, C, R, R)) * np.sqrt(2.0 / (C * R * R))).astype(np.float32)).astype(np.float32)
    yb = oracle.dwm_bf16_f64(x, w, stride, pad)
    yd = oracle.direct_f64(x, w, stride, pad)
    err = np.max(np.abs(yb - yd)) / np.max(np.abs(yd))
    assert 1e-5 < err < 8 * 2.0 ** -8
    rms = np.sqrt(np.mean((yb - yd) ** 2)) / np.sqrt(np.mean(yd ** 2))
    assert 2.0 ** -11 < rms < 2 * 2.0 ** -8
    # eight times coarser than binary16 storage of the same data would be
    yh = oracle.dwm_half_f64(x, w, stride, pad)  # bfloat16 values are binary16 values here (|x| < 1: exponents fit)
    rms16 = np.sqrt(np.mean((yh - yd) ** 2)) / np.sqrt(np.mean(yd ** 2))
    assert 3 < rms / rms16 < 20
