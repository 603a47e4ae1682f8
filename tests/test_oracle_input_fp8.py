"""Pins of the oracle's FP8 input quantization (App. "Input Quantization"): the two formats' value
sets built from their bit definition (every code decoded by hand), nearest-value rounding against
brute force over that set, ties to even, limits, the switch of format, idempotence and the error
bound of each format."""
import numpy as np
import pytest

from oracle import slim_oracle as O


def _all_values(exp_bits, man_bits, bias, e4m3):
    """Finite non-negative values of an 8-bit float from its bit fields."""
    vals = []
    for code in range(128):
        e, m = code >> man_bits, code & ((1 << man_bits) - 1)
        if e4m3:
            if code == 0x7F:                     # the only NaN of E4M3; there are no infinities
                continue
        elif e == (1 << exp_bits) - 1:           # E5M2 keeps IEEE's infinities and NaNs
            continue
        vals.append(m * 2.0 ** (1 - bias - man_bits) if e == 0 else (1 + m / (1 << man_bits)) * 2.0 ** (e - bias))
    return np.array(sorted(vals))


E4M3 = _all_values(4, 3, 7, True)
E5M2 = _all_values(5, 2, 15, False)


def test_value_sets():
    assert E4M3.max() == 448 and E4M3[1] == 2.0 ** -9 and len(E4M3) == 127
    assert E5M2.max() == 57344 and E5M2[1] == 2.0 ** -16 and len(E5M2) == 124
    for fmt, vals in (("e4m3", E4M3), ("e5m2", E5M2)):
        assert np.array_equal(O.fp8_round(vals, fmt), vals)              # representable values stay
        assert np.array_equal(O.fp8_round(-vals, fmt), -vals)


@pytest.mark.parametrize("fmt,vals", [("e4m3", E4M3), ("e5m2", E5M2)])
def test_rounding_is_nearest_value_by_brute_force(fmt, vals):
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.uniform(0, vals.max(), 4000), rng.uniform(0, vals[8], 2000), 10.0 ** rng.uniform(-6, 4.6, 4000)])
    x = x[x <= vals.max()]
    got = O.fp8_round(x, fmt)
    d = np.abs(x[:, None] - vals[None, :])
    best = d.min(axis=1)
    assert np.all(np.abs(got - x) <= best * (1 + 1e-12))
    assert np.all(np.isin(got, vals))
    # midpoints go to the neighbour with the even mantissa: every second value of the set
    mid = (vals[:-1] + vals[1:]) / 2
    r = O.fp8_round(mid, fmt)
    even = np.where(np.arange(len(vals) - 1) % 2 == 0, vals[:-1], vals[1:])
    assert np.array_equal(r, even)
    # beyond the largest value: limited, not infinite
    assert O.fp8_round(np.array([vals.max() * 1.5, -1e9]), fmt).tolist() == [vals.max(), -vals.max()]


def test_input_quant_format_switch_scale_and_bounds():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((16, 256)).astype(np.float16)
    Xq, s, fmt = O.input_quant_fp8(X)
    M = np.float32(np.abs(X.astype(np.float32)).max())
    assert fmt == "e4m3" and s == np.float32(M / np.float32(448))
    # 3 mantissa bits: relative error at most 2^-4 for values that are normal after scaling (+ the fp16 rounding)
    xf = X.astype(np.float64)
    big = np.abs(xf) >= float(s) * 2.0 ** -6
    assert np.all(np.abs(Xq.astype(np.float64) - xf)[big] <= np.abs(xf)[big] * (2.0 ** -4 + 2.0 ** -10))
    assert np.abs(Xq.astype(np.float64)).max() == float(M)                 # the maximum is kept exactly
    # an outlier beyond 448 switches the format: 2 mantissa bits
    X2 = X.copy()
    X2[3, 7] = np.float16(900.0)
    Xq2, s2, fmt2 = O.input_quant_fp8(X2)
    assert fmt2 == "e5m2" and s2 == np.float32(np.float32(900.0) / np.float32(57344.0))
    big2 = np.abs(X2.astype(np.float64)) >= float(s2) * 2.0 ** -14
    err = np.abs(Xq2.astype(np.float64) - X2.astype(np.float64))
    assert np.all(err[big2] <= np.abs(X2.astype(np.float64))[big2] * (2.0 ** -3 + 2.0 ** -10))
    assert Xq2[3, 7] == np.float16(900.0)
    # exactly 448 stays E4M3 with scale 1: the values then are the format's own
    X3 = np.array([[448.0, 1.0, 0.3, -17.0, 2.0 ** -9, 2.0 ** -11]], np.float16)
    Xq3, s3, fmt3 = O.input_quant_fp8(X3)
    assert fmt3 == "e4m3" and s3 == 1.0
    assert Xq3.tolist() == [[448.0, 1.0, 0.3125, -16.0, 2.0 ** -9, 0.0]]
    # a zero tensor
    Z, sz, fz = O.input_quant_fp8(np.zeros((2, 8), np.float16))
    assert sz == 1.0 and fz == "e4m3" and not Z.any()


def test_input_quant_is_idempotent_when_the_scale_is_a_power_of_two():
    rng = np.random.default_rng(3)
    X = (rng.standard_normal((8, 128)) * 3).astype(np.float16)
    X[0, 0] = np.float16(448.0 / 64)              # max -> scale 2^-6: scaling is exact
    X = np.clip(X, -7, 7).astype(np.float16)
    Xq, s, fmt = O.input_quant_fp8(X)
    assert s == np.float32(2.0 ** -6)
    Xqq, s2, _ = O.input_quant_fp8(Xq)
    assert s2 == s and np.array_equal(Xqq, Xq)


def test_signed_zero_is_kept():
    """Both formats have a negative zero: -0 stays -0, and a negative value below half the smallest
    subnormal rounds to -0 (IEEE 754 round to nearest), through the whole quantizer as well."""
    for fmt in ("e4m3", "e5m2"):
        r = O.fp8_round(np.array([-0.0, 0.0, -1e-9, 1e-9]), fmt)
        assert np.array_equal(np.signbit(r), [True, False, True, False]) and not r.any()
    X = np.array([[1.0, -0.0, 0.0, -6e-8, 6e-8]], np.float16)        # 6e-8: the smallest fp16 subnormal
    Xq, _, _ = O.input_quant_fp8(X)
    assert Xq.view(np.uint16).tolist() == [[0x3C00, 0x8000, 0x0000, 0x8000, 0x0000]]


def _decode(code, exp_bits, man_bits, bias):
    """Value of one 8-bit code from its bit fields (finite codes only)."""
    sign = -1.0 if code & 0x80 else 1.0
    e, m = (code & 0x7F) >> man_bits, code & ((1 << man_bits) - 1)
    return sign * (m * 2.0 ** (1 - bias - man_bits) if e == 0 else (1 + m / (1 << man_bits)) * 2.0 ** (e - bias))


@pytest.mark.parametrize("fmt,exp_bits,man_bits,bias", [("e4m3", 4, 3, 7), ("e5m2", 5, 2, 15)])
def test_codes_are_the_bit_fields_of_the_values(fmt, exp_bits, man_bits, bias):
    """fp8_encode against a decoder written from the formats' bit definition: every finite code decodes to a
    value whose code it is (both signs, both zeros), so encode is the inverse of the definition."""
    finite = [c for c in range(256) if not ((fmt == "e4m3" and (c & 0x7F) == 0x7F) or
                                             (fmt == "e5m2" and ((c & 0x7F) >> man_bits) == (1 << exp_bits) - 1))]
    vals = np.array([_decode(c, exp_bits, man_bits, bias) for c in finite])
    assert np.array_equal(O.fp8_encode(vals, fmt), np.array(finite, np.uint8))
    # a few known codes: 1.0, the largest value, the smallest subnormal, -2.0
    known = {"e4m3": {1.0: 0x38, 448.0: 0x7E, 2.0 ** -9: 0x01, -2.0: 0xC0},
             "e5m2": {1.0: 0x3C, 57344.0: 0x7B, 2.0 ** -16: 0x01, -2.0: 0xC0}}[fmt]
    for v, c in known.items():
        assert int(O.fp8_encode(np.array([v]), fmt)[0]) == c
    with pytest.raises(AssertionError):
        O.fp8_encode(np.array([1.0 + 2.0 ** -(man_bits + 1)]), fmt)           # not on the grid


def test_input_quant_codes_decode_to_the_quantized_values():
    rng = np.random.default_rng(4)
    for X in (rng.standard_normal((8, 200)).astype(np.float16), (rng.standard_normal((4, 64)) * 300).astype(np.float16),
              np.zeros((2, 16), np.float16)):
        codes, s, fmt = O.input_quant_fp8_codes(X)
        Xq, s2, fmt2 = O.input_quant_fp8(X)
        assert s == s2 and fmt == fmt2 and codes.dtype == np.uint8 and codes.shape == X.shape
        eb, mb, bias = (4, 3, 7) if fmt == "e4m3" else (5, 2, 15)
        vals = np.array([_decode(int(c), eb, mb, bias) for c in codes.ravel()]).reshape(X.shape)
        # the values the codes stand for, times the scale and rounded to fp16, are the quantizer's fp16 output
        assert np.array_equal((vals.astype(np.float32) * s).astype(np.float32).astype(np.float16).view(np.uint16) & 0x7FFF,
                              Xq.view(np.uint16) & 0x7FFF)
        assert np.array_equal(np.signbit(vals), np.signbit(Xq.astype(np.float32)))
