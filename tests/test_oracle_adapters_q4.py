"""Pins of the oracle's adapter group quantizer (Sec. 3.3): a hand-worked row,
exact rational arithmetic on small inputs, and the invariants of an AbsMax
quantizer.  No GPU."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import slim_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "handworked_adapter_group.txt")


def _rand(rows, cols, seed, scale=0.01):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((rows, cols)) * scale).astype(np.float16)


def test_handworked_row():
    idx, val, code = [], [], []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        i, v, c = line.split()
        idx.append(int(i)); val.append(float(v)); code.append(int(c))
    A = np.zeros((1, 132), np.float16)
    A[0, idx] = np.array(val, np.float16)
    assert np.array_equal(A[0, idx].astype(np.float64), np.array(val))       # the fixture is exact in binary16
    codes, scales = O.quantize_adapter(A)
    assert scales.shape == (1, 2)
    assert float(scales[0, 0]) == 0.125 and float(scales[0, 1]) == 0.0078125
    assert codes[0, idx].tolist() == code
    rest = np.setdiff1d(np.arange(132), idx)
    assert not codes[0, rest].any()


def test_against_exact_rational_arithmetic():
    """Every step redone with fractions: scale = binary16(binary32(max / 7)), code
    = round-half-even(binary32(a / scale)), clamped."""
    A = _rand(3, 300, 1, scale=0.3)
    A[1, 5] = np.float16(0.0)
    codes, scales = O.quantize_adapter(A)
    for r in range(A.shape[0]):
        for g in range(scales.shape[1]):
            seg = A[r, g * 128:(g + 1) * 128]
            amax = max(abs(Fraction(float(x))) for x in seg)
            s32 = np.float32(float(amax / 7))                   # correctly rounded twice = once: 11-bit operands
            s16 = np.float16(s32)
            assert float(scales[r, g]) == float(s16)
            for j, x in enumerate(seg):
                q = Fraction(float(x)) / Fraction(float(s16))
                q32 = Fraction(float(np.float32(float(q))))
                lo = q32.numerator // q32.denominator               # floor
                frac = q32 - lo
                rounded = lo + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and lo % 2 == 1) else 0)
                assert int(codes[r, g * 128 + j]) == max(-8, min(7, rounded))


@pytest.mark.parametrize("rows,cols", [(7, 128), (5, 416), (3, 130), (2, 4096), (1, 1)])
def test_invariants(rows, cols):
    A = _rand(rows, cols, rows * 1000 + cols)
    codes, scales = O.quantize_adapter(A)
    assert codes.dtype == np.int8 and scales.dtype == np.float16
    assert scales.shape == (rows, (cols + 127) // 128)
    assert codes.min() >= -8 and codes.max() <= 7
    D = O.dequantize_adapter(codes, scales)
    for g in range(scales.shape[1]):
        sl = slice(g * 128, min(cols, (g + 1) * 128))
        a = A[:, sl].astype(np.float64)
        s = scales[:, g].astype(np.float64)[:, None]
        amax = np.abs(a).max(axis=1)
        # the stored scale is max / 7 within half a binary16 ulp (relative 2^-11, plus the binary32 rounding)
        nz = amax > 0
        assert np.all(np.abs(s[nz, 0] - amax[nz] / 7) <= (amax[nz] / 7) * (2.0 ** -11 + 2.0 ** -23))
        # an element is reproduced within half a step (a hair more: the quotient is rounded to binary32)
        assert np.all(np.abs(D[:, sl] - a) <= s * (0.5 + 1e-6))
        # the largest element of a group gets code +-7
        j = np.abs(a).argmax(axis=1)
        top = codes[:, sl][np.arange(rows), j]
        assert np.all(np.abs(top[nz]) == 7)


def test_zero_group_and_tiny_group():
    A = np.zeros((2, 256), np.float16)
    A[0, 130] = np.float16(2.0 ** -24)          # smallest subnormal: max / 7 rounds to zero in binary16
    A[1, 0] = np.float16(1.0)
    codes, scales = O.quantize_adapter(A)
    assert float(scales[0, 0]) == 1.0 and not codes[0, :128].any()        # a group of zeros: scale 1, codes 0
    assert float(scales[0, 1]) == 2.0 ** -24 and int(codes[0, 130]) == 1  # the scale never becomes zero
    assert float(scales[1, 1]) == 1.0
    assert int(codes[1, 0]) == 7


def test_sign_symmetry():
    A = _rand(6, 500, 9)
    c1, s1 = O.quantize_adapter(A)
    c2, s2 = O.quantize_adapter(-A)
    assert np.array_equal(s1.view(np.uint16), s2.view(np.uint16))
    # rint is odd; the clamp is not (-8 exists, +8 does not), but |quotient| <= 7.004 never reaches it
    assert np.array_equal(c1, -c2)


def test_exact_reconstruction_on_a_power_of_two_grid():
    """A matrix that already lies on a 4-bit grid with a power-of-two step, with a
    +-7 in every group, comes back as exactly those codes and that step."""
    rng = np.random.default_rng(12)
    rows, cols = 5, 300
    codes = rng.integers(-7, 8, size=(rows, cols)).astype(np.int8)
    steps = np.array([2.0 ** -7, 2.0 ** -3, 2.0 ** -11], np.float64)          # one per group of the row
    for r in range(rows):
        for g in range(3):
            j = g * 128 + int(rng.integers(0, min(128, cols - g * 128)))
            codes[r, j] = 7 if (r + g) % 2 else -7
    A = np.empty((rows, cols), np.float64)
    for g in range(3):
        A[:, g * 128:(g + 1) * 128] = codes[:, g * 128:(g + 1) * 128] * steps[g]
    A16 = A.astype(np.float16)
    assert np.array_equal(A16.astype(np.float64), A)
    c, s = O.quantize_adapter(A16)
    assert np.array_equal(c, codes)
    assert np.array_equal(s.astype(np.float64), np.broadcast_to(steps, (rows, 3)))
    assert np.array_equal(O.dequantize_adapter(c, s), A)


def test_groups_do_not_leak_into_each_other():
    A = _rand(2, 384, 4)
    B = A.copy()
    B[:, 128:256] *= np.float16(8.0)
    ca, sa = O.quantize_adapter(A)
    cb, sb = O.quantize_adapter(B)
    for g in (0, 2):
        assert np.array_equal(ca[:, g * 128:(g + 1) * 128], cb[:, g * 128:(g + 1) * 128])
        assert np.array_equal(sa[:, g].view(np.uint16), sb[:, g].view(np.uint16))
    assert np.array_equal(ca[:, 128:256], cb[:, 128:256])       # a power-of-two factor moves only the scale
    assert np.array_equal((sa[:, 1].astype(np.float32) * 8).astype(np.float16).view(np.uint16), sb[:, 1].view(np.uint16))


def test_forward_with_quantized_adapters_is_the_forward_of_their_dequantized_values():
    """The layer with 4-bit adapters is, by definition, the layer whose adapters
    are the dequantized matrices: the oracle's forward takes them as they are."""
    rng = np.random.default_rng(5)
    W = rng.standard_normal((48, 256)).astype(np.float32) * 0.02
    L = _rand(48, 20, 6); R = _rand(20, 256, 7)
    X = rng.standard_normal((3, 256)).astype(np.float16)
    lc, ls = O.quantize_adapter(L); rc, rs = O.quantize_adapter(R)
    Ld, Rd = O.dequantize_adapter(lc, ls), O.dequantize_adapter(rc, rs)
    layer = O.compress(W)
    Y = O.forward(layer, Ld, Rd, X)
    Wd = O.dequant(layer.qvals, layer.meta, layer.scale)
    ref = X.astype(np.float64) @ (Wd + Ld @ Rd).T
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-12)
