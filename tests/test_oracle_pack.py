"""Pins for the oracle's mask / scale / quantize / pack / unpack steps.

Nothing here touches the GPU path.  Each test checks the C oracle against
something other than itself: brute force over all candidate answers, a
hand-worked row, bounds the definition implies, or a pure-Python decoder of
the documented byte layout.
"""
import itertools

import numpy as np
import pytest

from conftest import read_golden
from oracle import slim_oracle as O


def _rng_w(n, k, seed, ties=False):
    rng = np.random.default_rng(seed)
    if ties:
        # few distinct magnitudes, both signs, zeros and negative zeros: every
        # kind of tie shows up many times
        vals = np.array([0.0, -0.0, 0.25, -0.25, 0.5, -0.5, 1.0, -1.0], np.float32)
        return vals[rng.integers(0, len(vals), size=(n, k))]
    return (rng.standard_normal((n, k)) * 0.02).astype(np.float32)


# ---- hand-worked example -----------------------------------------------------

def test_handworked_row():
    g = read_golden("handworked_row.txt")
    w = np.array([float(v) for v in g["w"][0]], np.float32)[None, :]
    mask = O.mask_2of4(w)
    scale = O.row_scale(w)
    codes = O.quantize(w, mask, scale)
    qvals, meta = O.pack(codes, mask)
    assert scale[0] == np.float32(float(g["scale"][0][0]))
    assert mask[0].tolist() == [int(v) for v in g["mask"][0]]
    assert codes[0].tolist() == [int(v) for v in g["codes"][0]]
    assert qvals[0].tolist() == [int(v, 16) for v in g["qvals"][0]]
    assert meta[0].tolist() == [int(v, 16) for v in g["meta"][0]]
    x = np.array([float(v) for v in g["x"][0]], np.float64)[None, :]
    y = O.forward(O.PackedLayer(qvals, meta, scale), None, None, x)
    assert y.shape == (1, 1) and y[0, 0] == float(g["y"][0][0])
    # the tie case (two groups needed for k % 8: repeat it)
    tw = np.array([float(v) for v in g["tie_w"][0]] * 2, np.float32)[None, :]
    assert O.mask_2of4(tw)[0].tolist() == [int(v) for v in g["tie_mask"][0]] * 2


# ---- mask ----------------------------------------------------------------------

def _brute_force_pair(a4):
    """Of the 6 position pairs, the valid ones are those whose members are all
    >= every non-member in magnitude; the expected answer is the
    lexicographically smallest valid pair."""
    for pair in itertools.combinations(range(4), 2):
        rest = [i for i in range(4) if i not in pair]
        if all(a4[p] >= a4[q] for p in pair for q in rest):
            return pair
    raise AssertionError("no valid pair")


@pytest.mark.parametrize("ties", [False, True])
def test_mask_brute_force(ties):
    W = _rng_w(24, 64, seed=11 + ties, ties=ties)
    mask = O.mask_2of4(W)
    A = np.abs(W)
    for o in range(W.shape[0]):
        for g in range(W.shape[1] // 4):
            want = _brute_force_pair(A[o, 4 * g:4 * g + 4])
            got = tuple(np.nonzero(mask[o, 4 * g:4 * g + 4])[0].tolist())
            assert got == want, (o, g, W[o, 4 * g:4 * g + 4])


def test_mask_all_six_patterns_and_all_value_orders():
    # every permutation of 4 distinct magnitudes, and every tie pattern of
    # magnitudes drawn from {0, 1, 2}: 24 + 81 groups
    groups = [list(p) for p in itertools.permutations([1.0, 2.0, 3.0, 4.0])]
    groups += [list(p) for p in itertools.product([0.0, 1.0, 2.0], repeat=4)]
    groups += [[0.0, -0.0, 0.0, -0.0]]
    if len(groups) % 2:
        groups.append([0.0] * 4)
    W = np.array(groups, np.float32).reshape(1, -1)
    W[:, ::3] *= -1.0
    mask = O.mask_2of4(W)
    for g, vals in enumerate(groups):
        got = tuple(np.nonzero(mask[0, 4 * g:4 * g + 4])[0].tolist())
        assert got == _brute_force_pair(np.abs(np.array(vals))), (g, vals)


def test_mask_invariants_large():
    W = _rng_w(128, 1024, seed=5)
    mask = O.mask_2of4(W)
    m4 = mask.reshape(128, -1, 4)
    assert (m4.sum(-1) == 2).all()
    A = np.abs(W).reshape(128, -1, 4)
    kept_min = np.where(m4 == 1, A, np.inf).min(-1)
    drop_max = np.where(m4 == 0, A, -np.inf).max(-1)
    assert (drop_max <= kept_min).all()


# ---- scale -----------------------------------------------------------------------

def test_scale_pins():
    W = _rng_w(64, 256, seed=7)
    W[3] = 0.0
    s = O.row_scale(W)
    mask = O.mask_2of4(W)
    amax = np.abs(W).max(1)
    # the row maximum survives the mask, so the scale does not depend on
    # whether it is taken before or after pruning
    assert (np.abs(W * mask).max(1) == amax).all()
    assert s.dtype == np.float32 and s[3] == np.float32(1.0)
    rows = np.arange(64) != 3
    seven_s = (s.astype(np.float64) * 7.0)[rows]
    ulp = np.spacing(amax[rows]).astype(np.float64)
    assert (np.abs(seven_s - amax[rows].astype(np.float64)) <= ulp).all()
    # correctly rounded quotient: the exact a/7 lies within half an ulp of s
    exact = amax[rows].astype(np.float64) / 7.0
    assert (np.abs(s[rows].astype(np.float64) - exact) <= 0.5 * np.spacing(s[rows]).astype(np.float64)).all()


# ---- codes -----------------------------------------------------------------------

def test_code_pins():
    W = _rng_w(64, 512, seed=9)
    mask = O.mask_2of4(W)
    s = O.row_scale(W)
    codes = O.quantize(W, mask, s)
    assert codes.dtype == np.int8
    assert codes.min() >= -8 and codes.max() <= 7
    assert (codes[mask == 0] == 0).all()
    # the row maximum quantizes to exactly +-7
    j = np.abs(W).argmax(1)
    top = codes[np.arange(64), j]
    assert (np.abs(top) == 7).all()
    assert (np.sign(top) == np.sign(W[np.arange(64), j])).all()
    # uniform-quantizer error bound for kept entries: |w - c s| <= s/2
    err = np.abs(W.astype(np.float64) - codes.astype(np.float64) * s.astype(np.float64)[:, None])
    bound = 0.5 * s.astype(np.float64)[:, None] * (1 + 1e-6)
    assert (err[mask == 1] <= np.broadcast_to(bound, err.shape)[mask == 1]).all()
    # sign symmetry: quantizing -W negates every code (round-half-even is odd)
    codes_neg = O.quantize(-W, mask, s)
    assert (codes_neg == -codes).all()


def test_rounding_is_half_to_even_and_clamped():
    # scale 1.0 (row max 7): exact halves must go to the even neighbour
    w = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 6.5,
                   3.5, 4.5, 5.5, -6.5, -3.5, -4.5, -5.5, -7.0]], np.float32)
    mask = np.ones_like(w, dtype=np.uint8)       # quantize() itself takes any mask
    s = O.row_scale(w)
    assert s[0] == 1.0
    c = O.quantize(w, mask, s)
    assert c[0].tolist() == [7, 0, 2, 2, 0, -2, -2, 6, 4, 4, 6, -6, -4, -4, -6, -7]
    # the clamp: a scale smaller than max/7 pushes values outside [-8, 7]
    c2 = O.quantize(w, mask, np.array([0.5], np.float32))
    assert c2.min() == -8 and c2.max() == 7
    assert c2[0, 0] == 7 and c2[0, -1] == -8 and c2[0, 1] == 1


# ---- pack / unpack ---------------------------------------------------------------

def _python_decode(qrow, mrow, k):
    """Decoder of the canonical layout written from its description, in Python
    integers: per group g, byte qrow[g] holds the code of the lower kept
    position in its low nibble and of the higher one in its high nibble
    (two's complement); nibble (g & 1) of mrow[g >> 1] holds i0 | (i1 << 2)."""
    codes = [0] * k
    mask = [0] * k
    for g in range(k // 4):
        b = int(qrow[g])
        nib = (int(mrow[g >> 1]) >> (4 * (g & 1))) & 0xF
        i0, i1 = nib & 3, nib >> 2
        for pos, v in ((i0, b & 0xF), (i1, b >> 4)):
            codes[4 * g + pos] = v - 16 if v >= 8 else v
            mask[4 * g + pos] = 1
    return codes, mask


def test_pack_against_python_decoder():
    W = _rng_w(6, 64, seed=21)
    mask = O.mask_2of4(W)
    s = O.row_scale(W)
    codes = O.quantize(W, mask, s)
    qvals, meta = O.pack(codes, mask)
    assert qvals.shape == (6, 16) and meta.shape == (6, 8)
    for o in range(6):
        c, m = _python_decode(qvals[o], meta[o], 64)
        assert c == codes[o].tolist()
        assert m == mask[o].tolist()


def test_pack_unpack_round_trip_and_metadata_range():
    W = _rng_w(64, 512, seed=23, ties=False)
    Wt = _rng_w(64, 512, seed=24, ties=True)
    for w in (W, Wt):
        mask = O.mask_2of4(w)
        s = O.row_scale(w)
        codes = O.quantize(w, mask, s)
        qvals, meta = O.pack(codes, mask)
        c2, m2 = O.unpack(qvals, meta)
        assert (c2 == codes).all() and (m2 == mask).all()
        q2, me2 = O.pack(c2, m2)
        assert (q2 == qvals).all() and (me2 == meta).all()
        nib = np.stack([meta & 0xF, meta >> 4], -1)
        i0, i1 = nib & 3, nib >> 2
        assert (i0 < i1).all()
        # only 6 of the 16 nibble values can occur
        assert set(np.unique(nib).tolist()) <= {0x4, 0x8, 0xC, 0x9, 0xD, 0xE}


def test_unpack_pack_identity_on_arbitrary_valid_bytes():
    rng = np.random.default_rng(31)
    valid = np.array([0x4, 0x8, 0xC, 0x9, 0xD, 0xE], np.uint8)
    n, k = 16, 256
    qvals = rng.integers(0, 256, size=(n, k // 4), dtype=np.uint8)
    lo = valid[rng.integers(0, 6, size=(n, k // 8))]
    hi = valid[rng.integers(0, 6, size=(n, k // 8))]
    meta = (lo | (hi << 4)).astype(np.uint8)
    codes, mask = O.unpack(qvals, meta)
    assert codes.min() >= -8 and codes.max() <= 7
    assert (mask.reshape(n, -1, 4).sum(-1) == 2).all()
    q2, m2 = O.pack(codes, mask)
    assert (q2 == qvals).all() and (m2 == meta).all()


def test_pack_rejects_bad_mask_and_shapes():
    codes = np.zeros((2, 8), np.int8)
    mask = np.zeros((2, 8), np.uint8)
    mask[:, [0, 1, 4]] = 1                      # second group has one kept entry
    with pytest.raises(ValueError):
        O.pack(codes, mask)
    with pytest.raises(ValueError):
        O.mask_2of4(np.zeros((2, 6), np.float32))


def test_dequant_is_code_times_scale():
    W = _rng_w(8, 64, seed=41)
    layer = O.compress(W)
    codes, mask = O.unpack(layer.qvals, layer.meta)
    Wd = O.dequant(layer.qvals, layer.meta, layer.scale)
    assert Wd.dtype == np.float64
    want = codes.astype(np.float64) * layer.scale.astype(np.float64)[:, None]
    assert (Wd == want).all()
    # reconstruction error bound on kept entries, zero on dropped ones
    assert (Wd[mask == 0] == 0).all()
    err = np.abs(Wd - W)[mask == 1]
    assert (err <= np.broadcast_to(0.5 * layer.scale[:, None] * (1 + 1e-6), W.shape)[mask == 1]).all()


def test_all_zero_row_and_group():
    W = np.zeros((2, 16), np.float32)
    W[1, 8:] = [0, 0, 0, 0, 1, 0, 0, 0]
    layer = O.compress(W)
    assert layer.scale[0] == 1.0
    assert (layer.qvals[0] == 0).all()
    # zero groups keep positions 0 and 1: nibble 0 | (1 << 2) = 4
    assert (layer.meta[0] == 0x44).all()
    # group [1,0,0,0] keeps 0 and 1 as well; code 7 in the low nibble
    assert layer.qvals[1, 3] == 0x07 and layer.meta[1, 1] == 0x44
