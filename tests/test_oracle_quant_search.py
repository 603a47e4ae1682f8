"""Pins of the oracle's SLiM-Quant scale search (Sec. 3.1, Eq. 4-7, Alg. 1) and of
the saliency-weighted 2:4 mask.  No GPU."""
import numpy as np
import pytest

from oracle import slim_oracle as O


def test_bins_rule():
    # App. "Implementation Details": max(512, min(numel / 1000, 20000))
    assert O.quant_bins(512 * 512) == 512
    assert O.quant_bins(4096 * 4096) == 16777
    assert O.quant_bins(28672 * 8192) == 20000
    assert O.quant_bins(10) == 512


def test_histogram_counts_by_brute_force():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((40, 300)).astype(np.float32)
    counts, M = O.quant_histogram(W)
    assert counts.sum() == W.size and float(M) == float(np.abs(W).max())
    B = counts.shape[0]
    mine = np.zeros(B, np.int64)
    inv = np.float32(np.float32(B) / M)
    for v in np.abs(W).ravel():
        mine[min(B - 1, int(np.floor(np.float32(v) * inv)))] += 1
    assert np.array_equal(mine, counts)
    assert counts[-1] >= 1                     # the maximum itself lands in the last bin


def test_error_is_the_mse_of_the_quantizer_when_the_weights_sit_on_bin_centres():
    """Weights placed exactly on the centres of the histogram: the integral over the
    histogram is then the plain sum of squared errors of quantizing those weights with
    step alpha / 7 and clipping at alpha, computed here element by element."""
    B = 512
    M = 2.0
    centres = (np.arange(B) + 0.5) * (M / B)
    reps = np.random.default_rng(2).integers(0, 5, size=B)
    w = np.repeat(centres, reps)
    counts = reps.astype(np.int64)
    for alpha in (2.0, 1.3, 0.37, 0.05):
        step = alpha / 7
        total = 0.0
        for x in w:
            q = min(7, int(np.rint(x / step)))             # codes 0..7 on magnitudes
            total += (q * step - x) ** 2
        assert np.isclose(O.quant_error(counts, np.float32(M), alpha), total, rtol=1e-12)


def test_a_few_outliers_are_clipped():
    """Most of the mass near zero and a handful of large values: AbsMax wastes the grid on
    the outliers, the search picks an alpha far below the maximum and a smaller error."""
    rng = np.random.default_rng(3)
    W = (rng.standard_normal((600, 1000)) * 0.01).astype(np.float32)
    W[0, :4] = [1.0, -1.0, 0.9, 0.8]
    alpha, scale = O.quant_search(W)
    counts, M = O.quant_histogram(W)
    assert float(M) == 1.0
    assert float(alpha) < 0.2
    assert O.quant_error(counts, M, float(alpha)) < 0.25 * O.quant_error(counts, M, 1.0)
    assert float(scale) == float(np.float32(alpha) / np.float32(7.0))


def test_alpha_is_the_first_minimum_over_the_candidates_and_never_worse_than_absmax():
    rng = np.random.default_rng(4)
    W = rng.laplace(size=(300, 700)).astype(np.float32)
    alpha, _ = O.quant_search(W)
    counts, M = O.quant_histogram(W)
    eta = float(M) / 10
    coarse = [eta * i for i in range(1, 11)]
    e = [O.quant_error(counts, M, a) for a in coarse]
    lo = coarse[int(np.argmin(e))]
    fine = [lo + eta * (j / 10.0) for j in range(-10, 11)]
    fine = [a for a in fine if 0 < a <= float(M)]
    allc = coarse + fine
    best = min(O.quant_error(counts, M, a) for a in allc)
    assert O.quant_error(counts, M, float(alpha)) <= best * (1 + 1e-6)      # alpha is stored as binary32
    assert O.quant_error(counts, M, float(alpha)) <= O.quant_error(counts, M, float(M)) * (1 + 1e-6)
    assert np.float32(alpha) in [np.float32(a) for a in allc]


def test_scale_equivariance_and_symmetries():
    rng = np.random.default_rng(5)
    W = rng.standard_normal((128, 512)).astype(np.float32)
    a1, s1 = O.quant_search(W)
    a2, s2 = O.quant_search(W * np.float32(8.0))               # a power of two: exact
    assert float(a2) == 8.0 * float(a1) and float(s2) == 8.0 * float(s1)
    a3, _ = O.quant_search(-W)
    a4, _ = O.quant_search(W[::-1, ::-1])
    assert float(a3) == float(a1) and float(a4) == float(a1)


def test_zero_tensor():
    alpha, scale = O.quant_search(np.zeros((8, 64), np.float32))
    assert float(alpha) == 0.0 and float(scale) == 1.0


def test_quantizing_with_the_searched_scale_lowers_the_true_error():
    """The real test of the whole chain: codes computed with scale = alpha* / 7 (clamp now
    acting) reproduce a heavy-tailed W with a smaller squared error than AbsMax / 7."""
    rng = np.random.default_rng(6)
    W = rng.standard_t(3, size=(256, 1024)).astype(np.float32)
    keep = np.ones_like(W, np.uint8)
    _, s = O.quant_search(W)
    per_tensor = np.full(W.shape[0], s, np.float32)
    absmax = np.full(W.shape[0], np.float32(np.abs(W).max()) / np.float32(7.0), np.float32)
    e_search = np.sum((O.quantize(W, keep, per_tensor) * per_tensor[:, None].astype(np.float64) - W) ** 2)
    e_absmax = np.sum((O.quantize(W, keep, absmax) * absmax[:, None].astype(np.float64) - W) ** 2)
    assert e_search < 0.5 * e_absmax


# ---- saliency-weighted mask -----------------------------------------------------------

def test_saliency_mask_brute_force_and_special_cases():
    rng = np.random.default_rng(7)
    W = rng.standard_normal((16, 64)).astype(np.float32)
    sal = rng.uniform(0.1, 5.0, size=64).astype(np.float32)
    mask = O.mask_2of4(W, sal)
    assert np.all(mask.reshape(16, 16, 4).sum(axis=2) == 2)
    for o in range(16):
        for g in range(16):
            metric = (np.abs(W[o, 4 * g:4 * g + 4]) * sal[4 * g:4 * g + 4]).astype(np.float32)
            order = sorted(range(4), key=lambda i: (-float(metric[i]), i))
            want = np.zeros(4, np.uint8)
            want[order[:2]] = 1
            assert np.array_equal(mask[o, 4 * g:4 * g + 4], want)
    # a constant saliency is the magnitude mask; a zero saliency on two inputs drops them
    assert np.array_equal(O.mask_2of4(W, np.full(64, 2.0, np.float32)), O.mask_2of4(W))
    z = np.ones(64, np.float32)
    z[0::4] = 0
    z[1::4] = 0
    m = O.mask_2of4(W, z)
    assert not m[:, 0::4].any() and not m[:, 1::4].any()


def test_absmax_is_a_candidate_and_wins_when_the_weights_lie_on_its_grid():
    """Weights on the 4-bit grid of alpha = max|w| itself: nothing beats AbsMax, and the
    search must be able to return it (the tenth coarse sample)."""
    M = 0.875
    levels = np.arange(-7, 8) * (M / 7)
    W = np.tile(levels.astype(np.float32), (64, 40))[:, :512]
    alpha, scale = O.quant_search(W)
    assert float(alpha) == float(np.float32(M))
    assert float(scale) == 0.125


# ---- one scale per row ---------------------------------------------------------

def test_rows_search_is_the_tensor_search_of_every_row():
    rng = np.random.default_rng(31)
    W = rng.standard_t(4, size=(6, 2048)).astype(np.float32)
    W[2] = 0.0                                               # a zero row: scale 1
    W[3] *= np.float32(2.0 ** -7)                            # power-of-two scaling: alpha scales with it
    W[4] = W[3] * np.float32(2.0 ** 7)
    alpha, scale = O.quant_search_rows(W)
    assert alpha.shape == (6,) and scale.shape == (6,)
    for o in range(6):
        a, s = O.quant_search(W[o:o + 1])
        assert alpha[o] == a and scale[o] == s
    assert alpha[2] == 0 and scale[2] == 1
    assert alpha[4] == alpha[3] * np.float32(2.0 ** 7)
    # rows do not influence one another
    W2 = W.copy()
    W2[0] *= 3.0
    alpha2, _ = O.quant_search_rows(W2)
    assert np.array_equal(alpha2[1:], alpha[1:])


def test_rows_search_never_worse_than_absmax_per_row_on_its_histogram():
    rng = np.random.default_rng(32)
    W = rng.standard_normal((8, 4096)).astype(np.float32)
    W[:, 0] *= 12.0                                          # one outlier per row
    alpha, _ = O.quant_search_rows(W)
    for o in range(8):
        counts, M = O.quant_histogram(W[o])
        assert counts.shape[0] == 512 and counts.sum() == 4096
        assert O.quant_error(counts, M, float(alpha[o])) <= O.quant_error(counts, M, float(M))
        assert alpha[o] < M                                   # the outlier is clipped


def _row_with_two_equal_minima():
    """A row of 4560 heavy-tailed weights (seeded, numpy only) whose errors at
    alpha = 0.18 M and 0.19 M are the same rational number."""
    rng = np.random.default_rng(105)
    for _ in range(21):                                      # the generator's state is what matters
        n = int(rng.integers(1, 900))
        k = 8 * int(rng.integers(1, 700))
        dist = rng.integers(0, 3)
        W = (rng.standard_normal((n, k)) * 0.02 if dist == 0 else rng.standard_t(3, size=(n, k)) if dist == 1
             else np.round(rng.standard_normal((n, k)) * 2) / 4).astype(np.float32)
        rng.uniform(0, 3, size=k)
        rng.choice([1.0, 50.0, 3000.0])
    return W[426]


def test_candidates_can_tie_exactly_and_both_are_accepted():
    """alpha / M is a multiple of 1/100 and the bin centres are odd multiples of M / 2B, so
    the error over M^2 is a rational with a small denominator, and two candidates can
    have the same error exactly.  Which one a binary64 sum calls smaller depends on the
    order of its additions: quant_search_accepts takes both and nothing else."""
    from fractions import Fraction as F
    w = _row_with_two_equal_minima()
    counts, M = O.quant_histogram(w)
    B = counts.shape[0]

    def exact(num):                                          # error / M^2 at alpha = M num / 100
        a = F(num, 100)
        step = a / 7
        e = F(0)
        for b in np.nonzero(counts)[0]:
            x = F(2 * int(b) + 1, 2 * B)
            d = (round(x / step) * step - x) if x <= a else a - x       # round(): half to even, as rint
            e += int(counts[b]) * d * d
        return e

    errs = {num: exact(num) for num in range(10, 31)}        # the fine grid around 0.2 M
    assert errs[18] == errs[19] == min(errs.values())
    assert sorted(errs.values())[2] > errs[18]
    # the binary64 errors of the two agree to rounding, and are what the rational says
    cand, e64 = O.quant_search_candidates(w)
    eta = float(M) / 10.0
    i18 = cand.index(2 * eta + eta * (-2 / 10.0))
    i19 = cand.index(2 * eta + eta * (-1 / 10.0))
    assert abs(e64[i18] - e64[i19]) <= 4e-16 * 512 * e64[i18]
    assert abs(e64[i18] - float(errs[18]) * float(M) ** 2) <= 1e-12 * e64[i18]
    alpha, _ = O.quant_search(w)
    assert alpha in (np.float32(cand[i18]), np.float32(cand[i19]))
    assert O.quant_search_accepts(w, np.float32(cand[i18])) and O.quant_search_accepts(w, np.float32(cand[i19]))
    for i, a in enumerate(cand):
        if i not in (i18, i19) and np.float32(a) not in (np.float32(cand[i18]), np.float32(cand[i19])):
            assert not O.quant_search_accepts(w, np.float32(a))
    assert not O.quant_search_accepts(w, np.float32(cand[i18] * 1.0001))           # not a candidate at all


def test_accepts_is_the_search_itself_where_nothing_ties():
    rng = np.random.default_rng(33)
    for _ in range(20):
        w = rng.standard_normal((3, 700)).astype(np.float32)
        cand, errs = O.quant_search_candidates(w)
        alpha, _ = O.quant_search(w)
        srt = sorted(errs)
        if srt[1] <= srt[0] * (1 + 1e-9) and errs.count(srt[0]) == 1:
            continue                                         # a near tie of different candidates: not this test
        assert O.quant_search_accepts(w, alpha)
        ok = [np.float32(a) for a in cand if O.quant_search_accepts(w, np.float32(a))]
        assert set(ok) == {alpha}
    assert O.quant_search_accepts(np.zeros((2, 64), np.float32), np.float32(0.0))
    assert not O.quant_search_accepts(np.zeros((2, 64), np.float32), np.float32(1.0))
