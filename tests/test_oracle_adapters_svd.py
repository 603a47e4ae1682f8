"""Pins of the oracle's adapter computation (Sec. 3.2, Eq. 8-11, Alg. 2): values worked by hand, the
Eckart-Young residual on a planted spectrum, Naive-LoRA by an independent route (eigenvectors of
E E^T), exact recovery of a low-rank error, optimality in the weighted norm, and shapes that are
not square so that a transposed operand or a saliency on the wrong side fails."""
import os

import numpy as np
import pytest

from oracle import slim_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "handworked_adapters.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = np.array([float(v) for v in vals])
    return out


def test_handworked_rank1():
    g = _golden()
    E = g["E"].reshape(2, 2)
    assert np.array_equal(O.saliency_shift(g["xtilde"]), g["x"])
    L, R, s = O.compute_adapters(E, np.zeros((2, 2)), g["xtilde"], 1)
    np.testing.assert_allclose(L @ R, g["LR_slim"].reshape(2, 2), atol=1e-12)
    np.testing.assert_allclose(s, g["sigma_slim"], atol=1e-12)
    L, R, s = O.compute_adapters(E, np.zeros((2, 2)), None, 1)
    np.testing.assert_allclose(L @ R, g["LR_naive"].reshape(2, 2), atol=1e-12)


def _orth(rng, rows, cols):
    q, _ = np.linalg.qr(rng.standard_normal((rows, cols)))
    return q


@pytest.mark.parametrize("n,k,r", [(48, 32, 5), (24, 64, 7), (40, 40, 40)])
def test_planted_spectrum_eckart_young(n, k, r):
    """S = U0 diag(sigma) V0^T is planted through W = S diag(1/x), Wc = 0: the singular values come
    back, the weighted residual is the tail of the spectrum, L has orthonormal columns."""
    rng = np.random.default_rng(n * 1000 + k)
    p = min(n, k)
    sigma = np.sort(rng.uniform(0.5, 3.0, p))[::-1]
    S = (_orth(rng, n, p) * sigma) @ _orth(rng, k, p).T
    xt = rng.uniform(0.2, 5.0, k)
    x = O.saliency_shift(xt)
    W = S / x[None, :]
    L, R, s = O.compute_adapters(W, np.zeros((n, k)), xt, r)
    assert L.shape == (n, r) and R.shape == (r, k)
    np.testing.assert_allclose(s, sigma, rtol=1e-10)
    res = np.linalg.norm((W - L @ R) * x[None, :])
    np.testing.assert_allclose(res, np.sqrt(np.sum(sigma[r:] ** 2)), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(L.T @ L, np.eye(r), atol=1e-12)


def test_naive_lora_is_the_projection_on_top_eigenvectors():
    """x = 1: L R is E projected on the r leading eigenvectors of E E^T (computed with eigh, not svd)."""
    rng = np.random.default_rng(5)
    n, k, r = 20, 36, 6
    W = rng.standard_normal((n, k))
    Wc = W + 0.1 * rng.standard_normal((n, k))
    L, R, _ = O.compute_adapters(W, Wc, None, r)
    E = W - Wc
    lam, vec = np.linalg.eigh(E @ E.T)
    P = vec[:, np.argsort(lam)[::-1][:r]]
    np.testing.assert_allclose(L @ R, P @ (P.T @ E), atol=1e-10)
    # a constant x~ changes nothing: diag(x) is a multiple of the identity
    L2, R2, _ = O.compute_adapters(W, Wc, np.full(k, 0.7), r)
    np.testing.assert_allclose(L2 @ R2, L @ R, atol=1e-10)


def test_low_rank_error_is_recovered_exactly():
    rng = np.random.default_rng(6)
    n, k, r = 30, 44, 4
    Wc = rng.standard_normal((n, k))
    W = Wc + rng.standard_normal((n, r)) @ rng.standard_normal((r, k))
    xt = rng.uniform(0.1, 2.0, k)
    L, R, s = O.compute_adapters(W, Wc, xt, r)
    np.testing.assert_allclose(Wc + L @ R, W, atol=1e-10)
    assert np.all(s[r:] < 1e-10)
    # the sign of the error: W ~= Wc + L R, not Wc - L R
    assert np.linalg.norm(Wc - L @ R - W) > 1.0


def test_weighted_optimum_beats_naive_in_the_weighted_norm_only():
    rng = np.random.default_rng(7)
    n, k, r = 32, 48, 5
    W = rng.standard_normal((n, k))
    Wc = W + 0.2 * rng.standard_normal((n, k))
    xt = np.abs(rng.standard_normal(k)) + 0.05
    xt[:4] *= 30
    x = O.saliency_shift(xt)
    Ls, Rs, _ = O.compute_adapters(W, Wc, xt, r)
    Ln, Rn, _ = O.compute_adapters(W, Wc, None, r)
    E = W - Wc
    ws = np.linalg.norm((E - Ls @ Rs) * x[None, :])
    wn = np.linalg.norm((E - Ln @ Rn) * x[None, :])
    assert ws < wn * 0.999
    assert np.linalg.norm(E - Ln @ Rn) < np.linalg.norm(E - Ls @ Rs) * 0.999
    # and no other rank-r product does better in the weighted norm: random perturbations only lose
    for t in range(5):
        dL = 1e-3 * rng.standard_normal(Ls.shape)
        dR = 1e-3 * rng.standard_normal(Rs.shape)
        assert np.linalg.norm((E - (Ls + dL) @ (Rs + dR)) * x[None, :]) >= ws


def test_shift_requires_positive_entries():
    with pytest.raises(AssertionError):
        O.saliency_shift(np.array([1.0, 0.0, 2.0]))
    np.testing.assert_array_equal(O.saliency_shift(np.array([0.5, 2.0, 1.0])), np.array([1.0, 2.5, 1.5]))


def test_on_a_compressed_layer_the_adapters_reduce_the_forward_error():
    """End to end on the oracle's own compressed layer: the forward with the computed adapters is
    closer to the dense layer than without them (inputs with the channel magnitudes x~)."""
    rng = np.random.default_rng(8)
    n, k, r, m = 64, 128, 13, 32
    W = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    lay = O.compress(W)
    Wc = O.dequant(lay.qvals, lay.meta, lay.scale)
    amp = np.abs(rng.standard_normal(k)) + 0.1
    X = rng.standard_normal((m, k)) * amp[None, :]
    xt = np.mean(np.abs(X), axis=0)
    L, R, _ = O.compute_adapters(W, Wc, xt, r)
    ref = X @ W.astype(np.float64).T
    e0 = np.linalg.norm(X @ Wc.T - ref)
    e1 = np.linalg.norm(X @ (Wc + L @ R).T - ref)
    assert e1 < 0.95 * e0
