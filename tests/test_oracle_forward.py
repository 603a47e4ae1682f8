"""Pins for the oracle's forward pass (dequantized matmul + low-rank term).

The plain-loop C forward is checked against: a pure-Python exact evaluation
on dyadic inputs, numpy's matmul on the special cases where the layer reduces
to a library product, a dense brute-force L R, and the never-packs route.
Shapes are non-square everywhere (n != k != m != r) so that a transposed
operand cannot pass.
"""
from fractions import Fraction

import numpy as np

from oracle import slim_oracle as O


def _layer(n, k, r, m, seed):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    L = (rng.standard_normal((n, r)) * 0.01).astype(np.float16)
    R = (rng.standard_normal((r, k)) * 0.01).astype(np.float16)
    X = rng.standard_normal((m, k)).astype(np.float16)
    return W, L, R, X


def _relerr(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def test_forward_exact_on_dyadic_inputs():
    """Tiny layer with small-integer / power-of-two inputs: every product and
    sum is exact in fp64, so the C loops must equal rational arithmetic."""
    rng = np.random.default_rng(3)
    n, k, r, m = 3, 16, 2, 5
    W = rng.integers(-7, 8, size=(n, k)).astype(np.float32)
    W[:, 0] = 7.0                                  # scale 1.0 in every row
    L = (rng.integers(-4, 5, size=(n, r)) / 4).astype(np.float16)
    R = (rng.integers(-4, 5, size=(r, k)) / 8).astype(np.float16)
    X = (rng.integers(-8, 9, size=(m, k)) / 2).astype(np.float16)
    layer = O.compress(W)
    assert (layer.scale == 1.0).all()
    Y = O.forward(layer, L, R, X)
    codes, mask = O.unpack(layer.qvals, layer.meta)
    for i in range(m):
        for o in range(n):
            acc = Fraction(0)
            for c in range(k):
                acc += Fraction(float(X[i, c])) * int(codes[o, c])
            for j in range(r):
                t = sum(Fraction(float(X[i, c])) * Fraction(float(R[j, c])) for c in range(k))
                acc += t * Fraction(float(L[o, j]))
            assert Fraction(Y[i, o]) == acc, (i, o)


def test_lowrank_equals_dense_LR_product():
    n, k, r, m = 40, 96, 7, 5
    _, L, R, X = _layer(n, k, r, m, seed=1)
    zero = O.compress(np.zeros((n, k), np.float32))       # W = 0: pure low-rank
    Y = O.forward(zero, L, R, X)
    LR = np.zeros((n, k))
    for o in range(n):                                     # brute-force dense L R
        for c in range(k):
            LR[o, c] = sum(float(L[o, j]) * float(R[j, c]) for j in range(r))
    want = X.astype(np.float64) @ LR.T
    assert _relerr(Y, want) <= 1e-12
    # T alone
    T = O.xr(X, R)
    assert _relerr(T, X.astype(np.float64) @ R.astype(np.float64).T) <= 1e-13


def test_rank_one_is_an_outer_product_and_zero_padding_is_inert():
    n, k, m = 24, 64, 3
    _, L, R, X = _layer(n, k, 1, m, seed=2)
    zero = O.compress(np.zeros((n, k), np.float32))
    Y = O.forward(zero, L, R, X)
    t = X.astype(np.float64) @ R.astype(np.float64)[0]
    assert _relerr(Y, np.outer(t, L.astype(np.float64)[:, 0])) <= 1e-13
    Lp = np.concatenate([L, np.zeros((n, 5), np.float16)], 1)
    Rp = np.concatenate([R, np.zeros((5, k), np.float16)], 0)
    assert (O.forward(zero, Lp, Rp, X) == Y).all()


def test_route_packed_equals_route_explicit_dense():
    n, k, r, m = 48, 128, 9, 6
    W, L, R, X = _layer(n, k, r, m, seed=4)
    Y1 = O.forward(O.compress(W), L, R, X)
    Y2 = O.forward_explicit_dense(W, L, R, X)
    assert _relerr(Y1, Y2) <= 1e-12


def test_no_adapters_reduces_to_matmul_with_dequantized_weights():
    n, k, r, m = 32, 64, 4, 7
    W, L, R, X = _layer(n, k, r, m, seed=5)
    layer = O.compress(W)
    Wd = O.dequant(layer.qvals, layer.meta, layer.scale)
    want = X.astype(np.float64) @ Wd.T
    assert _relerr(O.forward(layer, None, None, X), want) <= 1e-13
    Lz = np.zeros_like(L)
    assert _relerr(O.forward(layer, Lz, R, X), want) <= 1e-13


def test_identity_input_returns_the_layer_matrix():
    n, k, r = 24, 32, 3
    W, L, R, _ = _layer(n, k, r, 1, seed=6)
    layer = O.compress(W)
    Y = O.forward(layer, L, R, np.eye(k))
    Wd = O.dequant(layer.qvals, layer.meta, layer.scale)
    want = (Wd + L.astype(np.float64) @ R.astype(np.float64)).T
    assert Y.shape == (k, n)
    assert np.abs(Y - want).max() <= 1e-15
    # and without adapters each one-hot input reads one column of Wd exactly
    assert (O.forward(layer, None, None, np.eye(k)) == Wd.T).all()


def test_row_subset_matches_full_forward():
    n, k, r, m = 64, 128, 5, 4
    W, L, R, X = _layer(n, k, r, m, seed=7)
    layer = O.compress(W)
    Y = O.forward(layer, L, R, X)
    rows = [63, 0, 17, 17, 40]
    Ys = O.forward(layer, L, R, X, rows=rows)
    assert Ys.shape == (m, len(rows))
    assert (Ys == Y[:, rows]).all()


def test_forward_is_linear_in_x_and_respects_scale():
    n, k, r, m = 16, 64, 3, 2
    W, L, R, X = _layer(n, k, r, m, seed=8)
    layer = O.compress(W)
    Y = O.forward(layer, L, R, X)
    Y2 = O.forward(layer, L, R, 2.0 * X.astype(np.float64))
    assert _relerr(Y2, 2 * Y) <= 1e-15
    # doubling the row scales doubles only the quantized term
    doubled = O.PackedLayer(layer.qvals, layer.meta, layer.scale * np.float32(2))
    Yq = O.forward(layer, None, None, X)
    assert _relerr(O.forward(doubled, L, R, X), Y + Yq) <= 1e-13


def test_configured_tiny_layer_routes_agree():
    """The configured tiny layer (512 x 512, r = 51, 8 tokens), generated by the
    shared seeded generator."""
    from paper_2410_09615_amd import workloads as wl
    W, L, R, X = wl.make_layer(wl.TINY, 8)
    W, L, R, X = W.numpy(), L.numpy(), R.numpy(), X.numpy()
    layer = O.compress(W)
    Y1 = O.forward(layer, L, R, X)
    Y2 = O.forward_explicit_dense(W, L, R, X)
    assert _relerr(Y1, Y2) <= 1e-12
    _, mask = O.unpack(layer.qvals, layer.meta)
    assert (mask.reshape(512, -1, 4).sum(-1) == 2).all()
