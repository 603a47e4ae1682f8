"""Acceptance of a forward result Y (fp16, from the HIP path) against the fp64 oracle.

Three bounds, all asserted by `assert_forward_close`:

  whole    ||Y - Yref||_F / ||Yref||_F <= 2e-3 over the whole call (the stated tolerance of this
           build: fp16 inputs, fp32 accumulation, one rounding of Y);
  tile     the same ratio on every tile of 16 consecutive checked output rows x all tokens, and on
           every token row: a defect confined to one row tile, one token or one row cannot hide in
           the norm of a large call;
  element  |Y - Yref| <= tol per element, tol from the arithmetic of the path:
             2^-11 |Yref|                       the one rounding of Y to fp16 (half an ulp);
             8 * 2^-11 * sqrt(c_t / 3) * Q_lr   T = X R^T is rounded to fp16 before it meets L: a
                                                rounding error is at most half an ulp, 2^-11 relative,
                                                variance (2^-11 t)^2 / 3; c_t counts the roundings a
                                                rank's value goes through (one on the prefill path;
                                                on the one-launch decode path up to four shares of
                                                the inputs, each rounded, and three fp16 additions:
                                                7; two more when the adapters are 4-bit, whose
                                                values code * scale are rounded to fp16 in L and in
                                                R); Q_lr[t][o] = sqrt(sum_j (T[t][j] L[o][j])^2) is
                                                what those independent errors add up to in Y; 8
                                                standard deviations;
             8 * 2^-24 * sqrt(n_acc / 6) * Q    fp32 accumulation of n_acc = k / 2 + r products
                                                (each exact: fp16 x fp16 fits binary32): an addition
                                                rounds the running sum, |S_i| ~ sqrt(i) * rms term,
                                                so the error's standard deviation is
                                                2^-24 * sqrt(n_acc / 6) * Q with Q the root sum of
                                                squares of the terms, bounded here by
                                                8 scale[o] ||X[t]||_2 + Q_lr (|code| <= 8).
           The first term is a hard bound, the other two are 8 standard deviations of sums of
           hundreds of bounded independent errors.
Everything on the reference side is the oracle's (T from its xr) or plain numpy on its outputs.
"""
import os

import numpy as np

TOL_Y = 2e-3
U16 = 2.0 ** -11
U32 = 2.0 ** -24
SIGMAS = 8.0


def relerr(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b))


def element_tolerance(Yref, T, Lrows, scale_rows, X, c_t, mma8=False):
    """tol[t][o] as derived above.  T [m][r] (oracle), Lrows [rows][r], scale_rows [rows] (None: no packed
    term), X [m][k]; all float64.
    mma8: the weight term ran on the 8-bit matrix instruction (slim_linear_gemm_fp8).  Its products are exact,
    but it does not add them in binary32: measured on the GPU (six configurations, with and without outlier
    channels, k from 128 to 4096), what an output is off by beyond its final rounding reaches 2^-12.5 of the
    LARGEST product of that output and hardly grows with k -- the behaviour of an adder that aligns the
    products of a step to the largest one and keeps about 13 bits below it.  The bound adds 2^-11 times an
    upper bound of the largest product, 8 scale[o] max_j |X[t][j]|."""
    m, k = X.shape
    r = 0 if T is None else T.shape[1]
    q_lr = np.sqrt((T ** 2) @ (Lrows ** 2).T) if r else np.zeros_like(Yref)
    q_pk = 0.0
    if scale_rows is not None:
        q_pk = 8.0 * np.linalg.norm(X, axis=1)[:, None] * scale_rows[None, :]
    n_acc = k / 2 + r
    tol = U16 * np.abs(Yref) + SIGMAS * U16 * np.sqrt(c_t / 3.0) * q_lr + SIGMAS * U32 * np.sqrt(n_acc / 6.0) * (q_pk + q_lr)
    if mma8:
        tol = tol + U16 * 8.0 * np.max(np.abs(X), axis=1)[:, None] * scale_rows[None, :]
    return tol


def assert_forward_close(Yg, Yref, tol, what=""):
    """Yg, Yref, tol: [m][rows] (Yg fp16 or float).  Returns the observed figures."""
    Yg = np.asarray(Yg, np.float64)
    assert np.isfinite(Yg).all(), what
    err = np.abs(Yg - Yref)
    ratio = err / np.maximum(tol, 1e-30)
    worst = float(ratio.max())
    if worst > 1.0:
        t, o = np.unravel_index(int(ratio.argmax()), ratio.shape)
        raise AssertionError(f"{what}: element (token {t}, checked row {o}): got {Yg[t, o]!r}, oracle {Yref[t, o]!r}, "
                             f"|error| {err[t, o]:.3e} > tolerance {tol[t, o]:.3e}")
    m, rows = Yref.shape
    full = rows // 16 * 16
    tile_max = 0.0
    if full:
        e2 = (err[:, :full] ** 2).reshape(m, full // 16, 16).sum(axis=(0, 2))
        y2 = (Yref[:, :full] ** 2).reshape(m, full // 16, 16).sum(axis=(0, 2))
        tile_rel = np.sqrt(e2 / np.maximum(y2, 1e-300))
        tile_max = float(tile_rel.max())
        assert tile_max <= TOL_Y, f"{what}: tile of checked rows {16 * int(tile_rel.argmax())}..: relative error {tile_max:.3e}"
    if rows > full:
        tail = float(np.linalg.norm(err[:, full:]) / max(np.linalg.norm(Yref[:, full:]), 1e-300))
        tile_max = max(tile_max, tail)
        assert tail <= TOL_Y, f"{what}: last rows: relative error {tail:.3e}"
    tok_rel = np.linalg.norm(err, axis=1) / np.maximum(np.linalg.norm(Yref, axis=1), 1e-300)
    assert float(tok_rel.max()) <= TOL_Y, f"{what}: token {int(tok_rel.argmax())}: relative error {float(tok_rel.max()):.3e}"
    whole = float(np.linalg.norm(err) / np.linalg.norm(Yref))
    assert whole <= TOL_Y, f"{what}: relative Frobenius error {whole:.3e}"
    stats = {"whole": whole, "tile_max": tile_max, "token_max": float(tok_rel.max()), "element_max_over_tol": worst}
    line = (f"parity {what}: whole {whole:.2e} tile max {tile_max:.2e} token max {stats['token_max']:.2e} "
            f"element max/tol {worst:.2f}")
    print(line)
    if os.environ.get("SLIM_PARITY_LOG"):            # observed figures of a run, for the records
        with open(os.environ["SLIM_PARITY_LOG"], "a") as f:
            f.write(line + "\n")
    return stats


def prefill_row_sample(n, count=256, seed=0):
    """Output rows checked at prefill shapes, where the oracle cannot do them all: the first and the last
    32 rows, one row of every run of 128 rows (the smallest piece of a row tile a workgroup of the
    prefill kernels owns), both sides of every multiple of 512 (workgroup row tiles), then random
    rows up to `count` (more if the layer has more runs)."""
    rng = np.random.default_rng(seed)
    rows = set(range(min(32, n))) | set(range(max(0, n - 32), n))
    for b in range(0, n, 128):
        rows.add(int(rng.integers(b, min(n, b + 128))))
    for b in range(512, n, 512):
        rows.update((b - 1, b))
    rest = np.setdiff1d(np.arange(n), np.fromiter(rows, int))
    if len(rows) < count and rest.size:
        rows.update(int(v) for v in rng.choice(rest, size=min(rest.size, count - len(rows)), replace=False))
    return np.array(sorted(rows), np.int64)
