"""The acceptance rule of the GPU parity tests (tests/parity.py), checked on the CPU: it takes a result that
carries exactly the roundings the path is allowed (T to fp16, fp32 sums, Y to fp16) and refuses planted
defects that the 2e-3 norm over a whole call would let through: one wrong element, one wrong row, one wrong
token, one row tile computed from the neighbouring tile's weights."""
import numpy as np
import pytest

from oracle import slim_oracle as O
from paper_2410_09615_amd import workloads as wl
from parity import TOL_Y, assert_forward_close, element_tolerance, prefill_row_sample, relerr


def _case(m=16, seed=5):
    shape = wl.LayerShape("t", 640, 1024, 51, True)
    W, L, R, X = wl.make_layer(shape, m, seed=seed)
    ref = O.compress(W.numpy())
    Xn, Ln, Rn = (a.numpy().astype(np.float64) for a in (X, L, R))
    Yref, T = O.forward(ref, Ln, Rn, Xn, return_t=True)
    assert np.array_equal(T, O.xr(Xn, Rn))                       # the T handed out is the one of xr
    tol = element_tolerance(Yref, T, Ln, ref.scale.astype(np.float64), Xn, 7)
    # the allowed roundings, applied to the oracle's own numbers: T through fp16, sums in fp32, Y to fp16
    packed = O.forward(ref, None, None, Xn).astype(np.float32)
    t16 = T.astype(np.float16).astype(np.float32)
    Y = (packed + t16 @ Ln.astype(np.float32).T).astype(np.float16)
    return Y, Yref, tol


def test_a_correctly_rounded_result_is_accepted():
    Y, Yref, tol = _case()
    stats = assert_forward_close(Y, Yref, tol, "emulated roundings")
    assert stats["whole"] < 4e-4 and stats["element_max_over_tol"] <= 1.0


@pytest.mark.parametrize("defect", ["element", "row", "token", "tile_shifted", "t_dropped_rank"])
def test_planted_defects_are_refused_although_the_whole_norm_passes(defect):
    Y, Yref, tol = _case()
    Y = Y.astype(np.float64)
    if defect == "element":
        Y[3, 77] *= 1.01
    elif defect == "row":
        Y[:, 100] *= 1.004
    elif defect == "token":
        Y[5, :] *= 1.003
    elif defect == "tile_shifted":
        Y[:, 160:176] = Y[:, 176:192]                             # a row tile that read its neighbour's weights
    else:
        shape = wl.LayerShape("t", 640, 1024, 51, True)
        _, L, R, X = wl.make_layer(shape, 16, seed=5)
        t_last = O.xr(X.numpy(), R.numpy())[:, -1:]
        Y = Y - t_last @ L.numpy().astype(np.float64)[:, -1:].T   # the last rank never added
    if defect != "tile_shifted":
        assert relerr(Y, Yref) <= TOL_Y or defect == "t_dropped_rank"    # the norm alone would have passed
    with pytest.raises(AssertionError):
        assert_forward_close(Y, Yref, tol, defect)


def test_prefill_row_sample_covers_every_piece_of_every_row_tile():
    for n in (4096, 5120, 11008, 13824, 28672, 130):
        rows = prefill_row_sample(n, 256, seed=1)
        assert rows.size >= min(n, 256) and rows.size == np.unique(rows).size and rows.max() < n
        assert set(range(min(32, n))) <= set(rows) and set(range(max(0, n - 32), n)) <= set(rows)
        assert np.unique(rows // 128).size == (n + 127) // 128    # a row in every run of 128
        for b in range(512, n, 512):
            assert b - 1 in rows and b in rows
