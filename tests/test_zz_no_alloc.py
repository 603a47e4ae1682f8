"""slim_linear_gemv_static: the decode forward on the library's own scratch array.

The entry point is for callers that cannot allocate (graph capture, serving loops): it must give
what slim_linear_gemv gives on a caller-owned workspace -- the same kernels run, so the outputs are
compared bit for bit where the one-launch kernel runs and to the forward tolerance where the
two-launch kernels (whose T is summed with atomic adds) run -- on calls in a row that share the
array, the second on a smaller input, and it must allocate nothing on the way.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import slim_oracle as O
from paper_2410_09615_amd import binding as B
from paper_2410_09615_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL_Y = 2e-3


def _relerr(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b))


def _case(n, k, r, m, seed, adapter_bits=16):
    shape = wl.LayerShape(f"t_{n}x{k}_r{r}", n, k, r, True)
    W, L, R, X = wl.make_layer(shape, m, seed=seed)
    layer = B.compress(W.to(DEV), L.to(DEV), R.to(DEV), adapter_bits=adapter_bits)
    if adapter_bits == 4:
        lc, ls = O.quantize_adapter(L.numpy())
        rc, rs = O.quantize_adapter(R.numpy())
        Lr, Rr = O.dequantize_adapter(lc, ls), O.dequantize_adapter(rc, rs)
    else:
        Lr, Rr = L.numpy(), R.numpy()
    Yref = O.forward(O.compress(W.numpy()), Lr, Rr, X.numpy())
    return layer, X.to(DEV), Yref


def test_static_scratch_matches_the_workspace_call_on_calls_in_a_row():
    """A larger layer at 16 tokens, then a smaller one at 3 tokens (it finds the first call's pieces of
    T in the array), then the first again; every output against the workspace call and the oracle."""
    big = _case(1000, 4096, 100, 16, seed=21)
    small = _case(300, 1024, 37, 3, seed=22)
    q4 = _case(640, 2048, 70, 5, seed=23, adapter_bits=4)
    torch.cuda.synchronize()
    for layer, X, Yref in (big, small, big, q4, small):
        m = X.shape[0]
        assert B.slim_decode_plan(layer.n, layer.k, layer.rank, m, layer.adapter_bits)["path"] == 2
        Y = torch.full((m, layer.n), float("nan"), dtype=torch.float16, device=DEV)
        before = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]
        B.slim_linear_gemv_static(layer, X, Y)
        assert torch.cuda.memory_stats(DEV)["allocation.all.allocated"] == before     # torch allocated nothing
        torch.cuda.synchronize()
        Yw = B.slim_linear_gemv(layer, X)
        torch.cuda.synchronize()
        assert torch.equal(Y, Yw)
        assert _relerr(Y.cpu().numpy(), Yref) <= TOL_Y
    B.slim_workspace_check(None)                          # no call on the library's array gave up waiting


def test_static_scratch_on_the_two_launch_kernels(decode_override):
    """The two-launch kernels keep partial sums and T (fp32, atomic adds: the last bits differ from call to
    call) in the array: a call, then a smaller one."""
    decode_override("parts")
    for n, k, r, m, seed in ((1000, 4096, 100, 16, 31), (300, 1024, 37, 3, 32)):
        layer, X, Yref = _case(n, k, r, m, seed)
        assert B.slim_decode_plan(n, k, r, m)["path"] == 0
        Y = torch.full((m, n), float("nan"), dtype=torch.float16, device=DEV)
        B.slim_linear_gemv_static(layer, X, Y)
        Yw = B.slim_linear_gemv(layer, X)
        torch.cuda.synchronize()
        assert _relerr(Y.cpu().numpy(), Yref) <= TOL_Y
        assert _relerr(Y.cpu().numpy(), Yw.cpu().numpy().astype(np.float64)) <= 1e-3


def test_static_scratch_refuses_what_does_not_fit(decode_override):
    """A call that needs more than the array holds is refused on the host, with the workspace status, and Y
    is left alone: here the two-launch kernels on 28672 x 8192 with 4-bit adapters (their fp16 expansion
    alone is 60 MB); the same layer through the one-launch kernel fits and runs."""
    n, k, r, m = 28672, 8192, 820, 16
    rp = B.slim_rank_pad(r)
    sizes_l, sizes_r = B.slim_adapter_q4_sizes(n, r), B.slim_adapter_q4_sizes(r, k)
    ps = B.slim_packed_sizes(n, k, r)
    z = lambda nbytes: torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    layer = B.SlimLayer(n, k, r, rp, z(ps["qvals"]), z(ps["meta"]), torch.ones(n, dtype=torch.float32, device=DEV), None, None,
                        4, z(sizes_l["codes"]), z(sizes_l["scales"]).view(torch.float16), z(sizes_r["codes"]),
                        z(sizes_r["scales"]).view(torch.float16))
    assert B.slim_workspace_bytes(layer, m) > 8 << 20
    X = torch.ones(m, k, dtype=torch.float16, device=DEV)
    Y = torch.full((m, n), 3.0, dtype=torch.float16, device=DEV)
    decode_override("parts")
    with pytest.raises(B.SlimError) as e:
        B.slim_linear_gemv_static(layer, X, Y)
    assert e.value.status == B.SLIM_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(Y.float().min()) == 3.0 and float(Y.float().max()) == 3.0
    decode_override("auto")
    B.slim_linear_gemv_static(layer, X, Y)                # zero codes, zero adapters: Y = 0
    torch.cuda.synchronize()
    assert float(Y.float().abs().max()) == 0.0
    with pytest.raises(B.SlimError) as e:
        B.lib().slim_linear_gemv_static.restype = ctypes.c_int
        B._check("slim_linear_gemv_static",
                 B.lib().slim_linear_gemv_static(layer.c_ref(), X.data_ptr(), 17, Y.data_ptr(), None))
    assert e.value.status == B.SLIM_ERR_SHAPE
