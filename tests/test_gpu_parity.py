"""Parity of the HIP path (through the C-ABI binding) against the CPU oracle.

Packing, metadata and scales must be bit-exact.  Y must be within a relative
Frobenius error of 2e-3 of the fp64 oracle (fp16 inputs, fp32 accumulation,
one final rounding to fp16; T = X R^T is rounded once to fp16 on the prefill
path).  Inputs come from the shared seeded generator.
"""
import numpy as np
import pytest
import torch

from oracle import slim_oracle as O
from paper_2410_09615_amd import binding as B
from paper_2410_09615_amd import workloads as wl
import functools

from layouts import tile_fp16, tile_packed
from parity import TOL_Y, assert_forward_close, element_tolerance, prefill_row_sample, relerr as _relerr

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
# roundings a value of T = X R^T goes through before it meets L (see parity.py): the one-launch decode
# kernel rounds up to four shares and adds them in fp16; prefill rounds T once; 4-bit adapters add the
# fp16 rounding of code * scale in R and in L
CT_DECODE, CT_PREFILL, CT_Q4 = 7, 1, 2


def _shape(n, k, r, outliers=True):
    return wl.LayerShape(f"t_{n}x{k}_r{r}", n, k, r, outliers)


def _gpu_layer(W, L, R):
    Wd = W.to(DEV)
    return B.compress(Wd, None if L is None else L.to(DEV), None if R is None else R.to(DEV))


def _assert_pack_equal(layer, W):
    ref = O.compress(W.numpy())
    torch.cuda.synchronize()
    assert np.array_equal(layer.scale.cpu().numpy().view(np.uint32), ref.scale.view(np.uint32))
    qt, mt = tile_packed(ref.qvals, ref.meta)       # the oracle's canonical bytes in the device order
    assert np.array_equal(layer.qvals.cpu().numpy(), qt)
    assert np.array_equal(layer.meta.cpu().numpy(), mt)
    return ref


# ---- slim_pack / slim_unpack / slim_pack_adapters: bit-exact -------------------

@pytest.mark.parametrize("n,k", [(512, 512), (37, 136), (96, 1024), (3, 8), (130, 12800), (1, 4096)])
def test_pack_bit_exact_small(n, k):
    W = wl.make_weight(n, k, seed=n + k)
    if n > 2:
        W[1] = 0.0                                   # all-zero row
        W[2, : k // 2] = 0.0                         # zero groups
    layer = _gpu_layer(W, None, None)
    ref = _assert_pack_equal(layer, W)
    codes, mask = B.slim_unpack(layer.qvals, layer.meta, n, k)
    rc, rm = O.unpack(ref.qvals, ref.meta)
    assert np.array_equal(codes.cpu().numpy(), rc) and np.array_equal(mask.cpu().numpy(), rm)


def test_pack_bit_exact_with_ties():
    g = torch.Generator().manual_seed(5)
    vals = torch.tensor([0.0, -0.0, 0.25, -0.25, 0.5, -0.5, 1.0, -1.0, 0.75, 0.125])
    W = vals[torch.randint(0, len(vals), (256, 2048), generator=g)].contiguous()
    _assert_pack_equal(_gpu_layer(W, None, None), W)
    # exact halves of the scale (row max 7 -> s = 1): round-half-even cases
    halves = torch.tensor([0.5, 1.5, 2.5, 3.5, 4.5, 5.5, 6.5, -0.5, -1.5, -2.5, -3.5, -4.5, -5.5, -6.5, 7.0, -7.0])
    W2 = halves[torch.randint(0, len(halves), (64, 512), generator=g)].contiguous()
    W2[:, 0] = 7.0
    _assert_pack_equal(_gpu_layer(W2, None, None), W2)


@pytest.mark.parametrize("shape", [wl.L7B_ATTN, wl.L7B_UP, wl.L7B_DOWN, wl.L13B_ATTN, wl.L13B_UP, wl.L70B_ATTN,
                                   wl.L70B_UP], ids=lambda s: s.name)
def test_pack_bit_exact_full_size(shape):
    W = wl.make_weight(shape.n, shape.k)
    _assert_pack_equal(_gpu_layer(W, None, None), W)


@pytest.mark.parametrize("n,k,r", [(300, 640, 51), (64, 1024, 32), (33, 136, 1)])
def test_pack_adapters_pads_and_tiles(n, k, r):
    # zero padding to rank_pad (and to whole tiles), then the documented tile order
    L, R = wl.make_adapters(n, k, r)
    Lp, Rp = B.slim_pack_adapters(L.to(DEV), R.to(DEV))
    rp = B.slim_rank_pad(r)
    Lref = np.zeros((n, rp), np.float16)
    Lref[:, :r] = L.numpy()
    Rref = np.zeros((rp, k), np.float16)
    Rref[:r] = R.numpy()
    assert np.array_equal(Lp.cpu().numpy().view(np.uint16), tile_fp16(Lref).view(np.uint16))
    assert np.array_equal(Rp.cpu().numpy().view(np.uint16), tile_fp16(Rref).view(np.uint16))


def test_unpack_arbitrary_valid_bytes():
    rng = np.random.default_rng(3)
    valid = np.array([0x4, 0x8, 0xC, 0x9, 0xD, 0xE], np.uint8)
    n, k = 64, 1024
    q = rng.integers(0, 256, size=(n, k // 4), dtype=np.uint8)
    me = (valid[rng.integers(0, 6, size=(n, k // 8))] | (valid[rng.integers(0, 6, size=(n, k // 8))] << 4)).astype(np.uint8)
    qt, mt = tile_packed(q, me)
    codes, mask = B.slim_unpack(torch.from_numpy(qt).to(DEV), torch.from_numpy(mt).to(DEV), n, k)
    rc, rm = O.unpack(q, me)
    assert np.array_equal(codes.cpu().numpy(), rc) and np.array_equal(mask.cpu().numpy(), rm)


def _assert_lowrank_close(Y, X, R, L, Y0=None, what="slim_lowrank"):
    """Y against (X R^T) L^T (+ Y0) with T from the oracle, element by element and tile by tile."""
    Xn = X.numpy().astype(np.float64)
    L64 = L.numpy().astype(np.float64)
    T = O.xr(Xn, R.numpy())
    ref = T @ L64.T
    if Y0 is not None:
        ref = ref + Y0.astype(np.float64)
    c_t = CT_DECODE if X.shape[0] <= 16 else CT_PREFILL
    return assert_forward_close(Y.cpu().numpy(), ref, element_tolerance(ref, T, L64, None, Xn, c_t), what)


def _assert_layer_close(Y, ref, Lr, Rr, X, c_t=CT_DECODE, what="forward"):
    """Y (device, fp16) against the oracle's forward of a packed layer on X (host tensor or array)."""
    Xn = (X.numpy() if hasattr(X, "numpy") else X).astype(np.float64)
    L64 = None if Lr is None else np.asarray(Lr, np.float64)
    R64 = None if Rr is None else np.asarray(Rr, np.float64)
    Yref, T = O.forward(ref, L64, R64, Xn, return_t=True)
    tol = element_tolerance(Yref, T, L64, ref.scale.astype(np.float64), Xn, c_t)
    return assert_forward_close(Y.cpu().numpy(), Yref, tol, what)


@pytest.mark.parametrize("n,k,r,m", [(4096, 4096, 410, 16), (4096, 4096, 410, 1), (1000, 11008, 130, 5), (33, 256, 1, 16),
                                     (28672, 8192, 820, 16)])
def test_lowrank_decode_shapes(n, k, r, m):
    """The low-rank term alone on layers of the configured sizes (several rounds of row tiles, X in
    chunks, a rank of 1), plain and accumulating, on one workspace."""
    L, R = wl.make_adapters(n, k, r, 41, 42)
    X = wl.make_activations(m, k, True, 43, 44)
    Lp, Rp = B.slim_pack_adapters(L.to(DEV), R.to(DEV))
    tmp = B.SlimLayer(n, k, r, B.slim_rank_pad(r), Lp, Lp, Lp, Lp, Rp)
    ws = B.alloc_workspace(tmp, m)
    Y = B.slim_lowrank(X.to(DEV), Rp, Lp, n, r, workspace=ws)
    torch.cuda.synchronize()
    _assert_lowrank_close(Y, X, R, L)
    Y2 = B.slim_lowrank(X.to(DEV), Rp, Lp, n, r, Y=Y.clone(), accumulate=True, workspace=ws)
    torch.cuda.synchronize()
    _assert_lowrank_close(Y2, X, R, L, Y0=Y.cpu().numpy())
    assert int(ws.view(torch.int32)[2]) == 0


def test_lowrank_several_row_tiles():
    n, k, r, m = 1100, 1280, 100, 300
    L, R = wl.make_adapters(n, k, r, 31, 32)
    X = wl.make_activations(m, k, True, 33, 34)
    Lp, Rp = B.slim_pack_adapters(L.to(DEV), R.to(DEV))
    Y = B.slim_lowrank(X.to(DEV), Rp, Lp, n, r)
    torch.cuda.synchronize()
    _assert_lowrank_close(Y, X, R, L)


# ---- forward: decode ------------------------------------------------------------

@functools.lru_cache(maxsize=3)
def _compressed(shape, seed, bits):
    """One layer on both sides, kept for the cases that share it (the large shapes take seconds to
    generate and to compress): the library's layer on the device, the oracle's packed layer, and the
    adapters as the oracle's forward takes them (fp16 values, or the dequantized 4-bit ones)."""
    W = wl.make_weight(shape.n, shape.k, seed + 0)
    L = R = Lr = Rr = None
    if shape.r > 0:
        L, R = wl.make_adapters(shape.n, shape.k, shape.r, seed + 1, seed + 2)
        if bits == 4:
            lc, ls = O.quantize_adapter(L.numpy())
            rc, rs = O.quantize_adapter(R.numpy())
            Lr, Rr = O.dequantize_adapter(lc, ls), O.dequantize_adapter(rc, rs)
        else:
            Lr, Rr = L.numpy().astype(np.float64), R.numpy().astype(np.float64)
    layer = B.compress(W.to(DEV), None if L is None else L.to(DEV), None if R is None else R.to(DEV), adapter_bits=bits)
    torch.cuda.synchronize()
    return layer, O.compress(W.numpy()), Lr, Rr


def _check_forward(layer, ref, Lr, Rr, X, fn, rows, c_t, what):
    """fn(layer, X) on a workspace of its own against the oracle's forward on the same inputs: the three
    bounds of parity.py, and the workspace's error word still clear.  Returns the whole-call error."""
    m = X.shape[0]
    ws = B.alloc_workspace(layer, m)
    Y = fn(layer, X.to(DEV), workspace=ws)
    torch.cuda.synchronize()
    assert int(ws.view(torch.int32)[2]) == 0, "a decode call gave up waiting for its T"
    Xn = X.numpy().astype(np.float64)
    Yref, T = O.forward(ref, Lr, Rr, Xn, rows=rows, return_t=True)
    sel = slice(None) if rows is None else rows
    tol = element_tolerance(Yref, T, None if Lr is None else Lr[sel], ref.scale[sel].astype(np.float64), Xn, c_t)
    Yg = Y.cpu().numpy()
    return assert_forward_close(Yg if rows is None else Yg[:, rows], Yref, tol, what)["whole"]


def _forward_case(shape, m, fn, seed=0, rows=None, bits=16):
    layer, ref, Lr, Rr = _compressed(shape, seed, bits)
    X = wl.make_activations(m, shape.k, shape.outliers, seed + 3, seed + 4)
    c_t = (CT_DECODE if fn is B.slim_linear_gemv else CT_PREFILL) + (CT_Q4 if bits == 4 else 0)
    return _check_forward(layer, ref, Lr, Rr, X, fn, rows, c_t, f"{fn.__name__} {shape.name} m={m} bits={bits}")


# slim_linear_gemv has a one-launch path (wherever its geometry fits) and a two-part path (everything
# else); slim_decode_override forces one of them, "roles" runs the one-launch kernel's two roles as two launches.
@pytest.fixture(params=["auto", "parts", "roles", "fused"])
def decode_path(request, decode_override):
    decode_override(request.param)
    return request.param


@pytest.mark.parametrize("m", [1, 16])
def test_gemv_launch_geometries_agree(m, decode_override):
    """The same call through the three decode geometries (one launch, its two roles as two
    launches, the two-launch kernels): the results differ only by reassociation of fp32 sums,
    by the fp16 rounding of T's shares on the one-launch path and by the final rounding of Y
    (2^-11 relative per element where a sum falls on the other side of a rounding boundary):
    6e-4 in relative Frobenius norm, well inside the 2e-3 each has against the oracle; the two
    launch forms of the one-launch kernel do the same arithmetic and agree exactly."""
    shape = _shape(640, 2048, 102)
    W, L, R, X = wl.make_layer(shape, m, seed=4)
    layer = _gpu_layer(W, L, R)
    Xd = X.to(DEV)
    out = {}
    for path in ("parts", "roles", "fused"):
        decode_override(path)
        out[path] = B.slim_linear_gemv(layer, Xd).float().cpu().numpy().astype(np.float64)
    assert np.array_equal(out["roles"], out["fused"])
    assert _relerr(out["parts"], out["fused"]) <= 6e-4


@pytest.mark.parametrize("m", [1, 4, 8, 16])
def test_gemv_tiny_layer(m, decode_path):
    assert _forward_case(wl.TINY, m, B.slim_linear_gemv) <= TOL_Y


@pytest.mark.parametrize("m", [1, 4, 16])
def test_gemv_llama7b_attention(m, decode_path):
    assert _forward_case(wl.L7B_ATTN, m, B.slim_linear_gemv) <= TOL_Y


@pytest.mark.parametrize("n,k,r,m", [(1000, 1280, 37, 3), (17, 128, 1, 5), (2049, 640, 33, 16), (130, 11008, 410, 2),
                                     (5000, 2176, 100, 8), (48, 4096, 1024, 16)])
def test_gemv_ragged_shapes(n, k, r, m, decode_path):
    assert _forward_case(_shape(n, k, r), m, B.slim_linear_gemv, seed=7) <= TOL_Y


def test_gemv_without_adapters(decode_path):
    assert _forward_case(_shape(512, 1024, 0), 4, B.slim_linear_gemv, seed=3) <= TOL_Y


# every configured decode shape and token count (the 7B attention projection has its own test above),
# a few more, all output rows against the oracle, on the automatic path and on each forced one
@pytest.mark.parametrize("shape,m", [(wl.L13B_ATTN, 1), (wl.L13B_UP, 1), (wl.L70B_ATTN, 1), (wl.L70B_ATTN, 16), (wl.L70B_UP, 1),
                                     (wl.L70B_UP, 16), (wl.L70B_UP, 4), (wl.L7B_DOWN, 4), (wl.L7B_UP, 16)],
                         ids=lambda v: str(getattr(v, "name", v)))
def test_gemv_full_size_all_rows(shape, m, decode_path):
    assert _forward_case(shape, m, B.slim_linear_gemv) <= TOL_Y


@pytest.mark.parametrize("n,k,r,m,lds_kb", [(1000, 4096, 100, 16, 96), (1000, 4096, 100, 16, 72), (520, 11008, 410, 8, 64),
                                            (300, 2176, 37, 5, 24), (2049, 8192, 33, 16, 160), (64, 3072, 0, 16, 70)])
def test_gemv_one_launch_with_x_in_chunks(n, k, r, m, lds_kb, decode_override):
    """The one-launch kernel with X streamed through LDS in chunks (a smaller LDS
    budget forces the chunks on layers the oracle finishes quickly)."""
    decode_override("fused", lds_kb)
    plan = B.slim_decode_plan(n, k, r, m)
    assert plan["path"] == 2 and plan["chunks"] > 1            # the case really runs what it is meant to
    assert _forward_case(_shape(n, k, r), m, B.slim_linear_gemv, seed=13) <= TOL_Y


@pytest.mark.parametrize("m", list(range(1, 17)))
def test_gemv_every_token_count(m):
    assert _forward_case(_shape(777, 1408, 45), m, B.slim_linear_gemv, seed=100 + m) <= TOL_Y


def test_gemv_never_gives_up_waiting():
    """The one-launch kernel records in word 2 of the workspace if a helper ran out of
    polls; it never should."""
    W, L, R, X = wl.make_layer(wl.L7B_ATTN, 16, seed=1)
    layer = _gpu_layer(W, L, R)
    ws = B.alloc_workspace(layer, 16)
    Xd = X.to(DEV)
    for i in range(50):
        B.slim_linear_gemv(layer, Xd[: 1 + i % 16].contiguous(), workspace=ws)
    torch.cuda.synchronize()
    assert int(ws.view(torch.int32)[2]) == 0


def test_a_wait_that_gives_up_is_loud(decode_override):
    """The bounded wait of the one-launch kernel, forced from the host to run out (only the waiting half of the
    kernel is launched, with a short poll limit; every wavefront ends normally): the outputs are NaN, not
    plausible numbers, the workspace's error word is set, slim_workspace_check reports it once and clears
    it, and the next ordinary call on the same workspace is correct."""
    shape = _shape(640, 1024, 51)
    W, L, R, X = wl.make_layer(shape, 4, seed=17)
    layer = _gpu_layer(W, L, R)
    ref = O.compress(W.numpy())
    ws = B.alloc_workspace(layer, 4)
    B.slim_workspace_check(ws)                                  # a fresh workspace is clean
    decode_override("wait_test")
    Y = B.slim_linear_gemv(layer, X.to(DEV), workspace=ws)
    torch.cuda.synchronize()
    assert bool(torch.isnan(Y).all())
    assert int(ws.view(torch.int32)[2]) == 1
    with pytest.raises(B.SlimError) as e:
        B.slim_workspace_check(ws)
    assert e.value.status == B.SLIM_ERR_WAIT
    B.slim_workspace_check(ws)                                  # reported once, then clear again
    decode_override("auto")
    Y = B.slim_linear_gemv(layer, X.to(DEV), workspace=ws)
    torch.cuda.synchronize()
    _assert_layer_close(Y, ref, L.numpy(), R.numpy(), X, what="the call after a wait that gave up")
    B.slim_workspace_check(ws)


def test_gemv_repeated_calls_one_workspace(decode_override):
    """One workspace, many calls: the paths alternate, the token count changes, and
    every call must give the result of a call on a fresh workspace (no state of an
    earlier call may leak: flags, epochs, the T buffers)."""
    shape = _shape(1000, 2048, 70)
    W, L, R, X = wl.make_layer(shape, 16, seed=11)
    layer = _gpu_layer(W, L, R)
    ref_layer = O.compress(W.numpy())
    ws = torch.zeros(max(B.slim_workspace_bytes(layer, m) for m in range(1, 17)), dtype=torch.uint8, device=DEV)
    Xd = X.to(DEV)
    for i, (path, m) in enumerate([("fused", 16), ("parts", 3), ("fused", 3), ("fused", 1), ("roles", 16), ("parts", 16),
                                   ("fused", 8), ("fused", 16), ("parts", 1), ("fused", 2)]):
        decode_override(path)
        Y = B.slim_linear_gemv(layer, Xd[:m].contiguous(), workspace=ws)
        torch.cuda.synchronize()
        _assert_layer_close(Y, ref_layer, L.numpy(), R.numpy(), X[:m], what=f"call {i} ({path}, m={m})")
    assert int(ws.view(torch.int32)[2]) == 0


# ---- forward: prefill -----------------------------------------------------------

@pytest.mark.parametrize("m", [8, 128, 200])
def test_gemm_tiny_layer(m):
    assert _forward_case(wl.TINY, m, B.slim_linear_gemm) <= TOL_Y


@pytest.mark.parametrize("n,k,r,m", [(1000, 1280, 37, 200), (130, 256, 5, 77), (384, 640, 64, 129)])
def test_gemm_ragged_shapes(n, k, r, m):
    assert _forward_case(_shape(n, k, r), m, B.slim_linear_gemm, seed=11) <= TOL_Y


@pytest.mark.parametrize("stages", [1, 2, 3, 4, 5, 6, 7, 9, 12, 13])
@pytest.mark.parametrize("fp8", [False, True])
def test_gemm_every_stage_count_modulo_six(stages, fp8):
    """The main loops are written out for six stages of 128 inputs (three register sets of weights, two of X):
    every residue of the stage count, below and above one pass of the loop, on fp16 and on 8-bit inputs."""
    n, k, r, m = 200, 128 * stages, 20, 130
    if fp8:
        err, _ = _fp8_forward_case(n, k, r, m, seed=stages)
    else:
        err = _forward_case(_shape(n, k, r), m, B.slim_linear_gemm, seed=stages)
    assert err <= TOL_Y


def test_gemm_without_adapters():
    assert _forward_case(_shape(512, 1024, 0), 256, B.slim_linear_gemm, seed=4) <= TOL_Y


@pytest.mark.parametrize("shape,m", [(wl.L7B_UP, 2048), (wl.L7B_DOWN, 2048), (wl.L13B_ATTN, 4096), (wl.L13B_UP, 4096),
                                     (wl.L70B_ATTN, 4096), (wl.L70B_UP, 4096)], ids=lambda v: str(getattr(v, "name", v)))
def test_gemm_full_size_sampled_rows(shape, m):
    """Every configured prefill shape, all tokens, on at least 256 output rows: the first and last 32,
    one of every 128 (every piece of a row tile that some workgroup owns), both sides of every workgroup
    row tile, random ones."""
    rows = prefill_row_sample(shape.n, 256, seed=2)
    assert rows.size >= 256
    assert _forward_case(shape, m, B.slim_linear_gemm, rows=rows) <= TOL_Y


def test_gemm_whole_round_plus_remainder_tiles():
    # 3 row tiles x 100 token tiles = 300 workgroup tiles: one whole round of 256 and a
    # remainder that runs as half-height tiles; 3 stages of inputs (an odd count)
    shape = _shape(1536, 384, 37)
    rows = np.arange(0, 1536, 7)
    assert _forward_case(shape, 12800, B.slim_linear_gemm, seed=13, rows=rows) <= TOL_Y


def test_gemv_and_gemm_agree():
    W, L, R, X = wl.make_layer(wl.TINY, 16, seed=2)
    layer = _gpu_layer(W, L, R)
    Xd = X.to(DEV)
    a = B.slim_linear_gemv(layer, Xd).float()
    b = B.slim_linear_gemm(layer, Xd).float()
    assert float((a - b).norm() / a.norm()) <= 1e-3


# ---- slim_pack_ex / slim_quant_search (SLiM-Quant scale, saliency-weighted mask) ---------

def _assert_packed_equal(qvals, meta, scale, codes, mask, ref_scale):
    qv, me = O.pack(codes, mask)
    qt, mt = tile_packed(qv, me)
    torch.cuda.synchronize()
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), ref_scale.view(np.uint32))
    assert np.array_equal(qvals.cpu().numpy(), qt)
    assert np.array_equal(meta.cpu().numpy(), mt)


def _accepted_alpha(W, alpha_gpu):
    """The library's alpha has to be the oracle's, bit for bit, unless candidates of Alg. 1 tie
    within the rounding error of the binary64 error sums (they can tie exactly): then any of
    the tied ones.  Returns (alpha, scale = alpha / 7 in binary32, 1 for a zero tensor)."""
    ra, rs = O.quant_search(W)
    a = np.float32(alpha_gpu)
    if a.view(np.uint32) != ra.view(np.uint32):
        assert O.quant_search_accepts(W, a), (float(a), float(ra))
        rs = np.float32(a / np.float32(7.0))
    return a, rs


def _accepted_alpha_rows(W, alpha_gpu, scale_gpu):
    ra, rs = O.quant_search_rows(W)
    rs = rs.copy()
    for o in np.argwhere(alpha_gpu.view(np.uint32) != ra.view(np.uint32)).ravel():
        _, rs[o] = _accepted_alpha(W[o], alpha_gpu[o])
    assert np.array_equal(scale_gpu.view(np.uint32), rs.view(np.uint32))
    return rs


@pytest.mark.parametrize("n,k,dist", [(512, 512, "normal"), (300, 1280, "t3"), (4096, 4096, "normal"), (64, 256, "outliers"),
                                      (33, 136, "zero")])
def test_quant_search_matches_the_oracle(n, k, dist):
    rng = np.random.default_rng(n + k)
    if dist == "normal":
        W = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    elif dist == "t3":
        W = rng.standard_t(3, size=(n, k)).astype(np.float32)
    elif dist == "outliers":
        W = (rng.standard_normal((n, k)) * 0.01).astype(np.float32)
        W[0, :3] = [1.0, -0.7, 0.5]
    else:
        W = np.zeros((n, k), np.float32)
    scale, alpha = B.slim_quant_search(torch.from_numpy(W).to(DEV))
    torch.cuda.synchronize()
    ra, rs = _accepted_alpha(W, alpha.cpu().numpy()[0])
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), np.full(n, rs, np.float32).view(np.uint32))


@pytest.mark.parametrize("n,k,dist", [(512, 512, "normal"), (37, 136, "t3"), (300, 4096, "outliers"), (5000, 1024, "t3")])
def test_quant_search_rows_matches_the_oracle(n, k, dist):
    rng = np.random.default_rng(n * 3 + k)
    if dist == "normal":
        W = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    elif dist == "t3":
        W = rng.standard_t(3, size=(n, k)).astype(np.float32)
    else:
        W = (rng.standard_normal((n, k)) * 0.01).astype(np.float32)
        W[:, 5] *= 40.0
    W[n // 2] = 0.0                                          # a zero row
    scale, alpha = B.slim_quant_search_rows(torch.from_numpy(W).to(DEV))
    torch.cuda.synchronize()
    rs = _accepted_alpha_rows(W, alpha.cpu().numpy(), scale.cpu().numpy())
    # and the layer packed with these scales is the oracle's
    q, m, s = B.slim_pack_ex(torch.from_numpy(W).to(DEV), None, scale)
    mask = O.mask_2of4(W)
    _assert_packed_equal(q, m, s, O.quantize(W, mask, rs), mask, rs)


@pytest.mark.parametrize("n,k", [(512, 512), (37, 136), (130, 12800), (1000, 4096)])
def test_pack_ex_bit_exact(n, k):
    """Saliency-weighted mask and given scales, separately and together, against the
    oracle's mask / quantize / pack with the same inputs."""
    rng = np.random.default_rng(n * 7 + k)
    W = rng.standard_t(4, size=(n, k)).astype(np.float32)
    sal = rng.uniform(0.05, 8.0, size=k).astype(np.float32)
    sal[::17] = 0.0
    _, rs = O.quant_search(W)
    given = np.full(n, rs, np.float32)
    given[: n // 2] *= np.float32(1.5)                       # not all rows alike
    Wd = torch.from_numpy(W).to(DEV)
    for use_sal, use_scale in ((True, False), (False, True), (True, True), (False, False)):
        q, m, s = B.slim_pack_ex(Wd, torch.from_numpy(sal).to(DEV) if use_sal else None,
                                 torch.from_numpy(given).to(DEV) if use_scale else None)
        mask = O.mask_2of4(W, sal if use_sal else None)
        ref_scale = given if use_scale else O.row_scale(W)
        codes = O.quantize(W, mask, ref_scale)
        _assert_packed_equal(q, m, s, codes, mask, ref_scale)


def test_forward_of_a_layer_packed_with_searched_scale_and_saliency_mask():
    """The whole chain: search the scale, pack with it and a saliency vector, run the
    decode and prefill forwards against the oracle's forward of the same packed layer."""
    shape = _shape(640, 1024, 51)
    W, L, R, X = wl.make_layer(shape, 8, seed=9)
    sal = np.random.default_rng(8).uniform(0.1, 3.0, size=shape.k).astype(np.float32)
    Wd = W.to(DEV)
    scale, _ = B.slim_quant_search(Wd)
    q, m, s = B.slim_pack_ex(Wd, torch.from_numpy(sal).to(DEV), scale)
    Lp, Rp = B.slim_pack_adapters(L.to(DEV), R.to(DEV))
    layer = B.SlimLayer(shape.n, shape.k, shape.r, B.slim_rank_pad(shape.r), q, m, s, Lp, Rp)
    _, rs = O.quant_search(W.numpy())
    mask = O.mask_2of4(W.numpy(), sal)
    ref_scale = np.full(shape.n, rs, np.float32)
    qv, me = O.pack(O.quantize(W.numpy(), mask, ref_scale), mask)
    packed = O.PackedLayer(qv, me, ref_scale)
    for fn, c_t in ((B.slim_linear_gemv, CT_DECODE), (B.slim_linear_gemm, CT_PREFILL)):
        Y = fn(layer, X.to(DEV))
        torch.cuda.synchronize()
        _assert_layer_close(Y, packed, L.numpy(), R.numpy(), X, c_t, fn.__name__)


# ---- 4-bit adapters (Sec. 3.3) ------------------------------------------------------

def _q4_layer(W, L, R):
    return B.compress(W.to(DEV), L.to(DEV), R.to(DEV), adapter_bits=4)


@pytest.mark.parametrize("n,k,r", [(300, 640, 51), (64, 1024, 32), (33, 256, 1), (1000, 4096, 410), (520, 11008, 130)])
def test_pack_adapters_q4_bit_exact(n, k, r):
    """Codes and scales of both adapters equal the oracle's group quantizer bit for bit."""
    L, R = wl.make_adapters(n, k, r, 31, 32)
    L[0, : min(r, 3)] = 0                       # and a few special values: a zero run, a tiny value, a large one
    R[0, 128:256] = 0                           # a whole group of zeros
    R[r - 1, 5] = 2.0 ** -24
    L[n - 1, r - 1] = 3.0
    Lq, Ls, Rq, Rs = B.slim_pack_adapters_q4(L.to(DEV), R.to(DEV))
    for (q, s, A, rows, cols) in ((Lq, Ls, L, n, r), (Rq, Rs, R, r, k)):
        codes, scales = B.slim_unpack_adapters_q4(q, s, rows, cols)
        torch.cuda.synchronize()
        rc, rs = O.quantize_adapter(A.numpy())
        assert np.array_equal(scales.cpu().numpy().view(np.uint16), rs.view(np.uint16))
        assert np.array_equal(codes.cpu().numpy(), rc)


def test_pack_adapters_q4_in_place_outputs():
    """The form that allocates nothing writes the same bytes into tensors of an earlier call (first filled with junk)."""
    L, R = wl.make_adapters(300, 640, 51, 5, 6)
    ref = B.slim_pack_adapters_q4(L.to(DEV), R.to(DEV))
    out = tuple(torch.full_like(t, 77) for t in ref)
    again = B.slim_pack_adapters_q4(L.to(DEV), R.to(DEV), out=out)
    torch.cuda.synchronize()
    assert all(a.data_ptr() == o.data_ptr() for a, o in zip(again, out))
    for a, b in zip(out, ref):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    with pytest.raises(ValueError):
        B.slim_pack_adapters_q4(L.to(DEV), R.to(DEV), out=(out[0][:-1].contiguous(),) + out[1:])


def _forward_case_q4(shape, m, fn, seed=0, rows=None):
    return _forward_case(shape, m, fn, seed=seed, rows=rows, bits=4)


@pytest.mark.parametrize("m", [1, 4, 8, 16])
def test_gemv_q4_adapters_tiny_layer(m, decode_path):
    assert _forward_case_q4(wl.TINY, m, B.slim_linear_gemv) <= TOL_Y


@pytest.mark.parametrize("n,k,r,m", [(1000, 1280, 37, 3), (17, 128, 1, 5), (2049, 640, 33, 16), (130, 11008, 410, 2),
                                     (5000, 2176, 100, 8), (48, 4096, 1024, 16), (300, 8192, 600, 16)])
def test_gemv_q4_adapters_ragged_shapes(n, k, r, m):
    assert _forward_case_q4(_shape(n, k, r), m, B.slim_linear_gemv, seed=7) <= TOL_Y


@pytest.mark.parametrize("shape,m", [(wl.L7B_ATTN, 1), (wl.L7B_ATTN, 16), (wl.L70B_ATTN, 4), (wl.L70B_UP, 1), (wl.L70B_UP, 16)],
                         ids=lambda v: str(getattr(v, "name", v)))
def test_gemv_q4_adapters_full_size_all_rows(shape, m):
    assert _forward_case_q4(shape, m, B.slim_linear_gemv) <= TOL_Y


@pytest.mark.parametrize("shape,m", [(wl.L7B_UP, 2048), (wl.L7B_DOWN, 2048), (wl.L13B_ATTN, 4096), (wl.L13B_UP, 4096),
                                     (wl.L70B_ATTN, 4096), (wl.L70B_UP, 4096)], ids=lambda v: str(getattr(v, "name", v)))
def test_gemm_q4_adapters_full_size_sampled_rows(shape, m):
    """Every configured prefill shape on 4-bit adapters read directly by both adapter products (whole
    tiles and the remainder-tile kernels, k = 11008 with its odd number of 256-column code tiles)."""
    rows = prefill_row_sample(shape.n, 256, seed=3)
    assert _forward_case_q4(shape, m, B.slim_linear_gemm, rows=rows) <= TOL_Y


@pytest.mark.parametrize("n,k,r,m,lds_kb", [(1000, 4096, 100, 16, 96), (520, 11008, 410, 8, 64), (300, 2176, 37, 5, 24)])
def test_gemv_q4_adapters_with_x_in_chunks(n, k, r, m, lds_kb, decode_override):
    decode_override("fused", lds_kb)
    plan = B.slim_decode_plan(n, k, r, m, 4)
    assert plan["path"] == 2 and plan["chunks"] > 1
    assert _forward_case_q4(_shape(n, k, r), m, B.slim_linear_gemv, seed=17) <= TOL_Y


@pytest.mark.parametrize("n,k,r,m", [(512, 512, 51, 200), (1000, 1280, 37, 129), (384, 640, 90, 129), (1200, 1024, 160, 300),
                                     (2100, 4096, 410, 700), (130, 256, 5, 77), (700, 2048, 300, 40), (2000, 2048, 1100, 260)])
def test_gemm_q4_adapters(n, k, r, m):
    """Prefill reads the 4-bit codes itself, in stages of 128 ranks or inputs taken in groups of 64:
    ranks that end 32 past such a group (90, 160, 410, 1100), below one group (5, 37, 51), several stages,
    more than 1024 ranks (five tiles of 256 code columns), ragged rows and tokens, the remainder-tile kernels
    (few tiles)."""
    assert _forward_case_q4(_shape(n, k, r), m, B.slim_linear_gemm, seed=5) <= TOL_Y


def test_gemm_q4_adapters_tokens_do_not_leak_into_each_other():
    """The adapter term runs whole groups of 64 ranks; where the padded rank ends inside a group the
    kernel must multiply zeros, not whatever follows the row of T -- the next token's T.  Tokens whose
    inputs are infinite make that visible: every other token still matches the oracle."""
    shape, m = _shape(384, 640, 90), 260
    layer, ref, Lr, Rr = _compressed(shape, 9, 4)
    X = wl.make_activations(m, shape.k, shape.outliers, 12, 13)
    bad = [1, 127, 128, 259]
    Xg = X.clone()
    Xg[bad] = float("inf")
    Y = B.slim_linear_gemm(layer, Xg.to(DEV)).cpu().numpy()
    keep = np.setdiff1d(np.arange(m), bad)
    Xn = X.numpy().astype(np.float64)[keep]
    Yref, T = O.forward(ref, Lr, Rr, Xn, return_t=True)
    tol = element_tolerance(Yref, T, Lr, ref.scale.astype(np.float64), Xn, CT_PREFILL + CT_Q4)
    assert np.isfinite(Y[keep]).all()
    assert assert_forward_close(Y[keep], Yref, tol, "q4 prefill beside infinite tokens")["whole"] <= TOL_Y


def test_q4_adapters_change_the_result_as_much_as_the_quantization_says():
    """The 4-bit layer is not the fp16 layer: the two forwards differ by about the
    quantization error of the adapter term (a guard against a path that silently
    reads the fp16 adapters)."""
    W, L, R, X = wl.make_layer(wl.TINY, 4, seed=3)
    y16 = B.slim_linear_gemv(_gpu_layer(W, L, R), X.to(DEV)).float()
    y4 = B.slim_linear_gemv(_q4_layer(W, L, R), X.to(DEV)).float()
    d = float((y16 - y4).norm() / y16.norm())
    assert 1e-4 < d < 0.2


# ---- slim_lowrank -----------------------------------------------------------------

@pytest.mark.parametrize("m", [1, 16, 300])
@pytest.mark.parametrize("accumulate", [False, True])
@pytest.mark.parametrize("path", ["auto", "parts"])
def test_lowrank(m, accumulate, path, decode_override):
    """Up to 16 tokens the call is the one-launch decode kernel without its packed items; "parts"
    keeps the two-part kernels that serve where that geometry does not fit."""
    if path == "parts":
        if m > 16:
            pytest.skip("the decode paths differ up to 16 tokens only")
        decode_override("parts")
    n, k, r = 640, 1280, 51
    L, R = wl.make_adapters(n, k, r, 21, 22)
    X = wl.make_activations(m, k, True, 23, 24)
    Lp, Rp = B.slim_pack_adapters(L.to(DEV), R.to(DEV))
    Y0 = Y0h = None
    if accumulate:
        std = float((O.xr(X.numpy(), R.numpy()) @ L.numpy().astype(np.float64).T).std())
        Y0h = (torch.randn(m, n, generator=torch.Generator().manual_seed(9)) * std).to(torch.float16)
        Y0 = Y0h.to(DEV)
    Y = B.slim_lowrank(X.to(DEV), Rp, Lp, n, r, Y=Y0, accumulate=accumulate)
    torch.cuda.synchronize()
    _assert_lowrank_close(Y, X, R, L, Y0=None if Y0h is None else Y0h.numpy())


# ---- measurement aids -------------------------------------------------------------

def test_probes_run_and_report_their_work():
    buf = torch.ones(8 << 20, dtype=torch.uint8, device=DEV)
    sink = torch.zeros(4, dtype=torch.float32, device=DEV)
    B.slim_probe_read(buf, 4 << 20, 2, 4 << 20, sink)
    for sparse in (False, True):
        flops = B.slim_probe_mfma(sparse, 8, 16, sink)
        assert flops == 16 * 4 * 8 * 4 * 2 * 32 * 32 * (32 if sparse else 16)
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0                    # the sinks are never written
    with pytest.raises(B.SlimError):
        B.slim_probe_read(buf, 1024, 1, 0, sink)
    with pytest.raises(ValueError):
        B.slim_probe_read(buf, 8 << 20, 2, 4 << 20, sink)


# ---- FP8 input quantization (App. "Input Quantization") ---------------------------------

@pytest.mark.parametrize("case", ["normal", "outliers", "beyond_e4m3", "tiny", "zero", "ragged"])
def test_input_quant_fp8_bit_exact(case):
    rng = np.random.default_rng(len(case))
    if case == "normal":
        X = rng.standard_normal((16, 4096)).astype(np.float16)
    elif case == "outliers":
        X = wl.make_activations(16, 4096, seed=5).numpy()
    elif case == "beyond_e4m3":
        X = (rng.standard_normal((8, 1024)) * 40).astype(np.float16)
        X[2, 3] = np.float16(-3000.0)
    elif case == "tiny":
        X = (rng.standard_normal((4, 512)) * 1e-4).astype(np.float16)          # fp16 subnormals among them
        X[0, :8] = np.array([-0.0, 0.0, -6e-8, 6e-8, -1e-7, 1e-7, -0.0, 0.0], np.float16)   # round to zero, sign kept
    elif case == "zero":
        X = np.zeros((2, 128), np.float16)
        X[1, ::3] = np.float16(-0.0)                                           # signed zeros stay what they are
    else:
        X = rng.standard_normal((3, 1001)).astype(np.float16)                  # a tail that is no 16-byte piece
        X[2, -3:] = np.array([-0.0, -6e-8, 0.0], np.float16)                   # signed zeros in that tail too
    Xq, info = B.slim_input_quant_fp8(torch.from_numpy(X).to(DEV))
    torch.cuda.synchronize()
    rq, rs, rf = O.input_quant_fp8(X)
    info = info.cpu().numpy()
    assert info[0].view(np.uint32) == np.float32(rs).view(np.uint32)
    assert info[1] == (1.0 if rf == "e5m2" else 0.0)
    assert np.array_equal(Xq.cpu().numpy().view(np.uint16), rq.view(np.uint16))


@pytest.mark.parametrize("case", ["normal", "beyond_e4m3", "tiny", "ragged"])
def test_input_quant_fp8_codes_bit_exact(case):
    """The 8-bit codes equal the oracle's (the bit fields of its quantized values), and the fp16 output and the
    scale are those of the call without codes."""
    rng = np.random.default_rng(len(case) + 7)
    if case == "normal":
        X = wl.make_activations(16, 4096, seed=6).numpy()
    elif case == "beyond_e4m3":
        X = (rng.standard_normal((8, 1024)) * 40).astype(np.float16)
        X[1, 5] = np.float16(2500.0)
    elif case == "tiny":
        X = (rng.standard_normal((4, 512)) * 1e-4).astype(np.float16)
        X[0, :6] = np.array([-0.0, 0.0, -6e-8, 6e-8, -1e-7, 1e-7], np.float16)
    else:
        X = rng.standard_normal((3, 1001)).astype(np.float16)
    Xq, info, codes = B.slim_input_quant_fp8(torch.from_numpy(X).to(DEV), codes=True)
    Xq2, info2 = B.slim_input_quant_fp8(torch.from_numpy(X).to(DEV))
    torch.cuda.synchronize()
    rc, rs, rf = O.input_quant_fp8_codes(X)
    assert info.cpu().numpy()[0].view(np.uint32) == np.float32(rs).view(np.uint32)
    assert float(info[1]) == (1.0 if rf == "e5m2" else 0.0)
    assert np.array_equal(codes.cpu().numpy(), rc)
    assert torch.equal(Xq.view(torch.int16), Xq2.view(torch.int16)) and torch.equal(info, info2)
    none, info3, codes3 = B.slim_input_quant_fp8(torch.from_numpy(X).to(DEV), Xq=False, codes=True)      # codes alone
    torch.cuda.synchronize()
    assert none is None and torch.equal(codes3, codes) and torch.equal(info3, info)


def _fp8_forward_case(n, k, r, m, seed=0, x_gain=1.0, rows=None, shape=None, bits=16):
    """slim_linear_gemm_fp8 against the oracle's forward on the exact quantized values value(code) * scale (both terms;
    the codes themselves are checked bit for bit in test_input_quant_fp8_codes_bit_exact).  bits = 4: on 4-bit
    adapters, the oracle's forward on their dequantized values."""
    shape = shape or _shape(n, k, r)
    W, L, R, X = wl.make_layer(shape, m, seed=seed)
    X = (X.float() * x_gain).half()
    if bits == 4:
        layer = _q4_layer(W, L, R)
        L = torch.from_numpy(O.dequantize_adapter(*O.quantize_adapter(L.numpy())))
        R = torch.from_numpy(O.dequantize_adapter(*O.quantize_adapter(R.numpy())))
    else:
        layer = _gpu_layer(W, L if shape.r else None, R if shape.r else None)
    _, info, codes = B.slim_input_quant_fp8(X.to(DEV), Xq=False, codes=True)
    torch.cuda.synchronize()
    fmt = int(info[1])
    ws = B.alloc_workspace(layer, m)
    Y = B.slim_linear_gemm_fp8(layer, codes, info, fmt, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws.view(torch.int32)[2]) == 0
    ref = O.compress(W.numpy())
    _, s, fname = O.input_quant_fp8(X.numpy())
    assert fmt == (1 if fname == "e5m2" else 0)
    xe = O.fp8_round((X.numpy().astype(np.float32) / s).astype(np.float32), fname).astype(np.float64) * np.float64(s)
    Lr = L.numpy().astype(np.float64) if shape.r else None
    Rr = R.numpy().astype(np.float64) if shape.r else None
    Yref, T = O.forward(ref, Lr, Rr, xe, rows=rows, return_t=True)
    sel = slice(None) if rows is None else rows
    tol = element_tolerance(Yref, T, None if Lr is None else Lr[sel], ref.scale[sel].astype(np.float64), xe,
                            CT_PREFILL + (CT_Q4 if bits == 4 else 0), mma8=True)
    Yg = Y.cpu().numpy()
    return assert_forward_close(Yg if rows is None else Yg[:, rows], Yref, tol,
                                f"slim_linear_gemm_fp8 {shape.name} m={m} fmt={fmt} bits={bits}")["whole"], fmt


@pytest.mark.parametrize("n,k,r,m", [(512, 128, 0, 128), (640, 1024, 0, 200), (1000, 2048, 64, 300), (33, 256, 1, 17),
                                     (2100, 4096, 410, 700), (1537, 1152, 100, 129)])
def test_gemm_fp8_inputs_small_and_ragged(n, k, r, m):
    err, fmt = _fp8_forward_case(n, k, r, m, seed=n % 7)
    assert err <= TOL_Y and fmt == 0


def test_gemm_fp8_inputs_e5m2():
    """Inputs beyond E4M3's range take the E5M2 form of the kernel."""
    err, fmt = _fp8_forward_case(512, 512, 32, 128, seed=1, x_gain=300.0)
    assert err <= TOL_Y and fmt == 1


@pytest.mark.parametrize("n,k,r,m,gain", [(1000, 2048, 64, 300, 1.0), (2100, 4096, 410, 700, 1.0), (384, 640, 90, 129, 1.0),
                                          (512, 512, 32, 128, 300.0)])
def test_gemm_fp8_inputs_with_q4_adapters(n, k, r, m, gain):
    """8-bit inputs and 4-bit adapters together: both operands of T = X R^T are codes (the last case in E5M2)."""
    err, fmt = _fp8_forward_case(n, k, r, m, seed=3, x_gain=gain, bits=4)
    assert err <= TOL_Y and fmt == (1 if gain > 1 else 0)


def test_gemm_fp8_inputs_with_q4_adapters_full_size_sampled_rows():
    shape = wl.L70B_ATTN
    rows = prefill_row_sample(shape.n, 256, seed=5)
    err, _ = _fp8_forward_case(shape.n, shape.k, shape.r, 4096, seed=4, rows=rows, shape=shape, bits=4)
    assert err <= TOL_Y


@pytest.mark.parametrize("shape,m", [(wl.L7B_UP, 2048), (wl.L70B_ATTN, 4096)])
def test_gemm_fp8_inputs_full_size_sampled_rows(shape, m):
    rows = prefill_row_sample(shape.n, 256, seed=3)
    err, _ = _fp8_forward_case(shape.n, shape.k, shape.r, m, seed=2, rows=rows, shape=shape)
    assert err <= TOL_Y


def test_forward_on_fp8_quantized_input():
    shape = _shape(512, 1024, 51)
    W, L, R, X = wl.make_layer(shape, 8, seed=13)
    layer = _gpu_layer(W, L, R)
    Xq, _ = B.slim_input_quant_fp8(X.to(DEV))
    Y = B.slim_linear_gemv(layer, Xq)
    torch.cuda.synchronize()
    ref = O.compress(W.numpy())
    rq, _, _ = O.input_quant_fp8(X.numpy())
    Yo = O.forward(ref, L.numpy(), R.numpy(), rq)
    _assert_layer_close(Y, ref, L.numpy(), R.numpy(), rq, what="forward on fp8-quantized input")
    # and the quantization of the input costs accuracy of the order of its 2 to 3 mantissa bits, not more
    Y0 = O.forward(ref, L.numpy(), R.numpy(), X.numpy())
    assert 1e-3 < _relerr(Yo, Y0) < 0.1


def test_quant_search_rows_on_a_row_whose_two_best_candidates_tie_exactly():
    """The errors at 0.18 M and 0.19 M of this row are the same rational number (pinned on the
    CPU): either is a correct answer, nothing else is, and the rows around it are unaffected."""
    from test_oracle_quant_search import _row_with_two_equal_minima
    w = _row_with_two_equal_minima()
    rng = np.random.default_rng(8)
    W = rng.standard_t(3, size=(9, w.size)).astype(np.float32)
    W[4] = w
    scale, alpha = B.slim_quant_search_rows(torch.from_numpy(W).to(DEV))
    torch.cuda.synchronize()
    _accepted_alpha_rows(W, alpha.cpu().numpy(), scale.cpu().numpy())
    ra, _ = O.quant_search_rows(W)
    keep = np.arange(9) != 4
    assert np.array_equal(alpha.cpu().numpy()[keep].view(np.uint32), ra[keep].view(np.uint32))
    # as a tensor of its own (more bins would need more elements: the same 512 here)
    scale1, alpha1 = B.slim_quant_search(torch.from_numpy(w[None, :].copy()).to(DEV))
    torch.cuda.synchronize()
    _, rs = _accepted_alpha(w[None, :], alpha1.cpu().numpy()[0])
    assert scale1.cpu().numpy()[0].view(np.uint32) == rs.view(np.uint32)


# ---- one workspace, several layers ---------------------------------------------------

@pytest.mark.parametrize("path", ["auto", "parts", "roles", "fused"])
def test_gemv_one_workspace_shared_by_layers_of_different_rank(path, decode_override):
    """Nothing is carried between calls: layers of different shape and rank, fp16 and 4-bit
    adapters, take turns on one workspace, on every decode geometry."""
    decode_override(path)
    cases = []
    for i, (n, k, r) in enumerate([(640, 1024, 51), (300, 2176, 37), (1000, 4096, 100), (48, 4096, 1024)]):
        shape = _shape(n, k, r)
        W, L, R, _ = wl.make_layer(shape, 1, seed=70 + i)
        if i % 2:
            layer = _q4_layer(W, L, R)
            lc, ls = O.quantize_adapter(L.numpy())
            rc, rs = O.quantize_adapter(R.numpy())
            Lr, Rr = O.dequantize_adapter(lc, ls), O.dequantize_adapter(rc, rs)
        else:
            layer, Lr, Rr = _gpu_layer(W, L, R), L.numpy(), R.numpy()
        cases.append((shape, layer, O.compress(W.numpy()), Lr, Rr))
    ws = torch.zeros(max(B.slim_workspace_bytes(c[1], 16) for c in cases), dtype=torch.uint8, device=DEV)
    rng = np.random.default_rng(4)
    for step in range(24):
        shape, layer, ref, Lr, Rr = cases[int(rng.integers(0, len(cases)))]
        m = int(rng.integers(1, 17))
        X = wl.make_activations(m, shape.k, seed=90 + step)
        Y = B.slim_linear_gemv(layer, X.to(DEV), workspace=ws)
        torch.cuda.synchronize()
        _assert_layer_close(Y, ref, Lr, Rr, X, CT_DECODE + CT_Q4, f"step {step} {shape.name} m={m}")
    assert int(ws.view(torch.int32)[2]) == 0


def test_calls_follow_the_current_stream():
    """The binding hands torch's current stream to the library: work enqueued on a side stream is
    ordered after what that stream already holds (a fill of X) and is complete after its
    synchronization, without a device-wide one."""
    shape = _shape(640, 1024, 51)
    W, L, R, X = wl.make_layer(shape, 4, seed=31)
    layer = _gpu_layer(W, L, R)
    ref = O.compress(W.numpy())
    Yo = O.forward(ref, L.numpy(), R.numpy(), X.numpy())
    side = torch.cuda.Stream(device=DEV)                     # default priority
    Xd = torch.zeros_like(X, device=DEV)
    Xsrc = X.to(DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        Xd.copy_(Xsrc, non_blocking=True)                    # on the side stream, ahead of the calls
        Y1 = B.slim_linear_gemv(layer, Xd)
        Y2 = B.slim_linear_gemm(layer, Xd)
    side.synchronize()
    assert _relerr(Y1.cpu().numpy(), Yo) <= TOL_Y and _relerr(Y2.cpu().numpy(), Yo) <= TOL_Y
    _assert_layer_close(Y1, ref, L.numpy(), R.numpy(), X, CT_DECODE, "gemv on a side stream")
    _assert_layer_close(Y2, ref, L.numpy(), R.numpy(), X, CT_PREFILL, "gemm on a side stream")


def test_forward_calls_captured_in_a_graph_replay_correctly():
    """The forward entry points enqueue kernels only, so they can be captured into a HIP graph.
    The one-launch decode kernel tags the pieces of T with a call number; under capture that number
    is advanced on the device by a one-thread kernel ahead of it, so that a replay never takes the
    previous replay's T for its own.  Several replays with different inputs, eager work and
    synchronizations in between, each compared with the eager result and the oracle."""
    shape_a, shape_b = _shape(640, 1024, 51), _shape(300, 2176, 37)
    Wa, La, Ra, _ = wl.make_layer(shape_a, 1, seed=51)
    Wb, Lb, Rb, _ = wl.make_layer(shape_b, 1, seed=52)
    la, lb = _gpu_layer(Wa, La, Ra), _gpu_layer(Wb, Lb, Rb)
    ra, rb = O.compress(Wa.numpy()), O.compress(Wb.numpy())
    ws = torch.zeros(max(B.slim_workspace_bytes(la, 1), B.slim_workspace_bytes(lb, 16), B.slim_workspace_bytes(la, 64)),
                     dtype=torch.uint8, device=DEV)
    x1 = torch.zeros(1, shape_a.k, dtype=torch.float16, device=DEV)
    x16 = torch.zeros(16, shape_b.k, dtype=torch.float16, device=DEV)
    x64 = torch.zeros(64, shape_a.k, dtype=torch.float16, device=DEV)
    y1 = torch.empty(1, shape_a.n, dtype=torch.float16, device=DEV)
    y16 = torch.empty(16, shape_b.n, dtype=torch.float16, device=DEV)
    y64 = torch.empty(64, shape_a.n, dtype=torch.float16, device=DEV)
    ylr = torch.empty(16, shape_b.n, dtype=torch.float16, device=DEV)      # the adapter term of layer b alone
    lowrank_b = lambda y: B.slim_lowrank(x16, lb.R, lb.L, shape_b.n, shape_b.r, y, False, ws)
    for _ in range(2):                                       # eager calls first: the workspace has history
        B.slim_linear_gemv(la, x1, y1, ws)
        B.slim_linear_gemv(lb, x16, y16, ws)
        B.slim_linear_gemm(la, x64, y64, ws)
        lowrank_b(ylr)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.slim_linear_gemv(la, x1, y1, ws)
        B.slim_linear_gemv(lb, x16, y16, ws)
        B.slim_linear_gemm(la, x64, y64, ws)
        lowrank_b(ylr)
    for rep in range(4):
        X1, X16, X64 = (wl.make_activations(m, k, seed=60 + 3 * rep + i) for i, (m, k) in
                        enumerate([(1, shape_a.k), (16, shape_b.k), (64, shape_a.k)]))
        x1.copy_(X1)
        x16.copy_(X16)
        x64.copy_(X64)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [y1.clone(), y16.clone(), y64.clone(), ylr.clone()]
        e1 = B.slim_linear_gemv(la, x1, workspace=ws)        # the program's own eager work between replays
        e16 = B.slim_linear_gemv(lb, x16, workspace=ws)
        e64 = B.slim_linear_gemm(la, x64, workspace=ws)
        elr = lowrank_b(torch.empty_like(ylr))
        torch.cuda.synchronize()
        for g, e in zip(got, (e1, e16, e64, elr)):
            assert torch.equal(g, e), rep
        _assert_lowrank_close(got[3], X16, Rb, Lb, what=f"replay {rep}: slim_lowrank")
        _assert_layer_close(got[0], ra, La.numpy(), Ra.numpy(), X1, CT_DECODE, f"replay {rep}: gemv a")
        _assert_layer_close(got[1], rb, Lb.numpy(), Rb.numpy(), X16, CT_DECODE, f"replay {rep}: gemv b")
        _assert_layer_close(got[2], ra, La.numpy(), Ra.numpy(), X64, CT_PREFILL, f"replay {rep}: gemm a")
    # replays back to back, nothing but new inputs in between: the pieces of T in the workspace are
    # those of the previous replay when the next one starts
    for rep in range(3):
        X1 = wl.make_activations(1, shape_a.k, seed=80 + rep)
        X16 = wl.make_activations(16, shape_b.k, seed=90 + rep)
        x1.copy_(X1)
        x16.copy_(X16)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _assert_layer_close(y1, ra, La.numpy(), Ra.numpy(), X1, CT_DECODE, f"back-to-back replay {rep}: gemv a")
        _assert_layer_close(y16, rb, Lb.numpy(), Rb.numpy(), X16, CT_DECODE, f"back-to-back replay {rep}: gemv b")
        _assert_lowrank_close(ylr, X16, Rb, Lb, what=f"back-to-back replay {rep}: slim_lowrank")
    assert int(ws.view(torch.int32)[2]) == 0
