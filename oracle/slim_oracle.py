"""Python face of the CPU oracle (oracle/slim_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark.  It imports nothing from the product
package and the product package imports nothing from here.

All arrays are numpy, on the host.  fp16 inputs (X, L, R) are widened to
float64 (exact) before they reach the C code.  Orientation is nn.Linear's:
W [n][k], L [n][r], R [r][k], X [m][k], Y [m][n]; the paper's
``Y = X W^C + (X L) R`` (Sec. 3.2) with every matrix transposed.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slim_oracle.c")
_LIB = os.path.join(_HERE, "libslim_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile slim_oracle.c with gcc (IEEE semantics, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.slim_oracle_threads.restype = ctypes.c_int
        for name, args in {
            "slim_oracle_mask": [p, i64, i64, p],
            "slim_oracle_scale": [p, i64, i64, p],
            "slim_oracle_quantize": [p, p, p, i64, i64, p],
            "slim_oracle_pack": [p, p, i64, i64, p, p],
            "slim_oracle_unpack": [p, p, i64, i64, p, p],
            "slim_oracle_dequant": [p, p, p, i64, i64, p],
            "slim_oracle_xr": [p, p, i64, i64, i64, p],
            "slim_oracle_forward": [p, p, p, p, p, p, i64, i64, i64, i64, p, i64, p, p],
        }.items():
            fn = getattr(lib, name)
            fn.argtypes = args
            fn.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().slim_oracle_threads())


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what} failed with code {rc}")


# ---- steps 1-3 ---------------------------------------------------------------

def mask_2of4(W: np.ndarray, saliency: np.ndarray | None = None) -> np.ndarray:
    """2:4 mask of W [n][k] (float32): uint8, 1 = kept.  Of every 4 consecutive
    inputs the two of largest |w| are kept; with `saliency` [k] (one non-negative
    number per input, e.g. the activation norm of Wanda's metric, Sec. 4) the two
    of largest |w| * saliency[input], the product taken in binary32.  Ties: the
    lower position first."""
    W = _c(W, np.float32)
    if saliency is not None:
        sal = _c(saliency, np.float32)
        assert sal.shape == (W.shape[1],) and np.all(sal >= 0)
        W = _c(np.abs(W) * sal[None, :], np.float32)         # binary32 products; the C code takes magnitudes of it
    n, k = W.shape
    mask = np.empty((n, k), np.uint8)
    _check(_load().slim_oracle_mask(_ptr(W), n, k, _ptr(mask)), "mask")
    return mask


def row_scale(W: np.ndarray) -> np.ndarray:
    """Per-row AbsMax scale max|w| / 7 in binary32 (1.0 for an all-zero row)."""
    W = _c(W, np.float32)
    n, k = W.shape
    s = np.empty((n,), np.float32)
    _check(_load().slim_oracle_scale(_ptr(W), n, k, _ptr(s)), "scale")
    return s


def quantize(W: np.ndarray, mask: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """int8 codes in [-8, 7] at kept positions, 0 elsewhere (Sec. 3.1 Eq. 2)."""
    W = _c(W, np.float32)
    mask = _c(mask, np.uint8)
    scale = _c(scale, np.float32)
    n, k = W.shape
    assert mask.shape == (n, k) and scale.shape == (n,)
    codes = np.empty((n, k), np.int8)
    _check(_load().slim_oracle_quantize(_ptr(W), _ptr(mask), _ptr(scale), n, k, _ptr(codes)),
           "quantize")
    return codes


# ---- steps 4-5 ---------------------------------------------------------------

def pack(codes: np.ndarray, mask: np.ndarray):
    """Canonical bytes: qvals [n][k/4], meta [n][k/8]."""
    codes = _c(codes, np.int8)
    mask = _c(mask, np.uint8)
    n, k = codes.shape
    assert mask.shape == (n, k)
    qvals = np.empty((n, k // 4), np.uint8)
    meta = np.empty((n, k // 8), np.uint8)
    _check(_load().slim_oracle_pack(_ptr(codes), _ptr(mask), n, k, _ptr(qvals), _ptr(meta)), "pack")
    return qvals, meta


def unpack(qvals: np.ndarray, meta: np.ndarray):
    """Inverse of pack: (codes int8 [n][k], mask uint8 [n][k])."""
    qvals = _c(qvals, np.uint8)
    meta = _c(meta, np.uint8)
    n, kq = qvals.shape
    k = kq * 4
    assert meta.shape == (n, k // 8)
    codes = np.empty((n, k), np.int8)
    mask = np.empty((n, k), np.uint8)
    _check(_load().slim_oracle_unpack(_ptr(qvals), _ptr(meta), n, k, _ptr(codes), _ptr(mask)),
           "unpack")
    return codes, mask


def dequant(qvals: np.ndarray, meta: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Dense dequantized weights Wd [n][k] in float64."""
    qvals = _c(qvals, np.uint8)
    meta = _c(meta, np.uint8)
    scale = _c(scale, np.float32)
    n, kq = qvals.shape
    k = kq * 4
    Wd = np.empty((n, k), np.float64)
    _check(_load().slim_oracle_dequant(_ptr(qvals), _ptr(meta), _ptr(scale), n, k, _ptr(Wd)),
           "dequant")
    return Wd


@dataclass
class PackedLayer:
    qvals: np.ndarray   # uint8 [n][k/4]
    meta: np.ndarray    # uint8 [n][k/8]
    scale: np.ndarray   # float32 [n]

    @property
    def n(self):
        return self.qvals.shape[0]

    @property
    def k(self):
        return self.qvals.shape[1] * 4


def compress(W: np.ndarray) -> PackedLayer:
    """Steps 1-4 in order: mask on the fp32 magnitudes, scale, quantize, pack."""
    mask = mask_2of4(W)
    scale = row_scale(W)
    codes = quantize(W, mask, scale)
    qvals, meta = pack(codes, mask)
    return PackedLayer(qvals, meta, scale)


# ---- step 6 --------------------------------------------------------------------

def xr(X: np.ndarray, R: np.ndarray) -> np.ndarray:
    """T = X R^T in float64, plain loops."""
    X = _c(X, np.float64)
    R = _c(R, np.float64)
    m, k = X.shape
    r = R.shape[0]
    assert R.shape == (r, k)
    T = np.empty((m, r), np.float64)
    _check(_load().slim_oracle_xr(_ptr(X), _ptr(R), m, k, r, _ptr(T)), "xr")
    return T


def forward(layer: PackedLayer, L, R, X, rows=None, return_t: bool = False):
    """Route (i): Y from the packed bytes, float64, [m][n] (or [m][len(rows)]).
    return_t: also the intermediate T = X R^T [m][r] the call used (None without adapters)."""
    X = _c(X, np.float64)
    m, k = X.shape
    n = layer.n
    assert k == layer.k
    r = 0
    if L is not None:
        L = _c(L, np.float64)
        R = _c(R, np.float64)
        r = L.shape[1]
        assert L.shape == (n, r) and R.shape == (r, k)
        if r == 0:
            L = R = None
    rows_arr = None
    nrows = n
    if rows is not None:
        rows_arr = _c(np.asarray(rows), np.int64)
        nrows = rows_arr.shape[0]
    Y = np.empty((m, nrows), np.float64)
    qv, me, sc = _c(layer.qvals, np.uint8), _c(layer.meta, np.uint8), _c(layer.scale, np.float32)
    T = np.empty((m, r), np.float64) if (return_t and r > 0) else None
    _check(_load().slim_oracle_forward(_ptr(qv), _ptr(me), _ptr(sc), _ptr(L), _ptr(R), _ptr(X),
                                       n, k, r, m, _ptr(rows_arr), nrows, _ptr(Y), _ptr(T)), "forward")
    return (Y, T) if return_t else Y


def forward_explicit_dense(W: np.ndarray, L, R, X) -> np.ndarray:
    """Route (ii): never packs.  Builds Wd = mask * codes * scale directly from
    steps 1-3, forms the dense n x k product L R, and multiplies once:
    Y = X (Wd + L R)^T.  For tiny shapes (it materialises n x k matrices)."""
    mask = mask_2of4(W)
    scale = row_scale(W)
    codes = quantize(W, mask, scale)
    Wd = mask.astype(np.float64) * codes.astype(np.float64) * scale.astype(np.float64)[:, None]
    X = np.asarray(X, np.float64)
    if L is not None and np.asarray(L).shape[1] > 0:
        Wd = Wd + np.asarray(L, np.float64) @ np.asarray(R, np.float64)
    return X @ Wd.T


# ---- quantized adapters (Sec. 3.3, "Low-rank Adapter Quantization") -----------------
# Plain numpy, one group at a time.  The steps that decide an integer (the scale
# that is stored, the division, the rounding) are taken in the precision the
# stored format fixes: the scale is a binary16 number, the quotient is binary32.

ADAPTER_GROUP = 128


def quantize_adapter(A: np.ndarray):
    """4-bit AbsMax group quantization of one adapter matrix A [rows][cols] (fp16).

    Every row is cut into groups of 128 consecutive elements (the last group of
    a row may be shorter).  Per group: scale = max|a| / 7 in binary32, rounded to
    binary16 (that is the number stored); a group of zeros gets scale 1, a scale
    that rounds to zero gets the smallest positive binary16 number.  Codes:
    clamp(rint(a / scale), -8, 7) with the quotient in binary32 and ties to even
    (the clamp never acts: |a / scale| <= 7 (1 + 2^-11)).
    Returns (codes int8 [rows][cols], scales float16 [rows][ceil(cols / 128)])."""
    A = np.asarray(A)
    assert A.dtype == np.float16 and A.ndim == 2
    rows, cols = A.shape
    groups = (cols + ADAPTER_GROUP - 1) // ADAPTER_GROUP
    codes = np.zeros((rows, cols), np.int8)
    scales = np.ones((rows, groups), np.float16)
    tiny = np.float16(2.0 ** -24)
    for r in range(rows):
        for g in range(groups):
            seg = A[r, g * ADAPTER_GROUP:(g + 1) * ADAPTER_GROUP].astype(np.float32)
            amax = np.float32(np.max(np.abs(seg)))
            if amax == 0:
                s16 = np.float16(1.0)
            else:
                s16 = np.float16(np.float32(amax / np.float32(7.0)))
                if s16 == 0:
                    s16 = tiny
            q = np.rint(seg / np.float32(s16))              # binary32 quotient, ties to even
            codes[r, g * ADAPTER_GROUP:(g + 1) * ADAPTER_GROUP] = np.clip(q, -8, 7).astype(np.int8)
            scales[r, g] = s16
    return codes, scales


def dequantize_adapter(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """code * scale of its group, exact in float64: [rows][cols]."""
    codes = np.asarray(codes, np.int8)
    scales = np.asarray(scales, np.float16)
    rows, cols = codes.shape
    out = np.empty((rows, cols), np.float64)
    for g in range(scales.shape[1]):
        sl = slice(g * ADAPTER_GROUP, min(cols, (g + 1) * ADAPTER_GROUP))
        out[:, sl] = codes[:, sl].astype(np.float64) * scales[:, g].astype(np.float64)[:, None]
    return out


# ---- SLiM-Quant: per-tensor scale by numerical integration over the histogram --------
# (Sec. 3.1, Eq. 4-7 and Alg. 1.)  Plain numpy, float64 for the error sums; the
# bin of an element is decided in binary32 so that the counts are integers that
# any implementation reproduces.

def quant_bins(numel: int) -> int:
    """Histogram resolution: one bin per 1000 elements, between 512 and 20000
    (App. "Implementation Details")."""
    return max(512, min(numel // 1000, 20000))


def quant_histogram(W: np.ndarray):
    """(counts int64 [B], M): histogram of |W| over [0, M], M = max|W|, B uniform
    bins; bin = min(B - 1, floor(|w| * (B / M))) with B / M and the product in
    binary32.  M == 0: all counts in bin 0."""
    a = np.abs(np.asarray(W, np.float32)).ravel()
    B = quant_bins(a.size)
    M = np.float32(a.max())
    if M == 0:
        counts = np.zeros(B, np.int64)
        counts[0] = a.size
        return counts, M
    inv = np.float32(np.float32(B) / M)
    b = np.minimum(np.floor(a * inv).astype(np.int64), B - 1)
    return np.bincount(b, minlength=B).astype(np.int64), M


def quant_error(counts: np.ndarray, M, alpha: float) -> float:
    """E_quant(alpha) + E_clip(alpha) (Eq. 5-7) with the density replaced by the
    histogram: every element of a bin sits at the bin's centre.  Symmetric 4-bit
    grid with 7 steps up to alpha: a magnitude x <= alpha becomes
    rint(x / (alpha / 7)) * (alpha / 7), a larger one is clipped to alpha."""
    B = counts.shape[0]
    x = (np.arange(B, dtype=np.float64) + 0.5) * (float(M) / B)
    step = alpha / 7.0
    inside = x <= alpha
    err = np.where(inside, np.rint(x / step) * step - x, alpha - x)
    return float(np.dot(counts.astype(np.float64), err * err))


def quant_search_candidates(W: np.ndarray, coarse_pick=None):
    """The candidates of Alg. 1 in the order they are tried, and their errors:
    10 uniform samples alpha = M i / 10, i = 1..10 (the last one is AbsMax), then 21
    samples of a tenth of that spacing around the best one (those inside (0, M]).
    `coarse_pick` puts the fine samples around that coarse candidate instead (0..9;
    for the treatment of ties only).  Returns (candidates, errors), lists of float;
    empty for a zero tensor."""
    counts, M = quant_histogram(W)
    if M == 0:
        return [], []
    eta = float(M) / 10.0
    cand = [eta * i for i in range(1, 11)]
    errs = [quant_error(counts, M, a) for a in cand]
    lo = cand[int(np.argmin(errs)) if coarse_pick is None else coarse_pick]
    for j in range(-10, 11):
        a = lo + eta * (j / 10.0)
        if 0.0 < a <= float(M):
            cand.append(a)
            errs.append(quant_error(counts, M, a))
    return cand, errs


def quant_search(W: np.ndarray):
    """alpha* of Alg. 1: the first minimum of the error over quant_search_candidates.
    Returns (alpha float32, scale float32 = alpha / 7 in binary32, or 1 for a zero
    tensor).

    The errors are sums of up to 20000 non-negative binary64 terms.  With alpha / M a
    multiple of 1/100 and the bin centres multiples of M / 2B they are, up to the
    factor M^2, rationals with a small common denominator, so two candidates CAN have
    exactly equal errors; which of them a binary64 evaluation calls smaller then
    depends on the order of its additions.  A caller comparing another
    implementation against this one has to accept any candidate whose error is
    within that rounding error of the minimum (tests: quant_search_accepts)."""
    cand, errs = quant_search_candidates(W)
    if not cand:
        return np.float32(0.0), np.float32(1.0)
    alpha = np.float32(cand[int(np.argmin(errs))])
    return alpha, np.float32(alpha / np.float32(7.0))


def quant_search_accepts(W: np.ndarray, alpha, rel: float = 1e-12) -> bool:
    """True if `alpha` (binary32) is what Alg. 1 can return for W when errors closer
    than `rel` (relative; the rounding error of a sum of 20000 binary64 terms is below
    5e-12, of 512 terms below 2e-13) count as equal: a candidate whose error is within
    `rel` of the smallest one, on the fine grid around a coarse candidate that is
    itself within `rel` of the best coarse one.  A zero tensor accepts alpha = 0 only."""
    cand, errs = quant_search_candidates(W)
    if not cand:
        return float(alpha) == 0.0
    coarse_best = min(errs[:10])
    for c in range(10):
        if errs[c] > coarse_best * (1.0 + rel):
            continue
        cv, ev = quant_search_candidates(W, coarse_pick=c)
        best = min(ev)
        if any(np.float32(a) == np.float32(alpha) and e <= best * (1.0 + rel) for a, e in zip(cv, ev)):
            return True
    return False


def quant_search_rows(W: np.ndarray):
    """Alg. 1 with one scale per output row (the granularity of the packed format):
    every row is searched as a tensor of its own.  Returns (alpha float32 [n],
    scale float32 [n])."""
    W = np.asarray(W, np.float32)
    res = [quant_search(W[o]) for o in range(W.shape[0])]
    return (np.array([r[0] for r in res], np.float32), np.array([r[1] for r in res], np.float32))

# ---- low-rank adapters: Naive-LoRA and SLiM-LoRA (Sec. 3.2, Eq. 8-11, Alg. 2) ----------
# Plain numpy in float64; the SVD is LAPACK's.  Orientation as everywhere in this
# file: the paper's matrices transposed.  The paper's saliency diag(x) W scales
# the input channels, which are the COLUMNS of W [n][k] here: S = E diag(x).

def saliency_shift(x_tilde: np.ndarray) -> np.ndarray:
    """x = x~ + min|x~| (Alg. 2, the step that keeps diag(x) invertible).  x~ is the
    per-input-channel average magnitude of the calibration inputs; it has to be
    positive and finite (with a zero entry the shift is zero and diag(x) singular)."""
    x_tilde = np.asarray(x_tilde, np.float64)
    assert x_tilde.ndim == 1 and np.all(np.isfinite(x_tilde)) and np.all(x_tilde > 0)
    return x_tilde + np.min(np.abs(x_tilde))


def compute_adapters(W: np.ndarray, Wc: np.ndarray, x_tilde, rank: int):
    """Adapters with W ~= Wc + L R (Sec. 3.2), rank r, minimising the saliency-weighted
    error ||(W - Wc - L R) diag(x)||_F (Eq. 9-11).

    Steps of Alg. 2: E = W - Wc (the sign that makes W ~= Wc + L R); x from
    saliency_shift (x_tilde None: x = 1, which is Naive-LoRA); S = E diag(x);
    S = U Sigma V^T; the factor on the input-channel side carries Sigma and the
    inverse saliency:  L = U_r [n][r],  R = Sigma_r V_r^T diag(1 / x) [r][k].
    Returns (L, R, singular values of S), float64."""
    W = np.asarray(W, np.float64)
    Wc = np.asarray(Wc, np.float64)
    n, k = W.shape
    assert Wc.shape == (n, k) and 1 <= rank <= min(n, k)
    x = np.ones(k) if x_tilde is None else saliency_shift(x_tilde)
    assert x.shape == (k,)
    E = W - Wc
    S = E * x[None, :]
    U, s, Vt = np.linalg.svd(S, full_matrices=False)
    L = U[:, :rank]
    R = (s[:rank, None] * Vt[:rank, :]) / x[None, :]
    return L, R, s


# ---- 8-bit input quantization (App. "Input Quantization") ------------------------------
# AbsMax quantization of an input tensor to an FP8 format with one scale per tensor, as
# the paper evaluates it (the quantized values, put back on the fp16 grid, are what the
# layer then sees).  E4M3 and E5M2 are the OCP 8-bit formats: 4 exponent bits (bias 7),
# 3 mantissa bits, largest finite value 448, subnormal spacing 2^-9; and 5 exponent bits
# (bias 15), 2 mantissa bits, largest finite value 57344, subnormal spacing 2^-16.

FP8_FORMATS = {"e4m3": (3, -6, 448.0), "e5m2": (2, -14, 57344.0)}      # mantissa bits, smallest normal exponent, largest value


def fp8_round(v: np.ndarray, fmt: str) -> np.ndarray:
    """Nearest value of the format (ties to even mantissa), |v| limited to the largest finite one;
    the sign is kept also where the magnitude rounds to zero (IEEE 754 rounding, signed zeros)."""
    p, emin, fmax = FP8_FORMATS[fmt]
    v = np.asarray(v, np.float64)
    a = np.minimum(np.abs(v), fmax)
    e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.maximum(e, emin)
    q = np.exp2(e - p)                               # spacing of the format at this magnitude
    r = np.rint(a / q) * q                           # rint: ties to even; a / q is exact (power of two)
    return np.copysign(np.minimum(r, fmax), v)      # the formats have signed zeros: what rounds to zero keeps its sign


def fp8_encode(v: np.ndarray, fmt: str) -> np.ndarray:
    """8-bit codes (uint8) of values that lie on the format's grid, as fp8_round returns them: sign in
    bit 7, then the exponent field (bias 1 - smallest normal exponent: 7 for E4M3, 15 for E5M2) and the
    mantissa; below the smallest normal value the exponent field is 0 and the mantissa counts the
    format's smallest spacing."""
    p, emin, fmax = FP8_FORMATS[fmt]
    v = np.asarray(v, np.float64)
    a = np.abs(v)
    assert np.all(a <= fmax)
    e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    sub = a < 2.0 ** emin
    field = np.where(sub, 0.0, e + (1 - emin))
    mant = np.where(sub, a / 2.0 ** (emin - p), (a / np.exp2(e) - 1.0) * (1 << p))
    assert np.array_equal(mant, np.rint(mant)), "a value off the format's grid"
    return ((np.signbit(v).astype(np.int64) << 7) | (field.astype(np.int64) << p) | mant.astype(np.int64)).astype(np.uint8)


def input_quant_fp8_codes(X: np.ndarray):
    """(codes uint8, scale, format) of the same quantization as input_quant_fp8: the 8-bit codes of
    fp8_round(x / scale), i.e. of the quantized values before they go back to the fp16 grid."""
    X = np.asarray(X)
    _, s, fmt = input_quant_fp8(X)
    qv = fp8_round((X.astype(np.float32) / s).astype(np.float32), fmt)
    return fp8_encode(qv, fmt), s, fmt


def input_quant_fp8(X: np.ndarray):
    """X fp16 -> (X' fp16, scale float32, format name).  M = max|X|; the format is E4M3 unless
    M exceeds its largest value 448, then E5M2; scale = M / (largest value of the format) in
    binary32 (1 for a zero tensor); every element becomes fp8_round(x / scale) * scale, the
    quotient and the product in binary32, the result rounded to fp16."""
    X = np.asarray(X)
    assert X.dtype == np.float16
    xf = X.astype(np.float32)
    M = np.float32(np.max(np.abs(xf))) if xf.size else np.float32(0)
    fmt = "e4m3" if M <= np.float32(448.0) else "e5m2"
    fmax = np.float32(FP8_FORMATS[fmt][2])
    s = np.float32(1.0) if M == 0 else np.float32(M / fmax)
    qv = fp8_round((xf / s).astype(np.float32), fmt).astype(np.float32)
    return (qv * s).astype(np.float32).astype(np.float16), s, fmt
