"""ctypes binding of libslim (include/slim.h): argument marshalling only.

Every function here has the name and meaning of the C entry point it calls;
torch owns the device memory and the stream, the library does all the work.
There is no fallback: if libslim.so is not built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libslim.so")
_lib = None


class SlimError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__(f"{fn}: {text} (status {status})")
        self.status = status


class slim_shape(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("k", ctypes.c_int32), ("rank", ctypes.c_int32)]


class slim_layer(ctypes.Structure):
    _fields_ = [("shape", slim_shape), ("qvals", ctypes.c_void_p), ("meta", ctypes.c_void_p),
                ("scale", ctypes.c_void_p), ("L", ctypes.c_void_p), ("R", ctypes.c_void_p),
                ("rank_pad", ctypes.c_int32), ("adapter_bits", ctypes.c_int32), ("Lq", ctypes.c_void_p),
                ("Ls", ctypes.c_void_p), ("Rq", ctypes.c_void_p), ("Rs", ctypes.c_void_p)]


SLIM_OK, SLIM_ERR_NULL, SLIM_ERR_SHAPE, SLIM_ERR_ALIGN, SLIM_ERR_WORKSPACE, SLIM_ERR_HIP, SLIM_ERR_WAIT = 0, -1, -2, -3, -4, -5, -6

EXPORTS = ["slim_status_string", "slim_rank_pad", "slim_packed_sizes", "slim_pack", "slim_pack_adapters",
           "slim_unpack", "slim_workspace_bytes", "slim_workspace_check", "slim_decode_override", "slim_decode_plan", "slim_linear_gemv", "slim_linear_gemv_static", "slim_linear_gemm",
           "slim_lowrank",
           "slim_adapter_q4_sizes", "slim_pack_adapters_q4", "slim_unpack_adapters_q4", "slim_pack_ex",
           "slim_quant_workspace_bytes", "slim_quant_search", "slim_quant_search_rows", "slim_adapters_workspace_bytes",
           "slim_compute_adapters", "slim_input_quant_fp8", "slim_probe_read", "slim_probe_mfma", "slim_gemm_tile_order", "slim_input_quant_fp8_codes",
           "slim_linear_gemm_fp8"]


def lib():
    """Load libslim.so once; raise if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2410_09615_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        psz, pi32 = ctypes.POINTER(sz), ctypes.POINTER(i32)
        L.slim_status_string.argtypes = [ctypes.c_int]
        L.slim_status_string.restype = ctypes.c_char_p
        L.slim_rank_pad.argtypes = [i32]
        L.slim_rank_pad.restype = i32
        L.slim_packed_sizes.argtypes = [slim_shape, psz, psz, psz, pi32, psz, psz]
        L.slim_pack.argtypes = [vp, slim_shape, vp, vp, vp, vp]
        L.slim_pack_adapters.argtypes = [vp, vp, slim_shape, vp, vp, vp]
        L.slim_unpack.argtypes = [vp, vp, slim_shape, vp, vp, vp]
        L.slim_workspace_bytes.argtypes = [ctypes.POINTER(slim_layer), i32, psz]
        L.slim_decode_plan.argtypes = [ctypes.POINTER(slim_layer), i32, pi32]
        L.slim_workspace_check.argtypes = [vp, vp]
        L.slim_decode_override.argtypes = [i32, i32]
        L.slim_adapter_q4_sizes.argtypes = [i32, i32, psz, psz]
        L.slim_pack_ex.argtypes = [vp, slim_shape, vp, vp, vp, vp, vp, vp]
        L.slim_quant_workspace_bytes.argtypes = [slim_shape, psz]
        L.slim_quant_search.argtypes = [vp, slim_shape, vp, vp, vp, sz, vp]
        L.slim_quant_search_rows.argtypes = [vp, slim_shape, vp, vp, vp]
        L.slim_adapters_workspace_bytes.argtypes = [slim_shape, psz]
        L.slim_compute_adapters.argtypes = [vp, vp, vp, vp, slim_shape, vp, i32, ctypes.c_uint32, vp, vp, vp, vp, sz, vp]
        L.slim_input_quant_fp8.argtypes = [vp, sz, vp, vp, vp, sz, vp]
        L.slim_probe_read.argtypes = [vp, sz, i32, sz, vp, vp]
        L.slim_probe_mfma.argtypes = [i32, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.slim_pack_adapters_q4.argtypes = [vp, vp, slim_shape, vp, vp, vp, vp, vp]
        L.slim_unpack_adapters_q4.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        L.slim_linear_gemv.argtypes = [ctypes.POINTER(slim_layer), vp, i32, vp, vp, sz, vp]
        L.slim_linear_gemm.argtypes = [ctypes.POINTER(slim_layer), vp, i32, vp, vp, sz, vp]
        L.slim_linear_gemv_static.argtypes = [ctypes.POINTER(slim_layer), vp, i32, vp, vp]
        L.slim_lowrank.argtypes = [vp, i32, vp, vp, slim_shape, i32, vp, ctypes.c_int, vp, sz, vp]
        L.slim_gemm_tile_order.argtypes = [i32, i32, pi32, sz]
        L.slim_input_quant_fp8_codes.argtypes = [vp, sz, vp, vp, vp, vp, sz, vp]
        L.slim_linear_gemm_fp8.argtypes = [ctypes.POINTER(slim_layer), vp, vp, i32, i32, vp, vp, sz, vp]
        for name in EXPORTS[2:]:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(fn: str, status: int):
    if status != SLIM_OK:
        raise SlimError(fn, status, lib().slim_status_string(status).decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(t: torch.Tensor):
    """Raw handle of torch's current stream on t's device."""
    return ctypes.c_void_p(torch._C._cuda_getCurrentRawStream(t.device.index))


def _dev(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous {dtype}")
    return t


def slim_status_string(status: int) -> str:
    return lib().slim_status_string(status).decode()


def slim_rank_pad(rank: int) -> int:
    return int(lib().slim_rank_pad(rank))


def slim_packed_sizes(n: int, k: int, rank: int) -> dict:
    q, me, sc, lb, rb = (ctypes.c_size_t() for _ in range(5))
    rp = ctypes.c_int32()
    _check("slim_packed_sizes", lib().slim_packed_sizes(slim_shape(n, k, rank), q, me, sc, rp, lb, rb))
    return {"qvals": q.value, "meta": me.value, "scale": sc.value, "rank_pad": rp.value,
            "L": lb.value, "R": rb.value}


@dataclass
class SlimLayer:
    """Device buffers of one compressed layer (what `slim_layer` points at)."""
    n: int
    k: int
    rank: int
    rank_pad: int
    qvals: torch.Tensor            # uint8, packed (tiled) layout of the canonical [n][k/4]
    meta: torch.Tensor             # uint8, packed (tiled) layout of the canonical [n][k/8]
    scale: torch.Tensor            # float32 [n]
    L: torch.Tensor | None         # float16, tiled layout of [n][rank_pad]
    R: torch.Tensor | None         # float16, tiled layout of [rank_pad][k]
    adapter_bits: int = 16         # 4: the adapters are Lq, Ls, Rq, Rs (slim_pack_adapters_q4), L and R unused
    Lq: torch.Tensor | None = None
    Ls: torch.Tensor | None = None
    Rq: torch.Tensor | None = None
    Rs: torch.Tensor | None = None

    def c_struct(self) -> slim_layer:
        p = lambda t: t.data_ptr() if t is not None else None
        return slim_layer(slim_shape(self.n, self.k, self.rank), self.qvals.data_ptr(), self.meta.data_ptr(),
                          self.scale.data_ptr(), p(self.L), p(self.R), self.rank_pad, self.adapter_bits,
                          p(self.Lq), p(self.Ls), p(self.Rq), p(self.Rs))

    def c_ref(self):
        """Pointer argument for the forward calls: the struct is built once per layer and rebuilt after
        any field is assigned (a decode call is a few microseconds; building the struct costs one)."""
        ref = self.__dict__.get("_ref")
        if ref is None:
            cs = self.c_struct()
            ref = (ctypes.byref(cs), cs)
            self.__dict__["_ref"] = ref
        return ref[0]

    def __setattr__(self, name, value):
        self.__dict__.pop("_ref", None)
        object.__setattr__(self, name, value)


def slim_pack(W: torch.Tensor, qvals=None, meta=None, scale=None):
    """W fp32 [n][k] on the device -> (qvals, meta, scale) device tensors."""
    _dev(W, torch.float32, "W")
    n, k = W.shape
    sizes = slim_packed_sizes(n, k, 0)
    if qvals is None:
        qvals = torch.empty(sizes["qvals"], dtype=torch.uint8, device=W.device)
        meta = torch.empty(sizes["meta"], dtype=torch.uint8, device=W.device)
        scale = torch.empty(n, dtype=torch.float32, device=W.device)
    _check("slim_pack", lib().slim_pack(_ptr(W), slim_shape(n, k, 0), _ptr(qvals), _ptr(meta), _ptr(scale),
                                        _stream(W)))
    return qvals, meta, scale


def slim_pack_ex(W: torch.Tensor, saliency: torch.Tensor | None = None, scale_in: torch.Tensor | None = None):
    """slim_pack with a saliency-weighted 2:4 mask (saliency fp32 [k]) and/or given scales (fp32 [n])."""
    _dev(W, torch.float32, "W")
    n, k = W.shape
    if saliency is not None:
        _dev(saliency, torch.float32, "saliency")
    if scale_in is not None:
        _dev(scale_in, torch.float32, "scale_in")
    sizes = slim_packed_sizes(n, k, 0)
    qvals = torch.empty(sizes["qvals"], dtype=torch.uint8, device=W.device)
    meta = torch.empty(sizes["meta"], dtype=torch.uint8, device=W.device)
    scale = torch.empty(n, dtype=torch.float32, device=W.device)
    _check("slim_pack_ex", lib().slim_pack_ex(_ptr(W), slim_shape(n, k, 0), _ptr(saliency) if saliency is not None else None,
                                              _ptr(scale_in) if scale_in is not None else None, _ptr(qvals), _ptr(meta),
                                              _ptr(scale), _stream(W)))
    return qvals, meta, scale


def slim_quant_search(W: torch.Tensor):
    """SLiM-Quant scale search: (scale fp32 [n] = alpha* / 7 in every row, alpha* as a 1-element tensor)."""
    _dev(W, torch.float32, "W")
    n, k = W.shape
    nbytes = ctypes.c_size_t()
    _check("slim_quant_workspace_bytes", lib().slim_quant_workspace_bytes(slim_shape(n, k, 0), nbytes))
    ws = torch.empty(nbytes.value, dtype=torch.uint8, device=W.device)
    scale = torch.empty(n, dtype=torch.float32, device=W.device)
    alpha = torch.empty(1, dtype=torch.float32, device=W.device)
    _check("slim_quant_search", lib().slim_quant_search(_ptr(W), slim_shape(n, k, 0), _ptr(scale), _ptr(alpha), _ptr(ws),
                                                        ws.numel(), _stream(W)))
    return scale, alpha


def slim_quant_search_rows(W: torch.Tensor):
    """SLiM-Quant scale search per output row: (scale fp32 [n] = alpha*(o) / 7, alpha* fp32 [n])."""
    _dev(W, torch.float32, "W")
    n, k = W.shape
    scale = torch.empty(n, dtype=torch.float32, device=W.device)
    alpha = torch.empty(n, dtype=torch.float32, device=W.device)
    _check("slim_quant_search_rows", lib().slim_quant_search_rows(_ptr(W), slim_shape(n, k, 0), _ptr(scale), _ptr(alpha),
                                                                  _stream(W)))
    return scale, alpha


def slim_compute_adapters(W: torch.Tensor, qvals, meta, scale, rank: int, x_tilde: torch.Tensor | None = None,
                          iters: int = 0, seed: int = 1):
    """Adapters of a compressed layer (Naive-LoRA when x_tilde is None, else SLiM-LoRA):
    (L fp16 [n][rank], R fp16 [rank][k], diag fp32 [4] = ||S||^2, captured ||L^T S||^2, max|L^T L - I|, 0)."""
    _dev(W, torch.float32, "W")
    n, k = W.shape
    if x_tilde is not None:
        _dev(x_tilde, torch.float32, "x_tilde")
        if x_tilde.numel() != k:
            raise ValueError("x_tilde must have one entry per input")
    shape = slim_shape(n, k, rank)
    nbytes = ctypes.c_size_t()
    _check("slim_adapters_workspace_bytes", lib().slim_adapters_workspace_bytes(shape, nbytes))
    ws = torch.empty(nbytes.value, dtype=torch.uint8, device=W.device)
    L = torch.empty(n, rank, dtype=torch.float16, device=W.device)
    R = torch.empty(rank, k, dtype=torch.float16, device=W.device)
    diag = torch.empty(4, dtype=torch.float32, device=W.device)
    _check("slim_compute_adapters",
           lib().slim_compute_adapters(_ptr(W), _ptr(qvals), _ptr(meta), _ptr(scale), shape, _ptr(x_tilde), iters, seed,
                                       _ptr(L), _ptr(R), _ptr(diag), _ptr(ws), ws.numel(), _stream(W)))
    return L, R, diag


def slim_input_quant_fp8(X: torch.Tensor, Xq=None, info=None, workspace=None, codes=None):
    """FP8 AbsMax quantization of an input tensor, values back on the fp16 grid:
    (Xq fp16 like X, info fp32 [2] = scale, format (0: E4M3, 1: E5M2)).  Xq, info and a
    workspace of at least 1024 bytes may be passed in (a caller in a loop).  codes=True (or a uint8
    tensor of X's size): also the 8-bit codes, for slim_linear_gemm_fp8; returns (Xq, info, codes);
    Xq=False then skips the fp16 output (Xq is returned as None)."""
    _dev(X, torch.float16, "X")
    skip_xq = Xq is False
    if skip_xq and codes is None:
        raise ValueError("nothing to compute: Xq=False needs codes")
    if codes is True:
        codes = torch.empty(X.shape, dtype=torch.uint8, device=X.device)
    if codes is not None and (codes.dtype != torch.uint8 or codes.numel() != X.numel() or codes.device != X.device
                              or not codes.is_contiguous()):
        raise ValueError("codes must be contiguous uint8 with X's size on X's device")
    if skip_xq:
        Xq = None
    elif Xq is None:
        Xq = torch.empty_like(X)
    elif Xq.dtype != torch.float16 or Xq.numel() != X.numel() or Xq.device != X.device or not Xq.is_contiguous():
        raise ValueError("Xq must be contiguous float16 with X's size on X's device")
    if info is None:
        info = torch.empty(2, dtype=torch.float32, device=X.device)
    elif info.dtype != torch.float32 or info.numel() < 2 or info.device != X.device:
        raise ValueError("info must be float32 [2] on X's device")
    ws = workspace if workspace is not None else torch.empty(1024, dtype=torch.uint8, device=X.device)
    if ws.device != X.device:
        raise ValueError("workspace must be on X's device")
    if codes is not None:
        _check("slim_input_quant_fp8_codes", lib().slim_input_quant_fp8_codes(_ptr(X), X.numel(), _ptr(Xq), _ptr(codes), _ptr(info),
                                                                              _ptr(ws), ws.numel(), _stream(X)))
        return Xq, info, codes
    _check("slim_input_quant_fp8", lib().slim_input_quant_fp8(_ptr(X), X.numel(), _ptr(Xq), _ptr(info), _ptr(ws), ws.numel(),
                                                              _stream(X)))
    return Xq, info


def slim_probe_read(buf: torch.Tensor, nbytes: int, repeats: int, stride: int, sink: torch.Tensor):
    """`repeats` streaming reads of nbytes at buf + i * stride (measurement aid; the caller times it)."""
    if (repeats - 1) * stride + nbytes > buf.numel() * buf.element_size():
        raise ValueError("the reads would run past the end of buf")
    _check("slim_probe_read", lib().slim_probe_read(_ptr(buf), nbytes, repeats, stride, _ptr(sink), _stream(buf)))


def slim_probe_mfma(sparse: bool, iters: int, workgroups: int, sink: torch.Tensor) -> float:
    """Back-to-back matrix instructions (measurement aid); returns the FLOPs of the launch."""
    flops = ctypes.c_double()
    _check("slim_probe_mfma", lib().slim_probe_mfma(int(sparse), iters, workgroups, _ptr(sink), ctypes.byref(flops),
                                                    _stream(sink)))
    return flops.value


def slim_pack_adapters(L: torch.Tensor, R: torch.Tensor):
    """L fp16 [n][rank], R fp16 [rank][k] -> (L_pad, R_pad): zero-padded to rank_pad and laid out in
    the kernels' tiled order (flat tensors; sizes from slim_packed_sizes)."""
    _dev(L, torch.float16, "L")
    _dev(R, torch.float16, "R")
    n, rank = L.shape
    k = R.shape[1]
    if R.shape[0] != rank:
        raise ValueError("L and R disagree on the rank")
    sizes = slim_packed_sizes(n, k, rank)
    L_pad = torch.empty(sizes["L"] // 2, dtype=torch.float16, device=L.device)
    R_pad = torch.empty(sizes["R"] // 2, dtype=torch.float16, device=L.device)
    _check("slim_pack_adapters", lib().slim_pack_adapters(_ptr(L), _ptr(R), slim_shape(n, k, rank), _ptr(L_pad),
                                                          _ptr(R_pad), _stream(L)))
    return L_pad, R_pad


def slim_unpack(qvals: torch.Tensor, meta: torch.Tensor, n: int, k: int):
    """(codes int8 [n][k], mask uint8 [n][k]) from the packed bytes of an n x k layer."""
    _dev(qvals, torch.uint8, "qvals")
    _dev(meta, torch.uint8, "meta")
    sizes = slim_packed_sizes(n, k, 0)
    if qvals.numel() < sizes["qvals"] or meta.numel() < sizes["meta"]:
        raise ValueError("packed buffers are smaller than slim_packed_sizes says")
    codes = torch.empty(n, k, dtype=torch.int8, device=qvals.device)
    mask = torch.empty(n, k, dtype=torch.uint8, device=qvals.device)
    _check("slim_unpack", lib().slim_unpack(_ptr(qvals), _ptr(meta), slim_shape(n, k, 0), _ptr(codes), _ptr(mask),
                                            _stream(qvals)))
    return codes, mask


def slim_adapter_q4_sizes(rows: int, cols: int) -> dict:
    c, s = ctypes.c_size_t(), ctypes.c_size_t()
    _check("slim_adapter_q4_sizes", lib().slim_adapter_q4_sizes(rows, cols, c, s))
    return {"codes": c.value, "scales": s.value}


def slim_pack_adapters_q4(L: torch.Tensor, R: torch.Tensor, out=None):
    """L fp16 [n][rank], R fp16 [rank][k] -> (Lq, Ls, Rq, Rs): 4-bit group-128 codes in the kernels'
    layout and fp16 group scales (flat tensors; sizes from slim_adapter_q4_sizes).  `out`: the four
    tensors of an earlier call on the same shape, written in place (then nothing is allocated)."""
    _dev(L, torch.float16, "L")
    _dev(R, torch.float16, "R")
    n, rank = L.shape
    k = R.shape[1]
    if R.shape[0] != rank:
        raise ValueError("L and R disagree on the rank")
    if out is not None:
        Lq, Ls, Rq, Rs = out
        sl, sr = slim_adapter_q4_sizes(n, rank), slim_adapter_q4_sizes(rank, k)
        for t, dt, cnt, name in ((Lq, torch.uint8, sl["codes"], "Lq"), (Ls, torch.float16, sl["scales"] // 2, "Ls"),
                                 (Rq, torch.uint8, sr["codes"], "Rq"), (Rs, torch.float16, sr["scales"] // 2, "Rs")):
            _dev(t, dt, name)
            if t.numel() != cnt:
                raise ValueError(f"{name}: {t.numel()} elements, this shape needs {cnt}")
    else:
        sl, sr = slim_adapter_q4_sizes(n, rank), slim_adapter_q4_sizes(rank, k)
        Lq = torch.empty(sl["codes"], dtype=torch.uint8, device=L.device)
        Ls = torch.empty(sl["scales"] // 2, dtype=torch.float16, device=L.device)
        Rq = torch.empty(sr["codes"], dtype=torch.uint8, device=L.device)
        Rs = torch.empty(sr["scales"] // 2, dtype=torch.float16, device=L.device)
    _check("slim_pack_adapters_q4", lib().slim_pack_adapters_q4(_ptr(L), _ptr(R), slim_shape(n, k, rank), _ptr(Lq),
                                                                _ptr(Ls), _ptr(Rq), _ptr(Rs), _stream(L)))
    return Lq, Ls, Rq, Rs


def slim_gemm_tile_order(n: int, m: int):
    """(tiles, tiles of the whole-tile launch, [tile of workgroup w]) of slim_linear_gemm's main kernel; host logic."""
    tiles = ((n + 511) // 512) * ((m + 127) // 128)
    out = (ctypes.c_int32 * (tiles + 2))()
    _check("slim_gemm_tile_order", lib().slim_gemm_tile_order(n, m, out, tiles + 2))
    return out[0], out[1], list(out[2:2 + out[0]])


def slim_unpack_adapters_q4(codes: torch.Tensor, scales: torch.Tensor, rows: int, cols: int):
    """(codes int8 [rows][cols], scales fp16 [rows][ceil(cols / 128)]) from the 4-bit adapter layout."""
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float16, "scales")
    out_c = torch.empty(rows, cols, dtype=torch.int8, device=codes.device)
    out_s = torch.empty(rows, (cols + 127) // 128, dtype=torch.float16, device=codes.device)
    _check("slim_unpack_adapters_q4", lib().slim_unpack_adapters_q4(_ptr(codes), _ptr(scales), rows, cols, _ptr(out_c),
                                                                    _ptr(out_s), _stream(codes)))
    return out_c, out_s


def compress(W: torch.Tensor, L: torch.Tensor | None = None, R: torch.Tensor | None = None,
             adapter_bits: int = 16) -> SlimLayer:
    """slim_pack (+ slim_pack_adapters, or slim_pack_adapters_q4 with adapter_bits=4) into a SlimLayer."""
    n, k = W.shape
    qvals, meta, scale = slim_pack(W)
    if L is None or L.shape[1] == 0:
        return SlimLayer(n, k, 0, 0, qvals, meta, scale, None, None)
    rank = L.shape[1]
    rp = slim_rank_pad(rank)
    if adapter_bits == 4:
        Lq, Ls, Rq, Rs = slim_pack_adapters_q4(L, R)
        return SlimLayer(n, k, rank, rp, qvals, meta, scale, None, None, 4, Lq, Ls, Rq, Rs)
    Lp, Rp = slim_pack_adapters(L, R)
    return SlimLayer(n, k, rank, rp, qvals, meta, scale, Lp, Rp)


def compress_dense(W: torch.Tensor, rank: int, x_tilde: torch.Tensor | None = None, saliency: torch.Tensor | None = None,
                   scale_search: str = "absmax", adapter_bits: int = 16, iters: int = 0, seed: int = 1,
                   return_adapters: bool = False):
    """The whole offline chain on one dense layer, every step a call of the library:
    scales (AbsMax per row, or slim_quant_search ("tensor") / slim_quant_search_rows ("rows")), 2:4 mask (by magnitude,
    or weighted by `saliency`) and codes (slim_pack / slim_pack_ex), adapters of `rank` (slim_compute_adapters:
    SLiM-LoRA with x_tilde, Naive-LoRA without; rank 0: none), their layout (fp16, or 4-bit groups of 128).
    Returns the SlimLayer, or (SlimLayer, L fp16 [n][rank], R fp16 [rank][k]) with return_adapters."""
    if scale_search == "absmax":
        scale_in = None
    elif scale_search == "tensor":
        scale_in, _ = slim_quant_search(W)
    elif scale_search == "rows":
        scale_in, _ = slim_quant_search_rows(W)
    else:
        raise ValueError("scale_search is 'absmax', 'tensor' or 'rows'")
    n, k = W.shape
    if saliency is None and scale_in is None:
        qvals, meta, scale = slim_pack(W)
    else:
        qvals, meta, scale = slim_pack_ex(W, saliency, scale_in)
    if rank == 0:
        layer = SlimLayer(n, k, 0, 0, qvals, meta, scale, None, None)
        return (layer, None, None) if return_adapters else layer
    L, R, _ = slim_compute_adapters(W, qvals, meta, scale, rank, x_tilde, iters, seed)
    rp = slim_rank_pad(rank)
    if adapter_bits == 4:
        Lq, Ls, Rq, Rs = slim_pack_adapters_q4(L, R)
        layer = SlimLayer(n, k, rank, rp, qvals, meta, scale, None, None, 4, Lq, Ls, Rq, Rs)
    else:
        Lp, Rp = slim_pack_adapters(L, R)
        layer = SlimLayer(n, k, rank, rp, qvals, meta, scale, Lp, Rp)
    return (layer, L, R) if return_adapters else layer


def slim_workspace_bytes(layer: SlimLayer, m: int) -> int:
    out = ctypes.c_size_t()
    cs = layer.c_struct()
    _check("slim_workspace_bytes", lib().slim_workspace_bytes(ctypes.byref(cs), m, out))
    return out.value


def slim_workspace_check(workspace: torch.Tensor | None = None):
    """Raise (status SLIM_ERR_WAIT) if a decode call on this workspace gave up waiting for its own T since the
    last check; synchronizes the current stream.  None: the library's own scratch array."""
    dev = workspace.device.index if workspace is not None else torch.cuda.current_device()
    _check("slim_workspace_check", lib().slim_workspace_check(_ptr(workspace), ctypes.c_void_p(
        torch._C._cuda_getCurrentRawStream(dev))))


DECODE_PATHS = {"auto": -1, "parts": 0, "roles": 1, "fused": 2, "wait_test": 3}


def slim_decode_override(path: str = "auto", lds_kb: int = 0):
    """Test and measurement control: force a decode launch geometry ("parts", "roles", "fused"; "auto" = the
    product path) and/or the LDS the one-launch geometry plans with (0 = the device's)."""
    _check("slim_decode_override", lib().slim_decode_override(DECODE_PATHS[path], lds_kb))


def slim_decode_plan(n: int, k: int, rank: int, m: int, adapter_bits: int = 16) -> dict:
    """Launch geometry slim_linear_gemv would use (host logic only; no device needed)."""
    layer = slim_layer(slim_shape(n, k, rank), None, None, None, None, None, slim_rank_pad(rank), adapter_bits, None, None,
                       None, None)
    out = (ctypes.c_int32 * 12)()
    _check("slim_decode_plan", lib().slim_decode_plan(ctypes.byref(layer), m, out))
    keys = ("path", "workgroups", "threads", "lds_bytes", "r_workgroups", "r_shares", "wavefronts_per_row_tile",
            "working_wavefronts", "helper_wavefronts", "chunk_inputs", "chunks", "y_workgroups")
    return dict(zip(keys, list(out)))


def alloc_workspace(layer: SlimLayer, m: int) -> torch.Tensor:
    return torch.zeros(slim_workspace_bytes(layer, m), dtype=torch.uint8, device=layer.qvals.device)


def _forward(fn_name: str, layer: SlimLayer, X: torch.Tensor, Y, workspace):
    _dev(X, torch.float16, "X")
    m, k = X.shape
    if k != layer.k:
        raise ValueError("X has the wrong number of inputs")
    if Y is None:
        Y = torch.empty(m, layer.n, dtype=torch.float16, device=X.device)
    elif Y.dtype != torch.float16 or Y.numel() != m * layer.n or Y.device != X.device or not Y.is_contiguous():
        raise ValueError("Y must be contiguous float16 [m][n] on X's device")
    if workspace is None:
        workspace = alloc_workspace(layer, m)
    # plain integers for the pointers: with argtypes set ctypes converts them itself
    status = getattr(lib(), fn_name)(layer.c_ref(), X.data_ptr(), m, Y.data_ptr(), workspace.data_ptr(),
                                     workspace.numel(), torch._C._cuda_getCurrentRawStream(X.device.index))
    if status != SLIM_OK:
        _check(fn_name, status)
    return Y


def slim_linear_gemv(layer: SlimLayer, X: torch.Tensor, Y=None, workspace=None) -> torch.Tensor:
    """Decode-shaped forward, 1 <= m <= 16."""
    return _forward("slim_linear_gemv", layer, X, Y, workspace)


def slim_linear_gemv_static(layer: SlimLayer, X: torch.Tensor, Y: torch.Tensor) -> torch.Tensor:
    """slim_linear_gemv on the library's own scratch array: no workspace, and Y is the caller's
    (nothing is allocated on the way)."""
    _dev(X, torch.float16, "X")
    _dev(Y, torch.float16, "Y")
    m, k = X.shape
    if k != layer.k or Y.numel() != m * layer.n or Y.device != X.device:
        raise ValueError("X must be [m][k] and Y [m][n] on one device")
    status = lib().slim_linear_gemv_static(layer.c_ref(), X.data_ptr(), m, Y.data_ptr(),
                                           torch._C._cuda_getCurrentRawStream(X.device.index))
    if status != SLIM_OK:
        _check("slim_linear_gemv_static", status)
    return Y


def slim_linear_gemm(layer: SlimLayer, X: torch.Tensor, Y=None, workspace=None) -> torch.Tensor:
    """Prefill-shaped forward."""
    return _forward("slim_linear_gemm", layer, X, Y, workspace)


def slim_linear_gemm_fp8(layer: SlimLayer, codes: torch.Tensor, info: torch.Tensor, fmt: int, Y=None, workspace=None) -> torch.Tensor:
    """Prefill-shaped forward on 8-bit inputs: codes uint8 [m][k] and info (scale, format) as
    slim_input_quant_fp8(..., codes=True) returns them; fmt = 0 (E4M3) or 1 (E5M2), the format in info[1]."""
    _dev(codes, torch.uint8, "codes")
    _dev(info, torch.float32, "info")
    if codes.dim() != 2 or codes.shape[1] != layer.k or info.numel() < 2:
        raise ValueError("codes must be [m][k], info [2]")
    m = codes.shape[0]
    if Y is None:
        Y = torch.empty(m, layer.n, dtype=torch.float16, device=codes.device)
    if workspace is None:
        workspace = alloc_workspace(layer, m)
    _check("slim_linear_gemm_fp8", lib().slim_linear_gemm_fp8(layer.c_ref(), _ptr(codes), _ptr(info), int(fmt), m, _ptr(Y),
                                                              _ptr(workspace), workspace.numel(), _stream(codes)))
    return Y


def slim_lowrank(X: torch.Tensor, R_pad: torch.Tensor, L_pad: torch.Tensor, n: int, rank: int, Y=None,
                 accumulate: bool = False, workspace=None) -> torch.Tensor:
    """Y [m][n] (+)= (X R^T) L^T with the adapters as produced by slim_pack_adapters."""
    _dev(X, torch.float16, "X")
    _dev(R_pad, torch.float16, "R_pad")
    _dev(L_pad, torch.float16, "L_pad")
    m, k = X.shape
    rp = slim_rank_pad(rank)
    if Y is None:
        if accumulate:
            raise ValueError("accumulate needs Y")
        Y = torch.empty(m, n, dtype=torch.float16, device=X.device)
    if workspace is None:
        tmp = SlimLayer(n, k, rank, rp, X, X, X, L_pad, R_pad)
        workspace = torch.zeros(slim_workspace_bytes(tmp, m), dtype=torch.uint8, device=X.device)
    _check("slim_lowrank", lib().slim_lowrank(_ptr(X), m, _ptr(R_pad), _ptr(L_pad), slim_shape(n, k, rank), rp,
                                              _ptr(Y), 1 if accumulate else 0, _ptr(workspace), workspace.numel(),
                                              _stream(X)))
    return Y
