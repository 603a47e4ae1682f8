"""The library's device layouts, written out from their definition in include/slim.h.

Test-side only: independent of the HIP sources, used to compare device buffers
with row-major references.
"""
import numpy as np


def tile_fp16(mat: np.ndarray, rows_to: int = 32, cols_to: int = 16) -> np.ndarray:
    """Tiled layout of an fp16 matrix [rows][K]: tiles of 32 rows x 16 columns (1 KiB),
    row tile major; inside a tile the pieces of 8 columns are ordered (column half, row).
    Rows are padded to a multiple of 32 and columns to a multiple of 16 with zeros."""
    rows, cols = mat.shape
    rp = -(-rows // rows_to) * rows_to
    cp = -(-cols // cols_to) * cols_to
    full = np.zeros((rp, cp), dtype=mat.dtype)
    full[:rows, :cols] = mat
    # [row tile][row in tile][col tile][half][8] -> [row tile][col tile][half][row in tile][8]
    t = full.reshape(rp // 32, 32, cp // 16, 2, 8).transpose(0, 2, 3, 1, 4)
    return np.ascontiguousarray(t).reshape(-1)


def tile_packed(q: np.ndarray, meta: np.ndarray):
    """Packed layout of the canonical qvals [n][k/4] and meta [n][k/8]: tiles of 32 rows x 128
    inputs (32 code bytes / 16 position bytes per row), row tile major; inside a tile the pieces
    of 64 inputs are ordered (input half, row).  Rows padded to 32, inputs to 128, with zeros."""
    n, g = q.shape
    npad = -(-n // 32) * 32
    kt = -(-g // 32)
    qf = np.zeros((npad, kt * 32), np.uint8)
    qf[:n, :g] = q
    mf = np.zeros((npad, kt * 16), np.uint8)
    mf[:n, : meta.shape[1]] = meta
    qt = qf.reshape(npad // 32, 32, kt, 2, 16).transpose(0, 2, 3, 1, 4)
    mt = mf.reshape(npad // 32, 32, kt, 2, 8).transpose(0, 2, 3, 1, 4)
    return np.ascontiguousarray(qt).reshape(-1), np.ascontiguousarray(mt).reshape(-1)
