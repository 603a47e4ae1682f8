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
