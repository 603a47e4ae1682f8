"""Build libslim.so (the HIP kernels + C-ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys
import tempfile

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libslim.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-munsafe-fp-atomics",
    # The prefill kernel addresses the accumulation registers by number from asm;
    # the compiler must not park spilled values there.
    "-mllvm", "-amdgpu-spill-vgpr-to-agpr=0",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


# Sources whose kernels address the accumulation registers by number (slim_mma.h).
FIXED_ACC_SOURCES = ("slim_gemm", "slim_gemm_sparse")
_MATRIX_OP = re.compile(r"^\s*v_(mfma|smfmac)_")
_COMPILER_AGPR = re.compile(r"\ba\d+\b|\ba\[\d+:\d+\]")


def compiler_agpr_uses(asm_text: str) -> dict:
    """kernel -> instructions in which the compiler itself names an accumulation register.

    The hand-written asm of those sources spells single registers a[N] and only the matrix instructions
    take ranges; anything else (aN, or a range on a load or move) is the register allocator parking a
    value of its own there, where the kernel's matrix instructions will overwrite it."""
    out, name = {}, None
    for line in asm_text.splitlines():
        if line[:1] not in (" ", "\t", ""):
            head = line.split(":")[0]
            if line.rstrip().endswith(":") and not head.startswith("."):
                name = head
            continue
        code = line.split(";")[0]
        if name is None or not code.strip() or code.lstrip().startswith(".") or _MATRIX_OP.match(code):
            continue
        if _COMPILER_AGPR.search(code):
            out[name] = out.get(name, 0) + 1
    return out


def build(verbose: bool = False) -> str:
    """Compile the library; the device assembly of the fixed-accumulator kernels (a by-product of the same
    compilation) is checked for accumulation registers used by the compiler."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-save-temps", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    with tempfile.TemporaryDirectory(prefix="slim_build_") as tmp:
        subprocess.run(cmd, check=True, cwd=tmp)
        for stem in FIXED_ACC_SOURCES:
            with open(os.path.join(tmp, stem + "-hip-amdgcn-amd-amdhsa-gfx950.s")) as fh:
                bad = compiler_agpr_uses(fh.read())
            if bad:
                os.remove(LIB)
                raise RuntimeError(f"{stem}.hip: the compiler uses accumulation registers of kernels that address them "
                                   f"by number (their results would be overwritten): {bad}")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    print(LIB)
    sys.exit(0)
