"""Builds liboptgqa.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc.

    python -m paper_2505_02351_amd.build            # compile
    python -m paper_2505_02351_amd.build --asm      # also keep the device assembly in _build/

The build needs no GPU (hipcc cross-compiles).  Packed-fp32 instruction selection is
switched off for all device code.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = os.path.join(PKG, "csrc", "optgqa.hip")
LIB = os.path.join(PKG, "liboptgqa.so")
BUILD_DIR = os.path.join(ROOT, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build(keep_asm: bool = False, verbose: bool = False, defines=(), out: str = LIB) -> str:
    """Compile csrc/optgqa.hip.  `defines` (e.g. ["OPTGQA_RING_TILES=4"]) and `out` exist for
    tuning experiments; the product library is the default call."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    tmp = os.path.join(BUILD_DIR, f"liboptgqa.{os.getpid()}.so")
    cmd = ["hipcc", *HIPCC_FLAGS, *["-D" + d for d in defines], "-I" + os.path.join(ROOT, "include"),
           "-I" + os.path.join(PKG, "csrc"), SRC, "-o", tmp]
    if keep_asm:
        cmd.append("-save-temps=obj")
    res = subprocess.run(cmd, capture_output=True, text=True, cwd=BUILD_DIR)
    noise = "'-packed-fp32-ops' is not a recognized feature"       # host pass does not know the feature
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(keep_asm="--asm" in sys.argv, verbose=True))
