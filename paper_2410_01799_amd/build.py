"""Build libscd.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
SRC = [PKG / "csrc" / "scd_kernels.hip", PKG / "csrc" / "scd_resident.hip", PKG / "csrc" / "scd_sparse.hip", PKG / "csrc" / "scd_apply.hip", PKG / "csrc" / "scd_lsq.hip",
       PKG / "csrc" / "scd_api.hip"]
LIB = PKG / "libscd.so"

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    # keep the compiler from forming packed-FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and Path(cand).exists():
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, extra=()) -> Path:
    cmd = [hipcc(), *FLAGS, *extra, f"-I{ROOT / 'include'}", f"-I{PKG / 'csrc'}", "-o", str(LIB), *map(str, SRC)]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed")
    if verbose and res.stderr.strip():
        sys.stderr.write(res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
