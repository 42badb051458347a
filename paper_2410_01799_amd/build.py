"""Build libscd.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
SRC = [PKG / "csrc" / name for name in ("scd_kernels.hip", "scd_stream.hip", "scd_resident.hip", "scd_sparse.hip",
                                        "scd_apply.hip", "scd_lsq.hip", "scd_api.hip")]
LIB = PKG / "libscd.so"

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # keep the compiler from forming packed-FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and Path(cand).exists():
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(map(str, cmd)), flush=True)
    res = subprocess.run(list(map(str, cmd)), capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed")
    if verbose and res.stderr.strip():
        sys.stderr.write(res.stderr)


def build(verbose: bool = False, extra=()) -> Path:
    """Compile every source (one hipcc process per file, side by side) and link the shared library.
    Always compiles: nothing is cached between calls."""
    cc = hipcc()
    inc = [f"-I{ROOT / 'include'}", f"-I{PKG / 'csrc'}"]
    with tempfile.TemporaryDirectory(prefix="scd_build_") as tmp:
        objs = [Path(tmp) / (s.stem + ".o") for s in SRC]
        with ThreadPoolExecutor(max_workers=min(len(SRC), os.cpu_count() or 1)) as pool:
            jobs = [pool.submit(_run, [cc, *FLAGS, *extra, *inc, "-c", s, "-o", o], verbose) for s, o in zip(SRC, objs)]
            for j in jobs:
                j.result()
        _run([cc, "--offload-arch=gfx950", "-fno-gpu-rdc", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
