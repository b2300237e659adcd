"""Builds libadamas.so (HIP kernels + C ABI) in-tree with hipcc for gfx950."""

from __future__ import annotations

import os
import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
SRC = PKG / "csrc" / "adamas.hip"
LIB = PKG / "libadamas.so"

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [SRC] + sorted((PKG / "csrc").glob("*.hpp")) + [ROOT / "include" / "adamas.h"]


def is_stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    return any(s.stat().st_mtime > t for s in sources())


def build(verbose: bool = False, extra_flags=()) -> Path:
    """Compiles unconditionally; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + [
        "-I", str(ROOT / "include"), "-I", str(PKG / "csrc"), "-o", str(tmp), str(SRC)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
