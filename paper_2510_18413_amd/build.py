"""Builds libadamas.so (HIP kernels + C ABI) in-tree with hipcc for gfx950."""

from __future__ import annotations

import hashlib
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


BUILD_ID_TAG = b"ADAMAS_BUILD_ID="


def source_id() -> str:
    """Hash of every source file and of the compiler flags: what a library built now would carry."""
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for s in sources():
        h.update(s.name.encode() + b"\0" + s.read_bytes())
    return h.hexdigest()[:16]


def built_id(lib: Path = LIB):
    """Build id stored in a built library (read from the file, nothing is loaded); None if absent."""
    if not lib.exists():
        return None
    blob = lib.read_bytes()
    at = blob.find(BUILD_ID_TAG)
    if at < 0:
        return None
    at += len(BUILD_ID_TAG)
    return blob[at:at + 16].decode("ascii", "replace")


def is_stale() -> bool:
    """True when the built library is missing or was built from other sources than the tree's."""
    return built_id() != source_id()


def build(verbose: bool = False, extra_flags=()) -> Path:
    """Compiles unconditionally; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ['-DADAMAS_BUILD_ID="%s"' % source_id()] + [
        "-I", str(ROOT / "include"), "-I", str(PKG / "csrc"), "-o", str(tmp), str(SRC)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
