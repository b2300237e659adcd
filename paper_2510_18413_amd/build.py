"""Builds libadamas.so (HIP kernels + C ABI) in-tree with hipcc for gfx950.

The kernels of every (head dimension, metric) pair are instantiated in an object file of their
own (csrc/kernels_inst.hip compiled once per pair), so the pairs compile in parallel; adamas.hip
holds the C ABI and dispatches through the tables those objects export.
"""

from __future__ import annotations

import hashlib
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
API_SRC = CSRC / "adamas.hip"
INST_SRC = CSRC / "kernels_inst.hip"
LIB = PKG / "libadamas.so"
OBJ_DIR = PKG / "_build"

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]
METRICS = 4     # kMetricL1, kMetricL2, kMetricB1, kMetricB3 (csrc/device_utils.hpp)


def head_dims():
    """The head dimensions csrc/kernel_set.hpp lists (ADAMAS_FOR_EACH_HEAD_DIM)."""
    text = (CSRC / "kernel_set.hpp").read_text()
    line = re.search(r"#define ADAMAS_FOR_EACH_HEAD_DIM\(X\)(.*)", text).group(1)
    return [int(d) for d in re.findall(r"X\((\d+)\)", line)]


def sources():
    return sorted(CSRC.glob("*.hip")) + sorted(CSRC.glob("*.hpp")) + [ROOT / "include" / "adamas.h"]


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


def build(verbose: bool = False, extra_flags=(), jobs: int = 0, only=None, out: Path = LIB) -> Path:
    """Compiles everything unconditionally; returns the path of the shared library.

    only=(head_dim, metric) is a developer option for kernel work: a quick build of that single
    pair (metric 0 = the method); the resulting library refuses every other configuration.
    `out` is where the library goes (default: the in-tree libadamas.so that the binding loads).
    """
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(16, os.cpu_count() or 4)
    OBJ_DIR.mkdir(exist_ok=True)
    tag = ".tmp%d" % os.getpid()
    common = [hipcc] + HIPCC_FLAGS + list(extra_flags) + [
        "-I", str(ROOT / "include"), "-I", str(CSRC), "-c"]
    api_flags = ['-DADAMAS_BUILD_ID="%s"' % source_id()]
    pairs = [(d, m) for d in head_dims() for m in range(METRICS)]
    if only is not None:
        pairs = [tuple(only)]
        api_flags += ["-DADAMAS_ONLY_D=%d" % only[0], "-DADAMAS_ONLY_METRIC=%d" % only[1]]
    units = [(OBJ_DIR / ("adamas%s.o" % tag), common + api_flags + [str(API_SRC)])]
    for d, m in pairs:
        units.append((OBJ_DIR / ("kernels_d%d_m%d%s.o" % (d, m, tag)),
                      common + ["-DADAMAS_INST_D=%d" % d, "-DADAMAS_INST_METRIC=%d" % m,
                                str(INST_SRC)]))

    def compile_one(unit):
        obj, cmd = unit
        cmd = cmd + ["-o", str(obj)]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        # hipcc's host pass does not know the packed-fp32 feature and says so: harmless
        out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed (%d): %s\n%s" % (r.returncode, " ".join(cmd), out))
        if out.strip():
            print(out, flush=True)
        return obj

    try:
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            objs = list(pool.map(compile_one, units))
        tmp = Path(str(out) + tag)
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp)] + [str(o) for o in objs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
        os.replace(tmp, out)
    finally:
        for obj, _ in units:
            if obj.exists():
                obj.unlink()
    return out


TRACE_LIB = PKG / "libadamas_trace.so"


def build_phase_trace(verbose: bool = False) -> Path:
    """The profiling build `bench.py --phase-trace` loads: the method's own kernels (head
    dimension 128, Eq. 6) with phase stamps compiled in (-DADAMAS_PHASE_TRACE)."""
    return build(verbose=verbose, extra_flags=["-DADAMAS_PHASE_TRACE"], only=(128, 0), out=TRACE_LIB)


if __name__ == "__main__":
    import sys
    if "--phase-trace" in sys.argv[1:]:
        print(build_phase_trace(verbose=True))
    else:
        print(build(verbose=True))
