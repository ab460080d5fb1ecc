"""Build libsvdp.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "svdp.hip")
# every file the translation unit includes: the library is rebuilt when any of them is newer
DEPS = [SRC, os.path.join(os.path.dirname(HERE), "include", "svdp.h")] + sorted(glob.glob(os.path.join(HERE, "csrc", "*.h")))
LIB = os.path.join(HERE, "libsvdp.so")
PROBE_SRC = os.path.join(HERE, "csrc", "svdp_probe.hip")
PROBE_LIB = os.path.join(HERE, "libsvdp_probe.so")


def hipcc_path() -> str:
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def _hipcc(src: str, out: str, verbose: bool) -> None:
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-function", "-o", out, src]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)


def build_lib(force: bool = True, verbose: bool = False) -> str:
    """Compile the C-ABI library.  Packed-fp32 instructions are disabled on purpose."""
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(p) for p in DEPS):
        return LIB
    _hipcc(SRC, LIB, verbose)
    return LIB


def build_probe(force: bool = True, verbose: bool = False) -> str:
    """Compile the benchmark's measurement helpers (include/svdp_probe.h)."""
    deps = [PROBE_SRC, os.path.join(os.path.dirname(HERE), "include", "svdp_probe.h")]
    if not force and os.path.exists(PROBE_LIB) and all(os.path.getmtime(PROBE_LIB) >= os.path.getmtime(p) for p in deps):
        return PROBE_LIB
    _hipcc(PROBE_SRC, PROBE_LIB, verbose)
    return PROBE_LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
    print(build_probe(verbose=True))
