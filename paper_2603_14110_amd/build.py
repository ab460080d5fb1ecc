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


def hipcc_path() -> str:
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build_lib(force: bool = True, verbose: bool = False) -> str:
    """Compile the C-ABI library.  Packed-fp32 instructions are disabled on purpose."""
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(p) for p in DEPS):
        return LIB
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-function", "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
