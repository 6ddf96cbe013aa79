"""Builds libgrkan.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libgrkan.so"
SOURCES = [CSRC / "grkan_kernels.hip", CSRC / "grkan_plan.cpp", CSRC / "grkan_alg1_baseline.hip",
           CSRC / "grkan_linear.hip"]
HEADERS = [CSRC / "grkan_walk.h", CSRC / "grkan_plan.h", CSRC / "grkan_elem.h", PKG.parent / "include" / "grkan.h",
           PKG.parent / "include" / "grkan_alg1.h"]

# packed-fp32 code generation is switched off on purpose (hipcc flag, device side)
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not Path(exe).exists():
        raise RuntimeError("hipcc not found; the GR-KAN library cannot be built")
    return exe


def is_stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    return any(p.stat().st_mtime > t for p in SOURCES + HEADERS)


def build_library(force: bool = True, verbose: bool = False) -> Path:
    """Compile the shared library.  `force=False` skips an up-to-date build."""
    if not force and not is_stale():
        return LIB
    tmp = LIB.with_name("libgrkan.so.tmp%d" % os.getpid())
    cmd = [hipcc(), *HIPCC_FLAGS, *map(str, SOURCES), "-o", str(tmp)]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        tmp.unlink(missing_ok=True)
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
