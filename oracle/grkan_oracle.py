"""ctypes front end of the fp64 C oracle (oracle/grkan_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the bench's
CPU-baseline leg.  It never imports the GPU package and the GPU package never
imports it.

The functions follow the FlashKAT paper's definition of the group-wise rational
function (Eq. "pade") and of its gradients (Eq. "grad_a", "grad_b", "grad_x",
"accum", "accum2"); see the header comment of the C file for the formulas and
the readings taken where the paper is silent.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "grkan_oracle.c"
_LIB = _HERE / "libgrkan_oracle.so"

_lib = None


def build(force: bool = False) -> Path:
    """Compile the C oracle with the host gcc (no fast-math, so the compensated
    sums survive optimisation)."""
    if force or (not _LIB.exists()) or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
               "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        dp = ctypes.POINTER(ctypes.c_double)
        i64, i32 = ctypes.c_int64, ctypes.c_int
        lib.grkan_oracle_fwd.argtypes = [dp, dp, dp, dp, i64, i32, i32, i32, i32, i32]
        lib.grkan_oracle_fwd.restype = i32
        lib.grkan_oracle_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, i64, i32, i32, i32, i32, i32]
        lib.grkan_oracle_bwd.restype = i32
        lib.grkan_oracle_scales.argtypes = [dp, dp, dp, dp, dp, dp, dp, dp, i64, i32, i32, i32, i32, i32]
        lib.grkan_oracle_scales.restype = i32
        lib.grkan_oracle_max_threads.argtypes = []
        lib.grkan_oracle_max_threads.restype = i32
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _shapes(x, A, B):
    if x.ndim < 1:
        raise ValueError("x needs at least one dimension")
    D = int(x.shape[-1])
    rows = int(x.size // D) if D else 0
    if A.ndim != 2 or B.ndim != 2 or A.shape[0] != B.shape[0]:
        raise ValueError("A must be [G, m+1] and B [G, n]")
    G, m, n = int(A.shape[0]), int(A.shape[1]) - 1, int(B.shape[1])
    return rows, D, G, m, n


def max_threads() -> int:
    return int(_load().grkan_oracle_max_threads())


def fwd(x, A, B, threads: int = 1) -> np.ndarray:
    """y = P_g(x) / (1 + |Aden_g(x)|), fp64, same shape as x."""
    x, A, B = _f64(x), _f64(A), _f64(B)
    rows, D, G, m, n = _shapes(x, A, B)
    y = np.empty_like(x)
    rc = _load().grkan_oracle_fwd(_ptr(x), _ptr(A), _ptr(B), _ptr(y), rows, D, G, m, n, threads)
    if rc:
        raise ValueError("grkan_oracle_fwd failed with code %d" % rc)
    return y


def bwd(x, dy, A, B, threads: int = 1):
    """(dx, dA[G, m+1], dB[G, n]) in fp64."""
    x, dy, A, B = _f64(x), _f64(dy), _f64(A), _f64(B)
    if dy.shape != x.shape:
        raise ValueError("dy must have the shape of x")
    rows, D, G, m, n = _shapes(x, A, B)
    dx = np.empty_like(x)
    dA = np.empty((G, m + 1), dtype=np.float64)
    dB = np.empty((G, n), dtype=np.float64)
    rc = _load().grkan_oracle_bwd(_ptr(x), _ptr(dy), _ptr(A), _ptr(B), _ptr(dx), _ptr(dA), _ptr(dB),
                                  rows, D, G, m, n, threads)
    if rc:
        raise ValueError("grkan_oracle_bwd failed with code %d" % rc)
    return dx, dA, dB


def scales(x, dy, A, B, threads: int = 1):
    """Condition scales (Sy, Sdx, RA, RB) used by the parity error metric."""
    x, A, B = _f64(x), _f64(A), _f64(B)
    dy = _f64(dy) if dy is not None else None
    rows, D, G, m, n = _shapes(x, A, B)
    Sy = np.empty_like(x)
    Sdx = np.empty_like(x)
    RA = np.empty((G, m + 1), dtype=np.float64)
    RB = np.empty((G, n), dtype=np.float64)
    rc = _load().grkan_oracle_scales(_ptr(x), _ptr(dy), _ptr(A), _ptr(B), _ptr(Sy), _ptr(Sdx),
                                     _ptr(RA), _ptr(RB), rows, D, G, m, n, threads)
    if rc:
        raise ValueError("grkan_oracle_scales failed with code %d" % rc)
    return Sy, Sdx, RA, RB
