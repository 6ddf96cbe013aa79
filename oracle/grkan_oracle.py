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
        lib.grkan_oracle_linear_fwd.argtypes = [dp, dp, dp, dp, dp, dp, i64, i32, i32, i32, i32, i32, i32, i32]
        lib.grkan_oracle_linear_fwd.restype = i32
        lib.grkan_oracle_linear_bwd.argtypes = [dp] * 11 + [i64, i32, i32, i32, i32, i32]
        lib.grkan_oracle_linear_bwd.restype = i32
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


# ---------------------------------------------------------------- GR-KAN layer, out = W F(x) (Eq. "GR_KAN")
def _linear_shapes(x, A, B, W):
    rows, D_in, G, m, n = _shapes(x, A, B)
    if W.ndim != 2 or W.shape[1] != D_in:
        raise ValueError("W must be [D_out, D_in]")
    return rows, D_in, int(W.shape[0]), G, m, n


def linear_fwd(x, A, B, W, bias=None, round_operand: bool = False, threads: int = 1) -> np.ndarray:
    """out[r, o] = sum_c W[o, c] F_{g(c)}(x[r, c]) (+ bias[o]): plain loops in C, fp64.
    round_operand=True rounds F to bfloat16 (nearest even) before the product."""
    x, A, B, W = _f64(x), _f64(A), _f64(B), _f64(W)
    rows, D_in, D_out, G, m, n = _linear_shapes(x, A, B, W)
    bias = _f64(bias) if bias is not None else None
    if bias is not None and bias.shape != (D_out,):
        raise ValueError("bias must be [D_out]")
    out = np.empty(x.shape[:-1] + (D_out,), dtype=np.float64)
    rc = _load().grkan_oracle_linear_fwd(_ptr(x), _ptr(A), _ptr(B), _ptr(W), _ptr(bias), _ptr(out),
                                         rows, D_in, D_out, G, m, n, 1 if round_operand else 0, threads)
    if rc:
        raise ValueError("grkan_oracle_linear_fwd failed with code %d" % rc)
    return out


def linear_fwd_matmul(x, A, B, W, bias=None, round_operand: bool = False, threads: int = 1) -> np.ndarray:
    """The same result with the library matrix product as the summation step
    (fwd, then numpy's fp64 matmul): for the full-size cases, where the plain
    loops would take minutes.  The rounding of the operand, if asked for, is
    numpy's own arithmetic here (not the C helper)."""
    W = _f64(W)
    y = fwd(x, A, B, threads=threads)
    if round_operand:
        mant, e = np.frexp(y)
        y = np.ldexp(np.rint(np.ldexp(mant, 8)), e - 8)
    out = y @ W.T
    if bias is not None:
        out += _f64(bias)
    return out


def linear_term_scale(x, A, B, W, threads: int = 1) -> np.ndarray:
    """Root-sum-square of the summed terms, sqrt(sum_c (W[o, c] F(x[r, c]))^2):
    the scale of the rounding error of the contraction, used by the parity
    metric of the fused layer (not part of the method)."""
    W = _f64(W)
    y = fwd(x, A, B, threads=threads)
    return np.sqrt((y * y) @ (W * W).T)


def linear_largest_term(x, A, B, W, threads: int = 1) -> np.ndarray:
    """max_c |W[o, c] F(x[r, c])| per output: the size of the one term whose
    bfloat16 rounding can change an output most (used by the parity metric of the
    fused layer; not part of the method).  rows * D_out * D_in operations in
    numpy: small cases or a sample of rows."""
    W = np.abs(_f64(W))
    y = np.abs(fwd(x, A, B, threads=threads)).reshape(-1, W.shape[1])
    out = np.zeros((y.shape[0], W.shape[0]))
    for c in range(W.shape[1]):
        np.maximum(out, y[:, c, None] * W[None, :, c], out=out)
    return out.reshape(np.shape(x)[:-1] + (W.shape[0],))


def linear_bwd(x, dOut, A, B, W):
    """dict(dF, dx, dA, dB, dW, dbias) of the GR-KAN layer by the chain rule; sequential, small cases."""
    x, dOut, A, B, W = _f64(x), _f64(dOut), _f64(A), _f64(B), _f64(W)
    rows, D_in, D_out, G, m, n = _linear_shapes(x, A, B, W)
    if dOut.shape != x.shape[:-1] + (D_out,):
        raise ValueError("dOut must be [rows, D_out]")
    dF, dx = np.empty_like(x), np.empty_like(x)
    dA, dB = np.empty((G, m + 1)), np.empty((G, n))
    dW, dbias = np.empty_like(W), np.empty(D_out)
    rc = _load().grkan_oracle_linear_bwd(_ptr(x), _ptr(dOut), _ptr(A), _ptr(B), _ptr(W), _ptr(dF), _ptr(dx),
                                         _ptr(dA), _ptr(dB), _ptr(dW), _ptr(dbias), rows, D_in, D_out, G, m, n)
    if rc:
        raise ValueError("grkan_oracle_linear_bwd failed with code %d" % rc)
    return dict(dF=dF, dx=dx, dA=dA, dB=dB, dW=dW, dbias=dbias)
