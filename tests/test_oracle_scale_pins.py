"""Two-sided pins of the oracle's condition scales (grkan_oracle_scales).

Every GPU parity figure is |gpu - ref| / max(|ref|, S) with S one of the four
scales, so a scale that is too large loosens the tolerance silently.  These
tests therefore fix the VALUE of every scale, not only a bound on it:

  S1  identity initialisation (paper, Sec. "Results"): Sy = |x|, Sdx = |dy|,
      RA[g,i] = sqrt(sum (dy x^i)^2), RB = 0
  S2  one-term denominator with constant numerator: closed forms
  S3  each scale rebuilt from the pinned forward / backward functions themselves
      (the magnitude polynomials are forward/backward passes with |a|, |b| at
      |x|; a root-sum-square is a coefficient gradient for a squared upstream
      gradient), to 1e-12
  S4  a vectorised numpy evaluation on a random small case, to 1e-12
  S5  mistakes planted in a copy of the C source (a factor 2, a missing 1/Q, Q
      for Q^2, a dropped square root, the magnitude polynomial in RB) are each
      caught by S1-S4
"""
import ctypes
import subprocess
from pathlib import Path

import numpy as np
import pytest

ROOT = Path(__file__).resolve().parent.parent


def random_case(seed, rows=23, D=24, G=4, m=5, n=4):
    rng = np.random.default_rng(seed)
    A = rng.uniform(-1, 1, size=(G, m + 1)) / (np.arange(m + 1) + 1.0)
    B = rng.uniform(-0.5, 0.5, size=(G, n))
    x = rng.standard_t(3, size=(rows, D))
    dy = rng.standard_normal((rows, D))
    return x, dy, A, B


def per_group(v, G):
    """[rows, D] -> [G, rows * d_g]"""
    rows, D = v.shape
    return v.reshape(rows, G, D // G).transpose(1, 0, 2).reshape(G, -1)


# ------------------------------------------------------------------ the checks (run on the real oracle
# and, in S5, on mutated copies of it)
def check_identity(orc):
    x, dy, _, _ = random_case(1)
    G, m, n = 4, 5, 4
    A = np.zeros((G, m + 1))
    A[:, 1] = 1.0
    B = np.zeros((G, n))
    Sy, Sdx, RA, RB = orc.scales(x, dy, A, B)
    np.testing.assert_allclose(Sy, np.abs(x), rtol=1e-14)
    np.testing.assert_allclose(Sdx, np.abs(dy), rtol=1e-14)
    xg, dg = per_group(x, G), per_group(dy, G)
    want = np.stack([np.sqrt(np.sum((dg * xg ** i) ** 2, axis=1)) for i in range(m + 1)], axis=1)
    np.testing.assert_allclose(RA, want, rtol=1e-12)
    assert np.array_equal(RB, np.zeros((G, n)))


def check_one_term_denominator(orc):
    x, dy, _, _ = random_case(2, rows=31, D=8, G=2)
    b = np.array([0.7, -1.3])
    G, m, n = 2, 5, 4
    A = np.zeros((G, m + 1))
    A[:, 0] = 1.0  # P = 1
    B = np.zeros((G, n))
    B[:, 0] = b    # Aden = b x
    Sy, Sdx, RA, RB = orc.scales(x, dy, A, B)
    bb = np.repeat(b, 4)[None, :]
    Q = 1.0 + np.abs(bb * x)
    np.testing.assert_allclose(Sy, 1.0 / Q, rtol=1e-13)
    # P' = 0, Aden' = b: Sdx = |dy| |b| / Q^2
    np.testing.assert_allclose(Sdx, np.abs(dy) * np.abs(bb) / Q ** 2, rtol=1e-13)
    xg, dg, Qg = per_group(x, G), per_group(dy, G), per_group(Q, G)
    for i in range(m + 1):
        np.testing.assert_allclose(RA[:, i], np.sqrt(np.sum((dg * xg ** i / Qg) ** 2, axis=1)), rtol=1e-12)
    for j in range(1, n + 1):
        # s^2 = 1 wherever x != 0 (it is, for these draws)
        np.testing.assert_allclose(RB[:, j - 1], np.sqrt(np.sum((dg * xg ** j / Qg ** 2) ** 2, axis=1)), rtol=1e-12)


def check_against_forward_and_backward(orc):
    """The scales rebuilt from the oracle's own (separately pinned) fwd and bwd."""
    x, dy, A, B = random_case(3)
    G, m, n = A.shape[0], A.shape[1] - 1, B.shape[1]
    Sy, Sdx, RA, RB = orc.scales(x, dy, A, B)
    e0 = np.zeros_like(A)
    e0[:, 0] = 1.0
    zB = np.zeros_like(B)
    one = np.ones_like(x)
    r = orc.fwd(x, e0, B)                      # 1 / Q
    Pm = orc.fwd(np.abs(x), np.abs(A), zB)     # sum |a_i| |x|^i
    dPm = orc.bwd(np.abs(x), one, np.abs(A), zB)[0]
    Ab = np.zeros_like(A)                      # sum |b_j| t^j as a "numerator"
    Ab[:, 1:n + 1] = np.abs(B)
    dAm = orc.bwd(np.abs(x), one, Ab, zB)[0]
    np.testing.assert_allclose(Sy, Pm * r, rtol=1e-12)
    np.testing.assert_allclose(Sdx, np.abs(dy) * (dPm * r + dAm * Pm * r * r), rtol=1e-12)
    y = orc.fwd(x, A, B)                       # P / Q
    sgn = np.sign(orc.fwd(x, _embed(B, A), zB))  # sign(Aden): Aden as a polynomial-only forward pass
    for i in range(m + 1):
        # dA_i for the upstream gradient dy^2 x^i / Q is sum (dy x^i / Q)^2
        _, dA, _ = orc.bwd(x, dy * dy * x ** i * r, A, B)
        np.testing.assert_allclose(RA[:, i], np.sqrt(dA[:, i]), rtol=1e-12)
    for j in range(1, n + 1):
        # with w = dy x^j s P / Q^2 = dy x^j s y / Q, the upstream gradient dy w gives dB_j = -sum w^2
        _, _, dB = orc.bwd(x, dy * dy * x ** j * sgn * y * r, A, B)
        np.testing.assert_allclose(RB[:, j - 1], np.sqrt(-dB[:, j - 1]), rtol=1e-12)


def _embed(B, A):
    """B's entries placed where the denominator terms sit in a numerator row: [0, b_1..b_n, 0...]."""
    out = np.zeros_like(A)
    out[:, 1:B.shape[1] + 1] = B
    return out


def check_against_numpy(orc, m=5, n=4):
    x, dy, A, B = random_case(4 + m, rows=19, D=30, G=5, m=m, n=n)
    G = A.shape[0]
    Sy, Sdx, RA, RB = orc.scales(x, dy, A, B)
    rows, D = x.shape
    xg = x.reshape(rows, G, D // G)
    dg = dy.reshape(rows, G, D // G)
    a = A[None, :, :, None]
    b = B[None, :, :, None]
    xe = xg[:, :, None, :]
    I = np.arange(m + 1)[None, None, :, None]
    J = np.arange(1, n + 1)[None, None, :, None]
    P = (a * xe ** I).sum(2)
    aden = (b * xe ** J).sum(2)
    Q = 1 + np.abs(aden)
    Pm = (np.abs(a) * np.abs(xe) ** I).sum(2)
    dPm = (I[:, :, 1:] * np.abs(a[:, :, 1:]) * np.abs(xe) ** (I[:, :, 1:] - 1)).sum(2)
    dAm = (J * np.abs(b) * np.abs(xe) ** (J - 1)).sum(2)
    np.testing.assert_allclose(Sy, (Pm / Q).reshape(rows, D), rtol=1e-12)
    np.testing.assert_allclose(Sdx, (np.abs(dg) * (dPm / Q + dAm * Pm / Q ** 2)).reshape(rows, D), rtol=1e-12)
    ta = dg[:, :, None, :] * xe ** I / Q[:, :, None, :]
    np.testing.assert_allclose(RA, np.sqrt((ta ** 2).sum(axis=(0, 3))), rtol=1e-12)
    tb = dg[:, :, None, :] * xe ** J * (np.sign(aden) * P / Q ** 2)[:, :, None, :]
    np.testing.assert_allclose(RB, np.sqrt((tb ** 2).sum(axis=(0, 3))), rtol=1e-12)


CHECKS = [check_identity, check_one_term_denominator, check_against_forward_and_backward, check_against_numpy]


# ------------------------------------------------------------------ S1-S4 on the oracle as it stands
def test_s1_identity_initialisation(oracle):
    check_identity(oracle)


def test_s2_one_term_denominator(oracle):
    check_one_term_denominator(oracle)


def test_s3_scales_rebuilt_from_forward_and_backward(oracle):
    check_against_forward_and_backward(oracle)


@pytest.mark.parametrize("m,n", [(5, 4), (3, 2), (7, 6)])
def test_s4_numpy_evaluation(oracle, m, n):
    check_against_numpy(oracle, m, n)


# ------------------------------------------------------------------ S5: planted mistakes
MUTANTS = [
    # (what, text in the C source, replacement)
    ("Sy inflated 2x", "Sy[r * D + c] = Pm / Q;", "Sy[r * D + c] = 2.0 * Pm / Q;"),
    ("Sy without 1/Q", "Sy[r * D + c] = Pm / Q;", "Sy[r * D + c] = Pm;"),
    ("Sdx: Q for Q^2", "Sdx[r * D + c] = d * (dPm / Q + dAm * Pm / Q2);", "Sdx[r * D + c] = d * (dPm / Q + dAm * Pm / Q);"),
    ("Sdx: missing 1/Q", "Sdx[r * D + c] = d * (dPm / Q + dAm * Pm / Q2);", "Sdx[r * D + c] = d * (dPm + dAm * Pm / Q2);"),
    ("Sdx: dropped j", "dAm += (double)j * fabs(b[j - 1]) * axp[j - 1];", "dAm += fabs(b[j - 1]) * axp[j - 1];"),
    ("RA: missing 1/Q", "double t = d * axp[i] / Q;", "double t = d * axp[i];"),
    ("RA inflated 2x", "double t = d * axp[i] / Q;", "double t = 2.0 * d * axp[i] / Q;"),
    ("RB: Q for Q^2", "double t = d * axp[j] * fabs(e.s) * fabs(e.P) / Q2;", "double t = d * axp[j] * fabs(e.s) * fabs(e.P) / Q;"),
    ("RB: magnitude polynomial for P", "double t = d * axp[j] * fabs(e.s) * fabs(e.P) / Q2;",
     "double t = d * axp[j] * fabs(e.s) * Pm / Q2;"),
    ("RB: x^(j-1)", "double t = d * axp[j] * fabs(e.s) * fabs(e.P) / Q2;",
     "double t = d * axp[j - 1] * fabs(e.s) * fabs(e.P) / Q2;"),
    ("RA: dropped square root", "RA[(size_t)g * (m + 1) + i] = sqrt(sq[(size_t)g * nc + i]);",
     "RA[(size_t)g * (m + 1) + i] = sq[(size_t)g * nc + i];"),
    ("RB: dropped square root", "RB[(size_t)g * n + (j - 1)] = sqrt(sq[(size_t)g * nc + m + j]);",
     "RB[(size_t)g * n + (j - 1)] = sq[(size_t)g * nc + m + j];"),
    ("RB: wrong group stride", "sq[(size_t)g * nc + m + j] += t * t;", "sq[(size_t)g * n + m + j] += t * t;"),
]


class MutantOracle:
    """The front end's three calls on a mutated build of the C source."""

    def __init__(self, lib_path):
        lib = ctypes.CDLL(str(lib_path))
        dp, i64, i32 = ctypes.POINTER(ctypes.c_double), ctypes.c_int64, ctypes.c_int
        lib.grkan_oracle_fwd.argtypes = [dp, dp, dp, dp, i64, i32, i32, i32, i32, i32]
        lib.grkan_oracle_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, i64, i32, i32, i32, i32, i32]
        lib.grkan_oracle_scales.argtypes = [dp, dp, dp, dp, dp, dp, dp, dp, i64, i32, i32, i32, i32, i32]
        self.lib = lib

    @staticmethod
    def _p(a):
        return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))

    @staticmethod
    def _c(*arrays):
        return [np.ascontiguousarray(a, dtype=np.float64) for a in arrays]

    def fwd(self, x, A, B):
        x, A, B = self._c(x, A, B)
        y = np.empty_like(x)
        assert self.lib.grkan_oracle_fwd(self._p(x), self._p(A), self._p(B), self._p(y), x.shape[0], x.shape[1],
                                         A.shape[0], A.shape[1] - 1, B.shape[1], 1) == 0
        return y

    def bwd(self, x, dy, A, B):
        x, dy, A, B = self._c(x, dy, A, B)
        dx, dA, dB = np.empty_like(x), np.empty_like(A), np.empty_like(B)
        assert self.lib.grkan_oracle_bwd(self._p(x), self._p(dy), self._p(A), self._p(B), self._p(dx), self._p(dA),
                                         self._p(dB), x.shape[0], x.shape[1], A.shape[0], A.shape[1] - 1,
                                         B.shape[1], 1) == 0
        return dx, dA, dB

    def scales(self, x, dy, A, B):
        x, dy, A, B = self._c(x, dy, A, B)
        Sy, Sdx, RA, RB = np.empty_like(x), np.empty_like(x), np.empty_like(A), np.empty_like(B)
        assert self.lib.grkan_oracle_scales(self._p(x), self._p(dy), self._p(A), self._p(B), self._p(Sy),
                                            self._p(Sdx), self._p(RA), self._p(RB), x.shape[0], x.shape[1],
                                            A.shape[0], A.shape[1] - 1, B.shape[1], 1) == 0
        return Sy, Sdx, RA, RB


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_s5_planted_mistakes_are_caught(tmp_path, what, old, new):
    src = (ROOT / "oracle" / "grkan_oracle.c").read_text()
    assert src.count(old) == 1, "the mutation target must occur exactly once: %r" % old
    c_file = tmp_path / "mutant.c"
    c_file.write_text(src.replace(old, new))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-o", str(so), str(c_file), "-lm"], check=True)
    mutant = MutantOracle(so)
    caught = 0
    for check in CHECKS:
        try:
            check(mutant)
        except AssertionError:
            caught += 1
    assert caught >= 1, "%s: no scale pin noticed" % what
