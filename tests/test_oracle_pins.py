"""Pins of the fp64 oracle against what the paper and the mathematics fix.

None of these tests touches the GPU path.  Each pin is chosen so that a
plausible mistake in the oracle (dropped term, wrong sign, wrong group index,
transposed coefficient layout) fails at least one of them:

  P1  identity init (paper, Sec. "Results": first GR-KAN layer starts as the
      identity)                                  -> plain dot products
  P2  B = 0                                      -> numpy polyval / polyder
  P3  one-term denominator, constant numerator   -> closed form
  P3b P = c (1 + Aden)                           -> F = c where Aden >= 0
  P4  F is linear in a: sum_i a_i dA_i = sum dy y            (ties bwd to fwd)
  P5  d/dlambda F(lambda x) at 1: sum x dx = sum i a_i dA_i + sum j b_j dB_j
  P6  sum_j b_j dB_j = -sum dy y (Q-1)/Q
  P7  symmetries under B -> -B and x -> -x
  P8  group bookkeeping
  P9  central finite differences of L = sum dy*y w.r.t. every coefficient and
      every x of a small case
  P10 hand-worked integer example (tests/golden/worked_example.txt)
"""
import math
from pathlib import Path

import numpy as np
import numpy.polynomial.polynomial as npoly
import pytest

import grkan_inputs

GOLDEN = Path(__file__).resolve().parent / "golden"


def small_case(seed, rows=16, D=24, G=4, m=5, n=4, avoid_kink=False):
    rng = np.random.default_rng(seed)
    A = rng.uniform(-1, 1, size=(G, m + 1)) / (np.arange(m + 1) + 1.0)
    B = rng.uniform(-0.5, 0.5, size=(G, n))
    x = rng.standard_normal((rows, D))
    dy = rng.standard_normal((rows, D))
    if avoid_kink:
        dg = D // G
        for _ in range(100):
            xg = x.reshape(rows, G, dg)
            aden = sum(B[None, :, j, None] * xg ** (j + 1) for j in range(n))
            bad = np.abs(aden) < 1e-2
            if not bad.any():
                break
            xg[bad] = rng.standard_normal(int(bad.sum()))
            x = xg.reshape(rows, D)
        else:
            raise AssertionError("could not move x away from the kink")
    return x, dy, A, B


def group_view(a, G):
    rows, D = a.shape
    return a.reshape(rows, G, D // G)


# ---------------------------------------------------------------- P1
def test_p1_identity(oracle):
    x, dy, _, _ = small_case(1, rows=50, D=48, G=8)
    G = 8
    A = np.zeros((G, 6))
    A[:, 1] = 1.0
    B = np.zeros((G, 4))
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    assert np.array_equal(y, x)
    assert np.array_equal(dx, dy)
    xg, dg = group_view(x, G), group_view(dy, G)
    for i in range(6):
        want = np.einsum("rgc,rgc->g", dg, xg ** i)
        np.testing.assert_allclose(dA[:, i], want, rtol=1e-12, atol=1e-12)
    assert np.array_equal(dB, np.zeros((G, 4)))


# ---------------------------------------------------------------- P2
def test_p2_polynomial_only(oracle):
    x, dy, A, _ = small_case(2, rows=40, D=36, G=3)
    G = 3
    B = np.zeros((G, 4))
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    xg, dg = group_view(x, G), group_view(dy, G)
    yg, dxg = group_view(y, G), group_view(dx, G)
    for g in range(G):
        np.testing.assert_allclose(yg[:, g], npoly.polyval(xg[:, g], A[g]), rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(dxg[:, g], dg[:, g] * npoly.polyval(xg[:, g], npoly.polyder(A[g])),
                                   rtol=1e-13, atol=1e-13)
        for i in range(6):
            np.testing.assert_allclose(dA[g, i], np.sum(dg[:, g] * xg[:, g] ** i), rtol=1e-12, atol=1e-12)
    assert np.array_equal(dB, np.zeros_like(dB))


# ---------------------------------------------------------------- P3
@pytest.mark.parametrize("b", [0.7, -1.3])
def test_p3_one_term_denominator(oracle, b):
    x, dy, _, _ = small_case(3, rows=30, D=8, G=1)
    A = np.array([[1.0, 0, 0, 0, 0, 0]])
    B = np.array([[b, 0, 0, 0]])
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    q = 1.0 + np.abs(b * x)
    np.testing.assert_allclose(y, 1.0 / q, rtol=1e-14)
    np.testing.assert_allclose(dx, -dy * np.sign(b * x) * b / q ** 2, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(dB[0, 0], -np.sum(dy * np.abs(x) * np.sign(b) / q ** 2), rtol=1e-12)
    # d/db_j for j >= 2: -dy x^j sign(b x) / q^2
    for j in (2, 3, 4):
        np.testing.assert_allclose(dB[0, j - 1], -np.sum(dy * x ** j * np.sign(b * x) / q ** 2), rtol=1e-12)
    for i in range(6):
        np.testing.assert_allclose(dA[0, i], np.sum(dy * x ** i / q), rtol=1e-12)


def test_p3b_numerator_equals_denominator(oracle):
    # P = c (1 + Aden): F = c wherever Aden >= 0 and c (1+Aden)/(1-Aden) elsewhere;
    # the two terms of dF/dx must cancel exactly where Aden > 0.
    rng = np.random.default_rng(33)
    c = 1.75
    b = np.array([0.4, -0.3, 0.2, 0.1])
    A = np.array([np.concatenate(([c], c * b, [0.0]))])
    B = b[None, :]
    x = rng.standard_normal((64, 4))
    dy = rng.standard_normal((64, 4))
    aden = sum(b[j] * x ** (j + 1) for j in range(4))
    daden = sum((j + 1) * b[j] * x ** j for j in range(4))
    y = oracle.fwd(x, A, B)
    dx, _, _ = oracle.bwd(x, dy, A, B)
    pos = aden > 0
    assert pos.any() and (~pos).any()
    np.testing.assert_allclose(y[pos], c, rtol=1e-14)
    np.testing.assert_allclose(dx[pos], 0.0, atol=1e-13)
    neg = aden < 0
    np.testing.assert_allclose(y[neg], c * (1 + aden[neg]) / (1 - aden[neg]), rtol=1e-13)
    np.testing.assert_allclose(dx[neg], dy[neg] * c * 2 * daden[neg] / (1 - aden[neg]) ** 2, rtol=1e-11, atol=1e-13)


def test_sign_convention_at_zero(oracle):
    # Aden(0) = 0: sign taken as 0, so dx = dy * a_1 and the b-gradients get nothing.
    A = np.array([[0.3, -1.2, 0.5, 0.1, -0.2, 0.05]])
    B = np.array([[0.4, 0.3, -0.2, 0.1]])
    x = np.zeros((3, 2))
    dy = np.arange(1.0, 7.0).reshape(3, 2)
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    np.testing.assert_allclose(y, 0.3)
    np.testing.assert_allclose(dx, dy * -1.2)
    np.testing.assert_allclose(dA[0], [dy.sum(), 0, 0, 0, 0, 0])
    assert np.array_equal(dB, np.zeros((1, 4)))


# ---------------------------------------------------------------- P4, P5, P6
@pytest.mark.parametrize("m,n", [(5, 4), (3, 2), (7, 6)])
@pytest.mark.parametrize("seed,G", [(4, 1), (5, 4), (6, 12)])
def test_p4_p5_p6_invariants(oracle, seed, G, m, n):
    x, dy, A, B = small_case(seed, rows=64, D=48, G=G, m=m, n=n)
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    xg, dg, yg, dxg = (group_view(a, G) for a in (x, dy, y, dx))
    aden = sum(B[None, :, j, None] * xg ** (j + 1) for j in range(n))
    q = 1 + np.abs(aden)
    i = np.arange(m + 1)
    j = np.arange(1, n + 1)
    # P4
    np.testing.assert_allclose((A * dA).sum(1), (dg * yg).sum((0, 2)), rtol=1e-11, atol=1e-11)
    # P5
    np.testing.assert_allclose((xg * dxg).sum((0, 2)), (i * A * dA).sum(1) + (j * B * dB).sum(1),
                               rtol=1e-10, atol=1e-10)
    # P6
    np.testing.assert_allclose((B * dB).sum(1), -(dg * yg * (q - 1) / q).sum((0, 2)), rtol=1e-10, atol=1e-10)


# ---------------------------------------------------------------- P7
def test_p7_symmetries(oracle):
    x, dy, A, B = small_case(7, rows=32, D=24, G=4)
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    # B -> -B
    y2 = oracle.fwd(x, A, -B)
    dx2, dA2, dB2 = oracle.bwd(x, dy, A, -B)
    np.testing.assert_allclose(y2, y, rtol=1e-15)
    np.testing.assert_allclose(dx2, dx, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(dA2, dA, rtol=1e-13)
    np.testing.assert_allclose(dB2, -dB, rtol=1e-13)
    # x -> -x with a_i -> (-1)^i a_i, b_j -> (-1)^j b_j
    sa = (-1.0) ** np.arange(6)
    sb = (-1.0) ** np.arange(1, 5)
    y3 = oracle.fwd(-x, A * sa, B * sb)
    dx3, dA3, dB3 = oracle.bwd(-x, dy, A * sa, B * sb)
    np.testing.assert_allclose(y3, y, rtol=1e-13)
    np.testing.assert_allclose(dx3, -dx, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(dA3, dA * sa, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dB3, dB * sb, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- P8
def test_p8_group_bookkeeping(oracle):
    G = 6
    x, dy, A, B = small_case(8, rows=20, D=36, G=G)
    dg_ = 36 // G
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)

    # identical rows: G groups vs one group
    A1, B1 = np.tile(A[:1], (G, 1)), np.tile(B[:1], (G, 1))
    _, dAg, dBg = oracle.bwd(x, dy, A1, B1)
    _, dA1, dB1 = oracle.bwd(x, dy, A[:1], B[:1])
    np.testing.assert_allclose(dAg.sum(0), dA1[0], rtol=1e-12)
    np.testing.assert_allclose(dBg.sum(0), dB1[0], rtol=1e-12)

    # permuting coefficient rows together with channel blocks permutes the outputs
    perm = np.array([3, 0, 5, 1, 4, 2])
    cols = (perm[:, None] * dg_ + np.arange(dg_)[None, :]).reshape(-1)
    yp = oracle.fwd(x[:, cols], A[perm], B[perm])
    dxp, dAp, dBp = oracle.bwd(x[:, cols], dy[:, cols], A[perm], B[perm])
    assert np.array_equal(yp, y[:, cols])
    assert np.array_equal(dxp, dx[:, cols])
    np.testing.assert_allclose(dAp, dA[perm], rtol=1e-15)
    np.testing.assert_allclose(dBp, dB[perm], rtol=1e-15)

    # zero upstream gradient on one group's channels zeroes only that group's sums
    dy0 = dy.copy()
    dy0[:, 2 * dg_:3 * dg_] = 0.0
    _, dAz, dBz = oracle.bwd(x, dy0, A, B)
    assert np.array_equal(dAz[2], np.zeros(6)) and np.array_equal(dBz[2], np.zeros(4))
    keep = [0, 1, 3, 4, 5]
    assert np.array_equal(dAz[keep], dA[keep]) and np.array_equal(dBz[keep], dB[keep])

    # an element only feeds its own group: channel c -> group c // d_g
    for c in (0, dg_ - 1, dg_, 35):
        dy1 = np.zeros_like(dy)
        dy1[5, c] = 1.0
        _, dAe, dBe = oracle.bwd(x, dy1, A, B)
        nz = np.nonzero(np.abs(dAe).sum(1))[0]
        assert list(nz) == [c // dg_]


# ---------------------------------------------------------------- P9
@pytest.mark.parametrize("m,n", [(5, 4), (3, 2), (7, 6)])
def test_p9_finite_differences(oracle, m, n):
    x, dy, A, B = small_case(9, rows=6, D=12, G=3, m=m, n=n, avoid_kink=True)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    scale = np.abs(dy).sum()

    def fd(arr, idx):
        # L(v + h) - L(v - h) summed term by term, so that the elements the perturbation does
        # not reach contribute exactly zero instead of the roundoff of two large sums
        v = arr[idx]
        h = 1e-6 * max(1.0, abs(v))
        arr[idx] = v + h
        yp = oracle.fwd(x, A, B)
        arr[idx] = v - h
        ym = oracle.fwd(x, A, B)
        arr[idx] = v
        return math.fsum((dy * (yp - ym)).ravel()) / (2 * h)

    for idx in np.ndindex(*A.shape):
        assert abs(fd(A, idx) - dA[idx]) <= 1e-7 * max(abs(dA[idx]), scale * 1e-2), ("dA", idx)
    for idx in np.ndindex(*B.shape):
        assert abs(fd(B, idx) - dB[idx]) <= 1e-7 * max(abs(dB[idx]), scale * 1e-2), ("dB", idx)
    for idx in np.ndindex(*x.shape):
        assert abs(fd(x, idx) - dx[idx]) <= 1e-7 * max(abs(dx[idx]), abs(dy[idx])), ("dx", idx)


# ---------------------------------------------------------------- P10
def test_p10_worked_example(oracle):
    rows = [l.split("#")[0].split() for l in (GOLDEN / "worked_example.txt").read_text().splitlines()]
    vals = {r[0]: [float(v) for v in r[1:]] for r in rows if r}
    A = np.array([vals["A"]])
    B = np.array([vals["B"]])
    x = np.array([vals["x"]])
    dy = np.array([vals["dy"]])
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    np.testing.assert_allclose(y[0], vals["y"], rtol=1e-15)
    np.testing.assert_allclose(dx[0], vals["dx"], rtol=1e-15)
    np.testing.assert_allclose(dA[0], vals["dA"], rtol=1e-15)
    np.testing.assert_allclose(dB[0], vals["dB"], rtol=1e-15)


# ---------------------------------------------------------------- C oracle vs the numpy mirror
@pytest.mark.parametrize("rows,D,G", [(788, 192, 8), (7, 30, 1), (5, 30, 30), (33, 40, 5)])
def test_c_oracle_matches_numpy_mirror(oracle, oracle_np, rows, D, G):
    if (rows, D, G) == (788, 192, 8):
        c = grkan_inputs.make_case("tiny")
        x, dy, A, B = (c[k].astype(np.float64) for k in ("x", "dy", "A", "B"))
    else:
        x, dy, A, B = small_case(rows * 1000 + D + G, rows=rows, D=D, G=G)
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    y2 = oracle_np.fwd(x, A, B)
    dx2, dA2, dB2 = oracle_np.bwd(x, dy, A, B)
    np.testing.assert_allclose(y, y2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dx, dx2, rtol=1e-11, atol=1e-12)
    _, _, RA, RB = oracle.scales(x, dy, A, B)
    assert np.all(np.abs(dA - dA2) <= 1e-12 * np.maximum(np.abs(dA), RA))
    assert np.all(np.abs(dB - dB2) <= 1e-12 * np.maximum(np.abs(dB), RB))


def test_other_degrees_match_numpy_mirror(oracle, oracle_np):
    x, dy, A, B = small_case(11, rows=9, D=10, G=2, m=3, n=2)
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    np.testing.assert_allclose(y, oracle_np.fwd(x, A, B), rtol=1e-12)
    dx2, dA2, dB2 = oracle_np.bwd(x, dy, A, B)
    np.testing.assert_allclose(dx, dx2, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dA, dA2, rtol=1e-11)
    np.testing.assert_allclose(dB, dB2, rtol=1e-11)


def test_threads_do_not_change_the_result(oracle):
    c = grkan_inputs.make_case("tiny")
    x, dy, A, B = (c[k].astype(np.float64) for k in ("x", "dy", "A", "B"))
    dx1, dA1, dB1 = oracle.bwd(x, dy, A, B, threads=1)
    dx4, dA4, dB4 = oracle.bwd(x, dy, A, B, threads=4)
    assert np.array_equal(dx1, dx4)
    np.testing.assert_allclose(dA4, dA1, rtol=1e-13)
    np.testing.assert_allclose(dB4, dB1, rtol=1e-13)
    assert np.array_equal(oracle.fwd(x, A, B, threads=4), oracle.fwd(x, A, B, threads=1))


def test_oracle_rejects_bad_shapes(oracle):
    x = np.zeros((2, 10))
    with pytest.raises(ValueError):
        oracle.fwd(x, np.zeros((3, 6)), np.zeros((3, 4)))  # 10 % 3 != 0
    with pytest.raises(ValueError):
        oracle.bwd(x, np.zeros((2, 9)), np.zeros((2, 6)), np.zeros((2, 4)))


def test_empty_input(oracle):
    x = np.zeros((0, 16))
    A, B = np.ones((4, 6)), np.ones((4, 4))
    assert oracle.fwd(x, A, B).shape == (0, 16)
    dx, dA, dB = oracle.bwd(x, x, A, B)
    assert dx.shape == (0, 16)
    assert np.array_equal(dA, np.zeros((4, 6))) and np.array_equal(dB, np.zeros((4, 4)))


def test_scales_bound_the_values(oracle):
    x, dy, A, B = small_case(12, rows=10, D=16, G=4)
    y = oracle.fwd(x, A, B)
    dx, dA, dB = oracle.bwd(x, dy, A, B)
    Sy, Sdx, RA, RB = oracle.scales(x, dy, A, B)
    assert np.all(np.abs(y) <= Sy * (1 + 1e-12))
    assert np.all(np.abs(dx) <= Sdx * (1 + 1e-12))
    n_terms = 10 * 4
    assert np.all(np.abs(dA) <= RA * np.sqrt(n_terms) * (1 + 1e-12))
    assert np.all(np.abs(dB) <= RB * np.sqrt(n_terms) * (1 + 1e-12))


def test_scales_bound_a_float32_evaluation(oracle):
    """What the parity tolerance is relative to.  The scales replace every
    monomial of P, P', Aden' by its magnitude and take Q as exact.  On
    heavy-tailed inputs a float32 evaluation whose denominator polynomial is
    formed in double (what the float32-I/O kernels do) stays within 16 eps of
    them, so the tolerance is reachable and not orders of magnitude loose; an
    all-float32 evaluation does not, because Aden cancels next to the roots of
    the denominator polynomial -- which is why the kernels form it in double."""
    rng = np.random.default_rng(13)
    rows, D, G = 4000, 32, 4
    A = (rng.uniform(-1, 1, size=(G, 6)) / (np.arange(6) + 1.0)).astype(np.float32)
    B = rng.uniform(-0.5, 0.5, size=(G, 4)).astype(np.float32)
    x = rng.standard_t(3, size=(rows, D)).astype(np.float32)
    dy = rng.standard_normal((rows, D)).astype(np.float32)
    f = np.float32
    xg = x.reshape(rows, G, D // G)
    a = A[None, :, :, None]
    b = B[None, :, :, None]
    P = a[:, :, 5]
    for i in (4, 3, 2, 1, 0):
        P = (P * xg + a[:, :, i]).astype(f)
    dP = (f(5) * a[:, :, 5])
    for i in (4, 3, 2, 1):
        dP = (dP * xg + f(i) * a[:, :, i]).astype(f)
    dh = f(4) * b[:, :, 3]
    for j in (2, 1, 0):
        dh = (dh * xg + f(j + 1) * b[:, :, j]).astype(f)

    def evaluate(wide):
        t = np.float64 if wide else np.float32
        xs = xg.astype(t)
        h = b[:, :, 3].astype(t)
        for j in (2, 1, 0):
            h = (h * xs + b[:, :, j].astype(t)).astype(t)
        aden = (h * xs).astype(f)
        q = (f(1) + np.abs(aden)).astype(f)
        y32 = (P / q).astype(f)
        dx32 = (dy.reshape(xg.shape) * (dP / q - np.sign(aden) * dh * P / q / q)).astype(f)
        return y32.reshape(rows, D), dx32.reshape(rows, D)

    x64, dy64, A64, B64 = (v.astype(np.float64) for v in (x, dy, A, B))
    y = oracle.fwd(x64, A64, B64)
    dx, _, _ = oracle.bwd(x64, dy64, A64, B64)
    Sy, Sdx, _, _ = oracle.scales(x64, dy64, A64, B64)
    eps = 2.0 ** -24

    def rel(y32, dx32):
        return (np.abs(y32 - y) / np.maximum(np.abs(y), Sy)).max(), (np.abs(dx32 - dx) / np.maximum(np.abs(dx), Sdx)).max()

    ry, rdx = rel(*evaluate(wide=True))
    assert ry <= 16 * eps and rdx <= 16 * eps, (ry / eps, rdx / eps)
    assert ry >= 1e-3 * eps and rdx >= 1e-3 * eps
    ry32, rdx32 = rel(*evaluate(wide=False))
    assert max(ry32, rdx32) > 16 * eps, (ry32 / eps, rdx32 / eps)
    # and the plain relative error is unbounded by such a constant on these inputs either way
    plain = np.abs(evaluate(wide=True)[1] - dx) / np.abs(dx)
    assert plain.max() > 16 * eps


# ---------------------------------------------------------------- change detector
def test_oracle_results_have_not_moved(oracle):
    """tests/golden/oracle_tiny_digest.txt was written by the committed script beside it, from the
    oracle alone, when the pins above held.  Not a pin: it flags later edits that move the results."""
    import importlib.util

    spec = importlib.util.spec_from_file_location("write_oracle_digest", GOLDEN / "write_oracle_digest.py")
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = {}
    for line in (GOLDEN / "oracle_tiny_digest.txt").read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        m, n, key, *vals = line.split()
        stored[(int(m), int(n), key)] = np.array([float(v) for v in vals])
    for m, n in ((5, 4), (3, 2), (7, 6)):
        d = mod.digest(m, n)
        for key in ("sum_y", "wsum_y", "sum_dx", "wsum_dx", "dA", "dB"):
            got = np.atleast_1d(np.array(d[key], dtype=np.float64))
            want = stored[(m, n, key)]
            scale = np.maximum(np.abs(want), 1e-3 * np.max(np.abs(want)))
            assert np.all(np.abs(got - want) <= 1e-11 * scale), (m, n, key)
