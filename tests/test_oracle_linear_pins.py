"""Pins of the oracle's GR-KAN layer, out = W F(x) (paper, Eq. "GR_KAN"), and of
its backward pass, against what the mathematics fixes.  No GPU.

  L1  identity F (the paper's first-layer initialisation)  -> out = x W^T (numpy matmul)
  L2  W = I                                                 -> out = the pinned rational forward
  L3  brute force: Python loops over a tiny case, written from the equation
  L4  linear in W, bias adds, a row of x only reaches its own row of out
  L5  W is [D_out, D_in] (not its transpose): one-hot weight rows pick single channels
  L6  the library-matmul route used at full size equals the plain loops
  L7  bfloat16 operand rounding: representable values, half-ulp bound, ties to even
  L8  backward: central finite differences of L = sum dOut * out w.r.t. x, A, B, W, bias;
      W = I reduces it to the pinned rational backward; dF = dOut W
  L9  the term scale is the root-sum-square of the summed terms (brute force)
"""
import numpy as np
import pytest


def case(seed, rows=7, D_in=24, D_out=10, G=4, m=5, n=4):
    rng = np.random.default_rng(seed)
    A = rng.uniform(-1, 1, size=(G, m + 1)) / (np.arange(m + 1) + 1.0)
    B = rng.uniform(-0.5, 0.5, size=(G, n))
    x = rng.standard_normal((rows, D_in))
    W = rng.standard_normal((D_out, D_in)) / np.sqrt(D_in)
    bias = rng.standard_normal(D_out)
    dOut = rng.standard_normal((rows, D_out))
    return x, A, B, W, bias, dOut


def test_l1_identity_rational_gives_the_plain_product(oracle):
    x, _, _, W, bias, _ = case(1)
    A = np.zeros((4, 6))
    A[:, 1] = 1.0
    B = np.zeros((4, 4))
    np.testing.assert_allclose(oracle.linear_fwd(x, A, B, W), x @ W.T, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.linear_fwd(x, A, B, W, bias), x @ W.T + bias, rtol=1e-13, atol=1e-14)


def test_l2_identity_weights_give_the_rational_forward(oracle):
    x, A, B, _, _, _ = case(2)
    out = oracle.linear_fwd(x, A, B, np.eye(24))
    np.testing.assert_allclose(out, oracle.fwd(x, A, B), rtol=1e-14, atol=1e-15)


def test_l3_brute_force(oracle):
    x, A, B, W, bias, _ = case(3, rows=3, D_in=12, D_out=5, G=3)
    rows, D_in = x.shape
    dg = D_in // 3
    want = np.zeros((rows, 5))
    for r in range(rows):
        for o in range(5):
            acc = bias[o]
            for c in range(D_in):
                g = c // dg
                P = sum(A[g, i] * x[r, c] ** i for i in range(6))
                aden = sum(B[g, j - 1] * x[r, c] ** j for j in range(1, 5))
                acc += W[o, c] * P / (1.0 + abs(aden))
            want[r, o] = acc
    np.testing.assert_allclose(oracle.linear_fwd(x, A, B, W, bias), want, rtol=1e-12, atol=1e-13)


def test_l4_linearity_in_the_weights_and_row_independence(oracle):
    x, A, B, W, bias, _ = case(4)
    W2 = np.random.default_rng(40).standard_normal(W.shape)
    f = lambda w, b=None: oracle.linear_fwd(x, A, B, w, b)
    np.testing.assert_allclose(f(W + W2), f(W) + f(W2), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(f(-2.5 * W), -2.5 * f(W), rtol=1e-13)
    np.testing.assert_allclose(f(W, bias) - f(W), np.broadcast_to(bias, (x.shape[0], bias.size)), rtol=1e-12, atol=1e-13)
    x2 = x.copy()
    x2[3] += 1.0
    d = oracle.linear_fwd(x2, A, B, W) - f(W)
    assert np.all(d[[0, 1, 2, 4, 5, 6]] == 0.0) and np.any(d[3] != 0.0)


def test_l5_weight_layout_is_out_by_in(oracle):
    x, A, B, _, _, _ = case(5, D_in=24, D_out=3)
    W = np.zeros((3, 24))
    W[0, 5] = 1.0    # output 0 <- channel 5 (group 0)
    W[1, 23] = 2.0   # output 1 <- channel 23 (group 3)
    W[2, 12] = -1.0  # output 2 <- channel 12 (group 2)
    y = oracle.fwd(x, A, B)
    out = oracle.linear_fwd(x, A, B, W)
    np.testing.assert_allclose(out, np.stack([y[:, 5], 2.0 * y[:, 23], -y[:, 12]], axis=1), rtol=1e-14)


@pytest.mark.parametrize("round_operand", [False, True])
def test_l6_matmul_route_equals_the_plain_loops(oracle, round_operand):
    x, A, B, W, bias, _ = case(6, rows=33, D_in=96, D_out=40, G=8)
    a = oracle.linear_fwd(x, A, B, W, bias, round_operand=round_operand, threads=3)
    b = oracle.linear_fwd_matmul(x, A, B, W, bias, round_operand=round_operand)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


def test_l7_bfloat16_operand_rounding(oracle):
    # identity F and one-hot weights expose the rounded operand itself
    A = np.zeros((1, 6))
    A[0, 1] = 1.0
    B = np.zeros((1, 4))
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -8), 0.0,
                     3.1415926, 1e-3, -123456.789, 2.0 ** -8 * 1.0000001 + 1.0])
    x = vals[None, :].repeat(2, axis=0)
    W = np.eye(vals.size)
    got = oracle.linear_fwd(x, np.repeat(A, 1, 0), B, W, round_operand=True)[0]
    # exact ties go to the even 8-bit significand: 1 + 2^-8 -> 1, 1 + 3 2^-8 -> 1 + 2^-6 (= 1 + 4 2^-8)
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == 1.0 + 2.0 ** -6 and got[3] == 1.0 + 2.0 ** -7
    assert got[4] == -1.0 and got[5] == 0.0 and got[9] == 1.0 + 2.0 ** -7
    # representable in 8 significant bits, and within half an ulp (ulp = 2^-7 of the binade's lower end)
    mant, _ = np.frexp(got)
    assert np.all(np.ldexp(mant, 8) == np.rint(np.ldexp(mant, 8)))
    nz = vals != 0
    binade = 2.0 ** np.floor(np.log2(np.abs(vals[nz])))
    assert np.all(np.abs(got[nz] - vals[nz]) <= 2.0 ** -8 * binade)
    # numpy's own float32 -> bfloat16 style rounding agrees (through float32 bit patterns)
    u = vals.astype(np.float32).view(np.uint32)
    bf = (((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)).view(np.float32)
    exact32 = vals.astype(np.float32).astype(np.float64) == vals  # only where float32 holds the value exactly
    assert np.array_equal(got[exact32], bf.astype(np.float64)[exact32])


def test_l8_backward_by_finite_differences(oracle):
    x, A, B, W, bias, dOut = case(8, rows=5, D_in=12, D_out=6, G=3)
    # keep away from the kink of |Aden|
    for _ in range(50):
        xg = x.reshape(5, 3, 4)
        aden = sum(B[None, :, j, None] * xg ** (j + 1) for j in range(4))
        bad = np.abs(aden) < 1e-2
        if not bad.any():
            break
        xg[bad] += 0.37
        x = xg.reshape(5, 12)
    g = oracle.linear_bwd(x, dOut, A, B, W)
    L = lambda x_, A_, B_, W_, b_: float(np.sum(dOut * oracle.linear_fwd(x_, A_, B_, W_, b_)))

    def fd(arr, which):
        out = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            h = 1e-6 * max(1.0, abs(arr[idx]))
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += h
            lo[idx] -= h
            args = dict(x_=x, A_=A, B_=B, W_=W, b_=bias)
            args[which] = hi
            up = L(**args)
            args[which] = lo
            out[idx] = (up - L(**args)) / (2 * h)
        return out

    for name, arr, which in (("dx", x, "x_"), ("dA", A, "A_"), ("dB", B, "B_"), ("dW", W, "W_"), ("dbias", bias, "b_")):
        want = fd(arr, which)
        np.testing.assert_allclose(g[name], want, rtol=2e-6, atol=2e-7, err_msg=name)
    np.testing.assert_allclose(g["dF"], dOut @ W, rtol=1e-13, atol=1e-14)


def test_l8b_identity_weights_reduce_to_the_rational_backward(oracle):
    x, A, B, _, _, _ = case(9)
    dOut = np.random.default_rng(90).standard_normal(x.shape)
    g = oracle.linear_bwd(x, dOut, A, B, np.eye(24))
    dx, dA, dB = oracle.bwd(x, dOut, A, B)
    np.testing.assert_allclose(g["dx"], dx, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(g["dA"], dA, rtol=1e-13)
    np.testing.assert_allclose(g["dB"], dB, rtol=1e-13)
    # dW[o, c] = sum_r dOut[r, o] F(x[r, c])
    np.testing.assert_allclose(g["dW"], dOut.T @ oracle.fwd(x, A, B), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["dbias"], dOut.sum(0), rtol=1e-13)


def test_l9_term_scale_is_the_root_sum_square_of_the_terms(oracle):
    x, A, B, W, _, _ = case(10, rows=4, D_in=12, D_out=5, G=3)
    y = oracle.fwd(x, A, B)
    want = np.zeros((4, 5))
    for r in range(4):
        for o in range(5):
            want[r, o] = np.sqrt(sum((W[o, c] * y[r, c]) ** 2 for c in range(12)))
    np.testing.assert_allclose(oracle.linear_term_scale(x, A, B, W), want, rtol=1e-13)
    # and it bounds nothing from below: |out| <= sqrt(D_in) * scale (Cauchy-Schwarz)
    assert np.all(np.abs(oracle.linear_fwd(x, A, B, W)) <= np.sqrt(12) * want * (1 + 1e-12))


def test_l9b_largest_term(oracle):
    x, A, B, W, _, _ = case(12, rows=4, D_in=12, D_out=5, G=3)
    y = oracle.fwd(x, A, B)
    want = np.array([[max(abs(W[o, c] * y[r, c]) for c in range(12)) for o in range(5)] for r in range(4)])
    got = oracle.linear_largest_term(x, A, B, W)
    np.testing.assert_allclose(got, want, rtol=1e-14)
    # between the root-mean-square and the root-sum-square of the terms
    R = oracle.linear_term_scale(x, A, B, W)
    assert np.all(got <= R * (1 + 1e-12)) and np.all(got >= R / np.sqrt(12) * (1 - 1e-12))


def test_linear_oracle_rejects_bad_shapes(oracle):
    x, A, B, W, bias, _ = case(11)
    with pytest.raises(ValueError):
        oracle.linear_fwd(x, A, B, W.T)
    with pytest.raises(ValueError):
        oracle.linear_fwd(x, A, B, W, bias[:-1])
    with pytest.raises(ValueError):
        oracle.linear_bwd(x, np.zeros((7, 9)), A, B, W)
