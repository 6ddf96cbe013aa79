"""GPU tests of the PyTorch front end: autograd through the HIP kernels against
the fp64 oracle, with the paper's shared-numerator convention, and the KAT MLP
block against a float64 reference assembled from the oracle and numpy products."""
import numpy as np
import pytest

from parity_util import TOL

pytestmark = pytest.mark.gpu


def test_autograd_function_matches_the_oracle(oracle):
    import torch

    from paper_2505_13813_amd import nn as gnn

    rng = np.random.default_rng(3)
    rows, D, G = 301, 768, 8
    x = rng.standard_normal((4, rows // 4 + 1, D)).astype(np.float32)[:, :75]
    dy = rng.standard_normal(x.shape).astype(np.float32)
    a = (rng.uniform(-1, 1, 6) / (np.arange(6) + 1)).astype(np.float32)
    B = rng.uniform(-0.5, 0.5, (G, 4)).astype(np.float32)

    xt = torch.tensor(x, device="cuda:0", requires_grad=True)
    at = torch.tensor(a, device="cuda:0", requires_grad=True)      # shared numerator row
    Bt = torch.tensor(B, device="cuda:0", requires_grad=True)
    y = gnn.group_rational(xt, at.expand(G, 6), Bt)
    y.backward(torch.tensor(dy, device="cuda:0"))
    torch.cuda.synchronize()

    A = np.tile(a, (G, 1))
    x2, dy2 = x.reshape(-1, D).astype(np.float64), dy.reshape(-1, D).astype(np.float64)
    y_ref = oracle.fwd(x2, A, B, threads=4)
    dx_ref, dA_ref, dB_ref = oracle.bwd(x2, dy2, A, B, threads=4)
    Sy, Sdx, RA, RB = oracle.scales(x2, dy2, A, B, threads=4)
    err = lambda g, r, s: float(np.max(np.abs(g - r) / np.maximum(np.abs(r), s)))
    assert err(y.detach().cpu().numpy().reshape(-1, D), y_ref, Sy) <= TOL["f32"]["y"]
    assert err(xt.grad.cpu().numpy().reshape(-1, D), dx_ref, Sdx) <= TOL["f32"]["dx"]
    assert err(Bt.grad.cpu().numpy(), dB_ref, RB) <= TOL["f32"]["dB"]
    # the shared numerator receives the sum of the per-group gradients
    ra = np.sqrt((RA ** 2).sum(0))
    assert err(at.grad.cpu().numpy(), dA_ref.sum(0), ra) <= TOL["f32"]["dA"]


@pytest.mark.parametrize("degrees", [(5, 4), (3, 2), (7, 6)])
def test_kat_mlp_block_forward_backward(oracle, degrees):
    import torch

    from paper_2505_13813_amd import nn as gnn

    torch.manual_seed(0)
    dim, G = 192, 8
    mlp = gnn.KATMlp(dim, groups=G, degrees=degrees).to("cuda:0")
    # move the rationals away from their init so that every coefficient matters; the steps shrink with
    # the power they multiply, or the high powers would make F steep enough to amplify the float32
    # rounding of the library GEMM that feeds it beyond what this test is about
    with torch.no_grad():
        for r in (mlp.fc1.rational, mlp.fc2.rational):
            m, n = r.degrees
            ka = torch.arange(1, m + 2, device="cuda:0", dtype=torch.float32) ** 2
            kb = torch.arange(1, n + 1, device="cuda:0", dtype=torch.float32) ** 2
            r.numerator.add_(0.05 * torch.randn_like(r.numerator) / ka)
            r.denominator.add_(0.05 * torch.randn_like(r.denominator) / kb)
    x = torch.randn(2, 197, dim, device="cuda:0", requires_grad=True)
    y = mlp(x)
    g = torch.randn_like(y)
    y.backward(g)
    torch.cuda.synchronize()

    # float64 reference: oracle for the rationals, numpy for the products
    def rows_of(r):
        A, B = r.coefficient_rows()
        return A.detach().cpu().numpy().astype(np.float64), B.detach().cpu().numpy().astype(np.float64)

    W1 = mlp.fc1.linear.weight.detach().cpu().numpy().astype(np.float64)
    b1 = mlp.fc1.linear.bias.detach().cpu().numpy().astype(np.float64)
    W2 = mlp.fc2.linear.weight.detach().cpu().numpy().astype(np.float64)
    b2 = mlp.fc2.linear.bias.detach().cpu().numpy().astype(np.float64)
    A1, B1 = rows_of(mlp.fc1.rational)
    A2, B2 = rows_of(mlp.fc2.rational)
    x0 = x.detach().cpu().numpy().reshape(-1, dim).astype(np.float64)
    f1 = oracle.fwd(x0, A1, B1)
    h = f1 @ W1.T + b1
    f2 = oracle.fwd(h, A2, B2)
    y_ref = f2 @ W2.T + b2
    g0 = g.cpu().numpy().reshape(-1, dim).astype(np.float64)
    df2 = g0 @ W2
    dh, dA2, dB2 = oracle.bwd(h, df2, A2, B2)
    df1 = dh @ W1
    dx_ref, dA1, dB1 = oracle.bwd(x0, df1, A1, B1)

    def close(got, want, tol):
        got = got.detach().cpu().numpy().astype(np.float64).reshape(want.shape)
        scale = np.maximum(np.abs(want), np.sqrt(np.mean(want ** 2)))
        assert np.max(np.abs(got - want) / scale) <= tol, np.max(np.abs(got - want) / scale)

    # float32 products (library GEMMs) set the tolerance here, not the rational kernels
    close(y, y_ref, 2e-4)
    close(x.grad, dx_ref, 2e-4)
    close(mlp.fc2.rational.denominator.grad, dB2, 2e-4)
    close(mlp.fc2.rational.numerator.grad, dA2.sum(0), 2e-4)
    close(mlp.fc1.rational.denominator.grad, dB1, 2e-4)
    close(mlp.fc1.rational.numerator.grad, dA1.sum(0), 2e-4)
    close(mlp.fc2.linear.weight.grad, g0.T @ f2, 2e-4)
    close(mlp.fc1.linear.weight.grad, dh.T @ f1, 2e-4)


def test_fused_layer_module_forward_and_backward(oracle):
    """GRKANLinear(fused="always"): the forward pass is the one-kernel layer, the backward pass
    recomputes F(x); gradients against the oracle's chain rule (bfloat16 storage throughout, so the
    comparison is coarse: it checks the wiring -- which product, which transpose, which sum)."""
    import torch

    import paper_2505_13813_amd as grkan
    from paper_2505_13813_amd import nn as gnn

    torch.manual_seed(1)
    rows, D_in, D_out, G = 160, 256, 64, 8
    layer = gnn.GRKANLinear(D_in, D_out, G, init="swish", fused="always").to("cuda:0").to(torch.bfloat16)
    with torch.no_grad():
        layer.rational.numerator.add_(torch.randn_like(layer.rational.numerator) * 0.05)
        layer.rational.denominator.add_(torch.randn_like(layer.rational.denominator) * 0.05)
        layer.linear.bias.normal_(0.0, 0.1)
    x = torch.randn(rows, D_in, device="cuda:0").to(torch.bfloat16).requires_grad_(True)
    dout = torch.randn(rows, D_out, device="cuda:0").to(torch.bfloat16)
    A, B = layer.rational.coefficient_rows()
    assert gnn.fused_layer_supported(x, A, layer.linear.weight)
    out = layer(x)
    direct = grkan.grkan_linear_fwd(x.detach(), A.float().contiguous(), B.float().contiguous(),
                                    layer.linear.weight.detach(), layer.linear.bias.detach().float())
    assert torch.equal(out.detach().view(torch.int16), direct.view(torch.int16))
    out.backward(dout)
    torch.cuda.synchronize()

    f64 = lambda t: t.detach().to(torch.float32).cpu().numpy().astype(np.float64)
    A64, B64 = f64(A.float()), f64(B.float())
    ref = oracle.linear_bwd(f64(x), f64(dout), A64, B64, f64(layer.linear.weight))
    close = lambda g, r, tol: np.max(np.abs(g - r)) <= tol * np.max(np.abs(r))
    assert close(f64(x.grad), ref["dx"], 3e-2)
    assert close(f64(layer.linear.weight.grad), ref["dW"], 3e-2)
    assert close(f64(layer.linear.bias.grad), ref["dbias"], 3e-2)
    assert close(f64(layer.rational.denominator.grad), ref["dB"], 5e-2)
    # one shared numerator row: the sum of the per-group gradients
    assert close(f64(layer.rational.numerator.grad), ref["dA"].sum(0), 5e-2)
    # inference mode of the default setting takes the fused kernel, training the two-kernel path
    auto = gnn.GRKANLinear(D_in, D_out, G, init="swish").to("cuda:0").to(torch.bfloat16)
    auto.load_state_dict(layer.state_dict())
    with torch.no_grad():
        assert torch.equal(auto(x).view(torch.int16), direct.view(torch.int16))
        # the packed copy of the weights is remade when the weights are written to
        first = auto._packed[0]
        assert auto(x) is not None and auto._packed[0] is first
        auto.linear.weight.mul_(0.5)
        auto.linear.bias.add_(1.0)
        again = auto(x)
        assert auto._packed[0] is not first
        want = grkan.grkan_linear_fwd(x.detach(), A.float().contiguous(), B.float().contiguous(),
                                      auto.linear.weight.detach(), auto.linear.bias.detach().float())
        assert torch.equal(again.view(torch.int16), want.view(torch.int16))
        # ... and when the rational function's coefficients are
        auto.rational.denominator.add_(0.01)
        A2, B2 = auto.rational.coefficient_rows()
        want = grkan.grkan_linear_fwd(x.detach(), A2.float().contiguous(), B2.float().contiguous(),
                                      auto.linear.weight.detach(), auto.linear.bias.detach().float())
        assert torch.equal(auto(x).view(torch.int16), want.view(torch.int16))
