"""Model-level conventions of the PyTorch front end that need no GPU: the Swish
fit, the variance-preserving scale and the parameter layout."""
import math

import numpy as np
import pytest
import torch

from paper_2505_13813_amd import nn as gnn


def swish(x):
    return x / (1.0 + np.exp(-x))


def test_swish_fit_is_tight_and_uses_a_positive_denominator():
    a, b = gnn.swish_coefficients()
    assert len(a) == 6 and len(b) == 4
    xs = np.linspace(-3, 3, 997)
    assert np.abs(gnn._rational_np(xs, np.array(a), np.array(b)) - swish(xs)).max() < 5e-6
    xs = np.linspace(-6, 6, 997)
    assert np.abs(gnn._rational_np(xs, np.array(a), np.array(b)) - swish(xs)).max() < 2e-2
    aden = sum(b[j] * xs ** (j + 1) for j in range(4))
    assert aden.min() > -1e-9  # |.| never active: F is smooth


@pytest.mark.parametrize("m,n,tol", [(3, 2, 6e-3), (7, 6, 1e-8)])
def test_swish_fit_for_the_other_degree_pairs(m, n, tol):
    a, b = gnn.swish_coefficients(m, n)
    assert len(a) == m + 1 and len(b) == n
    xs = np.linspace(-3, 3, 997)
    assert np.abs(gnn._rational_np(xs, np.array(a), np.array(b)) - swish(xs)).max() < tol
    aden = sum(b[j] * xs ** (j + 1) for j in range(n))
    assert aden.min() > -1e-9
    layer = gnn.GroupRational(4, init="swish", degrees=(m, n))
    A, B = layer.coefficient_rows()
    assert A.shape == (4, m + 1) and B.shape == (4, n)
    with pytest.raises(ValueError):
        gnn.GroupRational(4, degrees=(4, 4))


def test_second_moment_matches_closed_forms():
    # identity: E[x^2] = 1; x^2: E[x^4] = 3; Swish fit: E[swish^2] by direct quadrature
    assert abs(gnn.second_moment([0, 1, 0, 0, 0, 0], [0, 0, 0, 0]) - 1.0) < 1e-12
    assert abs(gnn.second_moment([0, 0, 1, 0, 0, 0], [0, 0, 0, 0]) - 3.0) < 1e-10
    t, w = np.polynomial.hermite_e.hermegauss(200)
    want = float(np.sum(w * swish(t) ** 2) / math.sqrt(2 * math.pi))
    a, b = gnn.swish_coefficients()
    assert abs(gnn.second_moment(a, b) - want) < 2e-3


def test_parameter_layout_follows_the_paper():
    # one shared numerator row (6) + G denominator rows (4 each): m + n*g + 1 extra parameters
    layer = gnn.GRKANLinear(768, 3072, groups=8, init="swish", bias=False)
    n_rational = sum(p.numel() for p in layer.rational.parameters())
    assert n_rational == 5 + 4 * 8 + 1
    A, B = layer.rational.coefficient_rows()
    assert A.shape == (8, 6) and B.shape == (8, 4)
    assert torch.equal(A[0], A[7])
    # variance-preserving weights: std = sqrt(alpha / d_in)
    alpha = 1.0 / layer.rational.second_moment()
    assert abs(layer.linear.weight.std().item() - math.sqrt(alpha / 768)) < 5e-4
    # ... which is what keeps the variance: Var[W F(x)] = d_in * Var[w] * E[F^2] = 1
    assert abs(768 * (alpha / 768) * layer.rational.second_moment() - 1.0) < 1e-12
    mlp = gnn.KATMlp(192)
    assert mlp.fc1.linear.weight.shape == (768, 192) and mlp.fc2.linear.weight.shape == (192, 768)
    ident = mlp.fc1.rational.coefficient_rows()
    assert torch.equal(ident[0][0], torch.tensor([0.0, 1, 0, 0, 0, 0])) and torch.count_nonzero(ident[1]) == 0


def test_cpu_tensors_are_refused():
    layer = gnn.GroupRational(8)
    with pytest.raises(ValueError):
        layer(torch.zeros(4, 192))
    with pytest.raises(ValueError):
        gnn.GRKANLinear(100, 10, groups=8)


def test_fused_layer_size_rule():
    """The module takes the one-kernel layer only where it fills the chip (or the contraction is short)."""
    from paper_2505_13813_amd.nn import fused_layer_pays

    assert fused_layer_pays(25216, 3072, 768)          # KAT-B second layer at batch 128: 226 workgroups
    assert not fused_layer_pays(12608, 3072, 768)      # half the batch: 113 workgroups, the two kernels are faster
    assert not fused_layer_pays(197, 3072, 768)        # one image
    assert fused_layer_pays(25216, 1536, 384)          # KAT-S second layer
    assert not fused_layer_pays(6304, 1536, 384)
    assert fused_layer_pays(197, 768, 192)             # short contraction: one launch instead of two
    assert fused_layer_pays(6000, 3072, 3072)          # many channel blocks make up for few tokens
