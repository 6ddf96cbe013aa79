"""PyTorch front end of the GR-KAN layer: an autograd function over the HIP
kernels, the group-wise rational module with the paper's model-level
conventions, the GR-KAN linear layer and the KAT MLP block.

The rational function runs in this package's kernels; the matrix products are
torch's (library GEMMs), except where the one-kernel layer grkan_linear_fwd is
selected (GRKANLinear(fused=...)).  Conventions taken from the FlashKAT paper:
  * GR-KAN(x) = W F(x): the rational function is applied to the INPUT of each
    linear layer (Eq. "GR_KAN").
  * the groups use one common set of numerator coefficients and have their own
    denominator coefficients (Sec. "Results"): one numerator row, broadcast to
    the kernel's [G, m+1] layout; autograd's expand sums dA over the groups.
  * the first rational of an MLP block starts as the identity, the second as a
    Swish (Sec. "Results").  The paper prints no Swish coefficients, so they
    are obtained here by a (linearised) least-squares fit on [-3, 3].
  * variance-preserving weights (Sec. "Kolmogorov-Arnold Transformer"):
    W ~ N(0, alpha / d_in).  The paper prints alpha = E[F(x)^2] / Var[x], which
    would not preserve the variance (Var[W F(x)] = d_in * Var[w] * E[F^2]); the
    stated purpose decides, so alpha = Var[x] / E[F(x)^2] here, with
    x ~ N(0, 1) -- the usual gain (2 for ReLU).  Both readings coincide for the
    identity initialisation.
"""
from __future__ import annotations

import math
from functools import lru_cache
from typing import Tuple

import numpy as np
import torch
from torch import nn

from . import binding

M_DEGREE = binding.M_DEGREE
N_DEGREE = binding.N_DEGREE


_workspaces = {}


def _workspace(x, rows: int, D: int, G: int) -> torch.Tensor:
    """One backward workspace per (device, stream), grown on demand.  Calls on one
    stream run one after the other, so they can share it; the workspace's
    contents mean nothing between calls."""
    need = binding._workspace_bytes_cached(rows, D, G, binding._io_of(x), x.device.index or 0)
    key = (x.device.index or 0, torch.cuda.current_stream(x.device).cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.empty(max(need, 1 << 16), dtype=torch.uint8, device=x.device)
        _workspaces[key] = ws
    return ws


class GroupRationalFunction(torch.autograd.Function):
    """y = F(x) group-wise; backward through grkan_bwd (nothing but x, A, B is saved)."""

    @staticmethod
    def forward(ctx, x, A, B):
        x = x.contiguous()
        A = A.contiguous()
        B = B.contiguous()
        ctx.save_for_backward(x, A, B)
        return binding.grkan_fwd(x, A, B)

    @staticmethod
    def backward(ctx, dy):
        x, A, B = ctx.saved_tensors
        D = int(x.shape[-1])
        ws = _workspace(x, int(x.numel() // D) if D else 0, D, int(A.shape[0]))
        dx, dA, dB = binding.grkan_bwd(x, dy.contiguous(), A, B, workspace=ws)
        return dx, dA, dB


def fused_layer_supported(x, A, weight) -> bool:
    """Shapes and types the one-kernel layer (grkan_linear_fwd) covers: bfloat16 x and W on the GPU,
    degrees (5, 4), D_in a multiple of 64, d_g a multiple of 32, D_out a multiple of 4."""
    D_in, G = int(x.shape[-1]), int(A.shape[0])
    return (x.is_cuda and x.dtype == torch.bfloat16 and weight.dtype == torch.bfloat16 and int(A.shape[1]) == 6
            and D_in % 64 == 0 and D_in % G == 0 and (D_in // G) % 32 == 0 and int(weight.shape[0]) % 4 == 0)


def fused_layer_pays(rows: int, D_in: int, D_out: int) -> bool:
    """Whether the one-kernel layer is the faster route at this size (measured on MI355X, bfloat16).
    A workgroup owns 112 tokens x one channel block (768, 384 or 192 channels) and walks the whole
    contraction by itself, so the kernel needs about as many workgroups as the chip has compute units:
    at D_in = 3072 -> 768 it takes 109 us for anything up to 6,000 tokens (the two kernels: 34 - 53 us)
    and wins from about 20,000 tokens on (135 against 192 us at 25,216); with a short contraction
    (D_in <= 768) a workgroup is quick and one launch instead of two wins at every size measured."""
    bn = 768 if D_out % 768 == 0 else (384 if D_out % 384 == 0 else 192)
    workgroups = -(-int(rows) // 112) * -(-int(D_out) // bn)
    return workgroups >= 200 or D_in <= 768


class GRKANLayerFunction(torch.autograd.Function):
    """out = F(x) W^T + bias with the forward pass in one kernel (F never written to memory) and
    nothing but x, A, B, W saved.  The backward pass recomputes F(x) for dW = dOut^T F(x)
    (grkan_fwd + a library product), forms dF = dOut W (library product) and runs grkan_bwd on it:
    one extra elementwise forward kernel in exchange for not keeping F(x) alive between the passes."""

    @staticmethod
    def forward(ctx, x, A, B, weight, bias):
        x = x.contiguous()
        A = A.contiguous()
        B = B.contiguous()
        weight = weight.contiguous()
        ctx.save_for_backward(x, A, B, weight)
        ctx.has_bias = bias is not None
        ctx.bias_dtype = bias.dtype if bias is not None else None
        b32 = bias.to(torch.float32).contiguous() if bias is not None else None
        return binding.grkan_linear_fwd(x, A, B, weight, b32, out_dtype=x.dtype)

    @staticmethod
    def backward(ctx, dout):
        x, A, B, weight = ctx.saved_tensors
        D_in, D_out = int(x.shape[-1]), int(weight.shape[0])
        dout2 = dout.contiguous().view(-1, D_out)
        y = binding.grkan_fwd(x, A, B).view(-1, D_in)      # F(x), recomputed
        dW = dout2.t().mm(y)
        dF = dout2.mm(weight).view(x.shape)
        rows = int(x.numel() // D_in) if D_in else 0
        ws = _workspace(x, rows, D_in, int(A.shape[0]))
        dx, dA, dB = binding.grkan_bwd(x, dF, A, B, workspace=ws)
        dbias = dout2.sum(0).to(ctx.bias_dtype) if ctx.has_bias else None
        return dx, dA, dB, dW, dbias


def group_rational(x, A, B):
    """Functional form: x [..., D] float32 / bfloat16 / float16 on the GPU, A [G, m+1], B [G, n] float32."""
    return GroupRationalFunction.apply(x, A, B)


def _rational_np(x, a, b):
    p = sum(a[i] * x ** i for i in range(len(a)))
    q = 1.0 + np.abs(sum(b[j] * x ** (j + 1) for j in range(len(b))))
    return p / q


@lru_cache(maxsize=None)
def swish_coefficients(m: int = M_DEGREE, n: int = N_DEGREE) -> Tuple[Tuple[float, ...], Tuple[float, ...]]:
    """(a_0..a_m, b_1..b_n) of a safe Pade unit fitted to Swish, x * sigmoid(x).

    Linearised least squares on a uniform grid over [-3, 3]: minimise
    |P(x) - t(x) * sum_j b_j x^j - t(x)| over (a, b), which is linear.  The
    solution has an even, non-negative denominator polynomial (odd b_j = 0,
    even b_j > 0), so the absolute value of the safe unit is inactive; for
    (5, 4) the fit error of F itself is below 1e-6 on the grid (8e-3 on
    [-6, 6]), for (3, 2) 5e-3, for (7, 6) 1e-10.  Deterministic: plain linear
    algebra in float64.
    """
    xs = np.linspace(-3.0, 3.0, 601)
    target = xs / (1.0 + np.exp(-xs))
    cols = [xs ** i for i in range(m + 1)] + [-target * xs ** (j + 1) for j in range(n)]
    theta, *_ = np.linalg.lstsq(np.stack(cols, axis=1), target, rcond=None)
    return tuple(float(v) for v in theta[:m + 1]), tuple(float(v) for v in theta[m + 1:])


def second_moment(a, b, points: int = 128) -> float:
    """E[F(x)^2] for x ~ N(0, 1) by Gauss-Hermite quadrature."""
    t, w = np.polynomial.hermite_e.hermegauss(points)
    f = _rational_np(t, np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64))
    return float(np.sum(w * f * f) / math.sqrt(2.0 * math.pi))


class GroupRational(nn.Module):
    """The group-wise rational function with learnable coefficients.

    `init`: "identity" (a = e_1, b = 0) or "swish".  With `shared_numerator`
    (the paper's setting) there is one numerator row for all groups.
    `degrees` = (m, n), one of the pairs the library is built for.
    """

    def __init__(self, groups: int = 8, init: str = "identity", shared_numerator: bool = True,
                 degrees: Tuple[int, int] = (M_DEGREE, N_DEGREE)):
        super().__init__()
        m, n = (int(v) for v in degrees)
        if (m, n) not in binding.DEGREES:
            raise ValueError("degrees must be one of %s" % (binding.DEGREES,))
        self.degrees = (m, n)
        if init == "identity":
            a = [0.0, 1.0] + [0.0] * (m - 1)
            b = [0.0] * n
        elif init == "swish":
            a, b = swish_coefficients(m, n)
        else:
            raise ValueError("init must be 'identity' or 'swish'")
        self.groups = int(groups)
        self.shared_numerator = bool(shared_numerator)
        a_t = torch.tensor(a, dtype=torch.float32)
        b_t = torch.tensor(b, dtype=torch.float32)
        self.numerator = nn.Parameter(a_t.clone() if shared_numerator else a_t.repeat(self.groups, 1))
        self.denominator = nn.Parameter(b_t.repeat(self.groups, 1))

    def coefficient_rows(self):
        A = self.numerator.expand(self.groups, self.degrees[0] + 1) if self.shared_numerator else self.numerator
        return A, self.denominator

    def second_moment(self) -> float:
        """E[F(x)^2], x ~ N(0,1), averaged over the groups (they start identical)."""
        A, B = self.coefficient_rows()
        A = A.detach().cpu().numpy()
        B = B.detach().cpu().numpy()
        return float(np.mean([second_moment(A[g], B[g]) for g in range(self.groups)]))

    def forward(self, x):
        A, B = self.coefficient_rows()
        return group_rational(x, A.to(torch.float32), B.to(torch.float32))


class GRKANLinear(nn.Module):
    """GR-KAN(x) = W F(x) + bias (Eq. "GR_KAN"), variance-preserving init."""

    def __init__(self, in_features: int, out_features: int, groups: int = 8, init: str = "identity",
                 bias: bool = True, shared_numerator: bool = True,
                 degrees: Tuple[int, int] = (M_DEGREE, N_DEGREE), fused: str = "inference"):
        """`fused`: when the one-kernel layer (F inside the matrix product) is used where it applies
        (bfloat16, see fused_layer_supported): "inference" = when no gradient is recorded (in training
        its backward pass has to recompute F(x)) and the input is large enough for it to be the faster
        route (fused_layer_pays); "always" = wherever it applies; "never"."""
        super().__init__()
        if in_features % groups:
            raise ValueError("in_features must be a multiple of groups")
        if fused not in ("inference", "always", "never"):
            raise ValueError("fused must be 'inference', 'always' or 'never'")
        self.fused = fused
        self._packed = None      # inference: packed copy of the weights and float32 bias, remade when they change
        self._packed_key = None
        self.rational = GroupRational(groups, init, shared_numerator, degrees)
        self.linear = nn.Linear(in_features, out_features, bias=bias)
        alpha = 1.0 / self.rational.second_moment()  # Var[x] / E[F(x)^2] with Var[x] = 1
        with torch.no_grad():
            self.linear.weight.normal_(0.0, math.sqrt(alpha / in_features))
            if bias:
                self.linear.bias.zero_()

    def _inference_weights(self):
        """Packed weights (the kernel then fetches them in whole cache lines), the bias and the
        coefficient rows in float32, cached until a parameter is written to or replaced."""
        params = (self.linear.weight, self.linear.bias, self.rational.numerator, self.rational.denominator)
        key = tuple(None if p is None else (p.data_ptr(), p._version, p.device) for p in params)
        if self._packed_key != key:
            w, b = self.linear.weight, self.linear.bias
            A, B = self.rational.coefficient_rows()
            self._packed = (binding.grkan_linear_pack_w(w.detach().contiguous()),
                            None if b is None else b.detach().to(torch.float32).contiguous(),
                            A.detach().to(torch.float32).contiguous(), B.detach().to(torch.float32).contiguous())
            self._packed_key = key
        return self._packed

    def forward(self, x):
        if self.fused != "never":
            A, B = self.rational.coefficient_rows()
            if fused_layer_supported(x, A, self.linear.weight):
                rows = x.numel() // x.shape[-1]
                pays = self.fused == "always" or fused_layer_pays(rows, x.shape[-1], self.linear.weight.shape[0])
                if not torch.is_grad_enabled() and pays:
                    pw, b32, A32, B32 = self._inference_weights()
                    return binding.grkan_linear_fwd(x.contiguous(), A32, B32, pw, b32, out_dtype=x.dtype)
                if self.fused == "always":
                    return GRKANLayerFunction.apply(x, A.to(torch.float32), B.to(torch.float32), self.linear.weight,
                                                    self.linear.bias)
        return self.linear(self.rational(x))


class KATMlp(nn.Module):
    """The MLP of a KAT block: two GR-KAN layers, hidden width 4x by default;
    the first rational starts as the identity, the second as Swish."""

    def __init__(self, dim: int, hidden: int | None = None, groups: int = 8,
                 degrees: Tuple[int, int] = (M_DEGREE, N_DEGREE), fused: str = "inference"):
        super().__init__()
        hidden = 4 * dim if hidden is None else hidden
        # the one-kernel layer pays for the wide input (fc2: long contraction, few outputs); for fc1
        # the library product after the elementwise kernel is faster on this hardware
        self.fc1 = GRKANLinear(dim, hidden, groups, init="identity", degrees=degrees, fused="never")
        self.fc2 = GRKANLinear(hidden, dim, groups, init="swish", degrees=degrees, fused=fused)

    def forward(self, x):
        return self.fc2(self.fc1(x))
