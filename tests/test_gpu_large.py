"""Maximum-size edge case: tensors larger than 4 GiB, so that every byte offset
the kernels form has to be 64-bit.  The inputs are drawn on the GPU (4.7 GB per
tensor would take too long on the host); y and dx are checked against the
oracle on sampled rows from both sides of the 4 GiB boundary, dA / dB through
additivity over a split of the rows (each part below 4 GiB), a property that
holds at any size."""
import numpy as np
import pytest

from parity_util import TOL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("G", [8, 64])
def test_offsets_beyond_4_gib(oracle, G):
    import torch

    import paper_2505_13813_amd as grkan

    rows, D = 380_000, 3072  # 1.167e9 elements = 4.67 GB per float32 tensor
    assert rows * D * 4 > 2 ** 32
    gen = torch.Generator(device="cuda:0").manual_seed(77 + G)
    x = torch.randn(rows, D, device="cuda:0", generator=gen)
    dy = torch.randn(rows, D, device="cuda:0", generator=gen)
    A = ((torch.rand(G, 6, device="cuda:0", generator=gen) * 2 - 1) / torch.arange(1, 7, device="cuda:0"))
    B = torch.rand(G, 4, device="cuda:0", generator=gen) - 0.5

    y = grkan.grkan_fwd(x, A, B)
    dx, dA, dB = grkan.grkan_bwd(x, dy, A, B)
    torch.cuda.synchronize()

    boundary = 2 ** 32 // (D * 4)  # first row that starts beyond 4 GiB
    pick = np.unique(np.concatenate([np.arange(0, 4), np.arange(boundary - 3, boundary + 4),
                                     np.arange(rows - 4, rows), np.random.default_rng(G).integers(0, rows, 100)]))
    idx = torch.from_numpy(pick).to("cuda:0")
    xs = x[idx].cpu().numpy().astype(np.float64)
    dys = dy[idx].cpu().numpy().astype(np.float64)
    A64, B64 = A.cpu().numpy().astype(np.float64), B.cpu().numpy().astype(np.float64)
    y_ref = oracle.fwd(xs, A64, B64, threads=4)
    dx_ref, _, _ = oracle.bwd(xs, dys, A64, B64, threads=4)
    Sy, Sdx, _, _ = oracle.scales(xs, dys, A64, B64, threads=4)
    ey = np.max(np.abs(y[idx].cpu().numpy() - y_ref) / np.maximum(np.abs(y_ref), Sy))
    edx = np.max(np.abs(dx[idx].cpu().numpy() - dx_ref) / np.maximum(np.abs(dx_ref), Sdx))
    assert ey <= TOL["f32"]["y"] and edx <= TOL["f32"]["dx"], (ey, edx)

    # additivity of the coefficient gradients over a split of the rows
    cut = rows // 2
    _, dA1, dB1 = grkan.grkan_bwd(x[:cut], dy[:cut], A, B)
    _, dA2, dB2 = grkan.grkan_bwd(x[cut:], dy[cut:], A, B)
    torch.cuda.synchronize()
    tA = (dA1.double() + dA2.double()).cpu().numpy()
    tB = (dB1.double() + dB2.double()).cpu().numpy()
    gA, gB = dA.double().cpu().numpy(), dB.double().cpu().numpy()
    # scale: root-sum-square of the terms ~ sqrt(N) * typical term; use the totals' spread over groups
    sA = np.maximum(np.abs(tA), np.sqrt(np.mean(tA ** 2, axis=0, keepdims=True)))
    sB = np.maximum(np.abs(tB), np.sqrt(np.mean(tB ** 2, axis=0, keepdims=True)))
    assert np.max(np.abs(gA - tA) / sA) <= TOL["f32"]["dA"], np.max(np.abs(gA - tA) / sA)
    assert np.max(np.abs(gB - tB) / sB) <= TOL["f32"]["dB"], np.max(np.abs(gB - tB) / sB)
    assert np.all(np.isfinite(gA)) and np.all(np.isfinite(gB))
