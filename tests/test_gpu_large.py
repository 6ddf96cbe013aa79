"""Maximum-size edge case: tensors larger than 4 GiB, so that every byte offset
the kernels form has to be 64-bit.  The inputs are drawn on the GPU (4.7 GB per
tensor would take too long on the host).

What is checked, and against what:
  * y and dx against the oracle on a contiguous band of rows on each side of
    the 4 GiB boundary, the first and last rows, and random rows;
  * y and dx of the whole launch, bit for bit, against two launches on the two
    halves of the rows (each below 4 GiB; the per-element arithmetic does not
    depend on the launch geometry), so that no element of the large launch goes
    unchecked;
  * dA / dB of a prefix of 2e8 elements against the oracle, and dA / dB of the
    whole launch through additivity over the split of the rows, a property that
    holds at any size.
"""
import numpy as np
import pytest

from parity_util import TOL, format_stats, plain_stats

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("G", [8, 64])
def test_offsets_beyond_4_gib(oracle, G):
    import torch

    import paper_2505_13813_amd as grkan

    rows, D = 380_000, 3072  # 1.167e9 elements = 4.67 GB per float32 tensor
    assert rows * D * 4 > 2 ** 32
    threads = max(1, min(16, oracle.max_threads()))
    gen = torch.Generator(device="cuda:0").manual_seed(77 + G)
    x = torch.randn(rows, D, device="cuda:0", generator=gen)
    dy = torch.randn(rows, D, device="cuda:0", generator=gen)
    A = ((torch.rand(G, 6, device="cuda:0", generator=gen) * 2 - 1) / torch.arange(1, 7, device="cuda:0"))
    B = torch.rand(G, 4, device="cuda:0", generator=gen) - 0.5

    y = grkan.grkan_fwd(x, A, B)
    dx, dA, dB = grkan.grkan_bwd(x, dy, A, B)
    torch.cuda.synchronize()

    boundary = 2 ** 32 // (D * 4)  # first row that starts beyond 4 GiB
    band = 2048
    pick = np.unique(np.concatenate([np.arange(0, 64), np.arange(boundary - band, boundary + band),
                                     np.arange(rows - 64, rows), np.random.default_rng(G).integers(0, rows, 500)]))
    idx = torch.from_numpy(pick).to("cuda:0")
    xs = x[idx].cpu().numpy().astype(np.float64)
    dys = dy[idx].cpu().numpy().astype(np.float64)
    A64, B64 = A.cpu().numpy().astype(np.float64), B.cpu().numpy().astype(np.float64)
    y_ref = oracle.fwd(xs, A64, B64, threads=threads)
    dx_ref, _, _ = oracle.bwd(xs, dys, A64, B64, threads=threads)
    Sy, Sdx, _, _ = oracle.scales(xs, dys, A64, B64, threads=threads)
    y_s, dx_s = y[idx].cpu().numpy(), dx[idx].cpu().numpy()
    tiny = np.finfo(np.float64).tiny  # an upstream gradient drawn as exactly 0 gives dx = Sdx = 0
    ey = np.max(np.abs(y_s - y_ref) / np.maximum(np.maximum(np.abs(y_ref), Sy), tiny))
    edx = np.max(np.abs(dx_s - dx_ref) / np.maximum(np.maximum(np.abs(dx_ref), Sdx), tiny))
    print()
    print("  " + format_stats("y  (%d rows)" % len(pick), ey, plain_stats(y_s, y_ref)))
    print("  " + format_stats("dx (%d rows)" % len(pick), edx, plain_stats(dx_s, dx_ref)))
    assert ey <= TOL["f32"]["y"] and edx <= TOL["f32"]["dx"], (ey, edx)
    del xs, dys, y_ref, dx_ref, Sy, Sdx

    # the two halves of the rows, each launch below 4 GiB
    cut = rows // 2
    assert cut * D * 4 < 2 ** 32 and (rows - cut) * D * 4 < 2 ** 32
    tmp = torch.empty(rows - cut, D, device="cuda:0")
    dAh, dBh = [], []
    for lo, hi in ((0, cut), (cut, rows)):
        out = tmp[:hi - lo]
        grkan.grkan_fwd(x[lo:hi], A, B, out=out)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), y[lo:hi].view(torch.int32)), "y differs in rows %d..%d" % (lo, hi)
        a_, b_ = torch.empty_like(A), torch.empty_like(B)
        grkan.grkan_bwd(x[lo:hi], dy[lo:hi], A, B, out=(out, a_, b_))
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), dx[lo:hi].view(torch.int32)), "dx differs in rows %d..%d" % (lo, hi)
        dAh.append(a_.double().cpu().numpy())
        dBh.append(b_.double().cpu().numpy())
    tA, tB = dAh[0] + dAh[1], dBh[0] + dBh[1]
    gA, gB = dA.double().cpu().numpy(), dB.double().cpu().numpy()
    assert np.all(np.isfinite(gA)) and np.all(np.isfinite(gB))

    # a prefix of 2e8 elements against the oracle: coefficient gradients and their scales
    prefix = 200_000_000 // D
    _, dAp, dBp = grkan.grkan_bwd(x[:prefix], dy[:prefix], A, B, out=(tmp[:prefix], torch.empty_like(A),
                                                                      torch.empty_like(B)))
    torch.cuda.synchronize()
    xp = x[:prefix].cpu().numpy().astype(np.float64)
    dyp = dy[:prefix].cpu().numpy().astype(np.float64)
    _, dA_ref, dB_ref = oracle.bwd(xp, dyp, A64, B64, threads=threads)
    _, _, RA, RB = oracle.scales(xp, dyp, A64, B64, threads=threads)
    del xp, dyp
    eA = np.max(np.abs(dAp.double().cpu().numpy() - dA_ref) / np.maximum(np.abs(dA_ref), RA))
    eB = np.max(np.abs(dBp.double().cpu().numpy() - dB_ref) / np.maximum(np.abs(dB_ref), RB))
    print("  " + format_stats("dA (prefix of %d rows)" % prefix, eA, plain_stats(dAp.cpu().numpy(), dA_ref)))
    print("  " + format_stats("dB (prefix of %d rows)" % prefix, eB, plain_stats(dBp.cpu().numpy(), dB_ref)))
    assert eA <= TOL["f32"]["dA"] and eB <= TOL["f32"]["dB"], (eA, eB)

    # additivity over the split; the root-sum-square of all terms is sqrt(rows / prefix) times the
    # prefix's (independent, identically distributed rows)
    grow = np.sqrt(rows / prefix)
    eA = np.max(np.abs(gA - tA) / np.maximum(np.abs(tA), RA * grow))
    eB = np.max(np.abs(gB - tB) / np.maximum(np.abs(tB), RB * grow))
    print("  additivity over the two halves: dA %.2e dB %.2e" % (eA, eB))
    assert eA <= TOL["f32"]["dA"] and eB <= TOL["f32"]["dB"], (eA, eB)
