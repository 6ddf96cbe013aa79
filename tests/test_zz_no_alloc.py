"""The allocation-free backward entry point (grkan_bwd_noalloc): for callers that
cannot allocate device memory or hand over a workspace.  It runs the kernels of
grkan_bwd on the library's own fixed device array, so its outputs must equal
grkan_bwd's bit for bit -- on two calls in a row, the second with a smaller
input (the array then still holds the first call's rows), and again with a
flat-walk shape that writes many more workspace rows."""
import numpy as np
import pytest

import grkan_inputs
from parity_util import assert_parity, run_oracle, to_device, to_host

pytestmark = pytest.mark.gpu


def _both(grkan, torch, dev):
    ref = grkan.grkan_bwd(dev["x"], dev["dy"], dev["A"], dev["B"])
    out = (torch.full_like(dev["x"], float("nan")), torch.full_like(dev["A"], float("nan")),
           torch.full_like(dev["B"], float("nan")))
    before = torch.cuda.memory_allocated()
    grkan.grkan_bwd_noalloc(dev["x"], dev["dy"], dev["A"], dev["B"], out=out)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return ref, out


def _bits(t):
    import torch

    return t.contiguous().view(torch.uint8).cpu().numpy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_noalloc_backward_equals_grkan_bwd_on_two_calls_in_a_row(oracle, dtype):
    import torch

    import paper_2505_13813_amd as grkan

    # first call: KAT-B x2 rows (group walk); second call: a smaller input of another shape (flat walk,
    # 96-byte segments) while the array still holds the first call's rows; third: the tiny configuration
    shapes = [("kat_b", "x2", 6000), ("kat_t", "x1", 1500), ("tiny", "x", None)]
    for config, tensor, rows in shapes:
        case = grkan_inputs.make_case(config, tensor, dtype=dtype, rows=rows)
        dev = to_device(case)
        ref, out = _both(grkan, torch, dev)
        for name, a, b in zip(("dx", "dA", "dB"), ref, out):
            assert np.array_equal(_bits(a), _bits(b)), (config, tensor, name)
        if config == "tiny":
            orc = run_oracle(oracle, case)
            y = grkan.grkan_fwd(dev["x"], dev["A"], dev["B"])
            gpu = dict(y=to_host(y), dx=to_host(out[0]), dA=to_host(out[1]), dB=to_host(out[2]))
            assert_parity(gpu, orc, dtype, label="noalloc tiny/" + dtype)


def test_noalloc_backward_rejects_shapes_beyond_its_scratch():
    import torch

    import paper_2505_13813_amd as grkan

    # per-channel coefficients on a wide tensor: every workgroup writes a row for every group of its block
    rows, D, G = 4096, 3072, 3072
    need = grkan.grkan_bwd_workspace_bytes(rows, D, G, grkan.GRKAN_F32)
    if need <= grkan.binding.NOALLOC_SCRATCH_BYTES:
        pytest.skip("this shape fits the scratch on this device (%d bytes)" % need)
    x = torch.zeros(rows, D, device="cuda:0")
    A = torch.zeros(G, 6, device="cuda:0")
    B = torch.zeros(G, 4, device="cuda:0")
    out = (torch.empty_like(x), torch.empty_like(A), torch.empty_like(B))
    with pytest.raises(grkan.GrkanError) as e:
        grkan.grkan_bwd_noalloc(x, x, A, B, out=out)
    assert e.value.status == 9
    # and the same shape is fine through the entry point that takes a workspace
    grkan.grkan_bwd(x, x, A, B, out=out)
    torch.cuda.synchronize()


def test_noalloc_backward_with_no_rows():
    import torch

    import paper_2505_13813_amd as grkan

    x = torch.empty(0, 192, device="cuda:0")
    A = torch.ones(8, 6, device="cuda:0")
    B = torch.ones(8, 4, device="cuda:0")
    out = (torch.empty_like(x), torch.full_like(A, 7.0), torch.full_like(B, 7.0))
    grkan.grkan_bwd_noalloc(x, x, A, B, out=out)
    torch.cuda.synchronize()
    assert torch.count_nonzero(out[1]).item() == 0 and torch.count_nonzero(out[2]).item() == 0
