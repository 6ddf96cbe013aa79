"""The entry points only enqueue kernels (no allocation, no memset, no
synchronisation), so a whole forward+backward step can be captured in a HIP
graph.  The graph is replayed several times, with eager work and
synchronisations of the program's own in between, and every replay is compared
bit for bit with the eager result."""
import numpy as np
import pytest

import grkan_inputs
from parity_util import to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("config,tensors,dtype", [("tiny", ("x",), "f32"), ("kat_t", ("x1", "x2"), "f32"),
                                                    ("kat_t", ("x1", "x2"), "bf16")])
def test_step_captured_in_a_graph_replays_bit_identically(config, tensors, dtype):
    import torch

    import paper_2505_13813_amd as grkan

    layers = []
    for t in tensors:
        case = grkan_inputs.make_case(config, t, dtype=dtype, rows=2048 if config != "tiny" else None)
        dev = to_device(case)
        io = {"f32": grkan.GRKAN_F32, "bf16": grkan.GRKAN_BF16, "f16": grkan.GRKAN_F16}[dtype]
        ws = torch.empty(grkan.grkan_bwd_workspace_bytes(case["rows"], case["D"], case["G"], io), dtype=torch.uint8,
                         device="cuda:0")
        out = dict(y=torch.empty_like(dev["x"]), dx=torch.empty_like(dev["x"]), dA=torch.empty_like(dev["A"]),
                   dB=torch.empty_like(dev["B"]))
        layers.append((dev, ws, out))

    def step():
        for dev, ws, out in layers:
            grkan.grkan_fwd(dev["x"], dev["A"], dev["B"], out=out["y"])
        for dev, ws, out in reversed(layers):
            grkan.grkan_bwd(dev["x"], dev["dy"], dev["A"], dev["B"], workspace=ws, out=(out["dx"], out["dA"], out["dB"]))

    def snapshot():
        torch.cuda.synchronize()
        return [{k: v.clone().view(torch.uint8).cpu().numpy() for k, v in out.items()} for _, _, out in layers]

    def clear():
        for _, _, out in layers:
            for v in out.values():
                v.view(torch.uint8).fill_(0xA5)

    step()
    eager = snapshot()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm the per-kernel occupancy cache outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    for replay in range(4):
        clear()
        # eager work of the program's own between replays
        scratch = torch.randn(1 << 20, device="cuda:0")
        scratch = (scratch * 2).sum().item()
        graph.replay()
        got = snapshot()
        for a, b in zip(eager, got):
            for k in a:
                assert np.array_equal(a[k], b[k]), (replay, k)


def test_fused_layer_and_allocation_free_backward_in_a_graph():
    """The fused layer forward and the allocation-free backward are single enqueues as well: captured
    together, replayed with eager work in between, compared bit for bit with the eager results."""
    import torch

    import paper_2505_13813_amd as grkan

    lin = grkan_inputs.make_linear_case("kat_t", "x2", rows=1000)
    dev = grkan_inputs.upload_linear(lin)
    out = dict(o=torch.empty(lin["rows"], lin["D_out"], device="cuda:0", dtype=torch.bfloat16),
               dx=torch.empty_like(dev["x"]), dA=torch.empty_like(dev["A"]), dB=torch.empty_like(dev["B"]))

    def step():
        grkan.grkan_linear_fwd(dev["x"], dev["A"], dev["B"], dev["W"], dev["bias"], out=out["o"])
        grkan.grkan_bwd_noalloc(dev["x"], dev["dy"], dev["A"], dev["B"], out=(out["dx"], out["dA"], out["dB"]))

    def snapshot():
        torch.cuda.synchronize()
        return {k: v.clone().view(torch.uint8).cpu().numpy() for k, v in out.items()}

    step()  # also: first-call set-up (LDS size attribute, scratch address) outside the capture
    eager = snapshot()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(3):
        for v in out.values():
            v.view(torch.uint8).fill_(0xA5)
        scratch = torch.randn(1 << 20, device="cuda:0")
        scratch = (scratch * 2).sum().item()
        graph.replay()
        got = snapshot()
        for k in eager:
            assert np.array_equal(eager[k], got[k]), (replay, k)
