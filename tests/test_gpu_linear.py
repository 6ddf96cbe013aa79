"""GPU parity of the fused GR-KAN layer, out = W F(x) (+ bias) in one kernel
(paper, Eq. "GR_KAN"), against the fp64 oracle, element by element.

Two gates, both relative to max(|ref|, R) with R = sqrt(sum_c (W[o,c] F(x[r,c]))^2),
the root-sum-square of the summed terms (the scale of the rounding error of a
sum of D_in terms):

  gate 1, against the definition (fp64 F, fp64 sum).  The kernel feeds the matrix
      cores bfloat16 operands: F is rounded to 8 significant bits, an error of at
      most 2^-8 and of 2^-7 / sqrt(12) * sqrt(1/2) = 1.6e-3 rms per term (uniform
      within half an ulp, averaged over the binade), independent between terms, so
      the sum is off by sigma = 1.6e-3 R.  The largest of n such deviations is
      about sqrt(2 ln 2n) sigma: 6.1 sigma = 9.8e-3 R for the 7.7e7 outputs of the
      largest case.  Tolerance 7.5 sigma = 1.2e-2 for float32 output (exceeded by
      chance once in 1e5 such runs); a bfloat16 output adds its own rounding,
      2^-8 |ref|: 1.6e-2.
  gate 2, against the oracle with the operand rounded the same way (the rounding
      decision taken on both sides, as for a quantised code).  What is left is
      (a) float32 accumulation of D_in <= 3072 exact products, about
      sqrt(D_in) 2^-24 R = 3e-6 R, gated at 1e-4 max(|ref|, R); (b) the rare
      element whose float32 F falls on the other side of a rounding boundary than
      the fp64 F (probability about 4e-5 per term): each moves the output by one
      bfloat16 ulp of its term, at most 2^-7 T with T the largest term of that
      output; up to four such per output are allowed for; (c) for bfloat16 output
      its own rounding, 2^-8 |ref|.  T costs rows * D_out * D_in operations in
      numpy, so at full size this gate runs on a sample of rows (gate 1 on all).
"""
import numpy as np
import pytest

import grkan_inputs
from parity_util import format_stats, plain_stats

pytestmark = pytest.mark.gpu

TOL1 = {"f32": 1.2e-2, "bf16": 1.6e-2}
TOL2 = 1.0e-4     # what is left after allowing for operand flips and the output's own rounding
FLIPS = 4


def custom_linear_case(seed, rows, D_in, D_out, G, bias=True):
    rng = np.random.default_rng(seed)
    A = (rng.uniform(-1, 1, size=(G, 6)) / (np.arange(6) + 1.0)).astype(np.float32)
    B = rng.uniform(-0.5, 0.5, size=(G, 4)).astype(np.float32)
    x = rng.standard_normal((rows, D_in)).astype(np.float32)
    W = (rng.standard_normal((D_out, D_in)) / np.sqrt(D_in)).astype(np.float32)
    xb, Wb = grkan_inputs.round_to_bf16_bits(x), grkan_inputs.round_to_bf16_bits(W)
    return dict(dtype="bf16", rows=rows, D=D_in, D_in=D_in, D_out=D_out, G=G, m=5, n=4, A=A, B=B,
                x_bits=xb, x=grkan_inputs.bf16_bits_to_f32(xb), dy_bits=xb, dy=grkan_inputs.bf16_bits_to_f32(xb),
                W_bits=Wb, W=grkan_inputs.bf16_bits_to_f32(Wb),
                bias=(rng.standard_normal(D_out) * 0.1).astype(np.float32) if bias else None)


def run_gpu_linear(case, out_dtype):
    import torch

    import paper_2505_13813_amd as grkan

    dev = grkan_inputs.upload_linear(case)
    out = grkan.grkan_linear_fwd(dev["x"], dev["A"], dev["B"], dev["W"], dev["bias"],
                                 out_dtype=torch.float32 if out_dtype == "f32" else torch.bfloat16)
    torch.cuda.synchronize()
    return out.to(torch.float32).cpu().numpy()


def check(oracle, case, out_dtype, label, threads=4, full=False):
    gpu = run_gpu_linear(case, out_dtype).astype(np.float64)
    x, A, B, W = (case[k].astype(np.float64) for k in ("x", "A", "B", "W"))
    bias = case["bias"].astype(np.float64) if case["bias"] is not None else None
    fwd = oracle.linear_fwd_matmul if full else oracle.linear_fwd
    ref = fwd(x, A, B, W, bias, threads=threads)
    R = oracle.linear_term_scale(x, A, B, W, threads=threads)
    assert gpu.shape == ref.shape and np.all(np.isfinite(gpu)), label
    tiny = np.finfo(np.float64).tiny
    e1 = float(np.max(np.abs(gpu - ref) / np.maximum(np.maximum(np.abs(ref), R), tiny))) if ref.size else 0.0
    print()
    print(label, out_dtype, "all %d outputs" % ref.size)
    print("  " + format_stats("vs definition     ", e1, plain_stats(gpu, ref)))
    assert e1 <= TOL1[out_dtype], (label, e1)
    del ref

    # gate 2 on every output of the small cases, on a sample of rows at full size
    rows = x.shape[0]
    pick = np.arange(rows)
    if full and rows > 512:
        rng = np.random.default_rng(5)
        pick = np.unique(np.concatenate([np.arange(0, 16), np.arange(rows - 16, rows), rng.integers(0, rows, 480)]))
    xs = x[pick]
    ref2 = oracle.linear_fwd_matmul(xs, A, B, W, bias, round_operand=True, threads=threads)
    T = oracle.linear_largest_term(xs, A, B, W, threads=threads)
    allowed = FLIPS * 2.0 ** -7 * T
    if out_dtype == "bf16":
        allowed = allowed + 2.0 ** -8 * 1.01 * np.abs(ref2)
    excess = np.maximum(np.abs(gpu[pick] - ref2) - allowed, 0.0)
    e2 = float(np.max(excess / np.maximum(np.maximum(np.abs(ref2), R[pick]), tiny))) if ref2.size else 0.0
    e2_plain = float(np.max(np.abs(gpu[pick] - ref2) / np.maximum(np.maximum(np.abs(ref2), R[pick]), tiny))) if ref2.size else 0.0
    print("  vs rounded operand (%d rows): beyond the flip allowance %.2e, without any allowance %.2e"
          % (len(pick), e2, e2_plain))
    assert e2 <= TOL2, (label, e2)
    return e1, e2


SHAPES = [
    # rows, D_in, D_out, G        what it exercises
    (300, 768, 384, 8),         # several token blocks with a ragged tail, d_g = 96, one full channel block (BN = 384)
    (113, 768, 192, 8),         # one token past a block, BN = 192
    (1, 64, 4, 2),              # smallest shape: one row, one pair of stages, a sliver of a channel block
    (17, 128, 200, 4),          # partial channel block (edge variant), d_g = 32
    (225, 3072, 768, 8),        # KAT-B fc2 contraction length, one channel block of 768 (eight waves)
    (130, 192, 768, 2),         # d_g = 96 with D_in = 192
    (112, 256, 1152, 8),        # exactly one token block, three channel blocks of 384
    (500, 64, 64, 1),           # one group, short contraction
    (97, 1536, 388, 48),        # d_g = 32: the coefficient group changes every stage; edge block
]


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,D_in,D_out,G", SHAPES)
def test_fused_layer_shapes(oracle, rows, D_in, D_out, G, out_dtype):
    case = custom_linear_case(rows * 31 + D_in + D_out * 7 + G, rows, D_in, D_out, G, bias=(rows % 2 == 1))
    check(oracle, case, out_dtype, "%dx%d -> %d G=%d" % (rows, D_in, D_out, G))


def _random_shapes(count, seed):
    """Seeded shapes inside what the fused kernel covers: D_in a multiple of 64, d_g of 32, D_out of 4."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        rows = int(rng.integers(1, 400))
        D_in = 64 * int(rng.integers(1, 17))
        groups = [g for g in (1, 2, 3, 4, 6, 8, 12, 16, 24, 32) if D_in % g == 0 and (D_in // g) % 32 == 0]
        G = int(rng.choice(groups))
        kind = int(rng.integers(0, 4))  # whole blocks of each tile variant, or anything a multiple of 4
        D_out = [192 * int(rng.integers(1, 5)), 384 * int(rng.integers(1, 4)), 768 * int(rng.integers(1, 3)),
                 4 * int(rng.integers(1, 400))][kind]
        shapes.append((rows, D_in, D_out, G))
    return shapes


@pytest.mark.parametrize("rows,D_in,D_out,G", _random_shapes(12, 20250527))
def test_fused_layer_random_shapes(oracle, rows, D_in, D_out, G):
    # every tile variant, full and partial channel blocks, one to four token blocks, odd group counts
    case = custom_linear_case(rows + 3 * D_in + 5 * D_out + G, rows, D_in, D_out, G, bias=bool(D_out % 8))
    check(oracle, case, "bf16" if rows % 2 else "f32", "random %dx%d -> %d G=%d" % (rows, D_in, D_out, G))


def test_fused_layer_identity_rational_is_a_plain_matrix_product(oracle):
    # A = e_1, B = 0 (the paper's first-layer initialisation): F(x) = x exactly, also after rounding
    # (x is bfloat16 already), so the kernel must agree with an fp64 product to float32 accumulation accuracy
    case = custom_linear_case(5, 200, 768, 384, 8, bias=False)
    case["A"] = np.zeros((8, 6), np.float32)
    case["A"][:, 1] = 1.0
    case["B"] = np.zeros((8, 4), np.float32)
    gpu = run_gpu_linear(case, "f32").astype(np.float64)
    ref = case["x"].astype(np.float64) @ case["W"].astype(np.float64).T
    R = np.sqrt((case["x"].astype(np.float64) ** 2) @ (case["W"].astype(np.float64) ** 2).T)
    assert np.max(np.abs(gpu - ref) / np.maximum(np.abs(ref), R)) <= 1e-5


def test_fused_layer_one_hot_weights_pick_single_channels(oracle):
    # W[o] = e_{c(o)}: out[r, o] = bf16(F(x[r, c(o)])): every (token, k) position of the token operand
    # and every output position is hit exactly once; compared with the elementwise kernel's bfloat16 y
    import torch

    import paper_2505_13813_amd as grkan

    rows, D_in, G = 150, 256, 8
    case = custom_linear_case(6, rows, D_in, D_in, G, bias=False)
    perm = np.random.default_rng(7).permutation(D_in)
    W = np.zeros((D_in, D_in), np.float32)
    W[np.arange(D_in), perm] = 1.0
    case["W"] = W
    case["W_bits"] = grkan_inputs.round_to_bf16_bits(W)
    dev = grkan_inputs.upload_linear(case)
    out = grkan.grkan_linear_fwd(dev["x"], dev["A"], dev["B"], dev["W"], None, out_dtype=torch.bfloat16)
    y = grkan.grkan_fwd(dev["x"], dev["A"], dev["B"])
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), y[:, torch.from_numpy(perm).to("cuda:0")].contiguous().view(torch.int16))


def test_fused_layer_is_deterministic():
    import torch

    import paper_2505_13813_amd as grkan

    case = custom_linear_case(8, 1000, 768, 768, 8)
    dev = grkan_inputs.upload_linear(case)
    outs = []
    for _ in range(3):
        outs.append(grkan.grkan_linear_fwd(dev["x"], dev["A"], dev["B"], dev["W"], dev["bias"]).view(torch.int16).cpu())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_fused_layer_rejects_what_it_does_not_cover():
    import torch

    import paper_2505_13813_amd as grkan

    x = torch.zeros(8, 192, device="cuda:0", dtype=torch.bfloat16)
    A = torch.zeros(8, 6, device="cuda:0")
    B = torch.zeros(8, 4, device="cuda:0")
    W = torch.zeros(64, 192, device="cuda:0", dtype=torch.bfloat16)
    with pytest.raises(grkan.GrkanError) as e:    # d_g = 24 is not a multiple of 32
        grkan.grkan_linear_fwd(x, A, B, W)
    assert e.value.status == 8
    with pytest.raises(grkan.GrkanError) as e:    # degrees (3, 2) are not built for the fused layer
        grkan.grkan_linear_fwd(x, torch.zeros(2, 4, device="cuda:0"), torch.zeros(2, 2, device="cuda:0"), W)
    assert e.value.status == 3
    with pytest.raises(TypeError):
        grkan.grkan_linear_fwd(x.float(), A, B, W)
    with pytest.raises(ValueError):
        grkan.grkan_linear_fwd(x, A, B, W[:, :128])
    out = grkan.grkan_linear_fwd(x[:0], A[:2], B[:2], W)   # no rows: nothing to do
    assert out.shape == (0, 64)


FULL = [("kat_b", "x1"), ("kat_b", "x2"), ("kat_s", "x2"), ("kat_t", "x2")]


@pytest.mark.parametrize("out_dtype", ["bf16", "f32"])
@pytest.mark.parametrize("config,tensor", FULL)
def test_fused_layer_full_size(oracle, config, tensor, out_dtype):
    """The paper's model shapes (per-GPU batch 128): every output against the oracle."""
    if out_dtype == "f32" and (config, tensor) != ("kat_b", "x2"):
        pytest.skip("float32 output is checked at the headline shape")
    case = grkan_inputs.make_linear_case(config, tensor)
    threads = max(1, min(16, oracle.max_threads()))
    check(oracle, case, out_dtype, "%s %s [%d,%d] -> %d" % (config, tensor, case["rows"], case["D_in"], case["D_out"]),
          threads=threads, full=True)


def _packed_layout_numpy(W_bits, D_out, D_in, bn):
    """The packed copy as include/grkan.h describes it, from the bfloat16 bit patterns (data movement only)."""
    T = -(-D_out // bn) * (bn // 16)
    stages = D_in // 32
    Wp = np.zeros((stages, T, 64, 8), np.uint16)
    rows_pad = np.zeros((T * 16, D_in), np.uint16)
    rows_pad[:D_out] = W_bits.view(np.uint16).reshape(D_out, D_in)
    lanes = np.arange(64)
    g = ((lanes >> 4) ^ (lanes >> 3)) & 3
    piece = (lanes & 3) ^ g
    for s in range(stages):
        blk = rows_pad[:, 32 * s:32 * s + 32].reshape(T, 16, 4, 8)          # [tile, row in tile, piece, 8 values]
        Wp[s] = blk[:, lanes >> 2, piece, :]
    return Wp.reshape(-1)


@pytest.mark.parametrize("D_in,D_out,bn", [(256, 768, 768), (128, 384, 384), (64, 200, 192), (192, 1152, 384)])
def test_packed_weights_have_the_documented_layout(D_in, D_out, bn):
    import torch

    import paper_2505_13813_amd as grkan

    rng = np.random.default_rng(D_in + D_out)
    W_bits = grkan_inputs.round_to_bf16_bits(rng.standard_normal((D_out, D_in)).astype(np.float32))
    W = torch.from_numpy(np.ascontiguousarray(W_bits).view(np.int16)).to("cuda:0").view(torch.bfloat16)
    pw = grkan.grkan_linear_pack_w(W)
    torch.cuda.synchronize()
    got = pw.data.cpu().numpy().view(np.uint16)
    want = _packed_layout_numpy(W_bits, D_out, D_in, bn)
    assert got.shape == want.shape and np.array_equal(got, want)


@pytest.mark.parametrize("rows,D_in,D_out,G", SHAPES + _random_shapes(6, 77))
def test_packed_weights_give_bit_identical_outputs(rows, D_in, D_out, G):
    # same arithmetic and summation order, only the weights' addresses differ
    import torch

    import paper_2505_13813_amd as grkan

    case = custom_linear_case(rows + D_in + D_out + G, rows, D_in, D_out, G, bias=True)
    dev = grkan_inputs.upload_linear(case)
    pw = grkan.grkan_linear_pack_w(dev["W"])
    for dt in (torch.bfloat16, torch.float32):
        a = grkan.grkan_linear_fwd(dev["x"], dev["A"], dev["B"], dev["W"], dev["bias"], out_dtype=dt)
        b = grkan.grkan_linear_fwd(dev["x"], dev["A"], dev["B"], pw, dev["bias"], out_dtype=dt)
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (rows, D_in, D_out, G, dt)


def test_packed_weights_full_size_bit_identical():
    import torch

    import paper_2505_13813_amd as grkan

    case = grkan_inputs.make_linear_case("kat_b", "x2")
    dev = grkan_inputs.upload_linear(case)
    pw = grkan.grkan_linear_pack_w(dev["W"])
    a = grkan.grkan_linear_fwd(dev["x"], dev["A"], dev["B"], dev["W"], dev["bias"])
    b = grkan.grkan_linear_fwd(dev["x"], dev["A"], dev["B"], pw, dev["bias"])
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    with pytest.raises(ValueError):
        grkan.grkan_linear_fwd(dev["x"][:, :1536].contiguous(), dev["A"], dev["B"], pw)   # made for another D_in
