"""GPU parity: the HIP path through the C ABI against the fp64 oracle, element
by element, on the seeded synthetic inputs."""
import numpy as np
import pytest

import grkan_inputs
from parity_util import (ABS_FLOOR, TOL, assert_parity, format_stats, plain_stats, run_gpu, run_oracle,
                         to_device, to_host)

pytestmark = pytest.mark.gpu


def custom_case(seed, rows, D, G, dtype="f32", x_scale=1.0, m=5, n=4):
    rng = np.random.default_rng(seed)
    A = (rng.uniform(-1, 1, size=(G, m + 1)) / (np.arange(m + 1) + 1.0)).astype(np.float32)
    B = rng.uniform(-0.5, 0.5, size=(G, n)).astype(np.float32)
    x = (rng.standard_normal((rows, D)) * x_scale).astype(np.float32)
    dy = rng.standard_normal((rows, D)).astype(np.float32)
    case = dict(dtype=dtype, rows=rows, D=D, G=G, m=m, n=n, A=A, B=B, x=x, dy=dy)
    if dtype != "f32":
        to_bits, widen = ((grkan_inputs.round_to_bf16_bits, grkan_inputs.bf16_bits_to_f32) if dtype == "bf16"
                          else (grkan_inputs.round_to_f16_bits, grkan_inputs.f16_bits_to_f32))
        for k in ("x", "dy"):
            bits = to_bits(case[k])
            case[k + "_bits"] = bits
            case[k] = widen(bits)
    return case


@pytest.fixture(scope="module")
def threads(oracle):
    return max(1, min(16, oracle.max_threads()))


# ------------------------------------------------------------------ config 0
@pytest.mark.parametrize("m,n", [(5, 4), (3, 2), (7, 6)])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_tiny_config_elementwise(oracle, dtype, m, n):
    case = grkan_inputs.make_case("tiny", dtype=dtype, m=m, n=n)
    gpu = run_gpu(case)
    ref = run_oracle(oracle, case)
    err = assert_parity(gpu, ref, dtype, label="tiny/%s (%d,%d)" % (dtype, m, n))
    print("tiny", dtype, (m, n), err)


# ------------------------------------------------------------------ shapes that span tiles, tails, vector widths
SHAPES = [
    # rows, D, G            what it exercises
    (1000, 192, 8),       # KAT-T x1 segment (96 B): flat walk, ragged tail
    (999, 768, 8),        # KAT-T x2 / KAT-B x1 segment, odd row count
    (513, 384, 8),        # KAT-S x1 (192 B segments): flat walk
    (257, 1536, 8),       # KAT-S x2
    (301, 3072, 8),       # KAT-B x2 segment
    (129, 3072, 1),       # one group
    (131, 3072, 64),      # 64 groups
    (37, 40, 5),          # d_g = 8
    (33, 30, 5),          # d_g = 6  -> 2-wide vectors (fp32)
    (29, 35, 5),          # d_g = 7  -> scalar path
    (1, 192, 8), (2, 8, 8), (5, 7, 1), (64, 64, 1), (1, 1, 1),
    (3, 64 * 4 * 1009, 64),   # flat walk over very long rows
    (3, 64 * 64 * 1031, 64),  # group walk, general (non fixed-column) columns
    (3, 8 * 24 * 10007, 8),   # group walk, 4 groups per workgroup, general columns
    (700, 192, 48), (300, 96, 96),  # d_g = 4 and d_g = 1: many groups per workgroup in the flat walk
]


@pytest.mark.parametrize("rows,D,G", SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_shapes_elementwise(oracle, rows, D, G, dtype):
    case = custom_case(rows * 7919 + D * 31 + G, rows, D, G, dtype)
    gpu = run_gpu(case)
    ref = run_oracle(oracle, case, threads=4)
    assert_parity(gpu, ref, dtype, label="%dx%d G=%d %s" % (rows, D, G, dtype))


@pytest.mark.parametrize("rows,D,G", SHAPES)
@pytest.mark.parametrize("m,n,dtype", [(3, 2, "f32"), (3, 2, "bf16"), (7, 6, "f32"), (7, 6, "f16")])
def test_shapes_elementwise_other_degrees(oracle, rows, D, G, m, n, dtype):
    case = custom_case(rows * 7919 + D * 31 + G + 1000 * m, rows, D, G, dtype, m=m, n=n)
    gpu = run_gpu(case)
    ref = run_oracle(oracle, case, threads=4)
    assert_parity(gpu, ref, dtype, label="%dx%d G=%d %s (%d,%d)" % (rows, D, G, dtype, m, n))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("D,G", [(768, 8), (192, 8)])  # group walk / flat walk
def test_every_trip_count_of_the_streaming_loop(oracle, dtype, D, G):
    """The streaming loop handles two chunks per trip and finishes with one or two
    more.  With one workgroup per compute unit and these sizes the waves make
    between one and six visits, odd and even, so every exit of the loop is
    compared element by element at sizes that take seconds."""
    import paper_2505_13813_amd as grkan

    grkan.tuning_override(1, 1)
    try:
        vec = 4 if dtype == "f32" else 8
        per_pass = 256 * 4 * 64 * vec  # elements one pass of a 256-workgroup grid covers
        for k, visits in enumerate((1.0, 1.5, 2.0, 2.6, 3.0, 3.7, 4.2, 5.0, 5.5)):
            rows = int(visits * per_pass / D) + k
            case = custom_case(9000 + k, rows, D, G, dtype)
            gpu = run_gpu(case)
            ref = run_oracle(oracle, case, threads=8)
            assert_parity(gpu, ref, dtype, label="%dx%d G=%d %s (%.1f visits)" % (rows, D, G, dtype, visits))
    finally:
        grkan.tuning_override(0, 0)


@pytest.mark.parametrize("dtype,offset", [("f32", 1), ("f32", 2), ("bf16", 1), ("bf16", 2), ("bf16", 4),
                                          ("f16", 1), ("f16", 2), ("f16", 4)])
def test_misaligned_tensors_take_a_narrower_path(oracle, dtype, offset):
    import torch

    import paper_2505_13813_amd as grkan

    rows, D, G = 61, 192, 8
    case = custom_case(4242 + offset, rows, D, G, dtype)
    dev = to_device(case)
    n = rows * D

    def shifted(t):
        buf = torch.empty(n + 16, dtype=t.dtype, device=t.device)
        view = buf[offset:offset + n].view(rows, D)
        view.copy_(t)
        return view

    x, dy = shifted(dev["x"]), shifted(dev["dy"])
    y = shifted(torch.zeros_like(dev["x"]))
    dx = shifted(torch.zeros_like(dev["x"]))
    dA, dB = torch.empty_like(dev["A"]), torch.empty_like(dev["B"])
    grkan.grkan_fwd(x, dev["A"], dev["B"], out=y)
    grkan.grkan_bwd(x, dy, dev["A"], dev["B"], out=(dx, dA, dB))
    torch.cuda.synchronize()
    gpu = dict(y=to_host(y), dx=to_host(dx), dA=to_host(dA), dB=to_host(dB))
    ref = run_oracle(oracle, case)
    assert_parity(gpu, ref, dtype, label="misaligned %s +%d" % (dtype, offset))


# ------------------------------------------------------------------ degenerate cases of the method
def test_identity_init_is_exact(oracle):
    # A = e_1, B = 0 (the paper's first-layer init): y = x, dx = dy, dB = 0 exactly
    case = custom_case(5, 300, 192, 8)
    case["A"] = np.zeros((8, 6), np.float32)
    case["A"][:, 1] = 1.0
    case["B"] = np.zeros((8, 4), np.float32)
    gpu = run_gpu(case)
    assert np.array_equal(gpu["y"], case["x"].astype(np.float64))
    assert np.array_equal(gpu["dx"], case["dy"].astype(np.float64))
    assert np.array_equal(gpu["dB"], np.zeros((8, 4)))
    ref = run_oracle(oracle, case)
    assert_parity(gpu, ref, "f32", label="identity")


def test_sign_of_zero_denominator_polynomial_is_zero(oracle):
    # x = 0 everywhere: Aden = 0, so dx = dy * a_1 and the b-gradients vanish
    case = custom_case(6, 64, 48, 4)
    case["x"][:] = 0.0
    case["x"][::3, ::5] = 0.5
    gpu = run_gpu(case)
    ref = run_oracle(oracle, case)
    assert_parity(gpu, ref, "f32", label="zeros")
    zero = case["x"] == 0.0
    a1 = np.repeat(case["A"][:, 1].astype(np.float64), 12)[None, :]
    want = (case["dy"].astype(np.float64) * a1)[zero]
    np.testing.assert_allclose(gpu["dx"][zero], want, rtol=1e-6)


def test_large_inputs_stay_finite(oracle):
    case = custom_case(7, 128, 384, 8, x_scale=300.0)
    gpu = run_gpu(case)
    ref = run_oracle(oracle, case)
    assert_parity(gpu, ref, "f32", label="large |x|")


def test_float16_results_beyond_the_format_become_infinities(oracle):
    # B = 0 makes F a polynomial: with |x| up to 40 some |y| pass 65504, the largest binary16 number
    case = custom_case(13, 64, 96, 4, "f16", x_scale=10.0)
    case["B"] = np.zeros_like(case["B"])
    gpu = run_gpu(case)
    ref = run_oracle(oracle, case)
    over = np.abs(ref["y"]) > 65520.0          # rounds to infinity (half-way point above 65504)
    safe = np.abs(ref["y"]) < 65504.0
    assert over.any() and safe.any()
    assert np.all(np.isinf(gpu["y"][over])) and np.all(np.sign(gpu["y"][over]) == np.sign(ref["y"][over]))
    err = np.abs(gpu["y"][safe] - ref["y"][safe]) / np.maximum(np.abs(ref["y"][safe]), ref["Sy"][safe])
    assert np.max(np.maximum(err - 2.0 ** -25 / np.maximum(np.abs(ref["y"][safe]), 1e-30), 0.0)) <= TOL["f16"]["y"]
    # the coefficient sums are float32 and stay finite
    assert np.all(np.isfinite(gpu["dA"])) and np.all(gpu["dB"] == 0.0)


def test_device_query_reports_the_chip():
    import paper_2505_13813_amd as grkan

    q = grkan.device_query()
    assert q["compute_units"] >= 64 and q["engine_clock_khz"] > 500_000
    assert q["memory_clock_khz"] > 100_000 and q["memory_bus_bits"] >= 1024


def test_empty_input():
    import torch

    import paper_2505_13813_amd as grkan

    x = torch.empty(0, 192, device="cuda:0")
    A = torch.ones(8, 6, device="cuda:0")
    B = torch.ones(8, 4, device="cuda:0")
    y = grkan.grkan_fwd(x, A, B)
    dx, dA, dB = grkan.grkan_bwd(x, x, A, B)
    torch.cuda.synchronize()
    assert y.shape == (0, 192) and dx.shape == (0, 192)
    assert torch.count_nonzero(dA).item() == 0 and torch.count_nonzero(dB).item() == 0


@pytest.mark.parametrize("rows,dtype", [(200, "f32"), (9000, "f32"), (9000, "bf16")])
def test_outputs_may_alias_inputs(oracle, rows, dtype):
    """y over x, dx over dy, dx over x.  The larger cases make every wave stream several chunks, so
    the prefetch of the next chunk runs ahead of the aliased stores of the current one."""
    import torch

    import paper_2505_13813_amd as grkan

    case = custom_case(8, rows, 768, 8, dtype)
    dev = to_device(case)
    ref = run_oracle(oracle, case, threads=4)
    xa = dev["x"].clone()
    grkan.grkan_fwd(xa, dev["A"], dev["B"], out=xa)            # y over x
    dya = dev["dy"].clone()
    dA, dB = torch.empty_like(dev["A"]), torch.empty_like(dev["B"])
    grkan.grkan_bwd(dev["x"], dya, dev["A"], dev["B"], out=(dya, dA, dB))  # dx over dy
    torch.cuda.synchronize()
    gpu = dict(y=to_host(xa), dx=to_host(dya), dA=to_host(dA), dB=to_host(dB))
    assert_parity(gpu, ref, dtype, label="aliased")
    xb = dev["x"].clone()
    dA2, dB2 = torch.empty_like(dev["A"]), torch.empty_like(dev["B"])
    grkan.grkan_bwd(xb, dev["dy"], dev["A"], dev["B"], out=(xb, dA2, dB2))  # dx over x
    torch.cuda.synchronize()
    gpu2 = dict(y=gpu["y"], dx=to_host(xb), dA=to_host(dA2), dB=to_host(dB2))
    assert_parity(gpu2, ref, dtype, label="dx over x")
    # the same launch geometry and arithmetic whether or not the buffers alias
    assert np.array_equal(gpu2["dx"], gpu["dx"]) and np.array_equal(gpu2["dA"], gpu["dA"])
    assert np.array_equal(gpu2["dB"], gpu["dB"])


def test_errors_from_the_device_side_checks():
    import torch

    import paper_2505_13813_amd as grkan

    x = torch.zeros(4, 192, device="cuda:0")
    A = torch.zeros(8, 6, device="cuda:0")
    B = torch.zeros(8, 4, device="cuda:0")
    small = torch.empty(8, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(grkan.GrkanError) as e:
        grkan.grkan_bwd(x, x, A, B, workspace=small)
    assert e.value.status == 5
    with pytest.raises(grkan.GrkanError) as e:
        grkan.grkan_fwd(x, torch.zeros(8, 5, device="cuda:0"), B)  # (m, n) = (4, 4): not a built pair
    assert e.value.status == 3
    with pytest.raises(grkan.GrkanError) as e:
        grkan.grkan_bwd(x, x, torch.zeros(8, 8, device="cuda:0"), B)  # (7, 4)
    assert e.value.status == 3
    with pytest.raises(grkan.GrkanError) as e:
        grkan.grkan_fwd(x, torch.zeros(7, 6, device="cuda:0"), torch.zeros(7, 4, device="cuda:0"))
    assert e.value.status == 2


# ------------------------------------------------------------------ determinism
@pytest.mark.parametrize("config,tensor,dtype", [("tiny", "x", "f32"), ("kat_b", "x2", "f32"), ("kat_b", "x1", "bf16"),
                                                 ("kat_b", "x1", "f16")])
def test_coefficient_gradients_are_bit_identical_run_to_run(config, tensor, dtype):
    import torch

    import paper_2505_13813_amd as grkan

    case = grkan_inputs.make_case(config, tensor, dtype=dtype)
    dev = to_device(case)
    runs = []
    for _ in range(4):
        dx, dA, dB = grkan.grkan_bwd(dev["x"], dev["dy"], dev["A"], dev["B"])
        torch.cuda.synchronize()
        runs.append((dA.cpu().numpy().copy(), dB.cpu().numpy().copy(), dx.view(torch.int32 if dtype == "f32" else torch.int16).cpu().numpy().copy()))
    for dA, dB, dx in runs[1:]:
        assert np.array_equal(dA.view(np.uint32), runs[0][0].view(np.uint32))
        assert np.array_equal(dB.view(np.uint32), runs[0][1].view(np.uint32))
        assert np.array_equal(dx, runs[0][2])


# ------------------------------------------------------------------ full-size configurations
FULL = [
    ("kat_t", "x1", "f32", 8), ("kat_t", "x2", "f32", 8),
    ("kat_s", "x1", "f32", 8), ("kat_s", "x2", "f32", 8),
    ("kat_b", "x1", "f32", 8), ("kat_b", "x2", "f32", 8),
    ("kat_b", "x1", "bf16", 8), ("kat_b", "x2", "bf16", 8),
    ("kat_b", "x1", "f16", 8), ("kat_b", "x2", "f16", 8),
    ("stress", "x", "f32", 1), ("stress", "x", "f32", 8), ("stress", "x", "f32", 64),
]
# the neighbouring degree pairs at the headline shape
FULL_DEGREES = [("kat_b", "x2", "f32", 8, 3, 2), ("kat_b", "x2", "f32", 8, 7, 6), ("kat_b", "x2", "bf16", 8, 7, 6)]

_case_cache = {}


def full_case(config, tensor, dtype, G, m=5, n=4):
    key = (config, tensor, dtype)
    if key not in _case_cache:
        _case_cache.clear()
        _case_cache[key] = grkan_inputs.make_case(config, tensor, dtype=dtype)
    case = dict(_case_cache[key])
    cfg = grkan_inputs.CONFIGS[config]
    case["A"], case["B"] = grkan_inputs.coefficients(cfg, G, m, n)
    case.update(G=G, m=m, n=n)
    return case


@pytest.mark.parametrize("config,tensor,dtype,G", FULL)
def test_full_size_configuration(oracle, threads, config, tensor, dtype, G):
    """At the bench's sizes and launch configuration: every element of y and dx
    and every entry of dA / dB against the oracle."""
    check_full_size(oracle, threads, full_case(config, tensor, dtype, G))


@pytest.mark.parametrize("config,tensor,dtype,G,m,n", FULL_DEGREES)
def test_full_size_other_degrees(oracle, threads, config, tensor, dtype, G, m, n):
    check_full_size(oracle, threads, full_case(config, tensor, dtype, G, m, n))


def check_full_size(oracle, threads, case):
    """Every element of y and dx and every entry of dA and dB against the oracle,
    in row blocks so that the float64 temporaries stay bounded."""
    config, tensor, dtype, G = case["config"], case["tensor"], case["dtype"], case["G"]
    dev = to_device(case)
    import torch

    import paper_2505_13813_amd as grkan

    y_d = grkan.grkan_fwd(dev["x"], dev["A"], dev["B"])
    dx_d, dA_d, dB_d = grkan.grkan_bwd(dev["x"], dev["dy"], dev["A"], dev["B"])
    torch.cuda.synchronize()
    y_g = y_d.to(torch.float32).cpu().numpy()
    dx_g = dx_d.to(torch.float32).cpu().numpy()
    gpu = dict(dA=to_host(dA_d), dB=to_host(dB_d))
    del dev, y_d, dx_d

    rows = case["rows"]
    A, B = case["A"].astype(np.float64), case["B"].astype(np.float64)
    x = case["x"].astype(np.float64)
    dy = case["dy"].astype(np.float64)
    y = oracle.fwd(x, A, B, threads=threads)
    dx, dA, dB = oracle.bwd(x, dy, A, B, threads=threads)
    Sy, Sdx, RA, RB = oracle.scales(x, dy, A, B, threads=threads)
    del x, dy

    floor = ABS_FLOOR[dtype]
    tiny = np.finfo(np.float64).tiny
    err = dict(y=0.0, dx=0.0)
    block = 4096
    for r0 in range(0, rows, block):
        sl = slice(r0, min(rows, r0 + block))
        for name, g, r, s in (("y", y_g, y, Sy), ("dx", dx_g, dx, Sdx)):
            gb = g[sl].astype(np.float64)
            assert np.all(np.isfinite(gb)), "%s has non-finite values in rows %d.." % (name, r0)
            e = np.maximum(np.abs(gb - r[sl]) - floor, 0.0) / np.maximum(np.maximum(np.abs(r[sl]), s[sl]), tiny)
            err[name] = max(err[name], float(e.max()))
    eA = float(np.max(np.abs(gpu["dA"] - dA) / np.maximum(np.abs(dA), RA)))
    eB = float(np.max(np.abs(gpu["dB"] - dB) / np.maximum(np.abs(dB), RB)))
    print()
    print(config, tensor, dtype, "G=%d" % G, "(%d,%d)" % (case["m"], case["n"]), "all %d elements" % y.size)
    print("  " + format_stats("y ", err["y"], plain_stats(y_g, y)))
    print("  " + format_stats("dx", err["dx"], plain_stats(dx_g, dx)))
    print("  " + format_stats("dA", eA, plain_stats(gpu["dA"], dA)))
    print("  " + format_stats("dB", eB, plain_stats(gpu["dB"], dB)))
    assert err["y"] <= TOL[dtype]["y"], err
    assert err["dx"] <= TOL[dtype]["dx"], err
    assert np.all(np.isfinite(gpu["dA"])) and np.all(np.isfinite(gpu["dB"]))
    assert eA <= TOL[dtype]["dA"] and eB <= TOL[dtype]["dB"], (eA, eB)
    # plain relative error where the sums are well conditioned
    well = np.abs(dA) > 10 * RA
    if well.any():
        assert np.max(np.abs(gpu["dA"] - dA)[well] / np.abs(dA)[well]) <= TOL[dtype]["dA"]


# ------------------------------------------------------------------ non-finite values, streams, layout
def test_nan_propagates_only_where_it_must(oracle):
    """IEEE propagation, no clamping: a NaN input poisons its own y and dx and
    the coefficient sums of its own group, and nothing else."""
    case = custom_case(11, 64, 192, 8)
    case["x"][5, 30] = np.nan      # channel 30 -> group 1
    gpu = run_gpu(case)
    assert np.isnan(gpu["y"][5, 30]) and np.isnan(gpu["dx"][5, 30])
    mask = np.ones_like(gpu["y"], dtype=bool)
    mask[5, 30] = False
    assert np.all(np.isfinite(gpu["y"][mask])) and np.all(np.isfinite(gpu["dx"][mask]))
    assert np.all(np.isnan(gpu["dA"][1])) and np.all(np.isnan(gpu["dB"][1]))
    others = [0, 2, 3, 4, 5, 6, 7]
    clean = dict(case)
    clean["x"] = case["x"].copy()
    clean["x"][5, 30] = 0.25
    ref = run_oracle(oracle, clean)
    eA = np.abs(gpu["dA"][others] - ref["dA"][others]) / np.maximum(np.abs(ref["dA"][others]), ref["RA"][others])
    eB = np.abs(gpu["dB"][others] - ref["dB"][others]) / np.maximum(np.abs(ref["dB"][others]), ref["RB"][others])
    assert eA.max() <= TOL["f32"]["dA"] and eB.max() <= TOL["f32"]["dB"]
    ey = np.abs(gpu["y"][mask] - ref["y"][mask]) / np.maximum(np.abs(ref["y"][mask]), ref["Sy"][mask])
    assert ey.max() <= TOL["f32"]["y"]


def test_work_is_enqueued_on_the_callers_stream(oracle):
    import torch

    import paper_2505_13813_amd as grkan

    case = custom_case(12, 500, 768, 8)
    dev = to_device(case)
    ref = run_oracle(oracle, case, threads=4)
    side = torch.cuda.Stream()
    x_late = torch.empty_like(dev["x"])
    with torch.cuda.stream(side):
        # the input is produced on the side stream just before the calls: results are right only
        # if the kernels really run on that stream, after the copy
        x_late.copy_(dev["x"], non_blocking=True)
        y = grkan.grkan_fwd(x_late, dev["A"], dev["B"])
        dx, dA, dB = grkan.grkan_bwd(x_late, dev["dy"], dev["A"], dev["B"])
    side.synchronize()
    gpu = dict(y=to_host(y), dx=to_host(dx), dA=to_host(dA), dB=to_host(dB))
    assert_parity(gpu, ref, "f32", label="side stream")


def test_binding_rejects_non_contiguous_and_mismatched_tensors():
    import torch

    import paper_2505_13813_amd as grkan

    x = torch.zeros(8, 384, device="cuda:0")
    A = torch.zeros(8, 6, device="cuda:0")
    B = torch.zeros(8, 4, device="cuda:0")
    with pytest.raises(ValueError):
        grkan.grkan_fwd(x[:, ::2], A, B)
    with pytest.raises(ValueError):
        grkan.grkan_bwd(x, x[:4], A, B)
    with pytest.raises(TypeError):
        grkan.grkan_fwd(x.double(), A, B)
    with pytest.raises(TypeError):
        grkan.grkan_fwd(x, A.double(), B)


def test_random_small_shapes_against_the_oracle(oracle):
    """Seeded sweep over awkward shapes, dtypes and pointer offsets, so that every
    kernel variant (vector widths 1-8, group / flat / general walks) meets the
    oracle, not only the shapes of the paper."""
    import random

    import torch

    import paper_2505_13813_amd as grkan

    rng = random.Random(4242)
    for trial in range(96):
        G = rng.choice([1, 2, 3, 4, 5, 8, 16, 33])
        dg = rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 24, 31, 32, 48, 96, 100, 192, 384])
        rows = rng.choice([1, 2, 3, 17, 64, 65, 127, 301, 1000])
        dtype = rng.choice(["f32", "bf16"])
        offset = rng.choice([0, 0, 0, 1, 2, 4])  # elements the tensors are shifted off their allocation
        D = G * dg
        if rows * D > 600_000:
            rows = max(1, 600_000 // D)
        # the second half of the sweep also draws the 16-bit float format and the other degree pairs
        m, n = (5, 4)
        if trial >= 48:
            dtype = rng.choice(["f32", "bf16", "f16", "f16"])
            m, n = rng.choice([(5, 4), (3, 2), (7, 6)])
        case = custom_case(100 + trial, rows, D, G, dtype, m=m, n=n)
        dev = to_device(case)
        n = rows * D

        def shifted(t):
            buf = torch.empty(n + 16, dtype=t.dtype, device=t.device)
            view = buf[offset:offset + n].view(rows, D)
            view.copy_(t)
            return view

        x, dy = shifted(dev["x"]), shifted(dev["dy"])
        y = shifted(torch.zeros_like(dev["x"]))
        dx = shifted(torch.zeros_like(dev["x"]))
        dA, dB = torch.empty_like(dev["A"]), torch.empty_like(dev["B"])
        grkan.grkan_fwd(x, dev["A"], dev["B"], out=y)
        grkan.grkan_bwd(x, dy, dev["A"], dev["B"], out=(dx, dA, dB))
        torch.cuda.synchronize()
        gpu = dict(y=to_host(y), dx=to_host(dx), dA=to_host(dA), dB=to_host(dB))
        ref = run_oracle(oracle, case)
        assert_parity(gpu, ref, dtype,
                      label="trial %d: %dx%d G=%d %s (%d,%d) +%d" % (trial, rows, D, G, dtype, m, n, offset))
