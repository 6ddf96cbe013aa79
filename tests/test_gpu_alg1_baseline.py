"""The paper's Algorithm 1 (per-element global atomics) as a baseline on the GPU:
it computes the same gradients, and its coefficient gradients carry the larger,
run-to-run varying rounding error the paper reports (Sec. "Reduced Gradient
Rounding Error", Table 5; appendix "Reduced Gradient Rounding Error Expanded"),
while the two-stage reduction of grkan_bwd is deterministic and more accurate.

Protocol of the rounding experiment, as in the appendix: X, dO, A, B all drawn
from N(0,1); dA, dB in fp64 (here: the CPU oracle) against float32 results of
both methods; mean absolute error over the coefficient entries, repeated over
passes.  The paper uses [1024, 197, 768] and 100 passes; the committed test
uses the per-GPU share [128, 197, 768] and 12 passes to keep the run short
(GRKAN_ROUNDING_FULL=1 switches to the paper's shape with 10 passes).
"""
import os

import numpy as np
import pytest

import grkan_inputs
from parity_util import run_oracle, to_device, to_host

pytestmark = pytest.mark.gpu


def test_alg1_baseline_matches_the_oracle(oracle):
    import torch

    import paper_2505_13813_amd as grkan

    for rows, D, G in ((788, 192, 8), (301, 3072, 8), (37, 40, 5), (5, 7, 1)):
        rng = np.random.default_rng(rows + D)
        case = dict(dtype="f32", rows=rows, D=D, G=G,
                    A=(rng.uniform(-1, 1, (G, 6)) / (np.arange(6) + 1.0)).astype(np.float32),
                    B=rng.uniform(-0.5, 0.5, (G, 4)).astype(np.float32),
                    x=rng.standard_normal((rows, D)).astype(np.float32),
                    dy=rng.standard_normal((rows, D)).astype(np.float32))
        dev = to_device(case)
        dx, dA, dB = grkan.grkan_alg1_bwd(dev["x"], dev["dy"], dev["A"], dev["B"])
        torch.cuda.synchronize()
        ref = run_oracle(oracle, case, threads=4)
        e_dx = np.max(np.abs(to_host(dx) - ref["dx"]) / np.maximum(np.abs(ref["dx"]), ref["Sdx"]))
        e_dA = np.max(np.abs(to_host(dA) - ref["dA"]) / np.maximum(np.abs(ref["dA"]), ref["RA"]))
        e_dB = np.max(np.abs(to_host(dB) - ref["dB"]) / np.maximum(np.abs(ref["dB"]), ref["RB"]))
        # sequential float32 atomics lose more than the tree of grkan_bwd: looser bound on the sums
        assert e_dx <= 1e-5 and e_dA <= 1e-3 and e_dB <= 1e-3, (rows, D, G, e_dx, e_dA, e_dB)


def test_rounding_error_of_coefficient_gradients_vs_alg1(oracle):
    import torch

    import paper_2505_13813_amd as grkan

    full = os.environ.get("GRKAN_ROUNDING_FULL", "0") == "1"
    batch, passes = (1024, 10) if full else (128, 12)
    rows, D, G = batch * 197, 768, 8
    rng = np.random.Generator(np.random.PCG64(20250513))
    A = rng.standard_normal((G, 6)).astype(np.float32)
    B = rng.standard_normal((G, 4)).astype(np.float32)
    x = rng.standard_normal((rows, D), dtype=np.float32)
    dy = rng.standard_normal((rows, D), dtype=np.float32)

    threads = max(1, min(16, oracle.max_threads()))
    _, dA64, dB64 = oracle.bwd(x.astype(np.float64), dy.astype(np.float64), A.astype(np.float64),
                               B.astype(np.float64), threads=threads)

    case = dict(dtype="f32", A=A, B=B, x=x, dy=dy)
    dev = to_device(case)
    out = (torch.empty_like(dev["x"]), torch.empty_like(dev["A"]), torch.empty_like(dev["B"]))

    def mae(dA, dB):
        return float(np.mean(np.abs(to_host(dA) - dA64))), float(np.mean(np.abs(to_host(dB) - dB64)))

    ours = []
    bits = []
    for _ in range(3):
        grkan.grkan_bwd(dev["x"], dev["dy"], dev["A"], dev["B"], out=out)
        torch.cuda.synchronize()
        ours.append(mae(out[1], out[2]))
        bits.append((out[1].cpu().numpy().view(np.uint32).copy(), out[2].cpu().numpy().view(np.uint32).copy()))
    assert all(np.array_equal(b[0], bits[0][0]) and np.array_equal(b[1], bits[0][1]) for b in bits)

    alg1 = []
    for _ in range(passes):
        grkan.grkan_alg1_bwd(dev["x"], dev["dy"], dev["A"], dev["B"], out=out)
        torch.cuda.synchronize()
        alg1.append(mae(out[1], out[2]))
    alg1 = np.array(alg1)
    ours = np.array(ours)

    def ci(v):  # 95 % confidence interval of the mean
        return 1.96 * v.std(ddof=1) / np.sqrt(len(v)) if len(v) > 1 else 0.0

    scale_A, scale_B = float(np.mean(np.abs(dA64))), float(np.mean(np.abs(dB64)))
    print("\nrounding experiment, X,dO,A,B ~ N(0,1), [%d,197,%d], G=%d; mean |dA| = %.3e, mean |dB| = %.3e" %
          (batch, D, G, scale_A, scale_B))
    print("  Algorithm 1, float32 atomics (%d passes): dA MAE %.3e (+-%.2e) var %.2e | dB MAE %.3e (+-%.2e) var %.2e" %
          (passes, alg1[:, 0].mean(), ci(alg1[:, 0]), alg1[:, 0].var(ddof=1), alg1[:, 1].mean(), ci(alg1[:, 1]),
           alg1[:, 1].var(ddof=1)))
    print("  grkan_bwd, float32 two-stage reduction (3 passes, bit-identical): dA MAE %.3e | dB MAE %.3e" %
          (ours[0, 0], ours[0, 1]))
    # the deterministic reduction is the more accurate one, by a wide margin (the paper reports ~100x;
    # measured here: ~100x on dA, 70-120x on dB)
    assert ours[0, 0] * 10 < alg1[:, 0].mean() and ours[0, 1] * 10 < alg1[:, 1].mean()

    # The appendix closes with the remark that the smaller rounding error should matter most for
    # low-precision training.  The same experiment with 16-bit activations and upstream gradients
    # (rounded inputs on both sides, fp64 oracle on those): the sums never leave float32 registers, so
    # the coefficient gradients keep float32-level accuracy whatever the storage format.
    for dtype, to_bits, widen in (("bf16", grkan_inputs.round_to_bf16_bits, grkan_inputs.bf16_bits_to_f32),
                                  ("f16", grkan_inputs.round_to_f16_bits, grkan_inputs.f16_bits_to_f32)):
        xb, dyb = to_bits(x), to_bits(dy)
        low = dict(dtype=dtype, A=A, B=B, x=widen(xb), dy=widen(dyb), x_bits=xb, dy_bits=dyb)
        _, dA_low, dB_low = oracle.bwd(low["x"].astype(np.float64), low["dy"].astype(np.float64),
                                       A.astype(np.float64), B.astype(np.float64), threads=threads)
        dlow = to_device(low)
        _, dA_g, dB_g = grkan.grkan_bwd(dlow["x"], dlow["dy"], dlow["A"], dlow["B"])
        torch.cuda.synchronize()
        mA = float(np.mean(np.abs(to_host(dA_g) - dA_low)))
        mB = float(np.mean(np.abs(to_host(dB_g) - dB_low)))
        print("  grkan_bwd, %s I/O, float32 sums: dA MAE %.3e (%.1e of mean |dA|) | dB MAE %.3e (%.1e of mean |dB|)" %
              (dtype, mA, mA / np.mean(np.abs(dA_low)), mB, mB / np.mean(np.abs(dB_low))))
        assert mA <= 1e-4 * np.mean(np.abs(dA_low)) and mB <= 1e-4 * np.mean(np.abs(dB_low))
