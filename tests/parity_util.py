"""Helpers of the GPU parity tests: run a case through the C ABI (via the thin
binding) and measure its error against the fp64 oracle.

Error metric (both sides see the same inputs; bf16 outputs are widened):
    y  : max_e |gpu - ref| / max(|ref|, Sy)
    dx : max_e |gpu - ref| / max(|ref|, Sdx)
    dA : max   |gpu - ref| / max(|ref|, RA),   dB likewise with RB
Sy, Sdx, RA, RB come from the oracle (grkan_oracle_scales): the paper's
expressions with every monomial of P, P', Aden' replaced by its magnitude and
Q taken as exact,
    Sy = Pm/Q,  Sdx = |dy| (dPm/Q + dAm Pm/Q^2),
    RA = sqrt(sum (dy x^i/Q)^2),  RB = sqrt(sum (dy x^j s P/Q^2)^2)
(the root-sum-squares of the very terms the coefficient gradients add up).
Where nothing cancels inside the polynomials Sy, Sdx are |y| and about |dx|, so
the measure is the plain relative error there; where P cancels, no float32
evaluation can be accurate relative to the result itself and the measure stays
bounded.  Beside the gated figure the tests print, but do not gate, the plain
relative error (median, 99th percentile, maximum) and max|gpu - ref| / max|ref|.
"""
from __future__ import annotations

import numpy as np

# fp32: tolerances of the target statement; bf16 I/O likewise.  float16 I/O
# (an addition of this library): y and dx are float32 results rounded once to 11
# significant bits, half an ulp = 2^-11 = 4.9e-4 relative, so 1e-3; the sums see
# the same float32 arithmetic as for bfloat16 I/O.
TOL = {
    "f32": dict(y=1e-5, dx=1e-5, dA=1e-4, dB=1e-4),
    "bf16": dict(y=1e-2, dx=1e-2, dA=1e-3, dB=1e-3),
    "f16": dict(y=1e-3, dx=1e-3, dA=1e-3, dB=1e-3),
}
# Below 2^-14 binary16 is subnormal, with a fixed spacing of 2^-24: rounding a
# tiny y or dx to storage costs up to half of that in absolute terms, whatever
# the size of the value.  (float32 and bfloat16 subnormals start at 1e-38.)
ABS_FLOOR = {"f32": 0.0, "bf16": 0.0, "f16": 2.0 ** -25}


def to_device(case, device="cuda:0"):
    import grkan_inputs

    return grkan_inputs.upload(case, device)


def to_host(t) -> np.ndarray:
    import torch

    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def run_gpu(case, device="cuda:0"):
    import torch

    import paper_2505_13813_amd as grkan

    dev = to_device(case, device)
    y = grkan.grkan_fwd(dev["x"], dev["A"], dev["B"])
    dx, dA, dB = grkan.grkan_bwd(dev["x"], dev["dy"], dev["A"], dev["B"])
    torch.cuda.synchronize()
    return dict(y=to_host(y), dx=to_host(dx), dA=to_host(dA), dB=to_host(dB))


def run_oracle(oracle, case, threads=1, rows=None):
    sl = slice(None) if rows is None else rows
    x = case["x"][sl].astype(np.float64)
    dy = case["dy"][sl].astype(np.float64)
    A = case["A"].astype(np.float64)
    B = case["B"].astype(np.float64)
    y = oracle.fwd(x, A, B, threads=threads)
    dx, dA, dB = oracle.bwd(x, dy, A, B, threads=threads)
    Sy, Sdx, RA, RB = oracle.scales(x, dy, A, B, threads=threads)
    return dict(y=y, dx=dx, dA=dA, dB=dB, Sy=Sy, Sdx=Sdx, RA=RA, RB=RB)


def errors(gpu, ref, rows=None, dtype="f32"):
    sl = slice(None) if rows is None else rows
    tiny = np.finfo(np.float64).tiny
    floor = ABS_FLOOR[dtype]

    def rel(g, r, s, floor=0.0):
        if r.size == 0:
            return 0.0
        excess = np.maximum(np.abs(g - r) - floor, 0.0)
        return float(np.max(excess / np.maximum(np.maximum(np.abs(r), s), tiny)))

    out = dict(y=rel(gpu["y"][sl], ref["y"], ref["Sy"], floor), dx=rel(gpu["dx"][sl], ref["dx"], ref["Sdx"], floor))
    if "dA" in ref:
        out["dA"] = rel(gpu["dA"], ref["dA"], ref["RA"])
        out["dB"] = rel(gpu["dB"], ref["dB"], ref["RB"])
    return out


def plain_stats(g, r):
    """Reported, not gated: plain relative error |g - r| / |r| (median, 99th
    percentile, maximum over the elements with r != 0) and max|g - r| / max|r|."""
    g = np.asarray(g, dtype=np.float64).ravel()
    r = np.asarray(r, dtype=np.float64).ravel()
    if r.size == 0:
        return dict(p50=0.0, p99=0.0, max=0.0, linf=0.0)
    diff = np.abs(g - r)
    absr = np.abs(r)
    nz = absr > 0
    rel = (diff[nz] / absr[nz]).astype(np.float32)
    if rel.size == 0:
        p50 = p99 = mx = 0.0
    else:
        k50, k99 = rel.size // 2, min(rel.size - 1, int(rel.size * 0.99))
        part = np.partition(rel, (k50, k99))
        p50, p99, mx = float(part[k50]), float(part[k99]), float(rel.max())
    top = float(absr.max())
    return dict(p50=p50, p99=p99, max=mx, linf=float(diff.max()) / top if top > 0 else 0.0)


def format_stats(name, gated, st):
    return "%s gated %.2e | plain rel p50 %.1e p99 %.1e max %.1e | Linf/Linf %.1e" % (
        name, gated, st["p50"], st["p99"], st["max"], st["linf"])


def assert_parity(gpu, ref, dtype, rows=None, what=("y", "dx", "dA", "dB"), label=""):
    err = errors(gpu, ref, rows, dtype)
    for k in what:
        assert np.all(np.isfinite(gpu[k])), "%s: %s has non-finite values" % (label, k)
        assert err[k] <= TOL[dtype][k], "%s: %s error %.3e > %.1e" % (label, k, err[k], TOL[dtype][k])
    return err
