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
    RA = sqrt(sum (dy x^i/Q)^2),  RB = sqrt(sum (dy x^j s Pm/Q^2)^2).
Where nothing cancels inside the polynomials these are |y|, about |dx| and the
root-sum-square of the summed terms, so the measure is the plain relative
error there; where P cancels, no float32 evaluation can be accurate relative
to the result itself and the measure stays bounded.
"""
from __future__ import annotations

import numpy as np

# fp32: tolerances of the target statement; bf16 I/O likewise
TOL = {
    "f32": dict(y=1e-5, dx=1e-5, dA=1e-4, dB=1e-4),
    "bf16": dict(y=1e-2, dx=1e-2, dA=1e-3, dB=1e-3),
}


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


def errors(gpu, ref, rows=None):
    sl = slice(None) if rows is None else rows
    tiny = np.finfo(np.float64).tiny

    def rel(g, r, s):
        if r.size == 0:
            return 0.0
        return float(np.max(np.abs(g - r) / np.maximum(np.maximum(np.abs(r), s), tiny)))

    out = dict(y=rel(gpu["y"][sl], ref["y"], ref["Sy"]), dx=rel(gpu["dx"][sl], ref["dx"], ref["Sdx"]))
    if "dA" in ref:
        out["dA"] = rel(gpu["dA"], ref["dA"], ref["RA"])
        out["dB"] = rel(gpu["dB"], ref["dB"], ref["RB"])
    return out


def assert_parity(gpu, ref, dtype, rows=None, what=("y", "dx", "dA", "dB"), label=""):
    err = errors(gpu, ref, rows)
    for k in what:
        assert np.all(np.isfinite(gpu[k])), "%s: %s has non-finite values" % (label, k)
        assert err[k] <= TOL[dtype][k], "%s: %s error %.3e > %.1e" % (label, k, err[k], TOL[dtype][k])
    return err
