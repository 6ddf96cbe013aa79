"""Second, independent fp64 reference of the group-wise rational function in
vectorised numpy.

TEST INFRASTRUCTURE ONLY.  It exists to catch indexing slips in the C oracle:
it reshapes the channel axis to [G, d_g] and broadcasts one coefficient row per
group instead of looping over elements.  It shares no code with the GPU path
and no arithmetic helpers with the C oracle.

Formulas: FlashKAT paper, Eq. "pade" (F = P / (1 + |Aden|)) and
Eq. "grad_a", "grad_b", "grad_x", "accum", "accum2".  sign(0) is taken as 0.
"""
from __future__ import annotations

import numpy as np


def _grouped(x, G):
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    if D % G:
        raise ValueError("D must be a multiple of G")
    return x.reshape(-1, G, D // G)


def _parts(xg, A, B):
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    m, n = A.shape[1] - 1, B.shape[1]
    a = A[None, :, :, None]          # [1, G, m+1, 1]
    b = B[None, :, :, None]          # [1, G, n,   1]
    xe = xg[:, :, None, :]           # [rows, G, 1, d_g]
    pw_a = xe ** np.arange(m + 1)[None, None, :, None]
    P = (a * pw_a).sum(axis=2)
    i = np.arange(1, m + 1)[None, None, :, None]
    dP = (i * a[:, :, 1:, :] * xe ** (i - 1)).sum(axis=2)
    j = np.arange(1, n + 1)[None, None, :, None]
    pw_b = xe ** j
    Aden = (b * pw_b).sum(axis=2)
    dAden = (j * b * xe ** (j - 1)).sum(axis=2)
    Q = 1.0 + np.abs(Aden)
    s = np.sign(Aden)
    return P, dP, Aden, dAden, Q, s, pw_a, pw_b


def fwd(x, A, B):
    G = np.asarray(A).shape[0]
    xg = _grouped(x, G)
    P, _, _, _, Q, _, _, _ = _parts(xg, A, B)
    return (P / Q).reshape(np.shape(x))


def bwd(x, dy, A, B):
    G = np.asarray(A).shape[0]
    xg = _grouped(x, G)
    dg = _grouped(dy, G)
    P, dP, _, dAden, Q, s, pw_a, pw_b = _parts(xg, A, B)
    dx = dg * (dP / Q - s * dAden * P / Q ** 2)
    # [rows, G, k, d_g] -> sum over rows and the group's channels
    dA = (dg[:, :, None, :] * pw_a / Q[:, :, None, :]).sum(axis=(0, 3))
    dB = (-dg[:, :, None, :] * pw_b * (s * P / Q ** 2)[:, :, None, :]).sum(axis=(0, 3))
    return dx.reshape(np.shape(x)), dA, dB
