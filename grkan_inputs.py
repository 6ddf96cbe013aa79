"""Seeded synthetic inputs for the GR-KAN rational layer at the paper's shapes.

This module only draws random numbers and rounds storage formats.  It holds
none of the method's arithmetic and is the one piece of code that the fp64
oracle's tests and the GPU path's tests/bench both use (as data only).

Shapes follow the KAT variants of the FlashKAT paper (Appendix, table of model
configurations: hidden 192/384/768, MLP width 4x, 197 tokens for a 224x224
image at patch size 16) and its kernel micro-benchmark (Sec. "Insight 2":
8 groups, numerator degree 5, denominator degree 4).  The activations of a
trained KAT on ImageNet-1k are not available; x ~ N(0,1) is the distribution
the paper's initialisation analysis assumes for the inputs of F.

Recipe (fixed, so every consumer sees the same arrays):
  * generator: numpy PCG64; one SeedSequence(1000 + config index) per config,
    spawned into independent child streams in the fixed order
    [A, B, then (x, dy, aux) per tensor in the order the tensors are listed];
    aux feeds the chi-square draw of the Student-t case
  * A[g, i] = U(-1, 1) / (i + 1), i = 0..5;  B[g, j] = U(-0.5, 0.5), j = 0..3
  * x ~ N(0, 1) (or Student-t with 3 degrees of freedom, z / sqrt(chi2_3 / 3),
    for the stress config), dy ~ N(0, sigma^2); x and dy are drawn and stored
    as float32, A and B are drawn as float64 and stored as float32
  * bf16 / f16 variants: the float32 arrays rounded to nearest-even bfloat16 /
    IEEE binary16; both the uint16 bit patterns and their exact float32
    widening are returned
  * other degrees (m, n): the same two child streams with the shapes
    [G, m + 1] / [G, n] and the same scaling 1 / (i + 1)
  * a sweep over G redraws A and B from the same two child streams with the
    new shape [G, m + 1] / [G, n]; x and dy do not depend on G.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

M_DEGREE = 5  # numerator degree  -> 6 coefficients a_0..a_5
N_DEGREE = 4  # denominator degree -> 4 coefficients b_1..b_4
TOKENS = 197


@dataclass(frozen=True)
class Config:
    name: str
    index: int
    batch: int
    tensors: Tuple[Tuple[str, int], ...]  # (tensor name, D)
    G: int
    x_dist: str       # "normal" | "student_t3"
    dy_sigma: float

    @property
    def rows(self) -> int:
        return self.batch * TOKENS

    def D(self, tensor: str) -> int:
        return dict(self.tensors)[tensor]


CONFIGS: Dict[str, Config] = {
    c.name: c
    for c in (
        Config("tiny", 0, 4, (("x", 192),), 8, "normal", 1.0),
        Config("kat_t", 1, 128, (("x1", 192), ("x2", 768)), 8, "normal", 0.01),
        Config("kat_s", 2, 128, (("x1", 384), ("x2", 1536)), 8, "normal", 0.01),
        Config("kat_b", 3, 128, (("x1", 768), ("x2", 3072)), 8, "normal", 0.01),
        Config("stress", 4, 256, (("x", 3072),), 8, "student_t3", 1.0),
    )
}


def round_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even.
    Inputs are finite, so no NaN handling is needed."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _streams(cfg: Config, extra: int = 0):
    ss = np.random.SeedSequence(1000 + cfg.index)
    kids = ss.spawn(2 + 3 * len(cfg.tensors) + extra)
    return [np.random.Generator(np.random.PCG64(k)) for k in kids]


def coefficients(cfg: Config, G: Optional[int] = None, m: int = M_DEGREE,
                 n: int = N_DEGREE) -> Tuple[np.ndarray, np.ndarray]:
    """(A[G, m + 1], B[G, n]) as float32."""
    G = cfg.G if G is None else int(G)
    gens = _streams(cfg)
    A = gens[0].uniform(-1.0, 1.0, size=(G, m + 1)) / (np.arange(m + 1) + 1.0)
    B = gens[1].uniform(-0.5, 0.5, size=(G, n))
    return A.astype(np.float32), B.astype(np.float32)


def round_to_f16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> IEEE binary16 bit patterns (uint16), round to nearest, ties to even."""
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of binary16 bit patterns to float32."""
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def _draw_x(gen: np.random.Generator, aux: np.random.Generator, dist: str, shape) -> np.ndarray:
    if dist == "normal":
        return gen.standard_normal(size=shape, dtype=np.float32)
    if dist == "student_t3":
        z = gen.standard_normal(size=shape, dtype=np.float32)
        chi2 = aux.chisquare(3.0, size=shape).astype(np.float32)
        return (z / np.sqrt(chi2 / np.float32(3.0))).astype(np.float32)
    raise ValueError("unknown distribution %r" % dist)


def make_case(config: str, tensor: Optional[str] = None, G: Optional[int] = None,
              dtype: str = "f32", rows: Optional[int] = None, m: int = M_DEGREE, n: int = N_DEGREE) -> dict:
    """Build one test/bench case.

    Returns a dict with A, B (float32), x, dy (float32, [rows, D]; for
    dtype="bf16" / "f16" these hold exactly representable values of that format
    and `x_bits`, `dy_bits` hold the uint16 patterns), and the scalars rows, D,
    G, m, n.
    `rows` cuts the case to its first rows (the stream is drawn row-major, so a
    shorter case is a prefix of the full one).
    """
    cfg = CONFIGS[config]
    names = [t for t, _ in cfg.tensors]
    tensor = names[0] if tensor is None else tensor
    if tensor not in names:
        raise ValueError("config %s has tensors %s" % (config, names))
    if dtype not in ("f32", "bf16", "f16"):
        raise ValueError("dtype must be 'f32', 'bf16' or 'f16'")
    ti = names.index(tensor)
    D = cfg.D(tensor)
    G = cfg.G if G is None else int(G)
    if D % G:
        raise ValueError("D=%d is not a multiple of G=%d" % (D, G))
    nrows = cfg.rows if rows is None else int(rows)
    if nrows < 0 or nrows > cfg.rows:
        raise ValueError("rows must be in [0, %d]" % cfg.rows)

    gens = _streams(cfg)
    A, B = coefficients(cfg, G, m, n)
    x = _draw_x(gens[2 + 3 * ti], gens[4 + 3 * ti], cfg.x_dist, (nrows, D))
    dy = gens[3 + 3 * ti].standard_normal(size=(nrows, D), dtype=np.float32)
    dy *= np.float32(cfg.dy_sigma)

    case = dict(config=config, tensor=tensor, dtype=dtype, rows=nrows, D=D, G=G,
                m=int(m), n=int(n), A=A, B=B)
    if dtype == "bf16":
        xb, dyb = round_to_bf16_bits(x), round_to_bf16_bits(dy)
        case.update(x_bits=xb, dy_bits=dyb, x=bf16_bits_to_f32(xb), dy=bf16_bits_to_f32(dyb))
    elif dtype == "f16":
        xb, dyb = round_to_f16_bits(x), round_to_f16_bits(dy)
        case.update(x_bits=xb, dy_bits=dyb, x=f16_bits_to_f32(xb), dy=f16_bits_to_f32(dyb))
    else:
        case.update(x=x, dy=dy)
    return case


def upload(case: dict, device: str = "cuda:0") -> dict:
    """Copy a case to the GPU as torch tensors (A, B float32; x, dy float32, or
    bfloat16 / float16 from the stored bit patterns).  Data movement only."""
    import torch

    dev = {}
    for k in ("A", "B"):
        dev[k] = torch.from_numpy(np.ascontiguousarray(case[k])).to(device)
    for k in ("x", "dy"):
        if case["dtype"] in ("bf16", "f16"):
            bits = np.ascontiguousarray(case[k + "_bits"]).view(np.int16)
            dev[k] = torch.from_numpy(bits).to(device).view(
                torch.bfloat16 if case["dtype"] == "bf16" else torch.float16)
        else:
            dev[k] = torch.from_numpy(np.ascontiguousarray(case[k])).to(device)
    return dev


def make_linear_case(config: str, tensor: Optional[str] = None, D_out: Optional[int] = None,
                     rows: Optional[int] = None, bias: bool = True) -> dict:
    """A GR-KAN layer out = W F(x) + bias at the paper's shapes, bfloat16 storage.

    `tensor` names the layer's input among the config's tensors: "x1" feeds the
    first linear layer of the MLP block (D_out = 4 D_in), "x2" the second
    (D_out = D_in / 4); single-tensor configs default to D_out = D_in.  x, A, B
    are those of make_case(dtype="bf16").  W ~ N(0, 1 / D_in) (the paper's
    variance-preserving scale for an identity-like F), drawn from two further
    child streams per tensor (after all of make_case's, so those are unchanged),
    stored as bfloat16; bias ~ N(0, 0.1^2) float32.  Data only."""
    case = make_case(config, tensor, dtype="bf16", rows=rows)
    cfg = CONFIGS[config]
    names = [t for t, _ in cfg.tensors]
    ti = names.index(case["tensor"])
    D_in = case["D"]
    if D_out is None:
        D_out = 4 * D_in if case["tensor"] == "x1" else (D_in // 4 if case["tensor"] == "x2" else D_in)
    gens = _streams(cfg, extra=2 * len(cfg.tensors))
    base = 2 + 3 * len(cfg.tensors)
    W = gens[base + 2 * ti].standard_normal(size=(D_out, D_in), dtype=np.float32) / np.float32(np.sqrt(D_in))
    Wb = round_to_bf16_bits(W)
    case.update(D_in=D_in, D_out=int(D_out), W_bits=Wb, W=bf16_bits_to_f32(Wb))
    case["bias"] = (gens[base + 2 * ti + 1].standard_normal(size=(D_out,), dtype=np.float32) * np.float32(0.1)
                    if bias else None)
    return case


def upload_linear(case: dict, device: str = "cuda:0") -> dict:
    """upload() plus W (bfloat16) and bias (float32 or None).  Data movement only."""
    import torch

    dev = upload(case, device)
    dev["W"] = torch.from_numpy(np.ascontiguousarray(case["W_bits"]).view(np.int16)).to(device).view(torch.bfloat16)
    dev["bias"] = torch.from_numpy(case["bias"]).to(device) if case.get("bias") is not None else None
    return dev
