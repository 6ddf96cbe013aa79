#!/usr/bin/env python3
"""Writes tests/golden/oracle_tiny_digest.txt: a few sums of the fp64 oracle's
outputs on the seeded "tiny" configuration, for each built degree pair.

This is a change detector for the oracle, not a pin of it (the pins are the
closed forms, invariants and the hand-worked example): once the pins hold, any
later edit that moves the oracle's results shows up here and has to be
justified.  The script calls nothing but oracle/ and the seeded input module.

    python tests/golden/write_oracle_digest.py
"""
import sys
from pathlib import Path

import numpy as np

ROOT = Path(__file__).resolve().parents[2]
sys.path.insert(0, str(ROOT))

import grkan_inputs  # noqa: E402
from oracle import grkan_oracle  # noqa: E402

OUT = Path(__file__).resolve().parent / "oracle_tiny_digest.txt"


def digest(m, n):
    c = grkan_inputs.make_case("tiny", m=m, n=n)
    x, dy, A, B = (c[k].astype(np.float64) for k in ("x", "dy", "A", "B"))
    y = grkan_oracle.fwd(x, A, B)
    dx, dA, dB = grkan_oracle.bwd(x, dy, A, B)
    w = np.cos(np.arange(y.size, dtype=np.float64)).reshape(y.shape)  # position-dependent weights
    return {
        "sum_y": float(np.sum(y)), "wsum_y": float(np.sum(w * y)),
        "sum_dx": float(np.sum(dx)), "wsum_dx": float(np.sum(w * dx)),
        "dA": dA.ravel().tolist(), "dB": dB.ravel().tolist(),
    }


def main():
    lines = ["# written by tests/golden/write_oracle_digest.py from oracle/ alone; see that file"]
    for m, n in ((5, 4), (3, 2), (7, 6)):
        d = digest(m, n)
        for k in ("sum_y", "wsum_y", "sum_dx", "wsum_dx"):
            lines.append("%d %d %s %.17g" % (m, n, k, d[k]))
        lines.append("%d %d dA %s" % (m, n, " ".join("%.17g" % v for v in d["dA"])))
        lines.append("%d %d dB %s" % (m, n, " ".join("%.17g" % v for v in d["dB"])))
    OUT.write_text("\n".join(lines) + "\n")
    print("wrote", OUT)


if __name__ == "__main__":
    main()
