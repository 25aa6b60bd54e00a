"""Writes oracle_tiny_regression.txt: CPU-oracle outputs for a few rows of the `tiny` workload.
Imports the oracle and the seeded input generator only.  Run from the repository root:
    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2601_20655_amd import workloads as wl  # noqa: E402

ROWS = [0, 1, 63, 64, 100, 255]
CHANNELS = [0, 1, 21, 22, 42, 63]


def values():
    cfg = wl.CONFIGS["tiny"]
    q, k, v = wl.self_attn_inputs(cfg)
    out, lse = oracle.self_attn(q, k, v, cfg["grid"], cfg["split"], rows=np.array(ROWS), want_lse=True)
    lines = []
    for i, r in enumerate(ROWS):
        for h in range(cfg["H"]):
            lines.append("row %d head %d lse %.17e out %s" % (
                r, h, lse[0, h, i], " ".join("%.17e" % out[0, i, h, c] for c in CHANNELS)))
    return lines


if __name__ == "__main__":
    with open(os.path.join(HERE, "oracle_tiny_regression.txt"), "w") as f:
        f.write("# tiny workload (grid 4x8x8, 4 heads, d64, fp32 inputs, RoPE 22/20/22, base 10000): oracle lse and\n")
        f.write("# output channels %s of rows %s, written by make_golden.py\n" % (CHANNELS, ROWS))
        f.write("\n".join(values()) + "\n")
