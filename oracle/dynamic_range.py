#!/usr/bin/env python3
"""Synthetic version of the paper's dynamic-range analysis of the Winograd-domain output Y
(Figure "Dynamic ranges across different taps or pixels of the Winograd domain output", panels
(a) and (c)): the standard deviation of Y at each of the n x n locations of the output tile,
relative to the mean over the locations, with the standard scales and with the learned F(6,3)
scales the paper tabulates; and the signal-to-quantization-noise ratio of the fully-integer
pipeline (oracle/fullint.py) with either set.  Random Gaussian inputs, Kaiming-normal weights
(the paper analyses a trained diffusion model; none is available here).

    python -m oracle.dynamic_range            # prints the tables
"""
from __future__ import annotations

import os

import numpy as np

import oracle
from oracle import cook_toom as ct
from oracle import fullint

GOLDEN = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "tests", "golden",
                      "learned_scales_f63.txt")


def learned_f63():
    rows = [[float(t) for t in l.split()] for l in open(GOLDEN) if not l.startswith("#")]
    return ct.matrices_from_scales(6, [r[1] for r in rows], [r[2] for r in rows])


def run(seed: int = 0, Cin: int = 64, Cout: int = 64, size: int = 24, g: int = 32):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((2, size, size, Cin)).astype(np.float32)
    w = (rng.standard_normal((Cout, Cin, 3, 3)) * np.sqrt(2.0 / (9 * Cin))).astype(np.float32)
    ref = oracle.direct_conv(x, w, None)
    out = {}
    for name, m, mats in (("F(4,3) standard", 4, ct.standard_matrices(4)),
                          ("F(6,3) standard", 6, ct.standard_matrices(6)),
                          ("F(6,3) learned scales", 6, learned_f63())):
        r = fullint.fullint_pipeline(x, w, None, *mats, m, g)
        rel = fullint.tap_relative_std(r["Yt"], m)
        out[name] = dict(rel_std=rel, spread=float(rel.max() / rel.min()),
                         sqnr_db=fullint.sqnr_db(ref, r["y"]))
    return out


def main():
    np.set_printoptions(precision=2, suppress=True, linewidth=120)
    for name, r in run().items():
        print(f"{name}: relative std of Y per tile location (max/min = {r['spread']:.0f}), "
              f"fully-integer pipeline SQNR {r['sqnr_db']:.1f} dB")
        print(r["rel_std"])
        print()


if __name__ == "__main__":
    main()
