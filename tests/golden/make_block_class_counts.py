#!/usr/bin/env python3
"""Regenerates tests/golden/block_class_counts.txt.

For each of the five benchmark geometries the token-level candidate predicate of the paper's Eq. 7 is enumerated
literally, one band of Bs query rows at a time (a band is a [Bs, N] boolean matrix, so the 118 800-token geometry
fits in memory), and the density rule ("Density control within blocks") and the never-pruned t <= 1 zone are applied
to each block of the band exactly as they are worded.  The per-frame-distance quantities (window w(t), retained(t),
Eqs. 1-6) come from oracle.frame_table; nothing else of the oracle is used, in particular not its interval-counting
block classification, which this file is the second opinion on.  Nothing here touches the GPU library.

Usage (repository root):  python tests/golden/make_block_class_counts.py      (about five minutes on 8 cores)
"""
from __future__ import annotations

import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import dynamicrad_oracle as o          # noqa: E402
from workloads import CONFIGS                      # noqa: E402

GAMMA, THETA_C, THETA_M = 1.0, 0.15, 0.60
HEADER = """# Counts of forced / candidate blocks and selectable-per-row min, max for the five
# benchmark geometries with gamma = 1, theta_c = 0.15, theta_m = 0.60.
# Written by tests/golden/make_block_class_counts.py: a literal token-level enumeration of
# the paper's Eq. 7 + the density rule, band by band, that uses the oracle's per-t table
# (Eqs. 1-6) and none of its block classification.  A second opinion on that
# classification, not numbers from the paper.
# name forced candidates sel_min sel_max
"""


def counts(name: str):
    wl = CONFIGS[name]
    N, Nt, Bs = wl.N, wl.Nt, wl.Bs
    tab = o.frame_table(wl.Nf, Nt, Bs, GAMMA, wl.lam)
    retained, w = tab["retained"], tab["w"]
    Sb = -(-N // Bs)
    q = np.arange(N)
    fq, vq = q // Nt, q % Nt                         # frame and in-frame index of every key token
    starts = np.arange(Sb) * Bs
    n_cols = np.minimum(N, starts + Bs) - starts
    forced = cand = 0
    sel_min, sel_max = None, None
    for qb in range(Sb):
        r0, r1 = qb * Bs, min(N, (qb + 1) * Bs)
        fp, up = fq[r0:r1, None], vq[r0:r1, None]
        t = np.abs(fp - fq[None, :])                                     # [rows, N] frame distance
        band = retained[t] & (np.abs(up - vq[None, :]) <= w[t])          # Eq. 7, every token pair of the band
        col_ratio = band.sum(axis=0) / float(r1 - r0)                    # retained-token ratio of each key column
        active = col_ratio > THETA_C
        n_active = np.add.reduceat(active.astype(np.int64), starts)
        aggregated = (n_active / n_cols.astype(np.float64)) > THETA_M    # active-column fraction of each key block
        t_min = np.minimum.reduceat(t.min(axis=0), starts)               # smallest frame distance inside the block pair
        is_forced = t_min <= 1
        selectable = aggregated & ~is_forced
        forced += int(is_forced.sum())
        cand += int((is_forced | aggregated).sum())
        n_sel = int(selectable.sum())
        sel_min = n_sel if sel_min is None else min(sel_min, n_sel)
        sel_max = n_sel if sel_max is None else max(sel_max, n_sel)
    return forced, cand, sel_min, sel_max


def main():
    lines = []
    for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
        f, c, lo, hi = counts(name)
        lines.append(f"{name} {f} {c} {lo} {hi}")
        print(lines[-1], flush=True)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "block_class_counts.txt")
    with open(path, "w") as fh:
        fh.write(HEADER + "\n".join(lines) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
