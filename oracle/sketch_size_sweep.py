"""TEST INFRASTRUCTURE ONLY -- accuracy of the AMS estimate M2 as a function of the sketch size.

The paper fixes one size (l x m = 5 x 250, "epsilon about 6 % with probability about 95 %",
Section 3.3) and skips the sweep.  This script measures, with the CPU oracle only, how the
relative error of M2(sk(v)) against ||v||^2 depends on (l, m): for every size it sketches
`trials` random vectors under fresh hash coefficients and prints the 50 % / 95 % / 99 % quantiles
of |M2 / ||v||^2 - 1| and how often the over-estimate  H = n - M2/(1+eps) >= n - ||v||^2  of
Theorem 1 fails for eps = 0.06 * sqrt(250 / m)  (the m = O(1/eps^2) scaling of the paper's point).

    python -m oracle.sketch_size_sweep [--d 20000] [--trials 400] [--tail gauss|t3] [--json FILE]

tests/golden/sketch_size_sweep.json is this script's output for --trials 300 --json (it calls nothing
but the oracle).
"""
from __future__ import annotations

import argparse
import json

import numpy as np

from . import fda_oracle as O

P = (1 << 31) - 1
SIZES = [(1, 250), (3, 250), (5, 125), (5, 250), (5, 500), (5, 1000), (7, 250), (7, 1000), (9, 250),
         (5, 2000)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--d", type=int, default=20000)
    ap.add_argument("--trials", type=int, default=400)
    ap.add_argument("--tail", choices=("gauss", "t3"), default="gauss")
    ap.add_argument("--json", default=None, help="also write the table to this file")
    args = ap.parse_args()
    rows = sweep(args.d, args.trials, args.tail, SIZES, verbose=True)
    if args.json:
        with open(args.json, "w") as f:
            json.dump({"_citation": "Section 3.3, 'Choice of l and m' (the paper gives the one point l x m = 5 x 250, "
                                    "eps about 6 %, confidence about 95 %, and skips the sweep); Section 3.1, "
                                    "m = O(1/eps^2).  Written by `python -m oracle.sketch_size_sweep --trials "
                                    f"{args.trials} --json` (oracle only).",
                       "d": args.d, "trials": args.trials, "drift": args.tail, "seed": SEED, "rows": rows}, f, indent=1)
            f.write("\n")


SEED = 2405_20988


def sweep(d, trials, tail, sizes, verbose=False):
    """One row per (l, m): quantiles of |M2 / ||v||^2 - 1| over `trials` vectors and hash draws."""
    rng = np.random.default_rng(SEED)
    if verbose:
        print(f"d={d} trials={trials} drift={tail}")
        print(" l     m    eps(m)   q50      q95      q99     P[Thm 1 bound fails]")
    rows = []
    for l, m in sizes:
        eps = 0.06 * np.sqrt(250.0 / m)
        rel = np.empty(trials)
        for t in range(trials):
            coef = rng.integers(0, P, size=(l, 2, 4), dtype=np.int64).astype(np.uint32)
            v = rng.normal(size=d) if tail == "gauss" else rng.standard_t(3, size=d)
            rel[t] = O.m2_estimate(O.ams_sketch(v, coef, m)) / float(v @ v) - 1.0
        q = np.quantile(np.abs(rel), [0.5, 0.95, 0.99])
        fails = float(np.mean(1.0 + rel > 1.0 + eps))          # M2/(1+eps) > ||v||^2
        rows.append({"l": l, "m": m, "eps": round(float(eps), 6), "q50": round(float(q[0]), 5),
                     "q95": round(float(q[1]), 5), "q99": round(float(q[2]), 5), "bound_fails": round(fails, 4)})
        if verbose:
            print(f"{l:2d} {m:5d}   {eps:.4f}   {q[0]:.4f}   {q[1]:.4f}   {q[2]:.4f}   {fails:.3f}")
    return rows


if __name__ == "__main__":
    main()
