"""TEST INFRASTRUCTURE ONLY -- bucket and sign of every coordinate of one sketch row, written to files.

A child process of the full-size parity tests (tests/fullsize_oracle.py): hashing 3.5e8 coordinates
for seven rows takes the CPU oracle minutes on one core, so each row gets a process of its own.
Calls nothing but oracle.fda_oracle.bucket_and_sign, over blocks of coordinates.

    python tests/oracle_hash_rows.py --row 3 --d 350000000 --m 1000 --coef '[[c0,c1,c2,c3],[c0,c1,c2,c3]]' --out DIR
"""
import argparse
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from oracle import fda_oracle as O  # noqa: E402

BLOCK = 1 << 20


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--row", type=int, required=True)
    ap.add_argument("--d", type=int, required=True)
    ap.add_argument("--m", type=int, required=True)
    ap.add_argument("--coef", required=True)
    ap.add_argument("--out", required=True)
    a = ap.parse_args()
    coef = np.array(json.loads(a.coef), np.uint32)
    bucket = np.lib.format.open_memmap(os.path.join(a.out, f"bucket_{a.row}.npy"), mode="w+",
                                       dtype=np.uint16, shape=(a.d,))
    negative = np.lib.format.open_memmap(os.path.join(a.out, f"negative_{a.row}.npy"), mode="w+",
                                         dtype=np.bool_, shape=(a.d,))
    for lo in range(0, a.d, BLOCK):
        hi = min(lo + BLOCK, a.d)
        b, s = O.bucket_and_sign(coef, np.arange(lo, hi, dtype=np.uint64), a.m)
        bucket[lo:hi] = b
        negative[lo:hi] = s < 0
    bucket.flush()
    negative.flush()


if __name__ == "__main__":
    main()
