"""Helpers that let the CPU oracle cover the benchmark configurations at their full sizes.

Nothing here is arithmetic of its own: the hash of a sketch row comes from
oracle.fda_oracle.bucket_and_sign, evaluated once per row over blocks of coordinates and kept
(the hash depends on the row and the coordinate only), and a sketch row of a vector is then
numpy's bincount over those buckets with weights sign * v -- ams_sketch's own statement, without
re-hashing for every vector.  Vectors are handled one worker at a time, so the host never holds a
[K, d] array in fp64.
"""
import json
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import fda_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BLOCK = 1 << 20
THREADS = 16                      # the CPU share of a one-GPU machine


def hash_rows(coef, rows, d, m, threads=THREADS):
    """{row: (bucket uint16 [d], negative bool [d])} by O.bucket_and_sign over blocks of coordinates
    (numpy releases the interpreter lock inside its loops, so the blocks run on several threads)."""
    out = {i: (np.empty(d, np.uint16), np.empty(d, np.bool_)) for i in rows}

    def one(job):
        i, a = job
        b = min(a + BLOCK, d)
        bucket, sign = O.bucket_and_sign(coef[i], np.arange(a, b, dtype=np.uint64), m)
        out[i][0][a:b] = bucket
        out[i][1][a:b] = sign < 0
    jobs = [(i, a) for i in rows for a in range(0, d, BLOCK)]
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(one, jobs))
    return out


def start_hash_processes(coef, rows, d, m, folder):
    """The same for very long vectors: one child process per sketch row (tests/oracle_hash_rows.py)
    writes bucket and sign of every coordinate to .npy files in `folder`.  Returns the children;
    collect with finish_hash_processes."""
    os.makedirs(folder, exist_ok=True)
    env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1")
    kids = []
    for i in rows:
        cmd = [sys.executable, os.path.join(ROOT, "tests", "oracle_hash_rows.py"), "--row", str(i),
               "--d", str(d), "--m", str(m), "--coef", json.dumps(np.asarray(coef[i]).tolist()),
               "--out", folder]
        kids.append((i, subprocess.Popen(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    return kids


def finish_hash_processes(kids, folder, timeout=600):
    out = {}
    for i, proc in kids:
        text, _ = proc.communicate(timeout=timeout)
        assert proc.returncode == 0, text.decode(errors="replace")[-2000:]
        out[i] = (np.load(os.path.join(folder, f"bucket_{i}.npy"), mmap_mode="r"),
                  np.load(os.path.join(folder, f"negative_{i}.npy"), mmap_mode="r"))
    return out


def sketch_row(v, hashed_row, m):
    """Row of sk(v): cell b = sum over the coordinates of bucket b of sign * v (Section 3.1)."""
    bucket, negative = hashed_row
    return np.bincount(bucket, weights=np.where(negative, -v, v), minlength=m)


def sketch_row_blocks(v, hashed_row, m, threads=THREADS):
    """sketch_row over blocks of coordinates on several threads (the blocks add: linearity)."""
    bucket, negative = hashed_row
    d = v.shape[0]

    def one(a):
        b = min(a + 8 * BLOCK, d)
        return np.bincount(bucket[a:b], weights=np.where(negative[a:b], -v[a:b], v[a:b]), minlength=m)
    with ThreadPoolExecutor(threads) as ex:
        return sum(ex.map(one, range(0, d, 8 * BLOCK)))


def cell_counts(hashed_row, m):
    return np.bincount(hashed_row[0], minlength=m).astype(np.float64)


def row_to_numpy(t):
    """Host copy of one slab row in the form the oracle takes (float32, or uint16 bf16 bit patterns)."""
    import torch
    r = t.detach().cpu()
    if r.dtype == torch.bfloat16:
        return r.view(torch.int16).numpy().view(np.uint16)
    return r.numpy()
