"""TEST INFRASTRUCTURE ONLY -- plain CPU fp64 oracle for the FDA local-state /
variance-check / synchronization path.

Nothing in the product path may import this module: only the tests, the smoke
check and the benchmark's CPU-baseline leg use it.  It shares no code, header,
table or constant generator with the HIP library; the two only ever see the same
*input bits* (parameter slabs, hash coefficients), handed to each separately.

Every function follows a definition of the FDA paper (arxiv 2405.20988) and says
which one.  All floating-point arithmetic is IEEE fp64 over inputs widened
exactly from their storage type (fp32, or bf16 given as uint16 bit patterns).
No blocking, fusion or reordering beyond what the definitions state.

Readings taken where the paper is silent (all listed again in the design notes):
  * AMS hash family (Section 3.1 only cites Cormode & Garofalakis 2005): per
    sketch row two independent cubic polynomials over the prime p = 2^31 - 1,
    g(j) = c3 j^3 + c2 j^2 + c1 j + c0 (mod p), coefficients given as data
    coef[row][which][e] = c_e with which = 0 for the bucket polynomial and 1 for
    the sign polynomial;  bucket = floor(g_b(j) * m / 2^31),
    sign = +1 if g_s(j) is even else -1.
  * No 1/sqrt(m) scaling: M2 is the median of the plain squared row norms
    (Section 3.1, definition of M2).
  * Median over an even number of rows = mean of the two middle values.
  * Decision is the strict comparison H > Theta (Algorithm 1, line 8).
  * A non-finite estimate means the round invariant cannot be guaranteed, so it
    synchronizes (Section 3, paragraph after Eq. 2).
  * xi with a zero denominator is the zero vector.

Pinned by tests/test_oracle_*.py (closed forms, hand cases, identities, brute
force), the absolute-sum scales of the tolerances (abs_projections,
ams_sketch_abs, ams_sketch_counts, u_mean_abs) included: hand values and
pure-Python loops.  The numeric *contents* of a sketch are fixed only through the
hash reading above -- the paper prints no worked sketch -- so sketch cell values
are "parity unpinned" with respect to the paper itself; their structure
(linearity, signed-permutation case, tug-of-war case, column sums, unbiasedness)
is pinned.
"""
from __future__ import annotations

import numpy as np

MERSENNE_P = (1 << 31) - 1


# --------------------------------------------------------------------------- #
# storage types
# --------------------------------------------------------------------------- #
def widen(x, dtype: str) -> np.ndarray:
    """Exact widening of stored parameters to fp64.

    dtype "f32": x is float32.  dtype "bf16": x holds bfloat16 bit patterns as
    uint16 (a bf16 is the upper half of an fp32, so shifting left by 16 is exact).
    """
    if dtype == "f32":
        a = np.asarray(x)
        if a.dtype != np.float32:
            raise TypeError("f32 slab must be float32")
        return a.astype(np.float64)
    if dtype == "bf16":
        a = np.asarray(x)
        if a.dtype != np.uint16:
            raise TypeError("bf16 slab must be given as uint16 bit patterns")
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (ties to even) of fp64 values, as uint16 bit patterns.

    bfloat16 = 1 sign, 8 exponent, 7 fraction bits: 8 significant bits, fp32's
    exponent range.  Written from that format definition, directly from fp64 (no
    intermediate fp32 rounding).  Finite inputs only; overflow goes to infinity.
    """
    x = np.asarray(x, np.float64)
    mant, expo = np.frexp(x)                 # x = mant * 2^expo, 0.5 <= |mant| < 1
    expo = np.maximum(expo, -125)            # below 2^-126 the spacing stays 2^-133
    quantum = np.ldexp(1.0, expo - 8)        # spacing of bf16 numbers around x
    r = np.rint(x / quantum) * quantum       # rint = round half to even; exact in fp64
    r32 = r.astype(np.float32)               # representable (or inf): exact
    return (r32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------- #
# exact variance (ground truth)
# --------------------------------------------------------------------------- #
def mean_model(w64: np.ndarray) -> np.ndarray:
    """Average model  w_bar = (1/K) sum_k w_k   (Section 3, Notation)."""
    K = w64.shape[0]
    return w64.sum(axis=0) / K


def true_variance(w64: np.ndarray) -> float:
    """Model variance, Eq. 1:  (1/K) sum_k || w_k - w_bar ||^2, by brute force."""
    K = w64.shape[0]
    wbar = mean_model(w64)
    total = 0.0
    for k in range(K):
        diff = w64[k] - wbar
        total += float(np.dot(diff, diff))
    return total / K


# --------------------------------------------------------------------------- #
# local drift and the scalar state components
# --------------------------------------------------------------------------- #
def drift(w64: np.ndarray, w_t0_64: np.ndarray) -> np.ndarray:
    """Local drifts  u_k = w_k - w_t0   (Section 3, 'Efficiently Monitoring the RI')."""
    return w64 - w_t0_64[None, :]


def sq_norms(u: np.ndarray) -> np.ndarray:
    """||u_k||^2 for every worker: first component of both local states (Thm 1, Thm 2)."""
    return np.einsum("kj,kj->k", u, u)


def projections(u: np.ndarray, xi64: np.ndarray) -> np.ndarray:
    """<xi, u_k> for every worker: LinearFDA's second state component (Thm 2)."""
    return u @ xi64


def abs_projections(u: np.ndarray, xi64: np.ndarray) -> np.ndarray:
    """sum_j |xi_j u_kj|: the scale a rounding-error bound on <xi,u_k> is relative to."""
    return np.abs(u) @ np.abs(xi64)


# --------------------------------------------------------------------------- #
# AMS sketch (Section 3.1; hash family = the reading in the module header)
# --------------------------------------------------------------------------- #
def poly_hash(c, j: np.ndarray) -> np.ndarray:
    """g(j) = c[3] j^3 + c[2] j^2 + c[1] j + c[0]  (mod 2^31 - 1), for keys j < p.

    Evaluated by Horner's rule in uint64: every intermediate is below
    p*p + p < 2^63, so nothing wraps.
    """
    j = np.asarray(j).astype(np.uint64)
    p = np.uint64(MERSENNE_P)
    if j.size and int(j.max()) >= MERSENNE_P:
        raise ValueError("keys must be below the prime 2^31 - 1")
    c = [np.uint64(int(v)) for v in c]
    if any(int(v) >= MERSENNE_P for v in c):
        raise ValueError("coefficients must be below the prime 2^31 - 1")
    g = np.full(j.shape, c[3], dtype=np.uint64)
    g = (g * j + c[2]) % p
    g = (g * j + c[1]) % p
    g = (g * j + c[0]) % p
    return g


def bucket_and_sign(coef_row, j: np.ndarray, m: int):
    """Bucket in [0, m) and sign in {+1, -1} of keys j for one sketch row.

    coef_row[0] = bucket polynomial, coef_row[1] = sign polynomial.
    bucket = floor(g_b * m / 2^31) (integer arithmetic), sign = +1 iff g_s even.
    """
    gb = poly_hash(coef_row[0], j)
    gs = poly_hash(coef_row[1], j)
    bucket = ((gb * np.uint64(m)) >> np.uint64(31)).astype(np.int64)
    sign = np.where((gs & np.uint64(1)) == 0, 1.0, -1.0)
    return bucket, sign


def ams_sketch(v: np.ndarray, coef: np.ndarray, m: int, j0: int = 0) -> np.ndarray:
    """sk(v) in R^{l x m}: row i, cell b = sum over j with bucket_i(j) = b of sign_i(j) v_j.

    j0: the coordinate of v[0] (v is the slice [j0, j0 + len(v)) of a longer vector; the sketch of
    the whole is the sum of the sketches of its slices, by linearity).
    """
    v = np.asarray(v, np.float64)
    l = coef.shape[0]
    j = np.arange(j0, j0 + v.shape[0], dtype=np.uint64)
    sk = np.zeros((l, m), np.float64)
    for i in range(l):
        bucket, sign = bucket_and_sign(coef[i], j, m)
        sk[i] = np.bincount(bucket, weights=sign * v, minlength=m)
    return sk


def ams_sketch_abs(v: np.ndarray, coef: np.ndarray, m: int) -> np.ndarray:
    """Per cell sum of |v_j| over the cell's keys: the scale of a cell's rounding error."""
    v = np.abs(np.asarray(v, np.float64))
    l = coef.shape[0]
    j = np.arange(v.shape[0], dtype=np.uint64)
    out = np.zeros((l, m), np.float64)
    for i in range(l):
        bucket, _ = bucket_and_sign(coef[i], j, m)
        out[i] = np.bincount(bucket, weights=v, minlength=m)
    return out


def ams_sketch_counts(d: int, coef: np.ndarray, m: int) -> np.ndarray:
    """Number of coordinates of [0, d) that fall into each cell of each row."""
    l = coef.shape[0]
    j = np.arange(d, dtype=np.uint64)
    out = np.zeros((l, m), np.float64)
    for i in range(l):
        bucket, _ = bucket_and_sign(coef[i], j, m)
        out[i] = np.bincount(bucket, minlength=m)
    return out


def m2_estimate(sk: np.ndarray) -> float:
    """M2(sk) = median over rows of the row's squared L2 norm (Section 3.1)."""
    row_sq = np.einsum("ib,ib->i", sk, sk)
    return float(np.median(row_sq))


# --------------------------------------------------------------------------- #
# local state of all K workers (Algorithm 1, line 6)
# --------------------------------------------------------------------------- #
def local_state(w, dtype: str, w_t0: np.ndarray, xi, coef, m: int, scales: bool = True, j0: int = 0):
    """States of all K workers.

    j0: the coordinate of column 0 (the inputs are the coordinates [j0, j0 + d) of longer vectors:
    n, p and sk of the whole are the sums over such blocks).  Only with scales=False.

    scales=False leaves out the absolute-sum scales (p_abs, sk_abs, sk_cnt: only the tests'
    tolerances use them; the method itself is n, p and sk) -- the benchmark's CPU-baseline leg
    times the method's own work that way.

    Returns a dict with
      n[K]        ||u_k||^2                              (Thm 1 / Thm 2, first component)
      p[K]        <xi, u_k>        (None if xi is None)  (Thm 2)
      p_abs[K]    sum_j |xi_j u_kj|
      sk[K,l,m]   sk(u_k)          (None if coef is None) (Thm 1)
      sk_abs[K,l,m]   per cell sum of |u_kj|
      sk_cnt[l,m]     per cell number of coordinates
      u_mean_abs[K]   mean_j |u_kj|
    """
    w64 = widen(w, dtype)
    w0 = np.asarray(w_t0, np.float32).astype(np.float64)
    u = drift(w64, w0)
    out = {"n": sq_norms(u), "p": None, "p_abs": None, "sk": None, "sk_abs": None, "sk_cnt": None,
           "u_mean_abs": np.abs(u).mean(axis=1)}
    if xi is not None:
        x = np.asarray(xi, np.float32).astype(np.float64)
        out["p"] = projections(u, x)
        if scales:
            out["p_abs"] = abs_projections(u, x)
    if coef is not None:
        K = u.shape[0]
        if scales and j0 != 0:
            raise ValueError("the tolerance scales are only computed for whole vectors")
        out["sk"] = np.stack([ams_sketch(u[k], coef, m, j0) for k in range(K)])
        if scales:
            out["sk_abs"] = np.stack([ams_sketch_abs(u[k], coef, m) for k in range(K)])
            out["sk_cnt"] = ams_sketch_counts(u.shape[1], coef, m)
    return out


def mean_state(w, dtype: str, w_t0: np.ndarray, xi, coef, m: int, scales: bool = True):
    """The average state of Algorithm 1, line 7, from the average drift.

    u_bar = (1/K) sum_k u_k;  the sketch and the inner product are linear (Section 3.1), so the
    average of the K states is (mean_k ||u_k||^2, <xi, u_bar>, sk(u_bar)): this function
    evaluates exactly that, sketching u_bar itself.  (That it equals the average of
    local_state's per-worker outputs is one of the pinned identities.)

    Returns a dict with n (float), p (float or None), sk[l,m] (or None) and (unless scales=False) the
    scales the tolerances use: p_abs = mean_k sum_j |xi_j u_kj|, sk_abs[l,m] = mean_k per-cell sum of
    |u_kj|, sk_cnt[l,m], u_mean_abs = mean over k, j of |u_kj|.
    """
    w64 = widen(w, dtype)
    w0 = np.asarray(w_t0, np.float32).astype(np.float64)
    u = drift(w64, w0)
    K = u.shape[0]
    u_bar = u.sum(axis=0) / K
    out = {"n": float(sq_norms(u).sum() / K), "p": None, "p_abs": None, "sk": None, "sk_abs": None,
           "sk_cnt": None, "u_mean_abs": float(np.abs(u).mean())}
    if xi is not None:
        x = np.asarray(xi, np.float32).astype(np.float64)
        out["p"] = float(u_bar @ x)
        if scales:
            out["p_abs"] = float(abs_projections(u, x).sum() / K)
    if coef is not None:
        out["sk"] = ams_sketch(u_bar, coef, m)
        if scales:
            out["sk_abs"] = ams_sketch_abs(np.abs(u).sum(axis=0) / K, coef, m)
            out["sk_cnt"] = ams_sketch_counts(u.shape[1], coef, m)
    return out


# --------------------------------------------------------------------------- #
# averaged state, estimates, decision (Algorithm 1, lines 7-8)
# --------------------------------------------------------------------------- #
def h_linear(n: np.ndarray, p: np.ndarray) -> float:
    """LinearFDA estimate (Thm 2):  mean_k ||u_k||^2 - ( mean_k <xi,u_k> )^2."""
    return float(np.mean(n) - np.mean(p) ** 2)


def h_sketch(n: np.ndarray, sk: np.ndarray, eps: float) -> float:
    """SketchFDA estimate (Thm 1):  mean_k ||u_k||^2 - M2( mean_k sk(u_k) ) / (1 + eps)."""
    sk_bar = sk.mean(axis=0)
    return float(np.mean(n) - m2_estimate(sk_bar) / (1.0 + eps))


def decide(h: float, theta: float, scale: float, tie_tol: float):
    """(sync, near_tie, nonfinite) for an estimate h against the threshold theta.

    sync = h > theta, strictly (Algorithm 1, line 8).  near_tie marks estimates
    within tie_tol * max(scale, |theta|) of theta, where a lower-precision
    evaluation may legitimately decide the other way.  A non-finite h
    synchronizes.
    """
    if not np.isfinite(h):
        return 1, 0, 1
    sync = 1 if h > theta else 0
    near = 1 if abs(h - theta) <= tie_tol * max(scale, abs(theta)) else 0
    return sync, near, 0


def estimate_variance(n, p, sk, eps: float, theta: float, tie_tol: float = 1e-5) -> dict:
    """Average the K states and evaluate both estimates and decisions."""
    n = np.asarray(n, np.float64)
    res = {"mean_sqnorm": float(np.mean(n)), "mean_proj": 0.0, "m2": 0.0,
           "h_linear": 0.0, "h_sketch": 0.0,
           "sync_linear": 0, "sync_sketch": 0,
           "near_tie_linear": 0, "near_tie_sketch": 0, "nonfinite": 0}
    scale = res["mean_sqnorm"]
    if p is not None:
        p = np.asarray(p, np.float64)
        res["mean_proj"] = float(np.mean(p))
        res["h_linear"] = h_linear(n, p)
        s, t, nf = decide(res["h_linear"], theta, scale, tie_tol)
        res["sync_linear"], res["near_tie_linear"] = s, t
        res["nonfinite"] |= nf
    if sk is not None:
        sk = np.asarray(sk, np.float64)
        res["m2"] = m2_estimate(sk.mean(axis=0))
        res["h_sketch"] = h_sketch(n, sk, eps)
        s, t, nf = decide(res["h_sketch"], theta, scale, tie_tol)
        res["sync_sketch"], res["near_tie_sketch"] = s, t
        res["nonfinite"] |= nf
    return res


# --------------------------------------------------------------------------- #
# synchronization and the LinearFDA direction (Algorithm 1, line 9; Section 3.2)
# --------------------------------------------------------------------------- #
def sync(w, dtype: str, w_t0: np.ndarray) -> dict:
    """Synchronize: every worker takes the average model (Section 3, Notation).

    Returns  mean[d] (fp64),  rows: what every slab row holds afterwards in the
    slab's storage type (fp32: the mean rounded to fp32; bf16: bit patterns of the
    mean rounded to nearest-even),  w_prev = the old w_t0 (the model after the
    second most recent synchronization, Table 'Notation').
    """
    w64 = widen(w, dtype)
    mean = mean_model(w64)
    if dtype == "f32":
        rows = mean.astype(np.float32)
    else:
        rows = round_to_bf16_bits(mean)
    return {"mean": mean, "rows": rows, "w_prev": np.asarray(w_t0, np.float32).copy()}


def update_xi(w_t0: np.ndarray, w_prev: np.ndarray) -> np.ndarray:
    """xi = (w_t0 - w_prev) / || w_t0 - w_prev ||_2   (Section 3.2, last display)."""
    diff = np.asarray(w_t0, np.float32).astype(np.float64) - \
        np.asarray(w_prev, np.float32).astype(np.float64)
    nrm = float(np.sqrt(np.dot(diff, diff)))
    if nrm == 0.0 or not np.isfinite(nrm):
        return np.zeros_like(diff)
    return diff / nrm
