"""The tolerances of the GPU parity tests, in one place (fp32 kernels against the fp64 oracle).

A sketch cell is a cancelling sum of n_cell terms.  Its bound is

    |cell_gpu - cell_oracle| <= 1e-5 * sum_{j in cell} |u_kj|                       (1)

on every cell that is not nearly empty of drift, i.e. whose sum of |u_kj| is at least half of
what n_cell average terms would give, sum_{j in cell} |u_kj| >= 0.5 * n_cell * mean_j |u_kj|.
The kernels add a term as the integer round(u * 2^e) with 2^e * mean|u| >= 2^17: every term is
off by at most 2^-18 of the mean |u|, a cell by at most n_cell * 2^-18 * mean|u| = 3.8e-6 *
n_cell * mean|u|, which is inside (1) on those cells.  A cell whose terms are all far below the
mean (a sparse or clustered drift) keeps the same absolute rounding while (1) shrinks with its
terms; only there the bound is

    1e-5 * (sum_{j in cell} |u_kj| + n_cell * mean_j |u_kj|)                        (2)

The functions return the worst error as a fraction of bound (1) over the cells that use it, so
that a test can print how far inside it the kernels sit.
"""
import numpy as np

RTOL = 1e-5


def cell_bounds(sk_abs, sk_cnt, u_mean_abs, rtol=RTOL):
    """(bound, dense) for sketch cells.

    sk_abs[..., l, m] per-cell sum of |u|; sk_cnt[l, m] coordinates per cell; u_mean_abs: mean |u|
    of the same vector(s), broadcastable against sk_abs once two axes are appended.
    dense marks the cells held to bound (1); the others get bound (2).
    """
    sk_abs = np.asarray(sk_abs, np.float64)
    typical = np.asarray(sk_cnt, np.float64) * np.asarray(u_mean_abs, np.float64)[..., None, None]
    dense = sk_abs >= 0.5 * typical
    bound = np.where(dense, rtol * sk_abs, rtol * (sk_abs + typical))
    return bound, dense


def check_cells(got, want, sk_abs, sk_cnt, u_mean_abs, rtol=RTOL, what="sketch"):
    """Assert every cell within its bound; returns (worst error / bound (1) over dense cells,
    fraction of dense cells)."""
    bound, dense = cell_bounds(sk_abs, sk_cnt, u_mean_abs, rtol)
    err = np.abs(np.asarray(got, np.float64) - np.asarray(want, np.float64))
    bad = err > bound + 1e-30
    assert not bad.any(), (what, int(bad.sum()), float((err / (bound + 1e-300)).max()))
    worst = float((err[dense] / (bound[dense] + 1e-300)).max()) if dense.any() else 0.0
    return worst, float(dense.mean())
