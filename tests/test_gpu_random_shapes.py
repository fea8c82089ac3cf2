"""Seeded random shapes: worker counts, vector lengths, sketch sizes, storage types and variants
that the named configurations never combine (odd group sizes, spare worker and row slots, more
than one row group, a single partition, ragged tails), each checked against the oracle for the
per-worker states, the average state and the estimate."""
import sys

import numpy as np
import pytest
import torch

import fda_synth as S
from fda_tolerance import check_cells
from oracle import fda_oracle as O

pytestmark = pytest.mark.gpu
RTOL = 1e-5
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def draw_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for t in range(n):
        K = int(rng.choice([1, 2, 3, 5, 7, 9, 12, 13, 19, 24, 31, 47]))
        d = int(rng.choice([1, 3, 17, 255, 2048, 2049, 6143, 20_000, 65_537, 131_075, 600_001]))
        l = int(rng.choice([1, 2, 3, 5, 6, 7, 8, 9, 12, 16]))
        m = int(rng.choice([1, 2, 7, 64, 250, 251, 1000, 1024, 4000, 9000]))
        dtype = str(rng.choice(["f32", "bf16"]))
        variants = int(rng.choice([1, 2, 3, 3]))
        heavy = bool(rng.integers(0, 2))
        cases.append((t, K, d, l, m, dtype, variants, heavy))
    return cases


@pytest.mark.parametrize("t,K,d,l,m,dtype,variants,heavy", draw_cases(72, 20240520))
def test_random_shape(t, K, d, l, m, dtype, variants, heavy):
    import paper_2405_20988_amd as F
    say(f"[case] random shape #{t}: K={K} d={d} {l}x{m} {dtype} variants={variants} heavy={heavy}")
    g = torch.Generator(device=DEV)
    g.manual_seed(1000 + t)
    w_t0 = torch.randn(d, generator=g, device=DEV) * 0.05
    xi = torch.randn(d, generator=g, device=DEV)
    xi /= xi.norm() + 1e-30
    u = torch.randn((K, d), generator=g, device=DEV)
    if heavy:   # Student-t(3): z / sqrt(chi2_3 / 3)
        chi = (torch.randn((3, K, d), generator=g, device=DEV) ** 2).sum(0) / 3.0
        u = u / chi.sqrt()
    u = u * 3e-4 + torch.randn(d, generator=g, device=DEV) * 1e-4          # private + shared drift
    w = (w_t0 + u).to(torch.float32 if dtype == "f32" else torch.bfloat16)
    coef = S.hash_coefficients(77 + t, l)
    eps = S.default_eps(m)
    mon = F.FdaMonitor(K, d, dtype, variants, l, m, eps, coef, device=DEV)
    say(f"       plan {mon.plan}")
    w_host = S.slab_to_numpy(w)
    w0_host = w_t0.cpu().numpy()
    xi_host = xi.cpu().numpy() if variants & 1 else None
    coef_o = coef if variants & 2 else None
    xi_dev = xi if variants & 1 else None

    # per-worker states (Algorithm 1 line 6) and the estimate on them
    mon.local_state(w, w_t0, xi_dev)
    ref = O.local_state(w_host, dtype, w0_host, xi_host, coef_o, m)
    n, p, sk = mon.state_numpy()
    assert np.allclose(n, ref["n"], rtol=RTOL, atol=0)
    if variants & 1:
        assert (np.abs(p - ref["p"]) <= RTOL * ref["p_abs"] + 1e-30).all()
    if variants & 2:
        check_cells(sk, ref["sk"], ref["sk_abs"], ref["sk_cnt"], ref["u_mean_abs"])
    var = O.true_variance(O.widen(w_host, dtype))
    for theta in (0.5 * var, 2.0 * var):
        est = mon.estimate_variance(theta)
        want = O.estimate_variance(ref["n"], ref["p"], ref["sk"], eps, theta)
        nbar = want["mean_sqnorm"]
        assert est.mean_sqnorm == pytest.approx(nbar, rel=RTOL)
        if variants & 1:
            assert abs(est.h_linear - want["h_linear"]) <= RTOL * nbar
            assert want["near_tie_linear"] or est.sync_linear == want["sync_linear"]
        if variants & 2:
            assert abs(est.h_sketch - want["h_sketch"]) <= RTOL * nbar
            assert want["near_tie_sketch"] or est.sync_sketch == want["sync_sketch"]

    # the average state directly (Algorithm 1 line 7 by linearity)
    mon.mean_state(w, w_t0, xi_dev)
    mref = O.mean_state(w_host, dtype, w0_host, xi_host, coef_o, m)
    nb, pb, skb = mon.mean_numpy()
    assert nb == pytest.approx(mref["n"], rel=RTOL)
    if variants & 1:
        assert abs(pb - mref["p"]) <= RTOL * mref["p_abs"] + 1e-30
    if variants & 2:
        check_cells(skb, mref["sk"], mref["sk_abs"], mref["sk_cnt"], mref["u_mean_abs"])
    mon.close()
