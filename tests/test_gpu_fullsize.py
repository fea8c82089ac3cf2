"""The benchmark configurations at their full sizes, in the launch configuration bench.py
times.  The oracle cannot finish a whole state there in seconds, so it computes sampled
outputs one by one -- the scalar state of a few workers and complete sketch rows of a few
(worker, row) pairs -- plus one property that holds at any size (the cells of a row add up to
the signed sum of the drift).  The average state of fda_mean_state is checked in the same pass:
the oracle walks over all K rows once, accumulating the mean drift, and sketches it for the
sampled rows."""
import sys

import numpy as np
import pytest
import torch

import fda_synth as S
from oracle import fda_oracle as O

pytestmark = pytest.mark.gpu
RTOL = 1e-5
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def row_to_numpy(wl, k):
    r = wl.w[k].cpu()
    if r.dtype == torch.bfloat16:
        return r.view(torch.int16).numpy().view(np.uint16)
    return r.numpy()


@pytest.mark.parametrize("name,workers,rows", [("cfg2", [0, 9, 15], [0, 4]),
                                                ("cfg3", [0, 17, 29], [0, 3]),
                                                ("cfg4", [0, 31, 59], [1, 4]),
                                                ("cfg5", [0, 7], [2])])
def test_full_size_sampled_outputs(name, workers, rows):
    import paper_2405_20988_amd as F
    say(f"[case] full size {name}: generating")
    wl = S.make(name, device=DEV, seed=0)
    mon = F.FdaMonitor(wl.K, wl.d, wl.dtype, 3, wl.l, wl.m, wl.eps, wl.hash_coef, device=DEV)
    say(f"       plan {mon.plan}")
    mon.local_state(wl.w, wl.w_t0, wl.xi)
    torch.cuda.synchronize()
    n, p, sk = mon.state_numpy()
    est = mon.estimate_variance(1e30)
    assert est.nonfinite == 0 and est.sync_linear == 0 and est.sync_sketch == 0
    assert est.mean_sqnorm == pytest.approx(float(np.mean(n.astype(np.float64))), rel=1e-6)

    w0 = wl.w_t0.cpu().numpy().astype(np.float64)
    xi = wl.xi.cpu().numpy().astype(np.float64)
    j = np.arange(wl.d, dtype=np.uint64)
    hashed = {}
    for i in rows:
        say(f"       oracle: hashing row {i} over {wl.d} keys")
        hashed[i] = O.bucket_and_sign(wl.hash_coef[i], j, wl.m)
    mon.mean_state(wl.w, wl.w_t0, wl.xi)
    torch.cuda.synchronize()
    nb, pb, skb = mon.mean_numpy()
    assert mon.last_state_path() == 0 and mon.last_mean_state_path() == 0
    usum = np.zeros(wl.d, np.float64)
    uabs = np.zeros(wl.d, np.float64)
    nsum = 0.0
    for k in range(wl.K):
        say(f"       oracle: worker {k}")
        u = O.widen(row_to_numpy(wl, k), wl.dtype) - w0
        usum += u
        uabs += np.abs(u)
        nsum += float(u @ u)
        if k not in workers:
            continue
        assert n[k] == pytest.approx(float(u @ u), rel=RTOL)
        want_p = float(u @ xi)
        assert abs(p[k] - want_p) <= RTOL * float(np.abs(u) @ np.abs(xi))
        for i in rows:
            bucket, sign = hashed[i]
            want = np.bincount(bucket, weights=sign * u, minlength=wl.m)
            scale = np.bincount(bucket, weights=np.abs(u), minlength=wl.m) + \
                np.bincount(bucket, minlength=wl.m) * np.abs(u).mean()
            err = np.abs(sk[k, i] - want)
            assert (err <= RTOL * scale).all(), float((err / scale).max())
            # any size: the cells of a row add up to the signed sum of the drift
            assert abs(float(sk[k, i].astype(np.float64).sum()) - float((sign * u).sum())) \
                <= RTOL * float(np.abs(u).sum())
        del u
    # the average state (Algorithm 1 line 7) from the average drift
    say("       oracle: mean state")
    usum /= wl.K
    uabs /= wl.K
    assert nb == pytest.approx(nsum / wl.K, rel=RTOL)
    assert abs(pb - float(usum @ xi)) <= RTOL * float(uabs @ np.abs(xi))
    for i in rows:
        bucket, sign = hashed[i]
        want = np.bincount(bucket, weights=sign * usum, minlength=wl.m)
        scale = np.bincount(bucket, weights=uabs, minlength=wl.m) + \
            np.bincount(bucket, minlength=wl.m) * uabs.mean()
        err = np.abs(skb[i] - want)
        assert (err <= RTOL * scale).all(), float((err / scale).max())
    est_m = mon.estimate_variance_mean(1e30)
    assert est_m.nonfinite == 0 and est_m.mean_sqnorm == pytest.approx(est.mean_sqnorm, rel=1e-6)
    assert est_m.h_sketch == pytest.approx(est.h_sketch, rel=1e-5)
    assert est_m.h_linear == pytest.approx(est.h_linear, rel=1e-5)
    mon.close()
