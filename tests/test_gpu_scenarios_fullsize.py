"""The benchmark configurations as they are stated, at their full sizes, against the CPU oracle.

  cfg3  K=30, d=7.0M fp32: the whole state of every worker, both estimates, the decisions and the
        near-tie flags at Theta in {1/4, 1/2, 1, 2} x the true variance (Eq. 1 by brute force).
  cfg4  K=60, d=20M fp32, SketchFDA only: the state pass, then a forced synchronization and the
        refresh of xi, every element of w_t0 and xi against the oracle, every row bit-equal.
  cfg2  K=16, d=2.6M fp32: T=100 steps enqueued on the device without reading anything back
        (decisions kept in device memory, logged on the device); the steps at which the GPU
        synchronized must be the oracle's.
  cfg5  K=8, d=350M bf16: T=20 steps with xi refreshed at every synchronization, again without a
        host read inside the run; the oracle evaluates the steps {0, a later synchronization,
        the last one} from snapshots of the device's inputs, and re-does the synchronization.

The oracle side streams one worker (or one block of coordinates) at a time and hashes every sketch
row once (tests/fullsize_oracle.py); heaviest case last.
"""
import shutil
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import fda_synth as S
from fda_tolerance import check_cells
from fullsize_oracle import (THREADS, cell_counts, finish_hash_processes, hash_rows, row_to_numpy,
                             sketch_row, sketch_row_blocks, start_hash_processes)
from oracle import fda_oracle as O

pytestmark = pytest.mark.gpu
RTOL = 1e-5
DEV = "cuda:0"


@pytest.fixture
def say(capsys):
    """Progress lines that reach the terminal also when pytest captures output."""
    t0 = time.time()

    def emit(msg):
        with capsys.disabled():
            print(f"[{time.time() - t0:6.1f}s] {msg}", flush=True)
            sys.stdout.flush()
    return emit


def monitor_for(wl, variants):
    import paper_2405_20988_amd as F
    return F.FdaMonitor(wl.K, wl.d, wl.dtype, variants, wl.l, wl.m, wl.eps, wl.hash_coef, device=DEV)


def check_estimate(est, want, variants, tol=RTOL):
    """Values within tol * mean||u||^2; decisions identical outside the near-tie band; the near-tie
    flags identical unless the estimate sits at the edge of the band itself."""
    nbar = want["mean_sqnorm"]
    assert est.mean_sqnorm == pytest.approx(nbar, rel=RTOL)
    assert est.nonfinite == want["nonfinite"] == 0
    for bit, name in ((1, "linear"), (2, "sketch")):
        if not variants & bit:
            continue
        h, hw = getattr(est, "h_" + name), want["h_" + name]
        assert abs(h - hw) <= tol * nbar, (name, h, hw)
        if not want["near_tie_" + name]:
            assert getattr(est, "sync_" + name) == want["sync_" + name], name
    if variants & 2:
        assert abs(est.m2 - want["m2"]) <= tol * max(nbar, want["m2"])


def near_tie_flags_agree(est, want, theta, name, tie_tol=1e-5):
    band = tie_tol * max(want["mean_sqnorm"], abs(theta))
    gap = abs(want["h_" + name] - theta)
    if abs(gap - band) <= RTOL * want["mean_sqnorm"]:
        return True                                  # on the edge of the band: either flag
    return getattr(est, "near_tie_" + name) == want["near_tie_" + name]


# --------------------------------------------------------------------------------------------
def test_cfg3_theta_sweep_full_size(say):
    wl = S.make("cfg3", device=DEV, seed=0)
    K, d, l, m = wl.K, wl.d, wl.l, wl.m
    mon = monitor_for(wl, 3)
    say(f"[case] cfg3 full size K={K} d={d}: plan {mon.plan}")
    mon.local_state(wl.w, wl.w_t0, wl.xi)
    torch.cuda.synchronize()
    n, p, sk = mon.state_numpy()
    assert mon.last_state_path() == 0

    w0 = wl.w_t0.cpu().numpy().astype(np.float64)
    xi = wl.xi.cpu().numpy().astype(np.float64)
    hashed = hash_rows(wl.hash_coef, range(l), d, m)
    cnt = np.stack([cell_counts(hashed[i], m) for i in range(l)])
    say("       oracle: hashed 5 rows; average model (Eq. 1 needs it)")
    wsum = np.zeros(d)
    for k in range(K):
        wsum += O.widen(row_to_numpy(wl.w[k]), "f32")
    wbar = wsum / K
    var = 0.0
    n_or, p_or, p_abs, u_mean_abs = np.zeros(K), np.zeros(K), np.zeros(K), np.zeros(K)
    sk_or, sk_abs = np.zeros((K, l, m)), np.zeros((K, l, m))
    for k in range(K):
        wk = O.widen(row_to_numpy(wl.w[k]), "f32")
        diff = wk - wbar
        var += float(diff @ diff)                      # Eq. 1, term by term
        u = O.drift(wk[None], w0)
        n_or[k] = O.sq_norms(u)[0]
        p_or[k] = O.projections(u, xi)[0]
        p_abs[k] = O.abs_projections(u, xi)[0]
        u_mean_abs[k] = np.abs(u[0]).mean()
        for i in range(l):
            sk_or[k, i] = sketch_row(u[0], hashed[i], m)
            sk_abs[k, i] = np.bincount(hashed[i][0], weights=np.abs(u[0]), minlength=m)
        if k % 10 == 9:
            say(f"       oracle: {k + 1} workers done")
    var /= K
    ubar = wbar - w0
    assert var == pytest.approx(float(n_or.mean() - ubar @ ubar), rel=1e-9)      # Eq. 3

    assert np.allclose(n, n_or, rtol=RTOL, atol=0)
    assert (np.abs(p - p_or) <= RTOL * p_abs).all()
    worst, dense = check_cells(sk, sk_or, sk_abs, cnt, u_mean_abs)
    say(f"       all {K * l * m} sketch cells: worst error {worst:.4f} of 1e-5 * sum|u| "
        f"({100 * dense:.1f} % of the cells held to that bound)")

    fired = {}
    for mult in (0.25, 0.5, 1.0, 2.0):
        theta = mult * var
        est = mon.estimate_variance(theta)
        want = O.estimate_variance(n_or, p_or, sk_or, wl.eps, theta)
        check_estimate(est, want, 3)
        for name in ("linear", "sketch"):
            assert near_tie_flags_agree(est, want, theta, name), (mult, name)
        fired[mult] = (want["sync_linear"], want["sync_sketch"], want["near_tie_linear"], want["near_tie_sketch"])
        say(f"       Theta = {mult} Var: H_lin {est.h_linear:.6e} H_sk {est.h_sketch:.6e} Var {var:.6e} "
            f"sync {est.sync_linear}/{est.sync_sketch} near-tie {est.near_tie_linear}/{est.near_tie_sketch}")
        assert want["h_linear"] >= var * (1 - 1e-12)                 # Thm 2
    # a random xi sees almost none of the drift: LinearFDA fires up to Theta = Var and not at 2 Var
    assert [fired[q][0] for q in (0.25, 0.5, 1.0, 2.0)] == [1, 1, 1, 0]
    assert [fired[q][1] for q in (0.25, 0.5, 2.0)] == [1, 1, 0]

    # the average state directly (fda_mean_state) must lead to the same estimates
    mon.mean_state(wl.w, wl.w_t0, wl.xi)
    for mult in (0.25, 0.5, 1.0, 2.0):
        theta = mult * var
        est = mon.estimate_variance_mean(theta)
        check_estimate(est, O.estimate_variance(n_or, p_or, sk_or, wl.eps, theta), 3)
    mon.close()


# --------------------------------------------------------------------------------------------
def test_cfg4_sketch_only_state_and_forced_sync_full_size(say):
    wl = S.make("cfg4", device=DEV, seed=0)
    K, d, l, m = wl.K, wl.d, wl.l, wl.m
    mon = monitor_for(wl, 2)                                          # SketchFDA only
    say(f"[case] cfg4 full size K={K} d={d}, sketch only: plan {mon.plan}")
    mon.local_state(wl.w, wl.w_t0, None)
    torch.cuda.synchronize()
    n, p, sk = mon.state_numpy()
    assert not p.any() and mon.last_state_path() == 0

    w0_32 = wl.w_t0.cpu().numpy().copy()
    w0 = w0_32.astype(np.float64)
    hashed = hash_rows(wl.hash_coef, range(l), d, m)
    cnt = np.stack([cell_counts(hashed[i], m) for i in range(l)])
    say("       oracle: hashed 5 rows; streaming the 60 workers")
    sampled = [0, 31, 59]
    wsum, wmax = np.zeros(d), np.zeros(d)
    n_or = np.zeros(K)
    for k in range(K):
        wk = O.widen(row_to_numpy(wl.w[k]), "f32")
        wsum += wk
        np.maximum(wmax, np.abs(wk), out=wmax)
        u = O.drift(wk[None], w0)
        n_or[k] = O.sq_norms(u)[0]
        if k in sampled:
            rows_or = np.stack([sketch_row(u[0], hashed[i], m) for i in range(l)])
            rows_abs = np.stack([np.bincount(hashed[i][0], weights=np.abs(u[0]), minlength=m) for i in range(l)])
            worst, _ = check_cells(sk[k][None], rows_or[None], rows_abs[None], cnt, np.array([np.abs(u[0]).mean()]))
            say(f"       worker {k}: all {l} sketch rows, worst cell error {worst:.4f} of 1e-5 * sum|u|")
    assert np.allclose(n, n_or, rtol=RTOL, atol=0)
    mean = wsum / K                                                   # the average model, Section 3 Notation
    ubar = mean - w0
    sk_bar = np.stack([sketch_row_blocks(ubar, hashed[i], m) for i in range(l)])   # = mean_k sk(u_k), linearity
    h_or = O.estimate_variance(n_or, None, sk_bar[None], wl.eps, 0.0)["h_sketch"]
    for mult in (0.5, 2.0):
        theta = mult * h_or
        est = mon.estimate_variance(theta)
        want = O.estimate_variance(n_or, None, sk_bar[None], wl.eps, theta)
        check_estimate(est, want, 2)
        assert est.sync_sketch == (1 if mult < 1 else 0) and est.h_linear == 0.0 and est.sync_linear == 0
    say(f"       H_sk {est.h_sketch:.6e} (oracle {h_or:.6e})")

    # forced synchronization (no predicate) and the refresh of xi
    w_prev = torch.zeros_like(wl.w_t0)
    xi_new = torch.zeros_like(wl.w_t0)
    mon.sync(wl.w, wl.w_t0, w_prev, pred=None)
    mon.update_xi(wl.w_t0, w_prev, xi_new, pred=None)
    torch.cuda.synchronize()
    assert np.array_equal(w_prev.cpu().numpy(), w0_32)                # the old model, bit for bit
    new_w0 = wl.w_t0.cpu().numpy()
    err = np.abs(new_w0.astype(np.float64) - mean)
    assert (err <= RTOL * wmax + 1e-30).all(), float((err / (wmax + 1e-300)).max())
    say(f"       w_t0: worst error {float((err / (wmax + 1e-300)).max()):.3e} of max_k |w_kj| over {d} coordinates")
    for k in range(K):                                                # every worker holds the same bits
        assert torch.equal(wl.w[k].view(torch.int32), wl.w_t0.view(torch.int32)), k
    assert np.array_equal(row_to_numpy(wl.w[K - 1]), new_w0)
    want_xi = O.update_xi(new_w0, w0_32)
    got_xi = xi_new.cpu().numpy().astype(np.float64)
    assert np.abs(got_xi - want_xi).max() <= RTOL * np.abs(want_xi).max()
    assert float(got_xi @ got_xi) == pytest.approx(1.0, rel=1e-5)
    # "after synchronization the model variance is zero": the state is exactly zero
    mon.local_state(wl.w, wl.w_t0, None)
    e = mon.estimate_variance(0.0)
    assert not mon.state.any() and (e.h_sketch, e.sync_sketch) == (0.0, 0)
    mon.close()


# --------------------------------------------------------------------------------------------
def est_from_log(log_row):
    import paper_2405_20988_amd as F
    return F.FdaEstimate.from_buffer_copy(log_row.tobytes())


def test_cfg2_hundred_steps_on_the_device(say):
    wl = S.make("cfg2", device=DEV, seed=0)
    K, d, l, m, T = wl.K, wl.d, wl.l, wl.m, wl.T
    assert T == 100
    mon = monitor_for(wl, 3)
    say(f"[case] cfg2 full size K={K} d={d} T={T}: plan {mon.plan}")
    # After a synchronization every worker drifts by N(0, 1e-4^2) per coordinate and step: s steps later
    # mean||u||^2 = s d 1e-8 and ||u_bar||^2 = s d 1e-8 / K, so H_sketch = s d 1e-8 (1 - 1/(K (1+eps)))
    # up to the sketch's few per cent of the second term.  Theta between s = 19 and s = 20 makes a
    # synchronization fire every 20 steps; the initial drift is far above it, so step 0 fires too.
    theta = 19.5 * d * 1e-8 * (1.0 - 1.0 / (K * (1.0 + wl.eps)))
    w_o = S.slab_to_numpy(wl.w)
    w0_o = wl.w_t0.cpu().numpy().copy()
    xi_o = wl.xi.cpu().numpy().copy()
    w_prev_o = w0_o.copy()
    noise = []
    for t in range(T):                                                # all the noise first: 16.6 GB of HBM
        noise.append(torch.stack([S._noise(d, wl.step_std, False, wl.gen, wl.w.device) for _ in range(K)]))
    w_prev = wl.w_t0.clone()
    log = torch.zeros((T, mon.est_dev.numel()), dtype=torch.uint8, device=DEV)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(T):                                                # nothing below reads the device
        wl.w += noise[t]
        mon.step(wl.w, wl.w_t0, w_prev, wl.xi, theta, decide_by="sketch", want_host=False)
        log[t].copy_(mon.est_dev)
    torch.cuda.synchronize()
    say(f"       100 steps enqueued and run in {time.perf_counter() - t0:.2f} s")
    log_host = log.cpu().numpy()
    gpu_syncs = [t for t in range(T) if est_from_log(log_host[t]).sync_sketch]

    hashed = hash_rows(wl.hash_coef, range(l), d, m)
    or_syncs, ties = [], []
    for t in range(T):
        w_o = w_o + noise[t].cpu().numpy()                            # the same fp32 additions
        w0 = w0_o.astype(np.float64)
        x64 = xi_o.astype(np.float64)
        n_or, p_or, usum = np.zeros(K), np.zeros(K), np.zeros(d)
        for k in range(K):
            u = O.drift(O.widen(w_o[k], "f32")[None], w0)
            n_or[k] = O.sq_norms(u)[0]
            p_or[k] = O.projections(u, x64)[0]
            usum += u[0]
        sk_bar = np.stack([sketch_row(usum / K, hashed[i], m) for i in range(l)])   # mean_k sk(u_k), linearity
        want = O.estimate_variance(n_or, p_or, sk_bar[None], wl.eps, theta)
        est = est_from_log(log_host[t])
        check_estimate(est, want, 3, tol=2 * RTOL)                    # the trajectories differ by roundings of the mean
        if want["near_tie_sketch"]:
            ties.append(t)
            break                                                     # the trajectories may part here
        if want["sync_sketch"]:
            or_syncs.append(t)
            s = O.sync(w_o, "f32", w0_o)
            w_prev_o = s["w_prev"]
            w0_o = s["mean"].astype(np.float32)
            w_o = np.tile(s["rows"], (K, 1))
            xi_o = O.update_xi(w0_o, w_prev_o).astype(np.float32)
        if t % 20 == 19:
            say(f"       oracle: step {t}, synchronizations so far {or_syncs}")
    say(f"       theta={theta:.4e} gpu syncs {gpu_syncs} oracle syncs {or_syncs} ties {ties}")
    assert not ties
    assert gpu_syncs == or_syncs and 4 <= len(or_syncs) <= 6
    got = wl.xi.cpu().numpy().astype(np.float64)
    change = float(np.linalg.norm(w0_o.astype(np.float64) - w_prev_o.astype(np.float64)))
    assert np.abs(got - xi_o).max() <= 8 * 2.0 ** -24 * float(np.abs(w0_o).max()) / change
    assert np.abs(wl.w_t0.cpu().numpy().astype(np.float64) - w0_o).max() <= RTOL * float(np.abs(w0_o).max())
    mon.close()


# --------------------------------------------------------------------------------------------
def run_cfg5(theta, snap_steps, say):
    """T steps of cfg5 on the device with no host read inside the run.  Returns the per-step result
    structs and, for the steps in snap_steps, clones of the inputs before and the outputs after."""
    wl = S.make("cfg5", device=DEV, seed=0)
    mon = monitor_for(wl, 3)
    T = wl.T
    w_prev = wl.w_t0.clone()
    log = torch.zeros((T, mon.est_dev.numel()), dtype=torch.uint8, device=DEV)
    import paper_2405_20988_amd as F
    off = F.FdaEstimate.sync_sketch.offset
    fired = mon.est_dev[off:off + 4].view(torch.int32)               # the decision, in device memory
    snaps = {}
    torch.cuda.synchronize()
    for t in range(T):
        wl.advance()
        if t in snap_steps:
            snaps[t] = {"w": wl.w.clone(), "w_t0": wl.w_t0.clone(), "xi": wl.xi.clone()}
        mon.step(wl.w, wl.w_t0, w_prev, wl.xi, theta, decide_by="sketch", want_host=False)
        log[t].copy_(mon.est_dev)
        if t in snap_steps:
            snaps[t].update({"w_after": wl.w.clone(), "w_t0_after": wl.w_t0.clone(),
                             "xi_after": wl.xi.clone(), "w_prev_after": w_prev.clone()})
        # the fp32 master copy follows the slab when the step synchronized (decided on the device)
        for k in range(wl.K):
            wl.latent[k] = torch.where(fired.bool(), wl.w[k].float(), wl.latent[k])
    torch.cuda.synchronize()
    plan = mon.plan
    mon.close()
    return wl, log.cpu().numpy(), snaps, plan


def mean_state_by_blocks(w_host, w0, xi, hashed, l, m, K, d, block=1 << 22):
    """(n[K], p[K], sk(u_bar)[l, m]) of a bf16 slab: blocks of coordinates on several threads, every
    block widened, differenced and sketched with the oracle's own statements (the blocks add)."""
    def one(a):
        b = min(a + block, d)
        n, p, usum = np.zeros(K), np.zeros(K), np.zeros(b - a)
        for k in range(K):
            u = O.drift(O.widen(w_host[k, a:b], "bf16")[None], w0[a:b])
            n[k] = O.sq_norms(u)[0]
            p[k] = O.projections(u, xi[a:b])[0]
            usum += u[0]
        ubar = usum / K
        sk = np.stack([np.bincount(hashed[i][0][a:b], weights=np.where(hashed[i][1][a:b], -ubar, ubar),
                                   minlength=m) for i in range(l)])
        return n, p, sk
    with ThreadPoolExecutor(THREADS) as ex:
        parts = list(ex.map(one, range(0, d, block)))
    return sum(q[0] for q in parts), sum(q[1] for q in parts), sum(q[2] for q in parts)


def test_cfg5_twenty_steps_with_refreshed_xi(say, tmp_path):
    K, d, l, m = (S.CONFIGS["cfg5"][q] for q in ("K", "d", "l", "m"))
    eps = S.default_eps(m)
    coef = S.hash_coefficients(0, l)
    folder = str(tmp_path / "hash")
    kids = start_hash_processes(coef, range(l), d, m, folder)         # they hash while the GPU runs
    try:
        # Theta: how fast H_sketch grows after a synchronization, measured by the oracle alone on a
        # short slab of the same recipe (H is a sum over coordinates: it scales with d)
        ds = 1_000_000
        small = S.make("cfg5", device="cpu", seed=3, d=ds)
        s0 = O.sync(S.slab_to_numpy(small.w), "bf16", small.w_t0.numpy())
        small.w.copy_(torch.from_numpy(np.tile(s0["rows"], (K, 1)).view(np.int16)).view(torch.bfloat16))
        small.w_t0.copy_(torch.from_numpy(s0["mean"].astype(np.float32)))
        small.after_sync()
        hs = []
        for _ in range(5):
            small.advance()
            ms = O.mean_state(S.slab_to_numpy(small.w), "bf16", small.w_t0.numpy(), None, small.hash_coef, m,
                              scales=False)
            hs.append(O.estimate_variance(np.array([ms["n"]]), None, ms["sk"][None], eps, 0.0)["h_sketch"])
        theta = 0.5 * (hs[3] + hs[4]) * d / ds                          # crossed 4-5 steps after a synchronization
        say(f"[case] cfg5 full size K={K} d={d} T=20: H/d after a synchronization {[f'{h / ds:.3e}' for h in hs]}, "
            f"theta {theta:.4e}")

        wl, log1, _, plan = run_cfg5(theta, (), say)
        T = wl.T
        del wl
        torch.cuda.empty_cache()
        import paper_2405_20988_amd as F
        ests = [F.FdaEstimate.from_buffer_copy(log1[t].tobytes()) for t in range(T)]
        gpu_syncs = [t for t in range(T) if ests[t].sync_sketch]
        say(f"       plan {plan}")
        say(f"       first run: synchronizations at {gpu_syncs}")
        # the first step meets the large initial drift and must fire; after that about every 4-5 steps
        # (the small slab's sketch error on the common bf16 residue differs from the full one's, so the
        # period is only roughly the intended one)
        assert gpu_syncs[0] == 0 and 2 <= len(gpu_syncs) <= 12
        later = gpu_syncs[len(gpu_syncs) // 2]
        steps = sorted({0, later, T - 1})
        wl, log2, snaps, _ = run_cfg5(theta, steps, say)
        assert np.array_equal(log1, log2)                               # the run is reproducible bit for bit
        say(f"       second run identical; oracle at steps {steps}")
        hashed = finish_hash_processes(kids, folder)
        kids = []
        say("       hashes of all 7 rows ready")
        for t in steps:
            sn = snaps[t]
            w_host = np.stack([row_to_numpy(sn["w"][k]) for k in range(K)])
            w0 = sn["w_t0"].cpu().numpy().astype(np.float64)
            xi = sn["xi"].cpu().numpy().astype(np.float64)
            n_or, p_or, sk_bar = mean_state_by_blocks(w_host, w0, xi, hashed, l, m, K, d)
            want = O.estimate_variance(n_or, p_or, sk_bar[None], eps, theta)
            check_estimate(ests[t], want, 3)
            say(f"       step {t}: H_sk {ests[t].h_sketch:.6e} (oracle {want['h_sketch']:.6e}) H_lin "
                f"{ests[t].h_linear:.6e} (oracle {want['h_linear']:.6e}) sync {ests[t].sync_sketch}")
            if not ests[t].sync_sketch:
                # no synchronization: nothing may have changed
                assert torch.equal(sn["w_after"].view(torch.int16), sn["w"].view(torch.int16))
                assert torch.equal(sn["w_t0_after"], sn["w_t0"]) and torch.equal(sn["xi_after"], sn["xi"])
                continue
            if t != later or not want["sync_sketch"]:
                continue
            # the synchronization of this step, re-done by the oracle block by block
            new_w0 = sn["w_t0_after"].cpu().numpy()
            assert torch.equal(sn["w_prev_after"], sn["w_t0"])          # the old model, bit for bit
            rows_gpu = row_to_numpy(sn["w_after"][0])
            for k in range(1, K):
                assert torch.equal(sn["w_after"][k].view(torch.int16), sn["w_after"][0].view(torch.int16)), k
            off_by_one = 0
            for a in range(0, d, 1 << 24):
                b = min(a + (1 << 24), d)
                s = O.sync(w_host[:, a:b], "bf16", new_w0[a:b])
                wmax = np.abs(O.widen(w_host[:, a:b], "bf16")).max(axis=0)
                assert (np.abs(new_w0[a:b].astype(np.float64) - s["mean"]) <= RTOL * wmax + 1e-30).all()
                diff = np.abs(rows_gpu[a:b].astype(np.int32) - s["rows"].astype(np.int32))
                assert diff.max() <= 1                                  # at most one bf16 step from the exact rounding
                off_by_one += int((diff != 0).sum())
            assert off_by_one < 1e-2 * d
            want_xi = O.update_xi(new_w0, sn["w_t0"].cpu().numpy())
            got_xi = sn["xi_after"].cpu().numpy().astype(np.float64)
            assert np.abs(got_xi - want_xi).max() <= RTOL * np.abs(want_xi).max()
            say(f"       step {t}: synchronization and xi agree with the oracle ({off_by_one} of {d} bf16 rows "
                f"one step from the exact rounding)")
    finally:
        for _, proc in kids:
            proc.kill()
        shutil.rmtree(folder, ignore_errors=True)
