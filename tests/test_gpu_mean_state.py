"""Parity of fda_mean_state / fda_estimate_variance_mean (the average state of Algorithm 1
line 7 computed directly, by linearity of the sketch) with the CPU fp64 oracle, and with the
average of the per-worker states fda_local_state writes.

Tolerances as for the per-worker states, with every scale averaged over the workers:
  mean ||u_k||^2       relative 1e-5
  <xi,u_bar>           1e-5 * mean_k sum_j |xi_j u_kj|
  sketch cell          1e-5 * mean_k sum_{j in cell} |u_kj| on every cell where that is at least
                       half of n_cell * mean_kj |u_kj|; the nearly empty rest: 1e-5 * (that +
                       n_cell * mean_kj |u_kj|)   (tests/fda_tolerance.py states why)
Integer-valued inputs must match bit for bit after the one division by K.
"""
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


def monitor_for(wl, variants=3, row_stride=None):
    import paper_2405_20988_amd as F
    return F.FdaMonitor(wl.K, wl.d, wl.dtype, variants, wl.l, wl.m, wl.eps, wl.hash_coef,
                        row_stride=row_stride, device=DEV)


def oracle_mean(wl, variants=3):
    return O.mean_state(S.slab_to_numpy(wl.w), wl.dtype, wl.w_t0.cpu().numpy(),
                        wl.xi.cpu().numpy() if variants & 1 else None,
                        wl.hash_coef if variants & 2 else None, wl.m)


def check_mean(mon, ref, variants=3):
    n, p, sk = mon.mean_numpy()
    assert n == pytest.approx(ref["n"], rel=RTOL)
    if variants & 1:
        assert abs(p - ref["p"]) <= RTOL * ref["p_abs"] + 1e-30, abs(p - ref["p"]) / ref["p_abs"]
    else:
        assert p == 0.0
    if variants & 2:
        worst, dense = check_cells(sk, ref["sk"], ref["sk_abs"], ref["sk_cnt"], ref["u_mean_abs"])
        say(f"       mean sketch cells: worst error {worst:.3f} of 1e-5 * mean_k sum|u| "
            f"({100 * dense:.1f} % of the cells are held to that bound)")


def check_estimate(est, ref, variants=3):
    nbar = ref["mean_sqnorm"]
    assert est.mean_sqnorm == pytest.approx(nbar, rel=RTOL)
    if variants & 1:
        assert abs(est.h_linear - ref["h_linear"]) <= RTOL * nbar
        if not ref["near_tie_linear"]:
            assert est.sync_linear == ref["sync_linear"]
    if variants & 2:
        assert abs(est.m2 - ref["m2"]) <= RTOL * max(nbar, ref["m2"])
        assert abs(est.h_sketch - ref["h_sketch"]) <= RTOL * nbar
        if not ref["near_tie_sketch"]:
            assert est.sync_sketch == ref["sync_sketch"]
    assert est.nonfinite == ref["nonfinite"]


# several tiles per workgroup where the partition count saturates, ragged tails, worker counts
# that are and are not multiples of the batch of slab rows (4 for fp32, 8 for bf16), sketches
# that need more than one row group
MEAN_CASES = [
    ("cfg1", None, {}),
    ("cfg2", 1_200_003, {}),
    ("cfg3", 300_007, {}),
    ("cfg4", 150_001, {}),
    ("cfg5", 1_100_005, {}),
    ("cfg5", 4099, {}),
    ("cfg5", 200_003, {"K": 11}),             # bf16, a full batch of 8 rows and a ragged one of 3
    ("cfg5", 100_001, {"K": 3}),              # bf16, a single ragged batch
    ("cfg1", 7, {"K": 3}),
    ("cfg2", 70_001, {"K": 1}),
    ("cfg3", 50_000, {"K": 17}),
    ("cfg4", 40_003, {"K": 33, "l": 4}),
    ("cfg1", 30_001, {"l": 16, "m": 64}),     # two row groups of 8 rows
    ("cfg1", 30_001, {"l": 1, "m": 1}),
    ("cfg2", 20_000, {"K": 3, "l": 3, "m": 19_000}),   # one row per row group: the sketch fills LDS
    ("cfg1", 5_000, {"K": 300, "l": 3, "m": 64}),      # many workers: 75 batches of rows per tile
]


@pytest.mark.parametrize("name,d,over", MEAN_CASES)
def test_mean_state_and_estimate_parity(name, d, over):
    say(f"[case] mean-state parity {name} d={d} {over}")
    wl = S.make(name, device=DEV, seed=1, d=d, **over)
    mon = monitor_for(wl)
    mon.mean_state(wl.w, wl.w_t0, wl.xi)
    torch.cuda.synchronize()
    ref = oracle_mean(wl)
    check_mean(mon, ref)
    var = O.true_variance(O.widen(S.slab_to_numpy(wl.w), wl.dtype))
    for mult in (0.25, 0.5, 1.0, 2.0):
        theta = mult * var
        est = mon.estimate_variance_mean(theta)
        want = O.estimate_variance(np.array([ref["n"]]), np.array([ref["p"]]), ref["sk"][None], wl.eps, theta)
        check_estimate(est, want)
    mon.close()


@pytest.mark.parametrize("variants", [1, 2])
def test_mean_state_single_variant(variants):
    say(f"[case] mean-state single variant {variants}")
    wl = S.make("cfg3", device=DEV, seed=2, d=90_001, K=30)
    mon = monitor_for(wl, variants)
    mon.mean_state(wl.w, wl.w_t0, wl.xi if variants & 1 else None)
    ref = oracle_mean(wl, variants)
    check_mean(mon, ref, variants)
    theta = 0.5 * O.true_variance(O.widen(S.slab_to_numpy(wl.w), wl.dtype))
    est = mon.estimate_variance_mean(theta)
    want = O.estimate_variance(np.array([ref["n"]]), None if ref["p"] is None else np.array([ref["p"]]),
                               None if ref["sk"] is None else ref["sk"][None], wl.eps, theta)
    check_estimate(est, want, variants)
    mon.close()


@pytest.mark.parametrize("dtype,K,d,l,m", [("f32", 4, 200_003, 5, 250), ("f32", 64, 30_001, 5, 500),
                                            ("bf16", 8, 300_007, 7, 1000), ("f32", 16, 5, 3, 4)])
def test_mean_state_integer_inputs_bit_exact(dtype, K, d, l, m):
    """Small-integer drifts and a power-of-two K: every sum and the division by K are exact, so
    the mean state must equal the oracle bit for bit -- any wrong bucket or sign would show."""
    say(f"[case] mean-state integer inputs {dtype} K={K} d={d} {l}x{m}")
    import paper_2405_20988_amd as F
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    w_t0 = torch.randint(-16, 17, (d,), generator=g, device=DEV).float()
    u = torch.randint(-4, 5, (K, d), generator=g, device=DEV).float()
    xi = torch.randint(-2, 3, (d,), generator=g, device=DEV).float()
    w = (w_t0 + u).to(torch.float32 if dtype == "f32" else torch.bfloat16)
    coef = S.hash_coefficients(5, l)
    mon = F.FdaMonitor(K, d, dtype, 3, l, m, 0.06, coef, device=DEV)
    mon.mean_state(w, w_t0, xi)
    n, p, sk = mon.mean_numpy()
    ref = O.mean_state(S.slab_to_numpy(w), dtype, w_t0.cpu().numpy(), xi.cpu().numpy(), coef, m)
    assert K & (K - 1) == 0
    assert n == ref["n"] and p == ref["p"]
    assert np.array_equal(sk.astype(np.float64), ref["sk"])
    assert mon.last_mean_state_path() == 0
    mon.close()


def test_mean_state_equals_average_of_local_states():
    """Linearity (Section 3.1) on the device's own numbers: both entry points quantize a drift
    the same way and add integers, so the mean state is the average of the K states up to the
    fp32 roundings of the K stored states (and the estimate agrees)."""
    say("[case] mean state vs average of the per-worker states")
    for name, d in (("cfg3", 400_003), ("cfg5", 900_001)):
        wl = S.make(name, device=DEV, seed=4, d=d)
        mon = monitor_for(wl)
        mon.local_state(wl.w, wl.w_t0, wl.xi)
        n, p, sk = mon.state_numpy()
        e1 = mon.estimate_variance(1e-9)
        mon.mean_state(wl.w, wl.w_t0, wl.xi)
        nb, pb, skb = mon.mean_numpy()
        e2 = mon.estimate_variance_mean(1e-9)
        assert mon.last_state_path() == 0 and mon.last_mean_state_path() == 0
        assert mon.estimate_variance_mean(1e30).state_path == 0
        assert nb == pytest.approx(n.astype(np.float64).mean(), rel=1e-6)
        w32 = wl.w.float() if wl.dtype == "bf16" else wl.w
        p_abs = float(((w32 - wl.w_t0).abs() * wl.xi.abs()).sum(dim=1).double().mean())
        assert abs(pb - p.astype(np.float64).mean()) <= 2e-6 * p_abs
        avg = sk.astype(np.float64).mean(axis=0)
        assert np.allclose(skb, avg, rtol=0, atol=2e-7 * np.abs(sk).mean(axis=0).max())
        assert e2.h_sketch == pytest.approx(e1.h_sketch, rel=1e-5)
        assert e2.h_linear == pytest.approx(e1.h_linear, rel=1e-5)
        assert (e2.sync_sketch, e2.sync_linear) == (e1.sync_sketch, e1.sync_linear)
        mon.close()


def test_mean_state_bit_reproducible():
    say("[case] mean state run-to-run bits")
    wl = S.make("cfg5", device=DEV, seed=5, d=2_000_003)
    mon = monitor_for(wl)
    a = mon.mean_state(wl.w, wl.w_t0, wl.xi).clone()
    for _ in range(3):
        b = mon.mean_state(wl.w, wl.w_t0, wl.xi)
        assert torch.equal(a, b)
    mon.close()


def test_mean_state_out_of_range_drifts_take_fp64_path():
    """A few drifts far above the sampled magnitudes cannot be held by the 32-bit terms: the call
    must notice, redo the sketch in fp64 and still meet the tolerance."""
    say("[case] mean-state fp64 path")
    wl = S.make("cfg3", device=DEV, seed=6, d=250_007, K=6)
    # coordinates the strided sample of the scale does not visit
    step = wl.d // 16384
    for k, j in ((0, 1), (3, 7 * step + 3), (5, wl.d - 2)):
        wl.w[k, j] += 4.0e3
    mon = monitor_for(wl)
    mon.mean_state(wl.w, wl.w_t0, wl.xi)
    assert mon.last_mean_state_path() == 1
    check_mean(mon, oracle_mean(wl))
    # and the next call on ordinary data is back on the integer path
    wl2 = S.make("cfg3", device=DEV, seed=7, d=250_007, K=6)
    wl2.hash_coef = wl.hash_coef              # the context keeps the coefficients it was created with
    mon.mean_state(wl2.w, wl2.w_t0, wl2.xi)
    assert mon.last_mean_state_path() == 0
    check_mean(mon, oracle_mean(wl2))
    mon.close()


def test_mean_state_all_zero_and_nonfinite():
    say("[case] mean-state zero drift / non-finite")
    wl = S.make("cfg1", device=DEV, seed=8, d=20_011)
    w = wl.w_t0.repeat(wl.K, 1).contiguous()
    mon = monitor_for(wl)
    out = mon.mean_state(w, wl.w_t0, wl.xi)
    assert not out.any()
    est = mon.estimate_variance_mean(0.0)
    assert est.sync_sketch == 0 and est.sync_linear == 0 and est.nonfinite == 0
    w[2, 777] = float("inf")
    mon.mean_state(w, wl.w_t0, wl.xi)
    est = mon.estimate_variance_mean(1.0)
    assert est.nonfinite == 1 and est.sync_sketch == 1 and est.sync_linear == 1
    w[2, 777] = float("nan")
    mon.mean_state(w, wl.w_t0, wl.xi)
    est = mon.estimate_variance_mean(1.0)
    assert est.nonfinite == 1 and est.sync_sketch == 1 and est.sync_linear == 1
    mon.close()


def test_mean_state_unaligned_and_strided():
    """Slab rows that are not 16-byte aligned, and a row stride larger than d."""
    say("[case] mean-state unaligned / strided")
    import paper_2405_20988_amd as F
    wl = S.make("cfg3", device=DEV, seed=9, d=60_001, K=5)
    # strided rows
    stride = wl.d + 24
    buf = torch.zeros((wl.K, stride), dtype=wl.w.dtype, device=DEV)
    buf[:, :wl.d] = wl.w
    mon = monitor_for(wl, row_stride=stride)
    mon.mean_state(buf, wl.w_t0, wl.xi)
    ref = oracle_mean(wl)
    check_mean(mon, ref)
    mon.close()
    # rows that start 4 bytes off a 16-byte boundary, odd stride
    stride = wl.d + 3
    flat = torch.zeros(wl.K * stride + 1, dtype=wl.w.dtype, device=DEV)
    view = flat[1:].view(wl.K, stride)
    view[:, :wl.d] = wl.w
    mon = monitor_for(wl, row_stride=stride)
    mon.mean_state(view, wl.w_t0, wl.xi)
    check_mean(mon, ref)
    mon.close()


@pytest.mark.parametrize("name,d,over", [("cfg4", 250_003, {}), ("cfg5", 400_005, {}),
                                         ("cfg1", None, {}), ("cfg2", 9, {"K": 2}),
                                         ("cfg3", 120_001, {"K": 7})])
def test_sync_from_mean_parity(name, d, over):
    """fda_mean_state with w_bar, then fda_sync_from_mean: the average model, the broadcast, w_prev
    and xi (Algorithm 1 line 9, Section 3.2) against the oracle's sync and update_xi."""
    say(f"[case] sync-from-mean parity {name} d={d} {over}")
    wl = S.make(name, device=DEV, seed=5, d=d, **over)
    mon = monitor_for(wl)
    w_host = S.slab_to_numpy(wl.w)
    w0_host = wl.w_t0.cpu().numpy().copy()
    ref = O.sync(w_host, wl.dtype, w0_host)
    scale = np.abs(O.widen(w_host, wl.dtype)).max(axis=0)
    w_prev = torch.full_like(wl.w_t0, 7.0)
    xi = torch.zeros_like(wl.w_t0)
    w_bar = torch.full_like(wl.w_t0, -3.0)

    mon.mean_state(wl.w, wl.w_t0, wl.xi, w_bar=w_bar)
    torch.cuda.synchronize()
    check_mean(mon, oracle_mean(wl))                    # the extra output does not disturb the state
    wb_host = w_bar.cpu().numpy()
    assert (np.abs(wb_host.astype(np.float64) - ref["mean"]) <= RTOL * scale + 1e-30).all()

    # predicate 0: nothing may change
    mon.estimate_variance_mean(1e30)
    before = wl.w.clone()
    mon.sync_from_mean(wl.w, wl.w_t0, w_bar, w_prev=w_prev, xi=xi, pred="sketch")
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.uint8), wl.w.view(torch.uint8))
    assert np.array_equal(wl.w_t0.cpu().numpy(), w0_host)
    assert (w_prev == 7.0).all() and not xi.any()

    # predicate 1
    est = mon.estimate_variance_mean(0.0)
    assert est.sync_sketch == 1
    mon.sync_from_mean(wl.w, wl.w_t0, w_bar, w_prev=w_prev, xi=xi, pred="sketch")
    torch.cuda.synchronize()
    assert np.array_equal(w_prev.cpu().numpy(), ref["w_prev"])            # bit-exact copy
    assert np.array_equal(wl.w_t0.cpu().numpy(), wb_host)                 # w_t0 <- w_bar, bit-exact
    rows = S.slab_to_numpy(wl.w)
    assert (rows == rows[0]).all()                                        # every worker holds the same bits
    if wl.dtype == "f32":
        assert np.array_equal(rows[0], wb_host)
    else:
        diff = np.abs(rows[0].astype(np.int32) - ref["rows"].astype(np.int32))
        assert diff.max() <= 1
        assert (diff != 0).mean() < 1e-2
        assert np.array_equal(rows[0], O.round_to_bf16_bits(wb_host.astype(np.float64)))
    # xi from the last two synchronized models, as the device now holds them
    want_xi = O.update_xi(wl.w_t0.cpu().numpy(), w_prev.cpu().numpy())
    got_xi = xi.cpu().numpy().astype(np.float64)
    assert np.abs(got_xi - want_xi).max() <= RTOL * np.abs(want_xi).max()
    assert float(got_xi @ got_xi) == pytest.approx(1.0, rel=1e-5)
    # "after synchronization the model variance is zero"
    out = mon.mean_state(wl.w, wl.w_t0, xi)
    if wl.dtype == "f32":
        assert not out.any()
    # without w_prev and xi, no predicate
    mon.mean_state(wl.w, wl.w_t0, xi, w_bar=w_bar)
    mon.sync_from_mean(wl.w, wl.w_t0, w_bar)
    torch.cuda.synchronize()
    assert np.array_equal(wl.w_t0.cpu().numpy(), w_bar.cpu().numpy())
    mon.close()


def test_sync_from_mean_unaligned():
    """w_bar, w_prev and xi off the 16-byte grid and an odd row stride (vector accesses at element
    alignment); the padding between rows must stay untouched."""
    say("[case] sync-from-mean unaligned")
    import paper_2405_20988_amd as F
    K, d, l, m = 6, 10_007, 5, 250
    stride = d + 5
    g = torch.Generator(device=DEV)
    g.manual_seed(6)
    coef = S.hash_coefficients(6, l)
    for dtype, tdt in (("f32", torch.float32), ("bf16", torch.bfloat16)):
        buf = torch.full((K * stride + 3,), 9.0, device=DEV, dtype=tdt)
        w_t0 = torch.zeros(d + 1, device=DEV)[1:]
        xi = torch.zeros(d + 1, device=DEV)[1:]
        w_prev = torch.zeros(d + 1, device=DEV)[1:]
        w_bar = torch.zeros(d + 1, device=DEV)[1:]
        w_t0.copy_(torch.randn(d, generator=g, device=DEV) * 0.05)
        xi.copy_(torch.randn(d, generator=g, device=DEV) / d ** 0.5)
        full = buf[3:].view(K, stride)
        w = full[:, :d]
        w.copy_((w_t0 + torch.randn((K, d), generator=g, device=DEV) * 1e-3).to(tdt))
        wc = w.contiguous()
        w0_host = w_t0.cpu().numpy().copy()
        mon = F.FdaMonitor(K, d, dtype, 3, l, m, 0.06, coef, row_stride=stride, device=DEV)
        from paper_2405_20988_amd import binding as B
        st = torch.cuda.current_stream().cuda_stream
        B.fda_mean_state(mon.ctx, w.data_ptr(), w_t0.data_ptr(), xi.data_ptr(), mon.mean.data_ptr(),
                         w_bar.data_ptr(), st)
        ref = O.mean_state(S.slab_to_numpy(wc), dtype, w0_host, xi.cpu().numpy(), coef, m)
        check_mean(mon, ref)
        B.fda_sync_from_mean(mon.ctx, w.data_ptr(), w_t0.data_ptr(), w_prev.data_ptr(), xi.data_ptr(),
                             w_bar.data_ptr(), None, st)
        torch.cuda.synchronize()
        sref = O.sync(S.slab_to_numpy(wc), dtype, w0_host)
        scale = np.abs(O.widen(S.slab_to_numpy(wc), dtype)).max(axis=0)
        assert (np.abs(w_t0.cpu().numpy().astype(np.float64) - sref["mean"]) <= RTOL * scale).all()
        assert np.array_equal(w_prev.cpu().numpy(), w0_host)
        assert (full[:, d:] == 9.0).all() and (buf[:3] == 9.0).all()
        rows = S.slab_to_numpy(w.contiguous())
        assert (rows == rows[0]).all()
        want_xi = O.update_xi(w_t0.cpu().numpy(), w_prev.cpu().numpy())
        assert np.abs(xi.cpu().numpy() - want_xi).max() <= RTOL * np.abs(want_xi).max()
        mon.close()
