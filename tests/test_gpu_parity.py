"""Parity of the HIP path (through the C ABI) with the CPU fp64 oracle, element by element,
on the same seeded input bits.

Tolerances (fp32 kernels against the fp64 oracle):
  ||u_k||^2, M2, sync outputs      relative 1e-5
  <xi,u_k>                         1e-5 * sum_j |xi_j u_kj|          (a cancelling sum)
  sketch cell                      1e-5 * sum_{j in cell} |u_kj|     (a cancelling sum) on every cell
                                   whose sum of |u_kj| is at least half of n_cell * mean_j |u_kj|;
                                   the nearly empty rest: 1e-5 * (that sum + n_cell * mean_j |u_kj|)
                                   (tests/fda_tolerance.py states why)
  H                                1e-5 * mean_k ||u_k||^2           (a difference of O(n) terms)
  decision                         identical, except inside the near-tie band
Integer-valued inputs make every fp32 sum exact, so there everything must be bit-identical;
that is how bucket indices and signs are checked for every coordinate.
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


def monitor_for(wl, variants=3, row_stride=None, flags=0):
    import paper_2405_20988_amd as F
    return F.FdaMonitor(wl.K, wl.d, wl.dtype, variants, wl.l, wl.m, wl.eps, wl.hash_coef,
                        row_stride=row_stride, device=DEV, flags=flags)


def oracle_state(wl, variants=3):
    w = S.slab_to_numpy(wl.w)
    return O.local_state(w, wl.dtype, wl.w_t0.cpu().numpy(),
                         wl.xi.cpu().numpy() if variants & 1 else None,
                         wl.hash_coef if variants & 2 else None, wl.m)


def check_state(mon, ref, variants=3):
    n, p, sk = mon.state_numpy()
    assert np.allclose(n, ref["n"], rtol=RTOL, atol=0), np.max(np.abs(n / ref["n"] - 1))
    if variants & 1:
        err = np.abs(p - ref["p"])
        assert (err <= RTOL * ref["p_abs"] + 1e-30).all(), (err / ref["p_abs"]).max()
    else:
        assert not p.any()
    if variants & 2:
        worst, dense = check_cells(sk, ref["sk"], ref["sk_abs"], ref["sk_cnt"], ref["u_mean_abs"])
        say(f"       sketch cells: worst error {worst:.3f} of 1e-5 * sum|u| "
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


# name, d, overrides: sizes the oracle finishes in seconds, several tiles per workgroup where
# the partition count saturates, and a ragged tail (d not a multiple of the vector width)
STATE_CASES = [
    ("cfg1", None, {}),                       # the full first configuration
    ("cfg2", 1_200_003, {}),
    ("cfg3", 300_007, {}),
    ("cfg4", 150_001, {}),
    ("cfg5", 1_100_005, {}),
    ("cfg5", 4099, {}),
    ("cfg1", 7, {"K": 3}),
    ("cfg2", 70_001, {"K": 1}),
    ("cfg3", 50_000, {"K": 17}),              # two unequal worker groups (9 + 8)
    ("cfg4", 40_003, {"K": 33, "l": 4}),      # even number of rows
    ("cfg1", 30_001, {"l": 16, "m": 64}),
    ("cfg1", 30_001, {"l": 1, "m": 1}),
    ("cfg2", 20_000, {"K": 3, "l": 1, "m": 19_000}),   # one worker per group: sketch fills LDS
    ("cfg1", 5_000, {"K": 300, "l": 3, "m": 64}),      # many workers: 38 worker groups
    # which kind of LDS rows the 32-bit-cell pass uses (expected plan: worker slots, sign-split rows)
    ("cfg2", 30_011, {"K": 2, "l": 3, "m": 6_000}),     # two workers in one 8-byte word, LDS too small to split the signs
    ("cfg2", 30_011, {"K": 4, "l": 2, "m": 4_500}),     # two groups of two rather than four slots: split rows fit
    ("cfg2", 30_011, {"K": 5, "l": 6, "m": 64}),        # 6 slots x 6 rows are not built: groups of 2, 2, 1 workers
    ("cfg2", 30_011, {"K": 5, "l": 5, "m": 64}),        # five workers in six slots: a spare high half
    ("cfg5", 40_009, {"K": 8, "l": 4, "m": 300}),       # bf16, eight slots
    ("cfg2", 20_011, {"K": 2, "l": 1, "m": 20_000}),    # about the widest sketch the LDS takes: 16-bit table fields up to 2 m - 1
]
EXPECTED_ROWS = {(2, 3, 6_000): (2, 0), (4, 2, 4_500): (2, 1), (5, 6, 64): (2, 1), (5, 5, 64): (6, 1), (8, 4, 300): (8, 1)}
PLAIN_TABLE_CASES = {(5, 5, 64)}        # planned without placed rows (FDA_DESC_PLAIN_TABLE): the same kernel on the plain table


@pytest.mark.parametrize("name,d,over", STATE_CASES)
def test_state_and_estimate_parity(name, d, over):
    say(f"[case] state parity {name} d={d} {over}")
    wl = S.make(name, device=DEV, seed=1, d=d, **over)
    key = (wl.K, wl.l, wl.m)
    mon = monitor_for(wl, flags=1 if key in PLAIN_TABLE_CASES else 0)
    say(f"       plan {mon.plan}")
    if key in EXPECTED_ROWS and "K" in over:
        assert (mon.plan["worker_slots"], mon.plan["sign_split_rows"]) == EXPECTED_ROWS[key], mon.plan
    mon.local_state(wl.w, wl.w_t0, wl.xi)
    torch.cuda.synchronize()
    ref = oracle_state(wl)
    check_state(mon, ref)
    var = O.true_variance(O.widen(S.slab_to_numpy(wl.w), wl.dtype))
    for mult in (0.25, 0.5, 1.0, 2.0):
        theta = mult * var
        est = mon.estimate_variance(theta)
        want = O.estimate_variance(ref["n"], ref["p"], ref["sk"], wl.eps, theta)
        check_estimate(est, want)
    # Theorem 2 holds for the GPU's numbers too (up to the tolerance)
    est = mon.estimate_variance(var)
    assert est.h_linear >= var - RTOL * est.mean_sqnorm
    mon.close()


def test_drifts_that_lean_one_way():
    """Sign-split rows keep the terms of one hash sign in a cell, so drifts that lean one way do not cancel
    there.  The planner keeps such cells at about 3500 expected terms at most; with a sketch so narrow that
    every workgroup's cells are about that full, drifts with a third of their mass leaning one way must
    finish on the 32-bit cells, and drifts that are all positive must match the oracle whichever cells
    they end on."""
    say("[case] leaning drifts, sketch 3 x 2")
    import paper_2405_20988_amd as F
    K, d, l, m = 2, 3_584_007, 3, 2
    g = torch.Generator(device=DEV)
    g.manual_seed(77)
    coef = S.hash_coefficients(5, l)
    w_t0 = torch.randn(d, generator=g, device=DEV) * 0.05
    xi = torch.randn(d, generator=g, device=DEV) / d ** 0.5
    mon = F.FdaMonitor(K, d, "f32", 3, l, m, 0.06, coef, device=DEV)
    say(f"       plan {mon.plan}")
    assert mon.plan["sign_split_rows"] == 1
    assert 2 * m * 1_500 <= mon.plan["chunk"] <= 2 * m * 3_500 + 2048      # the cells do get about that full
    noise = torch.randn((K, d), generator=g, device=DEV)
    for what, drift in (("a third leaning", (noise + 0.3) * 1e-3), ("all positive", noise.abs() * 1e-3)):
        w = (w_t0 + drift).contiguous()
        mon.local_state(w, w_t0, xi)
        path = mon.last_state_path()
        say(f"       {what}: sketch cells of kind {path}")
        assert path == 0 if what == "a third leaning" else path in (0, 1)
        check_state(mon, O.local_state(w.cpu().numpy(), "f32", w_t0.cpu().numpy(), xi.cpu().numpy(), coef, m))
    mon.close()


@pytest.mark.parametrize("variants", [1, 2])
def test_single_variant(variants):
    say(f"[case] single variant {variants}")
    wl = S.make("cfg3", device=DEV, seed=2, d=90_001, K=30)
    mon = monitor_for(wl, variants)
    assert mon.S == (2 if variants == 1 else 2 + wl.l * wl.m)
    mon.local_state(wl.w, wl.w_t0, wl.xi if variants & 1 else None)
    ref = oracle_state(wl, variants)
    check_state(mon, ref, variants)
    theta = 0.5 * O.true_variance(O.widen(S.slab_to_numpy(wl.w), wl.dtype))
    est = mon.estimate_variance(theta)
    check_estimate(est, O.estimate_variance(ref["n"], ref["p"], ref["sk"], wl.eps, theta), variants)
    if variants == 1:
        assert est.h_sketch == 0 and est.sync_sketch == 0 and est.m2 == 0
    else:
        assert est.h_linear == 0 and est.sync_linear == 0
    mon.close()


@pytest.mark.parametrize("dtype,K,d,l,m", [("f32", 5, 200_003, 5, 250), ("f32", 60, 30_001, 5, 500),
                                            ("bf16", 8, 300_007, 7, 1000), ("f32", 16, 5, 3, 4)])
def test_integer_inputs_bit_exact(dtype, K, d, l, m):
    """Small-integer drifts: every partial sum is exact in fp32, so the whole state must equal
    the oracle bit for bit -- any wrong bucket or sign of any coordinate would show."""
    say(f"[case] integer inputs {dtype} K={K} d={d} {l}x{m}")
    import paper_2405_20988_amd as F
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    w_t0 = torch.randint(-16, 17, (d,), generator=g, device=DEV).float()
    u = torch.randint(-4, 5, (K, d), generator=g, device=DEV).float()
    xi = torch.randint(-2, 3, (d,), generator=g, device=DEV).float()
    w = (w_t0 + u).to(torch.float32 if dtype == "f32" else torch.bfloat16)
    coef = S.hash_coefficients(5, l)
    mon = F.FdaMonitor(K, d, dtype, 3, l, m, 0.06, coef, device=DEV)
    mon.local_state(w, w_t0, xi)
    n, p, sk = mon.state_numpy()
    ref = O.local_state(S.slab_to_numpy(w), dtype, w_t0.cpu().numpy(), xi.cpu().numpy(), coef, m)
    assert np.array_equal(n.astype(np.float64), ref["n"])
    assert np.array_equal(p.astype(np.float64), ref["p"])
    assert np.array_equal(sk.astype(np.float64), ref["sk"])
    mon.close()


def test_one_hot_probe_reports_bucket_and_sign():
    """A drift with a single non-zero coordinate puts +-1 in exactly one cell per row."""
    say("[case] one-hot probes")
    import paper_2405_20988_amd as F
    K, d, l, m = 8, 100_000, 7, 1000
    coef = S.hash_coefficients(11, l)
    w_t0 = torch.zeros(d, device=DEV)
    w = torch.zeros((K, d), device=DEV)
    probes = [0, 1, 4095, 4096, 65_537, 99_990, 99_998, 99_999]
    for k, j in enumerate(probes):
        w[k, j] = 1.0
    mon = F.FdaMonitor(K, d, "f32", 2, l, m, 0.03, coef, device=DEV)
    mon.local_state(w, w_t0)
    _, _, sk = mon.state_numpy()
    for k, j in enumerate(probes):
        for i in range(l):
            b, s = O.bucket_and_sign(coef[i], np.array([j]), m)
            row = sk[k, i]
            assert np.count_nonzero(row) == 1
            assert row[b[0]] == s[0]
    mon.close()


def test_estimate_kernel_on_given_states():
    """fda_estimate_variance alone, fed a synthetic state: fp64 arithmetic on both sides."""
    say("[case] estimate kernel on given states")
    import paper_2405_20988_amd as F
    rng = np.random.default_rng(4)
    for (K, l, m) in [(5, 5, 250), (60, 5, 500), (8, 7, 1000), (3, 4, 10), (1, 1, 1), (2, 16, 33)]:
        coef = S.hash_coefficients(0, l)
        mon = F.FdaMonitor(K, 1000, "f32", 3, l, m, 0.06, coef, device=DEV)
        st = rng.normal(size=(K, 2 + l * m)).astype(np.float32)
        st[:, 0] = np.abs(st[:, 0]) * 50 + 40
        state = torch.from_numpy(st).to(DEV)
        n, p, sk = st[:, 0], st[:, 1], st[:, 2:].reshape(K, l, m)
        for theta in (0.0, 30.0, 60.0, 1e9):
            est = mon.estimate_variance(theta, tie_tol=1e-12, state=state)
            want = O.estimate_variance(n, p, sk, 0.06, theta, tie_tol=1e-12)
            for key, val in want.items():
                got = getattr(est, key)
                if isinstance(val, float):
                    assert got == pytest.approx(val, rel=1e-12, abs=1e-12), key
                else:
                    assert got == val, key
        mon.close()


def test_estimate_flags():
    say("[case] estimate flags")
    import paper_2405_20988_amd as F
    mon = F.FdaMonitor(2, 100, "f32", 3, 1, 2, 0.0, S.hash_coefficients(0, 1), device=DEV)
    st = torch.tensor([[4.0, 1.0, 1.0, 0.0], [4.0, 1.0, 1.0, 0.0]], device=DEV)
    e = mon.estimate_variance(3.0, tie_tol=0.0, state=st)       # both estimates are exactly 3
    assert (e.h_linear, e.h_sketch) == (3.0, 3.0)
    assert (e.sync_linear, e.sync_sketch) == (0, 0)             # tie: no synchronization
    assert (e.near_tie_linear, e.near_tie_sketch) == (1, 1)
    e = mon.estimate_variance(np.nextafter(3.0, 0.0), tie_tol=0.0, state=st)
    assert (e.sync_linear, e.sync_sketch, e.near_tie_linear) == (1, 1, 0)
    st[0, 0] = float("nan")
    e = mon.estimate_variance(3.0, state=st)
    assert e.nonfinite == 1 and e.sync_linear == 1 and e.sync_sketch == 1
    st[0, 0] = float("inf")
    e = mon.estimate_variance(3.0, state=st)
    assert e.nonfinite == 1 and e.sync_linear == 1
    # zero drift and Theta = 0: 0 > 0 is false (the Synchronous special case only fires on drift)
    e = mon.estimate_variance(0.0, state=torch.zeros((2, 4), device=DEV))
    assert (e.sync_linear, e.sync_sketch, e.nonfinite) == (0, 0, 0)
    mon.close()


@pytest.mark.parametrize("name,d,over", [("cfg4", 250_003, {}), ("cfg5", 400_005, {}),
                                         ("cfg1", None, {}), ("cfg2", 9, {"K": 2})])
def test_sync_and_xi_parity(name, d, over):
    say(f"[case] sync parity {name} d={d} {over}")
    wl = S.make(name, device=DEV, seed=5, d=d, **over)
    mon = monitor_for(wl)
    w_host = S.slab_to_numpy(wl.w)
    w0_host = wl.w_t0.cpu().numpy().copy()
    ref = O.sync(w_host, wl.dtype, w0_host)
    w_prev = torch.full_like(wl.w_t0, 7.0)
    xi = torch.zeros_like(wl.w_t0)

    # predicate 0: nothing may change
    mon.estimate_variance(1e30)
    before = wl.w.clone()
    mon.sync(wl.w, wl.w_t0, w_prev, pred="sketch")
    mon.update_xi(wl.w_t0, w_prev, xi, pred="sketch")
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.uint8), wl.w.view(torch.uint8))
    assert np.array_equal(wl.w_t0.cpu().numpy(), w0_host)
    assert (w_prev == 7.0).all() and not xi.any()

    # predicate 1
    mon.local_state(wl.w, wl.w_t0, wl.xi)
    est = mon.estimate_variance(0.0)
    assert est.sync_sketch == 1
    mon.sync(wl.w, wl.w_t0, w_prev, pred="sketch")
    mon.update_xi(wl.w_t0, w_prev, xi, pred="sketch")
    torch.cuda.synchronize()
    assert np.array_equal(w_prev.cpu().numpy(), ref["w_prev"])            # bit-exact copy
    new_w0 = wl.w_t0.cpu().numpy().astype(np.float64)
    scale = np.abs(O.widen(w_host, wl.dtype)).max(axis=0)
    assert (np.abs(new_w0 - ref["mean"]) <= RTOL * scale + 1e-30).all()
    rows = S.slab_to_numpy(wl.w)
    assert (rows == rows[0]).all()                                        # every worker holds the same bits
    if wl.dtype == "f32":
        assert np.array_equal(rows[0], wl.w_t0.cpu().numpy())
    else:
        # at most one bf16 step away from the oracle's rounding of the exact mean
        diff = np.abs(rows[0].astype(np.int32) - ref["rows"].astype(np.int32))
        assert diff.max() <= 1
        assert (diff != 0).mean() < 1e-2
    # xi from the last two synchronized models, as the device now holds them
    want_xi = O.update_xi(wl.w_t0.cpu().numpy(), w_prev.cpu().numpy())
    got_xi = xi.cpu().numpy().astype(np.float64)
    assert np.abs(got_xi - want_xi).max() <= RTOL * np.abs(want_xi).max()
    assert float(got_xi @ got_xi) == pytest.approx(1.0, rel=1e-5)
    # "after synchronization the model variance is zero"
    mon.local_state(wl.w, wl.w_t0, xi)
    n, p, sk = mon.state_numpy()
    if wl.dtype == "f32":
        assert not n.any() and not p.any() and not sk.any()
        e = mon.estimate_variance(0.0)
        assert (e.h_linear, e.h_sketch, e.sync_linear, e.sync_sketch) == (0, 0, 0, 0)
    else:
        # a bf16 slab keeps the rounding residue bf16(mean) - mean as drift, equal for all workers
        ref2 = O.local_state(S.slab_to_numpy(wl.w), "bf16", wl.w_t0.cpu().numpy(), None, None, 0)
        assert np.allclose(n, ref2["n"], rtol=RTOL)
        assert (n == n[0]).all()
    # forced synchronization with no predicate and no w_prev
    mon.sync(wl.w, wl.w_t0, None, pred=None)
    torch.cuda.synchronize()
    mon.close()


@pytest.mark.parametrize("name,d,over", [("cfg4", 250_003, {}), ("cfg5", 400_005, {}), ("cfg3", 1_300_001, {}),
                                         ("cfg1", None, {}), ("cfg2", 9, {"K": 2})])
def test_sync_xi_equals_sync_then_update_xi(name, d, over):
    """The synchronization that also takes the norm (Algorithm 1 line 9 with Section 3.2): rows, w_t0 and
    w_prev to the bit, xi to the rounding of a norm added up in another order; nothing moves under a
    zero predicate; a second synchronization right after the first gives the zero vector."""
    say(f"[case] sync_xi vs sync + update_xi {name} d={d} {over}")
    wl = S.make(name, device=DEV, seed=15, d=d, **over)
    mon = monitor_for(wl)
    a = [wl.w.clone(), wl.w_t0.clone(), torch.full_like(wl.w_t0, 7.0), torch.full_like(wl.w_t0, 5.0)]
    b = [t.clone() for t in a]
    mon.local_state(wl.w, wl.w_t0, wl.xi)
    mon.estimate_variance(1e30)
    mon.sync_xi(*b, pred="sketch")
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8))
    mon.estimate_variance(0.0)
    mon.sync(a[0], a[1], a[2], pred="sketch")
    mon.update_xi(a[1], a[2], a[3], pred="sketch")
    mon.sync_xi(*b, pred="sketch")
    torch.cuda.synchronize()
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8))
    xa, xb = a[3].cpu().numpy().astype(np.float64), b[3].cpu().numpy().astype(np.float64)
    assert np.abs(xa - xb).max() <= 4e-7 * np.abs(xa).max()
    want_xi = O.update_xi(b[1].cpu().numpy(), b[2].cpu().numpy())
    assert np.abs(xb - want_xi).max() <= RTOL * np.abs(want_xi).max()
    assert float(xb @ xb) == pytest.approx(1.0, rel=1e-5)
    K = wl.w.shape[0]
    if wl.dtype == "f32" and K & (K - 1) == 0:
        # the rows are the model already: their mean (exact for such K) is the model again, and xi of no
        # change is the zero vector
        mon.sync_xi(*b, pred=None)
        torch.cuda.synchronize()
        assert torch.equal(b[1], b[2]) and not b[3].any()
    mon.close()


def test_xi_zero_difference_gives_zero_vector():
    say("[case] xi of a zero difference")
    import paper_2405_20988_amd as F
    d = 5000
    mon = F.FdaMonitor(2, d, "f32", 1, device=DEV)
    a = torch.randn(d, device=DEV)
    xi = torch.ones(d, device=DEV)
    mon.update_xi(a, a.clone(), xi)
    torch.cuda.synchronize()
    assert not xi.any()
    mon.close()


def test_unaligned_and_strided_slab():
    """Pointers off the 16-byte grid and a row stride that is not a multiple of the vector width:
    the vector accesses only assume the alignment of the element type (the bf16 rows here start on
    odd 2-byte offsets); results must not change."""
    say("[case] unaligned / strided slab")
    import paper_2405_20988_amd as F
    K, d, l, m = 6, 10_007, 5, 250
    stride = d + 5
    g = torch.Generator(device=DEV)
    g.manual_seed(6)
    coef = S.hash_coefficients(6, l)
    for dtype, tdt in (("f32", torch.float32), ("bf16", torch.bfloat16)):
        buf = torch.zeros(K * stride + 3, device=DEV, dtype=tdt)
        w0b = torch.zeros(d + 1, device=DEV)
        xib = torch.zeros(d + 1, device=DEV)
        w_t0, xi = w0b[1:], xib[1:]
        w_t0.copy_(torch.randn(d, generator=g, device=DEV) * 0.05)
        xi.copy_(torch.randn(d, generator=g, device=DEV) / d ** 0.5)
        w = buf[3:].view(K, stride)[:, :d]
        w.copy_((w_t0 + torch.randn((K, d), generator=g, device=DEV) * 1e-3).to(tdt))
        mon = F.FdaMonitor(K, d, dtype, 3, l, m, 0.06, coef, row_stride=stride, device=DEV)
        from paper_2405_20988_amd import binding as B
        B.fda_local_state(mon.ctx, w.data_ptr(), w_t0.data_ptr(), xi.data_ptr(), mon.state.data_ptr(),
                          torch.cuda.current_stream().cuda_stream)
        wc = w.contiguous()
        ref = O.local_state(S.slab_to_numpy(wc), dtype, w_t0.cpu().numpy(), xi.cpu().numpy(), coef, m)
        check_state(mon, ref)
        # synchronize the strided slab; the padding between rows must stay untouched
        w_prev = torch.zeros(d + 1, device=DEV)[1:]
        B.fda_sync(mon.ctx, w.data_ptr(), w_t0.data_ptr(), w_prev.data_ptr(), None,
                   torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        sref = O.sync(S.slab_to_numpy(wc), dtype, w_prev.cpu().numpy())
        assert np.abs(w_t0.cpu().numpy() - sref["mean"]).max() <= RTOL * 0.3
        full = buf[3:].view(K, stride)
        assert not full[:, d:].any()
        assert torch.equal(full[0, :d], full[K - 1, :d])
        mon.close()


def test_simulated_run_cfg2_like():
    """T steps of Algorithm 1 lines 6-9 with the decision kept on the device: the sequence of
    synchronization steps must equal the oracle's (outside near ties), for both variants."""
    say("[case] simulated run (cfg2-like)")
    _simulate("cfg2", d=120_001, T=40, target_syncs=5, variant="sketch")
    _simulate("cfg2", d=120_001, T=40, target_syncs=5, variant="linear")


def test_simulated_run_cfg5_like():
    say("[case] simulated run (cfg5-like, bf16)")
    _simulate("cfg5", d=150_003, T=20, target_syncs=4, variant="sketch")


@pytest.mark.parametrize("mode", ["step", "step_mean", "step_mean_wbar"])
def test_simulated_run_through_fda_step(mode):
    """The same trajectories driven by the one-call step (per-worker states; the average state by
    linearity; the latter with the write-only synchronization)."""
    say(f"[case] simulated run through fda_step ({mode})")
    _simulate("cfg2", d=90_001, T=30, target_syncs=4, variant="sketch", mode=mode)
    _simulate("cfg5", d=100_003, T=16, target_syncs=3, variant="sketch", mode=mode)
    if mode != "step_mean_wbar":
        _simulate("cfg2", d=90_001, T=30, target_syncs=4, variant="linear", mode=mode)


def _simulate(name, d, T, target_syncs, variant, mode="calls"):
    wl = S.make(name, device=DEV, seed=7, d=d)
    # the oracle runs its own trajectory on host copies of the same starting bits and noise
    w_o = S.slab_to_numpy(wl.w)
    w0_o = wl.w_t0.cpu().numpy().copy()
    xi_o = wl.xi.cpu().numpy().copy()
    lat_o = wl.latent.cpu().numpy().copy() if wl.latent is not None else None
    key = "h_" + variant
    var_bit = 1 if variant == "linear" else 2

    # pass 1 (oracle only): how fast H grows from a freshly synchronized state, to pick a
    # Theta that is crossed about every T / target_syncs steps
    gen_state = wl.gen.get_state()
    s0 = O.sync(w_o, wl.dtype, w0_o)
    w_tmp = np.tile(s0["rows"], (wl.K, 1))
    w0_tmp = s0["mean"].astype(np.float32)
    xi_tmp = O.update_xi(w0_tmp, w0_o).astype(np.float32)
    lat_tmp = O.widen(w_tmp, "bf16").astype(np.float32) if lat_o is not None else None
    hs = []
    for t in range(T // target_syncs):
        w_tmp, lat_tmp = _apply_noise(w_tmp, lat_tmp, _draw_noise(wl), wl.dtype)
        st = O.local_state(w_tmp, wl.dtype, w0_tmp, xi_tmp if var_bit == 1 else None,
                           wl.hash_coef if var_bit == 2 else None, wl.m)
        hs.append(O.estimate_variance(st["n"], st["p"], st["sk"], wl.eps, 0.0)[key])
    theta = 0.5 * (hs[-1] + hs[-2])
    wl.gen.set_state(gen_state)

    mon = monitor_for(wl, var_bit)
    w_prev = wl.w_t0.clone()
    w_bar = torch.empty_like(wl.w_t0)
    w_prev_o = w0_o.copy()
    sync_steps_gpu, sync_steps_or, ties = [], [], []
    for t in range(T):
        noise = _draw_noise(wl)
        # device side
        noise_dev = torch.from_numpy(noise).to(DEV)
        if wl.dtype == "bf16":
            wl.latent += noise_dev
            wl.w.copy_(wl.latent.to(torch.bfloat16))
        else:
            wl.w += noise_dev
        if mode == "calls":
            mon.local_state(wl.w, wl.w_t0, wl.xi if var_bit == 1 else None)
            mon.estimate_variance(theta, want_host=False)
            mon.sync(wl.w, wl.w_t0, w_prev, pred=variant)
            mon.update_xi(wl.w_t0, w_prev, wl.xi, pred=variant)
            est = mon.estimate_variance(theta)          # same inputs again, now read back
        else:
            est = mon.step(wl.w, wl.w_t0, w_prev, wl.xi, theta, decide_by=variant,
                           mean=mode != "step", w_bar=w_bar if mode == "step_mean_wbar" else None,
                           want_host=True)
        if est.__getattribute__("sync_" + variant):
            sync_steps_gpu.append(t)
            wl.after_sync()
        # oracle side
        w_o, lat_o = _apply_noise(w_o, lat_o, noise, wl.dtype)
        st = O.local_state(w_o, wl.dtype, w0_o, xi_o if var_bit == 1 else None,
                           wl.hash_coef if var_bit == 2 else None, wl.m)
        want = O.estimate_variance(st["n"], st["p"], st["sk"], wl.eps, theta)
        assert abs(getattr(est, key) - want[key]) <= 2 * RTOL * want["mean_sqnorm"], t
        if want["near_tie_" + variant]:
            ties.append(t)
        if want["sync_" + variant]:
            sync_steps_or.append(t)
            s = O.sync(w_o, wl.dtype, w0_o)
            w_prev_o = s["w_prev"]
            w0_o = s["mean"].astype(np.float32)
            w_o = np.tile(s["rows"], (wl.K, 1))
            xi_o = O.update_xi(w0_o, w_prev_o).astype(np.float32)
            if lat_o is not None:
                lat_o = O.widen(w_o, "bf16").astype(np.float32)
        if ties:
            break                                    # trajectories may legitimately part here
    say(f"       theta={theta:.4e} gpu syncs {sync_steps_gpu} oracle syncs {sync_steps_or} ties {ties}")
    if not ties:
        assert sync_steps_gpu == sync_steps_or
        assert 2 <= len(sync_steps_or) <= 3 * target_syncs
        if var_bit == 1:
            # The two trajectories hold fp32 models that differ by a few roundings of the fp32 mean
            # (at most ~8 ulp of the largest |w|); xi divides such differences by the norm of the
            # (small) model change, which is what sets the scale of the comparison.
            got = wl.xi.cpu().numpy().astype(np.float64)
            change = float(np.linalg.norm(w0_o.astype(np.float64) - w_prev_o.astype(np.float64)))
            assert np.abs(got - xi_o).max() <= 8 * 2.0 ** -24 * float(np.abs(w0_o).max()) / change
    mon.close()


def _draw_noise(wl):
    out = np.empty((wl.K, wl.d), np.float32)
    for k in range(wl.K):
        out[k] = S._noise(wl.d, wl.step_std, wl.heavy_tail,
                          wl.gen, wl.w.device).cpu().numpy()
    return out


def _apply_noise(w, latent, noise, dtype):
    if dtype == "bf16":
        latent = latent + noise
        return O.round_to_bf16_bits(latent.astype(np.float64)), latent
    return w + noise, None


@pytest.mark.parametrize("name,d,over", [("cfg5", 700_003, {}), ("cfg4", 150_001, {}), ("cfg3", 300_007, {}),
                                         ("cfg5", 5_001, {"K": 2, "l": 9, "m": 250}), ("cfg1", None, {"l": 3, "m": 1024}),
                                         ("cfg2", 100_001, {"K": 2, "l": 8, "m": 500}),
                                         ("cfg5", 9_001, {"K": 2, "l": 11, "m": 700}),
                                         ("cfg5", 9_001, {"K": 6, "l": 7, "m": 2048}),
                                         ("cfg2", 100_001, {}),                               # four slots: a layout with a skew
                                         ("cfg5", 40_009, {"K": 8, "l": 4, "m": 300}),         # eight slots
                                         ("cfg2", 50_001, {"K": 4, "l": 5, "m": 251}),         # rows of 502 buckets take up 504
                                         ("cfg2", 50_001, {"K": 7, "l": 3, "m": 1023}),
                                         ("cfg5", 20_001, {"K": 8, "l": 3, "m": 251})])
def test_placed_rows_give_the_same_state(name, d, over):
    """A table whose row slots are chosen per coordinate (against LDS collisions) and the plain table:
    the same cells receive the same integer terms, so the states agree bit for bit -- and with the oracle."""
    say(f"[case] placed rows vs plain table {name} d={d} {over}")
    import paper_2405_20988_amd as F
    wl = S.make(name, device=DEV, seed=21, d=d, **over)
    placed = monitor_for(wl)
    plain = F.FdaMonitor(wl.K, wl.d, wl.dtype, 3, wl.l, wl.m, wl.eps, wl.hash_coef, device=DEV,
                         flags=F.FDA_DESC_PLAIN_TABLE)
    assert placed.plan["placed_row_group"] >= 2 and plain.plan["placed_row_group"] == 0
    for mon in (placed, plain):
        mon.local_state(wl.w, wl.w_t0, wl.xi)
    torch.cuda.synchronize()
    assert torch.equal(placed.state.view(torch.int32), plain.state.view(torch.int32))
    check_state(placed, oracle_state(wl))
    placed.close()
    plain.close()


def test_state_is_bit_reproducible():
    """The sketch cells are accumulated as integers and merged in a fixed order, the scalar
    components are reduced in a fixed shape: two runs must agree bit for bit."""
    say("[case] run-to-run reproducibility")
    wl = S.make("cfg3", device=DEV, seed=9, d=400_003)
    mon = monitor_for(wl)
    mon.local_state(wl.w, wl.w_t0, wl.xi)
    first = mon.state.clone()
    for _ in range(3):
        mon.local_state(wl.w, wl.w_t0, wl.xi)
        assert torch.equal(first.view(torch.int32), mon.state.view(torch.int32))
    mon.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_drifts_outside_the_sampled_range(dtype):
    """Drifts the sampled scale cannot represent -- isolated spikes 2^20 times larger than
    everything the sample sees, or a drift that is zero at every sampled coordinate -- must
    still give the oracle's sketch (the fp64 pass takes over)."""
    say(f"[case] out-of-range drifts {dtype}")
    import paper_2405_20988_amd as F
    K, d, l, m = 6, 300_000, 5, 250
    g = torch.Generator(device=DEV)
    g.manual_seed(10)
    coef = S.hash_coefficients(10, l)
    w_t0 = torch.randn(d, generator=g, device=DEV) * 0.05
    xi = torch.randn(d, generator=g, device=DEV) / d ** 0.5
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    for kind in ("spikes", "sparse"):
        if kind == "spikes":
            u = torch.randn((K, d), generator=g, device=DEV) * 1e-6
            u[1, 12_345] = 3.0
            u[4, 299_999] = -2.5
        else:
            u = torch.zeros((K, d), device=DEV)
            u[0, 7] = 1.0
            u[3, 100_001] = -0.25
            u[5, 250_003] = 0.5
        w = (w_t0 + u).to(tdt)
        if dtype == "bf16":
            w_t0_used = w_t0.to(torch.bfloat16).float() if kind == "sparse" else w_t0
        else:
            w_t0_used = w_t0
        mon = F.FdaMonitor(K, d, dtype, 3, l, m, 0.06, coef, device=DEV)
        mon.local_state(w, w_t0_used, xi)
        ref = O.local_state(S.slab_to_numpy(w), dtype, w_t0_used.cpu().numpy(), xi.cpu().numpy(), coef, m)
        check_state(mon, ref)
        # the 32-bit cells cannot hold these; fp32 spikes 10^6 times the rest need the fp64 cells
        # (with a bf16 slab the rounding residue narrows the range: which of the two wider kinds
        # takes over there depends on what the sample of the scale happens to see)
        assert mon.last_state_path() >= 1
        assert mon.estimate_variance(1e30).state_path == mon.last_state_path()
        if dtype == "f32" and kind == "spikes":
            assert mon.last_state_path() == 2
        mon.close()


def test_sketch_cell_paths():
    """The three kinds of sketch cell: ordinary drifts stay on the 32-bit cells; a few drifts
    thousands of times the mean go to the 64-bit cells; a 32-bit cell that leaves its safe band
    is noticed while the pass runs and the 64-bit cells redo the sketch."""
    say("[case] sketch cell paths")
    import paper_2405_20988_amd as F
    g = torch.Generator(device=DEV)
    g.manual_seed(12)
    # (a) ordinary
    wl = S.make("cfg4", device=DEV, seed=12, d=100_003)
    mon = monitor_for(wl)
    mon.local_state(wl.w, wl.w_t0, wl.xi)
    assert mon.last_state_path() == 0
    assert mon.estimate_variance(1e30).state_path == 0          # the same, reported without a stream wait
    check_state(mon, oracle_state(wl))
    mon.close()
    # (b) two drifts per worker 8000 times the mean, every coordinate sampled
    K, d, l, m = 4, 16_000, 5, 250
    coef = S.hash_coefficients(12, l)
    w_t0 = torch.zeros(d, device=DEV)
    u = torch.randn((K, d), generator=g, device=DEV) * 1e-6
    for k in range(K):
        u[k, 100 + k] = 1.0
        u[k, 9_000 + k] = -1.0
    xi = torch.randn(d, generator=g, device=DEV) / d ** 0.5
    mon = F.FdaMonitor(K, d, "f32", 3, l, m, 0.06, coef, device=DEV)
    mon.local_state(u, w_t0, xi)
    assert mon.last_state_path() == 1
    assert mon.estimate_variance(1e30).state_path == 1
    check_state(mon, O.local_state(u.cpu().numpy(), "f32", w_t0.cpu().numpy(), xi.cpu().numpy(), coef, m))
    mon.close()
    # (c) every coordinate in one bucket with one sign and equal positive drifts: the cell of a
    # workgroup collects 12288 terms of about 2^17.5 units and leaves [2^30, 3*2^30)
    d, m = 256 * 12_288, 4
    coef = np.array([[[1 << 30, 0, 0, 0], [0, 0, 0, 0]]], np.uint32)      # bucket 2, sign +1
    w_t0 = torch.zeros(d, device=DEV)
    w = torch.full((1, d), 0.5, device=DEV)
    mon = F.FdaMonitor(1, d, "f32", 2, 1, m, 0.06, coef, device=DEV)
    assert mon.plan["chunk"] == 12_288, mon.plan      # beyond 16384 terms a cell the call would not try 32-bit cells
    mon.local_state(w, w_t0)
    assert mon.last_state_path() == 1
    n, _, sk = mon.state_numpy()
    assert sk[0, 0].tolist() == [0.0, 0.0, 0.5 * d, 0.0]
    assert n[0] == 0.25 * d
    mon.close()
    # (d) the same with two workers, whose cells of a bucket are the two halves of one 8-byte word that
    # takes both additions at once: either half leaving its band, upwards or downwards (the low half
    # then borrows from the high one), must send the call to the 64-bit cells
    tiny = 2.0 ** -12
    for drifts in ((0.5, tiny), (-0.5, tiny), (tiny, 0.5), (tiny, -0.5), (-0.5, -0.5)):
        w = torch.empty((2, d), device=DEV)
        w[0].fill_(drifts[0])
        w[1].fill_(drifts[1])
        mon = F.FdaMonitor(2, d, "f32", 2, 1, m, 0.06, coef, device=DEV)
        assert mon.plan["workers_per_group"] == 2 and mon.plan["chunk"] == 12_288, mon.plan
        mon.local_state(w, w_t0)
        assert mon.last_state_path() == 1, drifts
        n, _, sk = mon.state_numpy()
        for k in range(2):
            assert sk[k, 0].tolist() == [0.0, 0.0, drifts[k] * d, 0.0], (drifts, k)
            assert n[k] == drifts[k] ** 2 * d
        mon.close()
    # ... and while both halves stay inside their bands they are exact and independent, whatever the
    # signs of the terms: drifts of alternating sign (the low half is added to and subtracted from all
    # the time), opposite in the two workers, a few coordinates changed by hand
    alt = torch.where(torch.arange(d, device=DEV) % 2 == 0, 2.0 ** -6, -(2.0 ** -6))
    w = torch.stack([alt, -alt]).contiguous()
    w[0, 5] = 2.0 ** -6
    w[1, 8] = -3 * 2.0 ** -6
    w[1, 77] = 5 * 2.0 ** -6
    mon = F.FdaMonitor(2, d, "f32", 2, 1, m, 0.06, coef, device=DEV)
    mon.local_state(w, w_t0)
    assert mon.last_state_path() == 0
    n, _, sk = mon.state_numpy()
    want = w.double().sum(dim=1).cpu().numpy()
    assert want.tolist() == [2.0 ** -5, -2.0 ** -5 + 2.0 ** -4]          # +2/64 and -2/64 + 4/64
    for k in range(2):
        assert sk[k, 0].tolist() == [0.0, 0.0, want[k], 0.0], k
    mon.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sync_propagates_nonfinite_values(dtype):
    """A NaN or an infinity in one worker's parameters must reach the average (and every row)
    instead of being rounded away -- in particular through the bf16 rounding of the stored rows."""
    say(f"[case] sync with non-finite parameters {dtype}")
    import paper_2405_20988_amd as F
    K, d = 4, 4099
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = torch.Generator(device=DEV)
    g.manual_seed(31)
    w = (torch.randn((K, d), generator=g, device=DEV) * 0.05).to(tdt)
    w[1, 5] = float("nan")
    w[2, 77] = float("inf")
    w[3, 78] = float("-inf")
    w[0, 4000] = float("inf")
    w[1, 4000] = float("-inf")                     # inf - inf: NaN
    w_t0 = torch.zeros(d, device=DEV)
    mon = F.FdaMonitor(K, d, dtype, 1, device=DEV)
    with np.errstate(invalid="ignore"):          # inf - inf in the oracle's mean is the point
        ref = O.sync(S.slab_to_numpy(w), dtype, w_t0.cpu().numpy())
    mon.sync(w, w_t0, None)
    torch.cuda.synchronize()
    got = w_t0.cpu().numpy()
    want = ref["mean"]
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isposinf(got), np.isposinf(want)) and np.array_equal(np.isneginf(got), np.isneginf(want))
    fin = np.isfinite(want)
    assert np.allclose(got[fin], want[fin], rtol=RTOL, atol=1e-7)
    rows = w.float().cpu().numpy()
    assert np.isnan(rows[:, 5]).all() and np.isnan(rows[:, 4000]).all()
    assert np.isposinf(rows[:, 77]).all() and np.isneginf(rows[:, 78]).all()
    assert np.isfinite(rows[:, :5]).all()
    mon.close()
