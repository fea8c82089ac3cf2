"""fda_step (Algorithm 1 lines 6-9 as one enqueue) against the same calls made one by one, and
the whole step under HIP graph capture and replay.  Parity with the oracle is established for
the individual calls elsewhere; here everything must agree bit for bit."""
import sys

import numpy as np
import pytest
import torch

import fda_synth as S

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def monitor_for(wl, variants=3):
    import paper_2405_20988_amd as F
    return F.FdaMonitor(wl.K, wl.d, wl.dtype, variants, wl.l, wl.m, wl.eps, wl.hash_coef, device=DEV)


def bits(t):
    return t.detach().contiguous().view(torch.uint8).cpu().numpy().copy()


def est_bytes(mon):
    torch.cuda.synchronize()
    return mon.est_dev.cpu().numpy().tobytes()


class Buffers:
    """One independent copy of a workload's tensors."""

    def __init__(self, wl):
        self.w, self.w_t0, self.xi = wl.w.clone(), wl.w_t0.clone(), wl.xi.clone()
        self.w_prev = torch.full_like(wl.w_t0, 3.0)
        self.w_bar = torch.zeros_like(wl.w_t0)

    def all_bits(self):
        return [bits(t) for t in (self.w, self.w_t0, self.xi, self.w_prev)]


def separate_calls(mon, b, theta, decide_by, mode):
    if mode == "workers":
        mon.local_state(b.w, b.w_t0, b.xi)
        mon.estimate_variance(theta, want_host=False)
    else:
        mon.mean_state(b.w, b.w_t0, b.xi, w_bar=b.w_bar if mode == "mean_wbar" else None)
        mon.estimate_variance_mean(theta, want_host=False)
    if mode == "mean_wbar":
        mon.sync_from_mean(b.w, b.w_t0, b.w_bar, w_prev=b.w_prev, xi=b.xi, pred=decide_by)
    else:
        mon.sync_xi(b.w, b.w_t0, b.w_prev, b.xi, pred=decide_by)


def one_step(mon, b, theta, decide_by, mode):
    return mon.step(b.w, b.w_t0, b.w_prev, b.xi, theta, decide_by=decide_by, mean=mode != "workers",
                    w_bar=b.w_bar if mode == "mean_wbar" else None)


@pytest.mark.parametrize("mode", ["workers", "mean", "mean_wbar"])
@pytest.mark.parametrize("name,d", [("cfg3", 200_003), ("cfg5", 300_001)])
def test_step_equals_separate_calls(name, d, mode):
    say(f"[case] fda_step vs separate calls {name} d={d} {mode}")
    wl = S.make(name, device=DEV, seed=11, d=d)
    mon_a, mon_b = monitor_for(wl), monitor_for(wl)
    for decide_by in ("sketch", "linear"):
        for theta in (1e30, 0.0):                      # no synchronization, then a forced one
            a, b = Buffers(wl), Buffers(wl)
            separate_calls(mon_a, a, theta, decide_by, mode)
            one_step(mon_b, b, theta, decide_by, mode)
            ea, eb = est_bytes(mon_a), est_bytes(mon_b)
            assert ea == eb
            st_a = mon_a.state if mode == "workers" else mon_a.mean
            st_b = mon_b.state if mode == "workers" else mon_b.mean
            assert np.array_equal(bits(st_a), bits(st_b))
            for x, y in zip(a.all_bits(), b.all_bits()):
                assert np.array_equal(x, y)
            changed = not np.array_equal(bits(b.w), bits(wl.w))
            assert changed == (theta == 0.0)
    mon_a.close()
    mon_b.close()


def test_step_argument_checks():
    import paper_2405_20988_amd as F
    from paper_2405_20988_amd import binding as B
    wl = S.make("cfg1", device=DEV, seed=12, d=5000)
    mon = F.FdaMonitor(wl.K, wl.d, wl.dtype, 2, wl.l, wl.m, wl.eps, wl.hash_coef, device=DEV)
    w_prev = wl.w_t0.clone()
    with pytest.raises(F.FdaError):                    # LINEAR is not one of the context's variants
        mon.step(wl.w, wl.w_t0, w_prev, wl.xi, 1.0, decide_by="linear")
    with pytest.raises(F.FdaError):                    # xi without w_prev
        mon.step(wl.w, wl.w_t0, None, wl.xi, 1.0)
    with pytest.raises(F.FdaError):                    # w_bar without the mean-state flag
        mon.step(wl.w, wl.w_t0, w_prev, wl.xi, 1.0, w_bar=w_prev)
    with pytest.raises(F.FdaError):                    # unknown flag
        B.fda_step(mon.ctx, wl.w.data_ptr(), wl.w_t0.data_ptr(), None, None, mon.state.data_ptr(), None,
                   1.0, 1e-5, B.FDA_VARIANT_SKETCH, 8, mon.est_dev.data_ptr())
    # no xi at all: allowed without LINEAR
    est = mon.step(wl.w, wl.w_t0, None, None, 1e30, want_host=True)
    assert est.sync_sketch == 0
    mon.close()


@pytest.mark.parametrize("mode", ["workers", "mean_wbar"])
def test_step_under_graph_capture(mode):
    """The library allocates nothing and records no memset, so a whole step can be captured in a
    HIP graph.  Every replay -- with eager work and synchronizations of the program in between --
    must leave exactly what the eager step leaves on the same inputs."""
    say(f"[case] fda_step under graph capture ({mode})")
    wl = S.make("cfg2", device=DEV, seed=13, d=150_001)
    mon_g, mon_e = monitor_for(wl), monitor_for(wl)
    g_buf, e_buf = Buffers(wl), Buffers(wl)
    theta_lo = 0.0
    noise = [torch.randn_like(wl.w) * 1e-4 for _ in range(4)]

    # eager warm-up on the capture stream: the once-per-context kernels must not be captured
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        scratch = Buffers(wl)
        one_step(mon_g, scratch, 1e30, "sketch", mode)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_step(mon_g, g_buf, theta_lo, "sketch", mode)
    torch.cuda.synchronize()
    for r in range(4):
        # program-side eager work between replays: move both slabs the same way
        g_buf.w += noise[r]
        e_buf.w += noise[r]
        torch.cuda.synchronize()
        graph.replay()
        one_step(mon_e, e_buf, theta_lo, "sketch", mode)
        torch.cuda.synchronize()
        assert est_bytes(mon_g) == est_bytes(mon_e), r
        for x, y in zip(g_buf.all_bits(), e_buf.all_bits()):
            assert np.array_equal(x, y), r
        st_g = mon_g.state if mode == "workers" else mon_g.mean
        st_e = mon_e.state if mode == "workers" else mon_e.mean
        assert np.array_equal(bits(st_g), bits(st_e)), r
    mon_g.close()
    mon_e.close()


def test_contexts_with_different_sketch_sizes_coexist():
    """Two contexts that use the same kernels with very different amounts of LDS, created large
    first and then small: the later one must not shrink what the earlier one may launch with."""
    say("[case] a large-sketch context stays usable after a small-sketch one is created")
    from oracle import fda_oracle as O
    big = S.make("cfg5", device=DEV, seed=14, d=100_003)           # 7 x 1000: 112 KB of LDS
    mon_big = monitor_for(big)
    small = S.make("cfg5", device=DEV, seed=15, d=50_001, K=2, l=7, m=8)   # same kernels (2 worker slots x 7

    def kernel_of(mon):
        return mon.plan["worker_slots"], mon.plan["rows_per_group"], mon.plan["sign_split_rows"]
    assert kernel_of(mon_big) == (2, 7, 1) and mon_big.plan["lds_bytes"] > 100_000    # rows per workgroup, split
    mon_small = monitor_for(small)                                                       # rows), ~2 KB of LDS
    assert kernel_of(mon_small) == kernel_of(mon_big) and mon_small.plan["lds_bytes"] < 10_000
    for mon, wl in ((mon_small, small), (mon_big, big), (mon_small, small)):
        mon.local_state(wl.w, wl.w_t0, wl.xi)
        mon.mean_state(wl.w, wl.w_t0, wl.xi)
        torch.cuda.synchronize()
        ref = O.local_state(S.slab_to_numpy(wl.w), wl.dtype, wl.w_t0.cpu().numpy(), wl.xi.cpu().numpy(),
                            wl.hash_coef, wl.m)
        n, _, _ = mon.state_numpy()
        assert np.allclose(n, ref["n"], rtol=1e-5)
        assert mon.mean_numpy()[0] == pytest.approx(float(ref["n"].mean()), rel=1e-5)
    mon_big.close()
    mon_small.close()
