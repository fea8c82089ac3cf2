"""The boundary from plain C: csrc/fda_c_example.c (compiled with the host C compiler, linked with
libfda.so and the HIP runtime, no Python or torch in the process) runs one step on a fixed
arithmetic pattern; its printed numbers are compared with the oracle's on the same pattern."""
import os
import subprocess
import sys

import numpy as np
import pytest

from fda_tolerance import cell_bounds
from oracle import fda_oracle as O

pytestmark = pytest.mark.gpu
RTOL = 1e-5


def pattern(K, d, l):
    j = np.arange(d, dtype=np.int64)
    w_t0 = (((j * 7 + 3) % 33 - 16) / 64.0).astype(np.float32)
    xi = (((j * 3 + 2) % 9 - 4) / 8.0).astype(np.float32)
    u = np.stack([(((j * 5 + k * 11 + 1) % 17 - 8) / 1024.0).astype(np.float32) for k in range(K)])
    coef = np.array([(1103515245 * (t + 1) + 12345) % 2147483647 for t in range(l * 8)],
                    np.uint32).reshape(l, 2, 4)
    return (w_t0[None, :] + u).astype(np.float32), w_t0, xi, coef


@pytest.mark.parametrize("K,d,l,m,theta", [(4, 100_003, 5, 250, 1e-3), (3, 5_000, 3, 64, 1e30)])
def test_c_example_against_oracle(K, d, l, m, theta):
    from paper_2405_20988_amd import build as B
    exe = B.EXAMPLE_PATH
    if not os.path.exists(exe):
        pytest.skip("the C example is not built (no host C compiler)")
    print(f"[case] C example K={K} d={d} {l}x{m} theta={theta}", flush=True)
    sys.stdout.flush()
    run = subprocess.run([exe, str(K), str(d), str(l), str(m), repr(theta)], capture_output=True, text=True,
                         timeout=120)
    assert run.returncode == 0, run.stderr
    got = {}
    for line in run.stdout.splitlines():
        name, value = line.split()
        got[name] = float(value)
    w, w_t0, xi, coef = pattern(K, d, l)
    st = O.local_state(w, "f32", w_t0, xi, coef, m)
    est = O.estimate_variance(st["n"], st["p"], st["sk"], 0.06, theta)
    assert got["state_floats"] == 2 + l * m
    for k in range(K):
        assert got[f"sqnorm_{k}"] == pytest.approx(st["n"][k], rel=RTOL)
        assert abs(got[f"proj_{k}"] - st["p"][k]) <= RTOL * st["p_abs"][k]
    bound, _ = cell_bounds(st["sk_abs"], st["sk_cnt"], st["u_mean_abs"])
    assert abs(got["sketch_0_0_0"] - st["sk"][0, 0, 0]) <= bound[0, 0, 0]
    nbar = est["mean_sqnorm"]
    assert got["mean_sqnorm"] == pytest.approx(nbar, rel=RTOL)
    for key in ("h_linear", "h_sketch"):
        assert abs(got[key] - est[key]) <= RTOL * nbar
        assert abs(got["mean_mode_" + key] - est[key]) <= RTOL * nbar
    assert got["m2"] == pytest.approx(est["m2"], rel=RTOL, abs=RTOL * nbar)
    assert got["nonfinite"] == 0
    if not est["near_tie_sketch"]:
        assert got["sync_sketch"] == est["sync_sketch"] == got["mean_mode_sync_sketch"]
    if not est["near_tie_linear"]:
        assert got["sync_linear"] == est["sync_linear"]
    if est["sync_sketch"] and not est["near_tie_sketch"]:
        s = O.sync(w, "f32", w_t0)
        want_xi = O.update_xi(s["mean"].astype(np.float32), w_t0)
        assert got["xi_sqnorm_after"] == pytest.approx(float(want_xi @ want_xi), rel=1e-5)
        assert got["w_t0_sum_after"] == pytest.approx(float(s["mean"].sum()), rel=1e-5, abs=1e-3)
    else:
        assert got["xi_sqnorm_after"] == pytest.approx(float(xi.astype(np.float64) @ xi.astype(np.float64)), rel=1e-6)
