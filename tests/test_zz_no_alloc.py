"""fda_estimate_variance_static (scratch in a static device array, nothing allocated) against
fda_estimate_variance (scratch in a context's workspace): the same kernel, so the 64-byte result must be
identical bit for bit -- on two calls in a row, the second with a smaller input, whose result must not
see anything the first call left in the shared array."""
import ctypes as C
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


def both_ways(K, l, m, variants, theta, seed, tie_tol=1e-5, eps=0.06):
    import paper_2405_20988_amd as F
    from paper_2405_20988_amd import binding as B
    rng = np.random.default_rng(seed)
    S_ = 2 + l * m if variants & 2 else 2
    st = rng.normal(size=(K, S_)).astype(np.float32)
    st[:, 0] = np.abs(st[:, 0]) * 50 + 40
    state = torch.from_numpy(st).to(DEV)
    mon = F.FdaMonitor(K, 1000, "f32", variants, l, m, eps, S.hash_coefficients(0, max(l, 1)), device=DEV)
    want = mon.estimate_variance(theta, tie_tol=tie_tol, state=state)
    want_bytes = bytearray(mon.est_dev.cpu().numpy().tobytes())
    # the last field says which sketch cells the context's last state pass used (none has run: 0);
    # the entry point without a context reports -1 there
    assert int.from_bytes(want_bytes[60:64], "little", signed=True) == (0 if variants & 2 else -1)
    want_bytes[60:64] = (-1).to_bytes(4, "little", signed=True)
    want_bytes = bytes(want_bytes)
    out = torch.full((C.sizeof(B.FdaEstimate),), 0xAB, dtype=torch.uint8, device=DEV)
    B.fda_estimate_variance_static(state.data_ptr(), K, l, m, variants, eps, theta, tie_tol, out.data_ptr(),
                                   torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got_bytes = out.cpu().numpy().tobytes()
    mon.close()
    return want, want_bytes, got_bytes


def test_static_scratch_estimate_equals_workspace_estimate():
    say("[case] fda_estimate_variance_static, two calls in a row (large, then small)")
    # the largest sketch the workspace path is built for in these tests, then a much smaller one
    want, a, b = both_ways(K=8, l=16, m=4000, variants=3, theta=30.0, seed=1)
    assert a == b
    assert want.m2 > 0 and want.nonfinite == 0
    want, a, b = both_ways(K=3, l=3, m=10, variants=3, theta=60.0, seed=2)
    assert a == b
    want, a, b = both_ways(K=5, l=0, m=0, variants=1, theta=10.0, seed=3)      # LinearFDA only: two floats per worker
    assert a == b and want.h_sketch == 0.0
    # again the large one: stale partial sums of the small calls must not matter either
    want, a, b = both_ways(K=60, l=5, m=500, variants=2, theta=1e9, seed=4)
    assert a == b and want.sync_sketch == 0


def test_static_scratch_rejects_sizes_beyond_its_maximum():
    from paper_2405_20988_amd import binding as B
    out = torch.zeros(C.sizeof(B.FdaEstimate), dtype=torch.uint8, device=DEV)
    st = torch.zeros(64, device=DEV)
    for bad in (dict(l=17, m=10), dict(l=5, m=32768), dict(l=0, m=10), dict(l=5, m=0)):
        with pytest.raises(B.FdaError) as e:
            B.fda_estimate_variance_static(st.data_ptr(), 2, bad["l"], bad["m"], 2, 0.06, 1.0, 1e-5, out.data_ptr(), 0)
        assert e.value.code == B.FDA_ERANGE
    with pytest.raises(B.FdaError) as e:
        B.fda_estimate_variance_static(None, 2, 1, 1, 2, 0.06, 1.0, 1e-5, out.data_ptr(), 0)
    assert e.value.code == B.FDA_EINVAL
