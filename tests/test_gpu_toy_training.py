"""Algorithm 1 end to end on a toy problem (quadratic objectives per worker, Optimize written
with torch; lines 6-9 in the HIP library through fda_step): the qualitative behaviour the paper
reports and the guarantees its theorems give.

  * Theta = 0 is the Synchronous special case: every step synchronizes (Section 3).
  * A larger Theta never needs more synchronizations on the same trajectory start, and an
    unreachable Theta needs none (Section 4: fewer synchronizations at higher Theta).
  * Round invariant with LinearFDA (Thm 2: Var <= H_linear): after every step that did not
    synchronize the true model variance is at most Theta.
"""
import sys

import pytest
import torch

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_toy_training_thresholds_and_round_invariant():
    from paper_2405_20988_amd import toy_training as T
    dev = torch.device("cuda:0")
    K, d, steps = 6, 40_000, 40
    unit = d * 1e-4
    for variant in ("linear", "sketch"):
        counts = []
        for theta in (0.0, 0.25 * unit, unit, 4 * unit, 16 * unit, 1e300):
            p = T.ToyProblem(K, d, dev, seed=3)
            syncs, loss, worst = T.run(p, theta, steps, variant, mean_state=True,
                                       check_invariant=(variant == "linear"))
            say(f"[toy] {variant} Theta={theta:.4g} syncs={len(syncs)} loss={loss:.5f} worst var={worst:.4g}")
            counts.append(len(syncs))
            if variant == "linear":
                assert worst <= theta * (1 + 1e-5) + 1e-30
        assert counts[0] == steps and counts[-1] == 0
        assert all(a >= b for a, b in zip(counts, counts[1:])), counts
        assert counts[1] > counts[-2]                    # the ladder actually spans the behaviour


def test_toy_training_mean_state_and_per_worker_states_agree():
    from paper_2405_20988_amd import toy_training as T
    dev = torch.device("cuda:0")
    K, d, steps = 5, 30_001, 30
    for variant in ("linear", "sketch"):
        runs = []
        for mean_state in (True, False):
            p = T.ToyProblem(K, d, dev, seed=4)
            syncs, loss, _ = T.run(p, 1.5 * d * 1e-4, steps, variant, mean_state=mean_state)
            runs.append((syncs, loss))
        say(f"[toy] {variant}: {runs}")
        assert runs[0][0] == runs[1][0]
        assert runs[0][1] == pytest.approx(runs[1][1], rel=1e-4)
