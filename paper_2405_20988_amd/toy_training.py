"""A toy run of Algorithm 1 around the FDA monitor: K workers descend their own quadratic
objectives and the monitor decides, step by step, when they must synchronize.

Only lines 6-9 of Algorithm 1 (state, estimate, decision, synchronization) run in the HIP
library; `Optimize` (line 5) is a stand-in written with torch operations: worker k minimizes
f_k(w) = 1/2 || a_k * (w - c_k) ||^2  (element-wise curvature a_k, its own optimum c_k) by noisy
gradient steps.  The global objective is the average of the f_k, minimized by the curvature-
weighted mean of the c_k; workers that never talk drift towards their own optima, workers that
synchronize at every step follow the global gradient (Section 3: the Synchronous special case
is Theta = 0).

    python -m paper_2405_20988_amd.toy_training [--K 8] [--d 200000] [--steps 200] [--variant sketch]
prints, for a ladder of thresholds, the number of synchronizations and the final global loss.
"""
from __future__ import annotations

import argparse
import math

import numpy as np
import torch

from .monitor import FdaMonitor


class ToyProblem:
    def __init__(self, K, d, device, seed=0, spread=0.05, noise=0.02, lr=0.2):
        g = torch.Generator(device=device)
        g.manual_seed(seed)
        self.K, self.d, self.lr, self.noise, self.gen = K, d, lr, noise, g
        self.a2 = 0.5 + torch.rand((K, d), generator=g, device=device)          # a_k^2 in [0.5, 1.5)
        shared = torch.randn(d, generator=g, device=device)
        self.c = shared + spread * torch.randn((K, d), generator=g, device=device)
        self.w_star = (self.a2 * self.c).sum(0) / self.a2.sum(0)                  # global optimum
        self.w0 = torch.zeros(d, device=device)

    def optimize(self, w):
        """One noisy gradient step of every worker on its own objective, in place."""
        grad = self.a2 * (w - self.c)
        w -= self.lr * (grad + self.noise * torch.randn(w.shape, generator=self.gen, device=w.device))

    def global_loss(self, v):
        return float((0.5 * self.a2 * (v[None, :] - self.c) ** 2).sum(1).mean())


def run(problem, theta, steps, variant="sketch", mean_state=True, l=5, m=250, eps=0.06, seed=0,
        check_invariant=False):
    """Returns (synchronization steps, final loss of the average model, largest variance seen
    right after a step that did not synchronize)."""
    dev = problem.w0.device
    K, d = problem.K, problem.d
    variants = 3
    # hash coefficients are data: any seeded uniform draw below the prime 2^31 - 1
    coef = np.random.default_rng(seed).integers(0, (1 << 31) - 1, size=(l, 2, 4), dtype=np.int64).astype(np.uint32)
    mon = FdaMonitor(K, d, "f32", variants, l, m, eps, coef, device=dev)
    w = problem.w0.repeat(K, 1).contiguous()
    w_t0, w_prev = problem.w0.clone(), problem.w0.clone()
    xi = torch.randn(d, generator=problem.gen, device=dev)
    xi /= xi.norm()
    syncs, worst = [], 0.0
    for t in range(steps):
        problem.optimize(w)
        est = mon.step(w, w_t0, w_prev, xi, theta, decide_by=variant, mean=mean_state, want_host=True)
        fired = est.sync_sketch if variant == "sketch" else est.sync_linear
        if fired:
            syncs.append(t)
        elif check_invariant:
            var = float(((w - w.mean(0, keepdim=True)) ** 2).sum(1).mean())
            worst = max(worst, var)
    loss = problem.global_loss(w.mean(0))
    mon.close()
    return syncs, loss, worst


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--K", type=int, default=8)
    ap.add_argument("--d", type=int, default=200_000)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--variant", choices=("sketch", "linear"), default="sketch")
    ap.add_argument("--per-worker-states", action="store_true")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    base = ToyProblem(args.K, args.d, dev)
    # the variance the workers reach if they never synchronize sets the scale of Theta
    ladder = [0.0] + [f * args.d * 1e-4 for f in (2.0, 8.0, 32.0, 128.0)] + [math.inf]
    print(f"K={args.K} d={args.d} steps={args.steps} variant={args.variant} "
          f"optimum loss={base.global_loss(base.w_star):.6f}")
    for theta in ladder:
        p = ToyProblem(args.K, args.d, dev)
        syncs, loss, _ = run(p, theta if math.isfinite(theta) else 1e300, args.steps, args.variant,
                             mean_state=not args.per_worker_states)
        print(f"Theta={theta:>10.4g}  synchronizations={len(syncs):>4d}  final global loss={loss:.6f}")


if __name__ == "__main__":
    main()
