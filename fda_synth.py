"""Seeded synthetic inputs for the FDA state / variance-check / sync path.

This module only draws random numbers and shapes them like the workloads the
benchmark configurations name (K workers, d parameters, storage type, sketch size);
it contains none of the method's arithmetic.  Both the HIP library (through its
binding) and the CPU oracle are fed from here, each getting the same bits.

The five recipes stand in for the paper's training runs (Table 1: LeNet-5 62K,
VGG16* 2.6M, DenseNet121 6.9M, DenseNet201 18M, a large fine-tuned ConvNet): only K
and d are taken from them; parameters and drifts are random.

All tensors are created with a torch.Generator on the requested device, so the same
call gives CPU tensors for the oracle-only tests and HBM-resident tensors on a GPU.
(The two devices draw different bits; parity tests copy one set of bits to both sides.)
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

MERSENNE_P = (1 << 31) - 1

# name -> (K, d, storage, l, m, T steps)
CONFIGS = {
    "cfg1": dict(K=5, d=61_706, dtype="f32", l=5, m=250, T=1),
    "cfg2": dict(K=16, d=2_600_000, dtype="f32", l=5, m=250, T=100),
    "cfg3": dict(K=30, d=7_000_000, dtype="f32", l=5, m=250, T=1),
    "cfg4": dict(K=60, d=20_000_000, dtype="f32", l=5, m=500, T=1),
    "cfg5": dict(K=8, d=350_000_000, dtype="bf16", l=7, m=1000, T=20),
}


def default_eps(m: int) -> float:
    """Sketch error for width m: 6 % at m = 250 (the paper's measured point), scaled by
    the m = O(1/eps^2) law for other widths."""
    return 0.06 * math.sqrt(250.0 / m)


def hash_coefficients(seed: int, l: int) -> np.ndarray:
    """[l][2][4] uint32 polynomial coefficients, uniform in [0, 2^31 - 1).

    [i][0] = bucket polynomial of sketch row i, [i][1] = its sign polynomial,
    last index e = coefficient of j^e.  Any seeded source works; this one is numpy's
    PCG64 seeded with (seed, 0x5eed).
    """
    rng = np.random.default_rng([int(seed), 0x5EED])
    return rng.integers(0, MERSENNE_P, size=(l, 2, 4), dtype=np.int64).astype(np.uint32)


@dataclass
class Workload:
    name: str
    K: int
    d: int
    dtype: str                      # "f32" or "bf16": storage type of the slab
    l: int
    m: int
    eps: float
    T: int
    w: torch.Tensor                 # [K, d] slab (float32 or bfloat16)
    w_t0: torch.Tensor              # [d] float32
    xi: torch.Tensor                # [d] float32, unit norm
    hash_coef: np.ndarray           # [l][2][4] uint32
    step_std: float                 # per-step drift scale used by advance()
    heavy_tail: bool
    gen: torch.Generator = field(repr=False, default=None)
    latent: torch.Tensor = field(repr=False, default=None)   # fp32 master copy (bf16 slabs)

    def advance(self) -> None:
        """One simulated local-training step: every worker's parameters move by fresh
        noise (the stand-in for Optimize in Algorithm 1, line 5).  For a bf16 slab the
        move is applied to an fp32 master copy and the slab is its rounding, as in
        mixed-precision training."""
        for k in range(self.K):
            noise = _noise(self.d, self.step_std, self.heavy_tail, self.gen, self.w.device)
            if self.dtype == "bf16":
                self.latent[k] += noise
                self.w[k] = self.latent[k].to(torch.bfloat16)
            else:
                self.w[k] += noise

    def after_sync(self) -> None:
        """Call after the slab was synchronized in place: the master copy follows it."""
        if self.dtype == "bf16":
            self.latent.copy_(self.w.to(torch.float32))


def _normal(n, std, gen, device):
    return torch.randn(n, generator=gen, device=device, dtype=torch.float32) * std


def _student_t3(n, scale, gen, device):
    """Student-t with 3 degrees of freedom: z / sqrt(chi2_3 / 3)."""
    z = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
    c = torch.zeros(n, device=device, dtype=torch.float32)
    for _ in range(3):
        g = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
        c.addcmul_(g, g)
    z.div_(torch.sqrt(c.div_(3.0)).clamp_min_(1e-20))
    return z.mul_(scale)


def _noise(n, std, heavy, gen, device):
    return _student_t3(n, std, gen, device) if heavy else _normal(n, std, gen, device)


def _unit(v: torch.Tensor) -> torch.Tensor:
    nrm = torch.linalg.vector_norm(v.double()).item()
    return (v.double() / nrm).float()


def make(name: str, device="cpu", seed: int = 0, d: int | None = None,
         K: int | None = None, l: int | None = None, m: int | None = None) -> Workload:
    """Build one of cfg1..cfg5; d / K / l / m may be overridden to get a scaled-down
    case with the same value distributions."""
    c = dict(CONFIGS[name])
    if d is not None:
        c["d"] = int(d)
    if K is not None:
        c["K"] = int(K)
    if l is not None:
        c["l"] = int(l)
    if m is not None:
        c["m"] = int(m)
    K_, d_, dt = c["K"], c["d"], c["dtype"]
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(seed))

    heavy = False
    if name == "cfg4":
        w_t0 = (torch.rand(d_, generator=gen, device=dev, dtype=torch.float32) * 0.2 - 0.1)
    else:
        w_t0 = _normal(d_, 0.05, gen, dev)
    xi = _unit(torch.randn(d_, generator=gen, device=dev, dtype=torch.float32))

    slab_dtype = torch.float32 if dt == "f32" else torch.bfloat16
    w = torch.empty((K_, d_), device=dev, dtype=slab_dtype)
    latent = None
    step_std = 1e-4

    if name in ("cfg1", "cfg2"):
        private = 1e-3 if name == "cfg1" else 5e-4
        shared = _normal(d_, 1e-3, gen, dev)
        for k in range(K_):
            w[k] = w_t0 + shared + _normal(d_, private, gen, dev)
    elif name == "cfg3":
        for k in range(K_):
            v = _unit(torch.randn(d_, generator=gen, device=dev, dtype=torch.float32)) * 0.01
            w[k] = w_t0 + v + _normal(d_, 1e-4, gen, dev)
    elif name == "cfg4":
        for k in range(K_):
            w[k] = w_t0 + _normal(d_, 2e-4, gen, dev)
    elif name == "cfg5":
        heavy = True
        step_std = 1e-5
        latent = torch.empty((K_, d_), device=dev, dtype=torch.float32)
        for k in range(K_):
            latent[k] = w_t0 + _student_t3(d_, 1e-4, gen, dev)
            w[k] = latent[k].to(torch.bfloat16)
    else:
        raise KeyError(name)

    return Workload(name=name, K=K_, d=d_, dtype=dt, l=c["l"], m=c["m"],
                    eps=default_eps(c["m"]), T=c["T"], w=w, w_t0=w_t0, xi=xi,
                    hash_coef=hash_coefficients(seed, c["l"]), step_std=step_std,
                    heavy_tail=heavy, gen=gen, latent=latent)


def slab_to_numpy(w: torch.Tensor) -> np.ndarray:
    """Host copy of a slab in the form the oracle takes: float32, or uint16 bit
    patterns for bfloat16."""
    w = w.detach().cpu()
    if w.dtype == torch.bfloat16:
        return w.view(torch.int16).numpy().view(np.uint16).copy()
    return w.numpy().copy()
