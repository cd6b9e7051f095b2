"""Seeded synthetic workloads for the DeepSqueeze step (inputs only).

This module makes *data*: the five benchmark configurations, and seeded
gradient streams with the shapes and value distributions those configurations
name.  It contains none of the method's arithmetic (no compression, no gossip)
and imports neither the GPU binding nor the CPU oracle, so both can be fed the
very same arrays.

The paper trains ResNet-20 on CIFAR-10 (its Experiments section); neither is
available here, so flat parameter vectors of ResNet-18/50 size with synthetic
gradients stand in for that workload.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

KIND_IDENTITY, KIND_QUANT_MAXABS, KIND_SIGN_MEANABS, KIND_TOPK, KIND_QUANT_L2NORM, KIND_RAND_SPARSE, KIND_GSPAR = 0, 1, 2, 3, 4, 5, 6
TOPO_RING, TOPO_TORUS2D, TOPO_CSR = 0, 1, 2
ALGO_DEEPSQUEEZE, ALGO_DCD_PSGD, ALGO_CHOCO_SGD = 0, 1, 2       # ds_algorithm

_TAG_CENTRE, _TAG_NOISE = 0x43454E54, 0x47524144   # 'CENT', 'GRAD'


@dataclass(frozen=True)
class Config:
    name: str
    n: int
    N: int
    topo: int
    kind: int
    gamma: float
    eta: float
    steps: int
    grad: str                 # 'quadratic' | 'normal' | 'student_t3'
    grad_scale: float         # noise sigma (quadratic) or overall scale
    bits: int = 0
    block: int = 0
    k: int = 0
    torus: Tuple[int, int] = (0, 0)
    seed: int = 0
    algo: int = 0             # 0 DeepSqueeze, 1 DCD-PSGD, 2 CHOCO-SGD (ds_algorithm)

    def scaled(self, N: int, steps: Optional[int] = None) -> "Config":
        """Same workload at another vector length (k follows as 1 % of N for top-k)."""
        k = max(1, N // 100) if self.kind in (KIND_TOPK, KIND_RAND_SPARSE, KIND_GSPAR) else 0
        return replace(self, N=N, k=k, steps=self.steps if steps is None else steps,
                       name=f"{self.name}@N={N}")

    @property
    def worker_params(self) -> int:
        return self.n * self.N


def configs():
    """The five benchmark configurations (index = position in the benchmark's config list)."""
    return [
        Config("cfg0_ring8_q4b512", n=8, N=65_536, topo=TOPO_RING, kind=KIND_QUANT_MAXABS, bits=4, block=512,
               gamma=0.1, eta=0.5, steps=100, grad="quadratic", grad_scale=0.1),
        Config("cfg1_ring16_q2b1024_resnet18", n=16, N=11_173_962, topo=TOPO_RING, kind=KIND_QUANT_MAXABS,
               bits=2, block=1024, gamma=0.05, eta=0.3, steps=200, grad="normal", grad_scale=0.01),
        Config("cfg2_ring8_sign256_resnet50", n=8, N=25_557_032, topo=TOPO_RING, kind=KIND_SIGN_MEANABS,
               block=256, gamma=0.05, eta=0.2, steps=100, grad="student_t3", grad_scale=1e-3),
        Config("cfg3_torus8x8_q4b512", n=64, N=4_194_304, topo=TOPO_TORUS2D, torus=(8, 8),
               kind=KIND_QUANT_MAXABS, bits=4, block=512, gamma=0.1, eta=0.4, steps=100,
               grad="quadratic", grad_scale=0.1),
        Config("cfg4_ring32_top1pct_resnet50", n=32, N=25_557_032, topo=TOPO_RING, kind=KIND_TOPK,
               k=25_557_032 // 100, gamma=0.05, eta=0.2, steps=50, grad="normal", grad_scale=1e-3),
    ]


def extra_configs():
    """Workloads beyond the benchmark's list: the compression of the paper's own experiments (b-bit codes plus
    the tensor's Euclidean norm) on its setting (8 workers on a ring, a vector of ResNet-20 size, 4 bits) and
    at a bandwidth-bound size (the shape of configuration 1, 2 bits); random sparsification at the shape of
    configuration 4 (1 % kept); the two comparison updates (DCD-PSGD, CHOCO-SGD) at the shapes and compressors of
    configurations 1 and 3."""
    c = configs()
    return [
        Config("x5_ring8_l2norm4b_resnet20", n=8, N=272_474, topo=TOPO_RING, kind=KIND_QUANT_L2NORM, bits=4,
               gamma=0.1, eta=0.5, steps=100, grad="normal", grad_scale=0.01),
        Config("x6_ring16_l2norm2b_resnet18", n=16, N=11_173_962, topo=TOPO_RING, kind=KIND_QUANT_L2NORM, bits=2,
               gamma=0.05, eta=0.3, steps=100, grad="normal", grad_scale=0.01),
        Config("x7_ring32_rand1pct_resnet50", n=32, N=25_557_032, topo=TOPO_RING, kind=KIND_RAND_SPARSE,
               k=25_557_032 // 100, gamma=0.05, eta=0.2, steps=50, grad="normal", grad_scale=1e-3),
        replace(c[1], name="x8_dcd_ring16_q2b1024_resnet18", algo=ALGO_DCD_PSGD),
        replace(c[1], name="x9_choco_ring16_q2b1024_resnet18", algo=ALGO_CHOCO_SGD),
        replace(c[3], name="x10_dcd_torus8x8_q4b512", algo=ALGO_DCD_PSGD),
        replace(c[3], name="x11_choco_torus8x8_q4b512", algo=ALGO_CHOCO_SGD),
        Config("x12_ring32_gspar1pct_resnet50", n=32, N=25_557_032, topo=TOPO_RING, kind=KIND_GSPAR,
               k=25_557_032 // 100, gamma=0.05, eta=0.2, steps=50, grad="normal", grad_scale=1e-3),
    ]


def _rng(seed: int, tag: int, t: int) -> np.random.Generator:
    key0 = (((seed << 32) ^ (seed >> 32)) & 0xFFFFFFFFFFFFFFFF) ^ tag          # 64-bit seeds fold into one key word
    return np.random.Generator(np.random.Philox(key=[key0, t]))


def centres(cfg: Config) -> np.ndarray:
    """c_i ~ N(0,1): the minimisers of the per-worker quadratics f_i(x) = 0.5 |x - c_i|^2."""
    return _rng(cfg.seed, _TAG_CENTRE, 0).standard_normal((cfg.n, cfg.N), dtype=np.float32)


def _noise(cfg: Config, t: int) -> np.ndarray:
    return _rng(cfg.seed, _TAG_NOISE, t).standard_normal((cfg.n, cfg.N), dtype=np.float32)


def gradient(cfg: Config, t: int, x: Optional[np.ndarray] = None, c: Optional[np.ndarray] = None) -> np.ndarray:
    """Stochastic gradients g_t (n x N, fp32) for step t.

    'quadratic'  : g = (x - c) + sigma * xi, xi ~ N(0,1)       (needs the current x and the centres)
    'normal'     : g = scale * N(0,1) i.i.d.
    'student_t3' : g = scale * Z / sqrt((Z1^2+Z2^2+Z3^2)/3)    (heavy tails, nu = 3)
    """
    if cfg.grad == "quadratic":
        assert x is not None and c is not None
        xi = _noise(cfg, t)
        d = (x.astype(np.float32) - c).astype(np.float64)
        return (d + np.float64(np.float32(cfg.grad_scale)) * xi.astype(np.float64)).astype(np.float32)
    if cfg.grad == "normal":
        return _noise(cfg, t) * np.float32(cfg.grad_scale)
    if cfg.grad == "student_t3":
        r = _rng(cfg.seed, _TAG_NOISE, t)
        z = r.standard_normal((cfg.n, cfg.N))
        chi = np.zeros((cfg.n, cfg.N))
        for _ in range(3):
            w = r.standard_normal((cfg.n, cfg.N))
            chi += w * w
        return (cfg.grad_scale * z / np.sqrt(chi / 3.0)).astype(np.float32)
    raise ValueError(cfg.grad)


def random_state(cfg: Config, seed: int, scale: float = 1.0):
    """A seeded non-trivial (x, delta) pair, for tests that should not start from zero."""
    r = np.random.Generator(np.random.Philox(key=[seed, 0x53544154]))
    x = (scale * r.standard_normal((cfg.n, cfg.N))).astype(np.float32)
    d = (0.1 * scale * r.standard_normal((cfg.n, cfg.N))).astype(np.float32)
    return x, d


def device_gradient(cfg: Config, t: int, device="cuda"):
    """Throughput-only gradients made on the GPU with torch's generator (same distributions).

    Values differ from `gradient` (different generator); used where only shape and
    distribution matter, or where the result is copied back to the host to feed the oracle.
    """
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed((cfg.seed << 20) + t)
    shape = (cfg.n, cfg.N)
    if cfg.grad in ("normal", "quadratic"):
        g = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
        return g.mul_(cfg.grad_scale)
    if cfg.grad == "student_t3":
        z = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
        chi = torch.zeros(shape, device=device, dtype=torch.float32)
        for _ in range(3):
            w = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
            chi.addcmul_(w, w)
        return z.mul_(cfg.grad_scale).div_(chi.div_(3.0).sqrt_())
    raise ValueError(cfg.grad)
