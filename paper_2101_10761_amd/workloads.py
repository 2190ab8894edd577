"""Seeded synthetic gradients shaped like the paper's workloads.

The paper measures on gradients of real models (Table 1: ResNet-20, VGG16,
ResNet-50, LSTM-PTB, VGG19) and on synthetic vectors of 0.26-260 M elements
(App. E, "Compression Complexity using Synthetic Gradients Vectors").  Those
datasets and trained weights are not available here, so these generators stand
in for them: the vector lengths are the benchmark configurations' and the
values are drawn from the sparsity-inducing laws the paper fits (Property 2:
double exponential, and heavier-tailed laws for the gamma / Pareto fits).

This module holds no arithmetic of the sparsifier itself.  Both the GPU tests
and the CPU oracle take their inputs from here and from nowhere else.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 210110761

DIST_EXP, DIST_GAMMA_GPD, DIST_GPD = 0, 1, 2


@dataclass
class Workload:
    name: str
    grad: np.ndarray                 # float32[d]
    residual: np.ndarray | None      # float32[d] or None (memoryless)
    delta: float
    dist: int
    stages: int
    delta1: float = 0.25
    tensor_offsets: np.ndarray | None = None   # int64[n+1] for multi-tensor vectors
    meta: dict = field(default_factory=dict)

    @property
    def d(self) -> int:
        return int(self.grad.size)


def _rng(seed_offset: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(SEED_BASE + seed_offset))


def laplace(d: int, b: float, rng: np.random.Generator) -> np.ndarray:
    """i.i.d. Laplace(0, b) drawn in float64, then cast to float32."""
    return rng.laplace(0.0, b, size=d).astype(np.float32)


def config1(d: int = 269_722) -> Workload:
    """ResNet-20-sized vector: i.i.d. Laplace(b=1e-3), zero residual, delta=0.01, one exponential stage."""
    rng = _rng(1)
    g = laplace(d, 1e-3, rng)
    return Workload("cfg1_resnet20_laplace", g, np.zeros(d, np.float32), 0.01, DIST_EXP, 1)


def config2(d: int = 14_714_688, clustered: bool = False) -> Workload:
    """VGG16-sized vector: 90 % Laplace(1e-4) + 10 % Laplace(1e-2), residual Laplace(1e-4),
    delta=0.001, two exponential stages with delta_1 = 0.05, error feedback on.
    `clustered` puts the wide 10 % in one contiguous block (clustered survivors)."""
    rng = _rng(2)
    narrow = rng.laplace(0.0, 1e-4, size=d)
    wide = rng.laplace(0.0, 1e-2, size=d)
    if clustered:
        start = d // 3
        pick = np.zeros(d, dtype=bool)
        pick[start:start + d // 10] = True
    else:
        pick = rng.random(d) < 0.1
    g = np.where(pick, wide, narrow).astype(np.float32)
    r = laplace(d, 1e-4, rng)
    return Workload("cfg2_vgg16_mixture" + ("_clustered" if clustered else ""), g, r, 0.001,
                    DIST_EXP, 2, delta1=0.05)


def config3(d: int = 25_557_032) -> Workload:
    """ResNet-50-sized vector: Student-t(nu=3) * 1e-3, zero residual, delta=0.001,
    three stages of generalized-Pareto fits (delta_1 = 0.25)."""
    rng = _rng(3)
    g = (rng.standard_t(3.0, size=d) * 1e-3).astype(np.float32)
    return Workload("cfg3_resnet50_student_t", g, np.zeros(d, np.float32), 0.001, DIST_GPD, 3)


def config4(d: int = 66_000_000, n_tensors: int = 50, ragged: bool = False) -> Workload:
    """LSTM-PTB-sized vector as `n_tensors` concatenated tensors, tensor t Laplace(b_t) with
    b_t log-uniform in [1e-5, 1e-2]; delta=1e-4, gamma first stage then one GPD stage.
    `ragged` draws unequal, unaligned tensor lengths."""
    rng = _rng(4)
    scales = np.exp(rng.uniform(np.log(1e-5), np.log(1e-2), size=n_tensors))
    if ragged:
        w = rng.uniform(0.2, 1.8, size=n_tensors)
        sizes = np.maximum(1, np.floor(w / w.sum() * d)).astype(np.int64)
        sizes[-1] += d - sizes.sum()
    else:
        sizes = np.full(n_tensors, d // n_tensors, dtype=np.int64)
        sizes[-1] += d - sizes.sum()
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    g = np.empty(d, dtype=np.float32)
    for t in range(n_tensors):
        g[offs[t]:offs[t + 1]] = laplace(int(sizes[t]), float(scales[t]), rng)
    return Workload("cfg4_lstm_ptb_multitensor", g, np.zeros(d, np.float32), 1e-4,
                    DIST_GAMMA_GPD, 2, tensor_offsets=offs, meta={"scales": scales})


def config5_grad(iteration: int, d: int = 138_357_544) -> np.ndarray:
    """VGG19-sized vector, fresh Laplace(b=1e-3) gradient of iteration `iteration`."""
    return laplace(d, 1e-3, _rng(5 + 1000 * (iteration + 1)))


def config5(d: int = 138_357_544, delta: float = 0.001) -> Workload:
    """First iteration of the 100-iteration run: zero residual, three exponential stages."""
    return Workload("cfg5_vgg19_iterated", config5_grad(0, d), np.zeros(d, np.float32), delta,
                    DIST_EXP, 3)
