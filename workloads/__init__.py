"""Seeded synthetic workloads shared by the oracle-side and the GPU-side tests.

This module only draws random inputs (features, labels, initial weights,
matrices with a prescribed spectrum).  It holds none of the method's
arithmetic and imports neither the oracle nor the HIP binding.

The five workloads C0..C4 stand in for the paper's speech data (Fisher
English, not available here): the shapes follow the paper's typical sizes
(Sec. 6.1, App. B.4), the values are Gaussian with per-dimension means and
scales, labels follow a Zipf law over the classes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

BASE_SEED = 14107455
TANH = 0
PNORM = 1


@dataclass
class NetSpec:
    name: str
    index: int                       # workload index, added to BASE_SEED
    dims: List[int]                  # dims[0] input, dims[1:] affine output dims
    nonlin: List[int]                # per hidden layer
    pnorm_group: int
    minibatch: int
    rank_in: int
    rank_out: int
    lr: float
    steps: int
    softmax_zero_init: bool
    label_law: str                   # "uniform" | "zipf"
    splice: int = 1                  # feature = base_dim x splice
    base_dim: int = 0
    alpha: float = 4.0
    num_samples_history: float = 2000.0
    epsilon: float = 1.0e-10
    update_period: int = 4
    in_dims: List[int] = field(default_factory=list)

    def __post_init__(self):
        d_in = self.dims[0]
        self.in_dims = []
        for l in range(len(self.dims) - 1):
            self.in_dims.append(d_in)
            if l < len(self.dims) - 2:
                d_in = self.dims[l + 1] // self.pnorm_group if self.nonlin[l] == PNORM else self.dims[l + 1]

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1

    @property
    def n_classes(self) -> int:
        return self.dims[-1]

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def n_params(self) -> int:
        return sum(self.dims[l + 1] * (self.in_dims[l] + 1) for l in range(self.n_layers))


def c0_tiny() -> NetSpec:
    """C0: 40 -> 128 tanh -> 128 tanh -> 50-way softmax, minibatch 64, ranks 4 / 8."""
    return NetSpec("c0_tiny_tanh", 0, [40, 128, 128, 50], [TANH, TANH], 10, 64, 4, 8, 0.01, 10,
                   softmax_zero_init=False, label_law="uniform", splice=1, base_dim=40)


def c1_pnorm() -> NetSpec:
    """C1: 360 -> 4 x (affine 3000, p-norm 10 -> 300) -> 5000-way softmax, minibatch 512, ranks 20 / 80."""
    return NetSpec("c1_pnorm_speech", 1, [360, 3000, 3000, 3000, 3000, 5000], [PNORM] * 4, 10, 512,
                   20, 80, 0.01, 200, softmax_zero_init=True, label_law="zipf", splice=9, base_dim=40)


def c3_wide_tanh() -> NetSpec:
    """C3: 440 -> 6 x tanh 2048 -> 8000-way softmax, minibatch 1024, ranks 20 / 80."""
    return NetSpec("c3_wide_tanh", 3, [440] + [2048] * 6 + [8000], [TANH] * 6, 10, 1024,
                   20, 80, 0.01, 200, softmax_zero_init=True, label_law="zipf", splice=11, base_dim=40)


def small_pnorm(minibatch: int = 96) -> NetSpec:
    """A reduced p-norm net (ragged sizes, several tiles) for parity tests the oracle finishes in seconds."""
    return NetSpec("small_pnorm", 7, [52, 170, 230, 203], [PNORM, PNORM], 10, minibatch, 5, 12, 0.01, 12,
                   softmax_zero_init=True, label_law="zipf", splice=4, base_dim=13)


def _rng(seed: int, *stream) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, *[int(s) for s in stream]]))


def initial_weights(spec: NetSpec, replica: int = 0):
    """N(0, 1/fan_in) weights with a zero bias column (App. C.7); softmax layer zero if the spec says so.

    `replica` does not change the weights: the paper's replicas start from the same model.
    """
    rng = _rng(spec.seed, 1)
    weights = []
    for l in range(spec.n_layers):
        d_out, d_in = spec.dims[l + 1], spec.in_dims[l]
        w = np.zeros((d_out, d_in + 1), dtype=np.float32)
        body = rng.standard_normal((d_out, d_in)).astype(np.float32) / np.float32(np.sqrt(d_in))
        if not (spec.softmax_zero_init and l == spec.n_layers - 1):
            w[:, :d_in] = body
        weights.append(w)
    return weights


def feature_law(spec: NetSpec):
    """Per-dimension mean and standard deviation of the spliced feature vector."""
    rng = _rng(spec.seed, 2)
    if spec.label_law == "uniform":          # C0: standard normal features
        return np.zeros(spec.dims[0], np.float32), np.ones(spec.dims[0], np.float32)
    mu = rng.uniform(-2.0, 2.0, spec.base_dim)
    sd = rng.uniform(0.5, 2.0, spec.base_dim)
    return (np.tile(mu, spec.splice).astype(np.float32), np.tile(sd, spec.splice).astype(np.float32))


def class_probabilities(spec: NetSpec) -> np.ndarray:
    k = np.arange(1, spec.n_classes + 1, dtype=np.float64)
    p = np.ones_like(k) if spec.label_law == "uniform" else k ** -1.1
    return p / p.sum()


def minibatch(spec: NetSpec, step: int, replica: int = 0, rows: int | None = None):
    """Minibatch `step` of replica `replica`: (x float32 N x D0, labels int32 N)."""
    n = spec.minibatch if rows is None else rows
    rng = _rng(spec.seed, 3, replica, step)
    mu, sd = feature_law(spec)
    x = (rng.standard_normal((n, spec.dims[0])).astype(np.float32) * sd[None, :] + mu[None, :]).astype(np.float32)
    labels = rng.choice(spec.n_classes, size=n, p=class_probabilities(spec)).astype(np.int32)
    return x, labels


# ---------------------------------------------------------------------------------------------
# C2: matrices with a decaying spectrum for the preconditioner alone
# ---------------------------------------------------------------------------------------------
@dataclass
class PrecondSpec:
    name: str
    rows: int
    dim: int
    rank: int
    ones_column: bool
    index: int = 2
    steps: int = 1000
    update_period: int = 1
    alpha: float = 4.0
    num_samples_history: float = 2000.0
    epsilon: float = 1.0e-10
    n_reflections: int = 4

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


def c2_input_side() -> PrecondSpec:
    return PrecondSpec("c2_x_512x3001_r20", 512, 3001, 20, True)


def c2_output_side() -> PrecondSpec:
    return PrecondSpec("c2_o_512x5000_r80", 512, 5000, 80, False)


def _reflectors(spec: PrecondSpec) -> np.ndarray:
    rng = _rng(spec.seed, 4, spec.dim)
    v = rng.standard_normal((spec.n_reflections, spec.dim))
    return v / np.linalg.norm(v, axis=1, keepdims=True)


def spectrum_matrix(spec: PrecondSpec, step: int, rows: int | None = None) -> np.ndarray:
    """M_t = G_t diag(1/k) Q^T with G_t fresh Gaussian and Q a fixed product of Householder reflections.

    Rows therefore have covariance Q diag(k^-2) Q^T (singular values ~ 1/k).  For the
    input-side case the last column is then overwritten with ones (the bias input).
    """
    n = spec.rows if rows is None else rows
    rng = _rng(spec.seed, 5, spec.dim, step)
    m = rng.standard_normal((n, spec.dim)) / np.arange(1, spec.dim + 1, dtype=np.float64)[None, :]
    for v in _reflectors(spec):
        m -= 2.0 * np.outer(m @ v, v)
    if spec.ones_column:
        m[:, -1] = 1.0
    return m.astype(np.float32)
