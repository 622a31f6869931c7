"""Seeded synthetic inputs for the subsampled Gauss-Newton path.

This module only *draws data*: feature matrices, labels, an initial parameter
vector, a subsample S and a probe vector.  It contains none of the method's
arithmetic (no forward pass, no derivatives, no products), so the fp64 oracle
and the HIP path can both take their inputs from here without sharing any
computation.

Every array comes from numpy's counter-based Philox generator keyed by
(base seed of the configuration, sub-stream id), so each piece can be
regenerated independently and in any order.

The five configurations mirror the shapes and value ranges of the paper's
workloads (Section 8, table of the data sets: features scaled to [0,1], one-hot
class targets; network sizes of the same order as Table 2) without
reproducing any data set.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Tuple

import numpy as np

_BASE_SEED = 1802_00130

# sub-stream identifiers
_ST_X, _ST_LABEL, _ST_THETA, _ST_SUBSET, _ST_PROBE, _ST_BIAS = 1, 2, 3, 4, 5, 6


@dataclasses.dataclass(frozen=True)
class Config:
    """One synthetic workload: network n_0-...-n_L, l samples, |S| subsample."""

    name: str
    dims: Tuple[int, ...]      # n_0, ..., n_L
    l: int                     # number of samples
    s: int                     # |S|
    C: float                   # regularisation parameter of the objective
    lam: float                 # Levenberg-Marquardt damping used in CG
    cg_iters: int
    features: str              # "uniform" (U[0,1)) or "normal3" (N(0,1) clipped to +-3)
    seed: int

    @property
    def L(self) -> int:
        return len(self.dims) - 1

    @property
    def n_classes(self) -> int:
        return self.dims[-1]

    @property
    def n_params(self) -> int:
        return num_params(self.dims)


def num_params(dims) -> int:
    """n = sum_m (n_{m-1} n_m + n_m)  (Section 2.1)."""
    return sum(dims[m - 1] * dims[m] + dims[m] for m in range(1, len(dims)))


def layer_offsets(dims) -> List[Tuple[int, int]]:
    """Offsets (weights, biases) of every layer inside theta.

    theta = [w^1; b^1; ...; w^L; b^L] with w^m the columns of W^m stacked
    (Section 2.1), i.e. the slice for layer m read row-major is the
    n_m x n_{m-1} matrix (W^m)^T, followed by the n_m biases.
    """
    offs = []
    o = 0
    for m in range(1, len(dims)):
        w = o
        o += dims[m - 1] * dims[m]
        b = o
        o += dims[m]
        offs.append((w, b))
    return offs


CONFIGS = (
    Config("cfg1_20-16-16-4", (20, 16, 16, 4), 200, 50, 1.0, 1.0, 5, "uniform", _BASE_SEED * 10 + 1),
    Config("cfg2_784-300-300-10", (784, 300, 300, 10), 60000, 3000, 60000.0, 1.0, 20, "uniform", _BASE_SEED * 10 + 2),
    Config("cfg3_3072-1000-500-10", (3072, 1000, 500, 10), 50000, 2500, 50000.0, 1.0, 20, "uniform", _BASE_SEED * 10 + 3),
    Config("cfg4_2048-2000x3-100", (2048, 2000, 2000, 2000, 100), 100000, 5000, 100000.0, 1.0, 50, "normal3", _BASE_SEED * 10 + 4),
    Config("cfg5_4096x5-1000", (4096, 4096, 4096, 4096, 4096, 1000), 200000, 2000, 200000.0, 1.0, 20, "uniform", _BASE_SEED * 10 + 5),
)


def config(index: int) -> Config:
    """Configuration by 1-based index (1 = tiny ... 5 = largest)."""
    return CONFIGS[index - 1]


def custom(dims, l, s, C=1.0, lam=1.0, cg_iters=5, features="uniform", seed=12345, name=None) -> Config:
    dims = tuple(int(d) for d in dims)
    return Config(name or ("custom_" + "-".join(map(str, dims))), dims, int(l), int(s), float(C), float(lam),
                  int(cg_iters), features, int(seed))


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def make_X(cfg: Config, rows: int | None = None) -> np.ndarray:
    """Feature matrix, fp32, [rows x n_0] row-major; the first `rows` samples."""
    rows = cfg.l if rows is None else min(rows, cfg.l)
    g = _rng(cfg.seed, _ST_X)
    n0 = cfg.dims[0]
    if cfg.features == "uniform":
        return g.random((rows, n0), dtype=np.float32)
    if cfg.features == "normal3":
        x = g.standard_normal((rows, n0), dtype=np.float32)
        np.clip(x, -3.0, 3.0, out=x)
        return x
    raise ValueError(cfg.features)


def make_labels(cfg: Config, rows: int | None = None) -> np.ndarray:
    """Uniform class ids in 0..K-1, int32, one per sample."""
    rows = cfg.l if rows is None else min(rows, cfg.l)
    g = _rng(cfg.seed, _ST_LABEL)
    return g.integers(0, cfg.n_classes, size=cfg.l, dtype=np.int32)[:rows]


def make_Y(cfg: Config, rows: int | None = None) -> np.ndarray:
    """Dense one-hot targets, fp32, [rows x n_L]."""
    lab = make_labels(cfg, rows)
    Y = np.zeros((lab.shape[0], cfg.n_classes), dtype=np.float32)
    Y[np.arange(lab.shape[0]), lab] = 1.0
    return Y


def make_theta(cfg: Config, bias_scale: float = 0.0, init: str = "xavier") -> np.ndarray:
    """Initial parameters, fp32, theta layout.

    init = "xavier": weights Xavier-uniform U(-a, a), a = sqrt(6 / (n_{m-1} + n_m)).
    init = "sparse": the sparse initialisation of Section 6.2 with the count given among the parameters in Section 8: of the n_{m-1}
        weights into each neuron of layer m, ceil(sqrt(n_{m-1})) chosen at random are N(0, 1), the rest zero.
    init = "dense": the dense initialisation of Section 8.2: N(0, 0.1^2) in the first layer, N(0, 0.001^2)
        in the output layer, N(0, 0.05^2) in the other layers.
    Biases: zero, or U(-bias_scale, bias_scale) when bias_scale > 0 so that
    tests exercise the bias paths.
    """
    if init not in ("xavier", "sparse", "dense"):
        raise ValueError(f"unknown init {init!r}")
    g = _rng(cfg.seed, _ST_THETA)
    gb = _rng(cfg.seed, _ST_BIAS)
    theta = np.zeros(cfg.n_params, dtype=np.float32)
    L = len(cfg.dims) - 1
    for m, (w, b) in enumerate(layer_offsets(cfg.dims), start=1):
        fan_in, fan_out = cfg.dims[m - 1], cfg.dims[m]
        if init == "xavier":
            a = math.sqrt(6.0 / (fan_in + fan_out))
            u = g.random(fan_in * fan_out, dtype=np.float32)
            theta[w:w + fan_in * fan_out] = (2.0 * u - 1.0) * np.float32(a)
        elif init == "sparse":
            k = math.isqrt(fan_in - 1) + 1 if fan_in > 0 else 0          # ceil(sqrt(fan_in))
            A = theta[w:w + fan_in * fan_out].reshape(fan_out, fan_in)     # row j: the weights into neuron j
            for j in range(fan_out):
                cols = g.permutation(fan_in)[:k]
                A[j, cols] = g.standard_normal(k, dtype=np.float32)
        else:
            sd = 0.1 if m == 1 else (0.001 if m == L else 0.05)
            theta[w:w + fan_in * fan_out] = g.standard_normal(fan_in * fan_out, dtype=np.float32) * np.float32(sd)
        if bias_scale > 0.0:
            ub = gb.random(fan_out, dtype=np.float32)
            theta[b:b + fan_out] = (2.0 * ub - 1.0) * np.float32(bias_scale)
    return theta


def make_subset(cfg: Config, rows: int | None = None) -> np.ndarray:
    """|S| distinct row ids drawn uniformly without replacement, int32.

    When `rows` is given the subset is drawn from 0..rows-1 (for parity runs
    on a prefix of the samples).
    """
    rows = cfg.l if rows is None else min(rows, cfg.l)
    g = _rng(cfg.seed, _ST_SUBSET)
    perm = g.permutation(rows)
    return np.ascontiguousarray(perm[:min(cfg.s, rows)].astype(np.int32))


def make_probe(cfg: Config, k: int = 0) -> np.ndarray:
    """Probe vector v ~ N(0,1), fp32, theta layout; k selects independent draws."""
    g = _rng(cfg.seed, _ST_PROBE + 16 * (k + 1))
    return g.standard_normal(cfg.n_params, dtype=np.float32)
