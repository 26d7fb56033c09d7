"""Seeded synthetic workloads: sparse layered networks, inputs, targets.

This module only *draws data*.  It holds none of the method's arithmetic (no
products, no activation, no gradient): the CPU oracle and the HIP library both
receive exactly the arrays built here and nothing else is shared between them.

Shapes follow the experimental setup of the paper (Section 6.1: layered nets
with the same number of neurons in every layer, 120+ layers, N = 1024 ... 65536,
binary input vectors) with synthetic stand-ins for the benchmark networks and
images, which are not available offline: every neuron has 32 incoming links at
distinct uniformly random source neurons, every weight is 1/16, one negative
bias per net size, activations capped at 32.  A fifth family models an
irregularly pruned net (heavy-tailed row degrees).

Layout conventions used everywhere in this repository:
  * W_l is n_out x n_in in CSR; entry (j, i) is the link from neuron i of layer
    l-1 to neuron j of layer l (Section 3.2).
  * activations are dense fp32 matrices [N][B]: row = neuron, column = sample
    (Section 5.1 places the batch vectors as the columns of X).
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np


@dataclass
class Layer:
    n_out: int
    n_in: int
    row_ptr: np.ndarray  # int32 [n_out+1]
    col_idx: np.ndarray  # int32 [nnz], ascending and distinct inside each row
    values: np.ndarray   # float32 [nnz]
    bias: np.ndarray     # float32 [n_out]

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])


@dataclass
class Workload:
    name: str
    layers: List[Layer]
    act_cap: float                 # np.inf = plain ReLU
    x_infer: np.ndarray            # float32 [N][B_infer]
    train_batch: int               # the first train_batch columns of x_infer
    loss: str                      # "mse" | "softmax_ce"
    lr: float
    targets: Optional[np.ndarray] = None   # float32 [N][train_batch]  (mse)
    labels: Optional[np.ndarray] = None    # int64 [train_batch]       (softmax_ce)
    n_classes: int = 0
    activation: str = "relu"               # "relu" (clamped at act_cap) | "sigmoid"
    meta: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return self.layers[0].n_in

    @property
    def total_nnz(self) -> int:
        return sum(l.nnz for l in self.layers)

    @property
    def x_train(self) -> np.ndarray:
        return np.ascontiguousarray(self.x_infer[:, : self.train_batch])


# ----------------------------------------------------------------------------
# pattern generators
# ----------------------------------------------------------------------------

def _distinct_sorted_columns(rng: np.random.Generator, n_rows: int, n_cols: int, d: int) -> np.ndarray:
    """[n_rows][d] int32, every row d distinct column ids in ascending order.

    Rows holding a repeated id are redrawn as a whole until none is left, so
    every d-subset stays equally likely.  Never builds an n_rows x n_cols table.
    """
    if d > n_cols:
        raise ValueError("more links per row than columns")
    cols = np.sort(rng.integers(0, n_cols, size=(n_rows, d), dtype=np.int64), axis=1)
    while True:
        bad = np.nonzero((cols[:, 1:] == cols[:, :-1]).any(axis=1))[0]
        if bad.size == 0:
            break
        cols[bad] = np.sort(rng.integers(0, n_cols, size=(bad.size, d), dtype=np.int64), axis=1)
    return cols.astype(np.int32)


def regular_layer(seed: int, n: int, d: int, value: float, bias: float,
                  n_in: Optional[int] = None) -> Layer:
    """n x n_in layer with exactly d links per row, constant weight and bias."""
    n_in = n if n_in is None else n_in
    rng = np.random.default_rng(seed)
    cols = _distinct_sorted_columns(rng, n, n_in, d)
    row_ptr = (np.arange(n + 1, dtype=np.int64) * d).astype(np.int32)
    return Layer(n, n_in, row_ptr, cols.reshape(-1),
                 np.full(n * d, value, dtype=np.float32),
                 np.full(n, bias, dtype=np.float32))


def strided_layer(seed: int, n: int, d: int = 32, scale: float = 0.25, bias_scale: float = 0.1,
                  value: Optional[float] = None, bias: Optional[float] = None) -> Layer:
    """Structured n x n layer in the manner of the butterfly-like benchmark topologies: neuron j is
    linked to the d neurons (j + k * n/d) mod n, k = 0..d-1, of the previous layer, so the d rows
    j, j + n/d, j + 2n/d, ... share one set of d columns while neighbouring rows share none.  Weights
    normal(0, scale) and biases normal(0, bias_scale) unless constants are given."""
    if n % d:
        raise ValueError("n must be a multiple of d")
    rng = np.random.default_rng(seed)
    stride = n // d
    cols = (np.arange(n, dtype=np.int64)[:, None] + stride * np.arange(d, dtype=np.int64)[None, :]) % n
    cols = np.sort(cols, axis=1).astype(np.int32)
    row_ptr = (np.arange(n + 1, dtype=np.int64) * d).astype(np.int32)
    values = (np.full(n * d, value, np.float32) if value is not None
              else (rng.standard_normal(n * d) * scale).astype(np.float32))
    b = (np.full(n, bias, np.float32) if bias is not None else (rng.standard_normal(n) * bias_scale).astype(np.float32))
    return Layer(n, n, row_ptr, cols.reshape(-1), values, b)


def heavy_tail_degrees(rng: np.random.Generator, n: int, s: float, cap: int, mean: float) -> np.ndarray:
    """Row degrees deg_i = clip(round(c * Z_i), 1, cap) with Z_i ~ Zipf(s).

    The scale c is found by bisection on the drawn Z so that the mean degree is
    `mean` (to within one link).  A plain clipped Zipf(1.2) has a much smaller
    mean than the ~820 the workload asks for, hence the scale.
    """
    z = rng.zipf(s, size=n).astype(np.float64)

    def deg(c):
        return np.clip(np.rint(c * z), 1, cap)

    lo, hi = 1e-6, float(cap)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if deg(mid).mean() < mean:
            lo = mid
        else:
            hi = mid
    return deg(hi).astype(np.int64)


def irregular_layer(seed: int, n: int, s: float = 1.2, cap: int = 2048, mean: float = 820.0,
                    mixed_sign: bool = True) -> Layer:
    """n x n layer with heavy-tailed row degrees, weights normal(0, sd=1/sqrt(deg)), bias 0."""
    rng = np.random.default_rng(seed)
    cap = min(cap, n)
    mean = min(mean, 0.4 * n)
    deg = heavy_tail_degrees(rng, n, s, cap, mean)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=row_ptr[1:])
    col_idx = np.empty(int(row_ptr[-1]), dtype=np.int32)
    for i in range(n):
        col_idx[row_ptr[i]:row_ptr[i + 1]] = np.sort(rng.choice(n, size=int(deg[i]), replace=False))
    sd = np.repeat(1.0 / np.sqrt(deg.astype(np.float64)), deg)
    values = (rng.standard_normal(col_idx.size) * sd).astype(np.float32)
    if not mixed_sign:
        values = np.abs(values)
    return Layer(n, n, row_ptr.astype(np.int32), col_idx, values, np.zeros(n, dtype=np.float32))


def random_layer(seed: int, n_out: int, n_in: int, density: float, scale: float = 1.0,
                 bias_scale: float = 0.5, allow_empty_rows: bool = True) -> Layer:
    """Small test layer: Bernoulli pattern, mixed-sign normal weights and biases."""
    rng = np.random.default_rng(seed)
    mask = rng.random((n_out, n_in)) < density
    if not allow_empty_rows:
        for i in range(n_out):
            if not mask[i].any():
                mask[i, rng.integers(0, n_in)] = True
    counts = mask.sum(axis=1)
    row_ptr = np.zeros(n_out + 1, dtype=np.int32)
    np.cumsum(counts, out=row_ptr[1:])
    col_idx = np.nonzero(mask)[1].astype(np.int32)
    values = (rng.standard_normal(col_idx.size) * scale).astype(np.float32)
    bias = (rng.standard_normal(n_out) * bias_scale).astype(np.float32)
    return Layer(n_out, n_in, row_ptr, col_idx, values, bias)


def ragged_layer(seed: int, n_out: int, n_in: int, density: float, n_long_rows: int, long_row_len: int,
                 n_long_cols: int, long_col_len: int, scale: float = 0.3) -> Layer:
    """Test layer with a few very long rows and a few very long columns in a sea of short ones
    (and some empty rows): a sparse Bernoulli pattern plus randomly placed dense stretches."""
    rng = np.random.default_rng(seed)
    mask = rng.random((n_out, n_in)) < density
    for r in rng.choice(n_out, size=n_long_rows, replace=False):
        mask[r, rng.choice(n_in, size=long_row_len, replace=False)] = True
    for c in rng.choice(n_in, size=n_long_cols, replace=False):
        mask[rng.choice(n_out, size=long_col_len, replace=False), c] = True
    counts = mask.sum(axis=1)
    row_ptr = np.zeros(n_out + 1, dtype=np.int32)
    np.cumsum(counts, out=row_ptr[1:])
    col_idx = np.nonzero(mask)[1].astype(np.int32)
    values = (rng.standard_normal(col_idx.size) * scale / np.sqrt(np.maximum(counts, 1)).repeat(counts)).astype(np.float32)
    bias = (rng.standard_normal(n_out) * 0.1).astype(np.float32)
    return Layer(n_out, n_in, row_ptr, col_idx, values, bias)


# ----------------------------------------------------------------------------
# inputs and targets
# ----------------------------------------------------------------------------

def binary_inputs(seed: int, n: int, b: int, density: float) -> np.ndarray:
    """Bernoulli(density) matrix [n][b] of 0.0 / 1.0.  Drawn in row chunks (the generator's stream is
    consumed in the same order as by one big draw, so the values do not depend on the chunking): the
    largest input set is 2^29 elements and a single draw would need 4 GB of temporaries."""
    rng = np.random.default_rng(seed)
    out = np.empty((n, b), dtype=np.float32)
    step = max(1, (1 << 20) // max(b, 1))
    buf = np.empty((step, b), dtype=np.float64)
    for r in range(0, n, step):
        k = min(step, n - r)
        rng.random(out=buf[:k])
        np.less(buf[:k], density, out=out[r:r + k], casting="unsafe")
    return out


def mixed_density_inputs(seed: int, n: int, b: int, densities: Sequence[float]) -> np.ndarray:
    """Binary inputs [n][b] whose column s is Bernoulli(densities[s % len(densities)]): samples that die
    at different depths next to samples that stay alive."""
    rng = np.random.default_rng(seed)
    dens = np.asarray([densities[s % len(densities)] for s in range(b)], dtype=np.float64)
    return (rng.random((n, b)) < dens[None, :]).astype(np.float32)


def normal_inputs(seed: int, n: int, b: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, b)).astype(np.float32)


def uniform_targets(seed: int, n: int, b: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.random((n, b)).astype(np.float32)


def class_labels(seed: int, b: int, n_classes: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(0, n_classes, size=b, dtype=np.int64)


# ----------------------------------------------------------------------------
# the five benchmark configurations (index 1..5) and their "live" companions
# ----------------------------------------------------------------------------

def _regular_job(job):
    seed, n, bias = job
    return regular_layer(seed, n, 32, 0.0625, bias)


def _irregular_job(job):
    seed, n = job
    return irregular_layer(seed, n)


def _build_layers(fn, jobs, threads: bool) -> List[Layer]:
    """Layers are independent (one seed each), so deep regular nets are drawn by several threads
    (numpy sorts and draws outside the interpreter lock); the result does not depend on how many.
    The heavy-tailed layers are drawn one after the other (a per-row Python loop dominates there)."""
    workers = min(len(jobs), 16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else 4)
    if not threads or workers <= 1 or len(jobs) < 4:
        return [fn(j) for j in jobs]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(workers) as ex:
        return list(ex.map(fn, jobs))


#        N      L    bias   B_infer density B_train
_REGULAR = {
    1: (1024, 120, -0.30, 64, 0.10, 64),
    2: (4096, 480, -0.32, 1024, 0.10, 128),
    3: (16384, 480, -0.35, 4096, 0.05, 128),
    4: (65536, 120, -0.45, 8192, 0.02, 64),
}


def make_config(cfg: int, *, n_layers: Optional[int] = None, n: Optional[int] = None,
                b_infer: Optional[int] = None, b_train: Optional[int] = None,
                density: Optional[float] = None, with_inputs: bool = True) -> Workload:
    """Build benchmark configuration `cfg` (1..5).

    Keyword overrides shrink or alter a configuration while keeping its
    generation rule and seeds (layer l of config c always uses seed 1000*c + l,
    inputs 1000*c + 900, targets/labels 1000*c + 901):
      n_layers  keep only the first n_layers layers (depth prefix)
      n         neurons per layer (tests use scaled-down nets)
      b_infer / b_train   number of samples
      density   input density of the binary inputs (the "live" companions use
                0.30 / 0.40: at the nominal densities these nets die after the
                first layer, every activation being exactly zero from layer 2)
    """
    if cfg in _REGULAR:
        N, L, bias, B, dens, Bt = _REGULAR[cfg]
        N = n or N
        L = n_layers or L
        B = b_infer or B
        Bt = min(b_train or Bt, B)
        dens = dens if density is None else density
        layers = _build_layers(_regular_job, [(1000 * cfg + l, N, bias) for l in range(1, L + 1)], threads=True)
        x = binary_inputs(1000 * cfg + 900, N, B, dens) if with_inputs else np.zeros((N, 0), np.float32)
        tg = uniform_targets(1000 * cfg + 901, N, Bt) if with_inputs else None
        return Workload(f"cfg{cfg}-N{N}-L{L}", layers, 32.0, x, Bt, "mse", 0.01, targets=tg,
                        meta=dict(cfg=cfg, density=dens, bias=bias))
    if cfg == 5:
        N = n or 8192
        L = n_layers or 30
        B = b_infer or 2048
        Bt = min(b_train or 256, B)
        layers = _build_layers(_irregular_job, [(5000 + l, N) for l in range(1, L + 1)], threads=False)
        x = normal_inputs(5900, N, B) if with_inputs else np.zeros((N, 0), np.float32)
        lab = class_labels(5901, Bt, 10)
        return Workload(f"cfg5-N{N}-L{L}", layers, float("inf"), x, Bt, "softmax_ce", 0.005,
                        labels=lab, n_classes=10, meta=dict(cfg=5))
    raise ValueError("cfg must be 1..5")


def paper_training_setup(n: int, n_layers: int = 120, n_inputs: int = 64, seed: int = 7000,
                         input_density: float = 0.19) -> Workload:
    """The paper's own training experiment (Section 6.1) on a synthetic stand-in net:
    sigmoid activation, MSE loss, weights uniform in [-1, 1], learning rate 0.01, ONE input
    vector per SGD step.  Topology as in configs 1-4 (32 links per neuron at distinct uniform
    sources: the benchmark nets themselves are not available offline); biases start at 0 and are
    trained (the paper folds the bias into W).  Inputs: `n_inputs` binary vectors (stand-ins for
    thresholded images; about 19 % of MNIST pixels are on), targets uniform in [0, 1).
    Use column s of x_infer / targets for step s."""
    layers = []
    for l in range(1, n_layers + 1):
        lay = regular_layer(seed + l, n, 32, 0.0, 0.0)
        rng = np.random.default_rng(seed + 500 + l)
        lay.values = rng.uniform(-1.0, 1.0, size=lay.nnz).astype(np.float32)
        layers.append(lay)
    x = binary_inputs(seed + 900, n, n_inputs, input_density)
    tg = uniform_targets(seed + 901, n, n_inputs)
    return Workload(f"paper-setup-N{n}-L{n_layers}", layers, float("inf"), x, 1, "mse", 0.01, targets=tg,
                    activation="sigmoid", meta=dict(setup="paper section 6.1"))


def tiny_net(seed: int, sizes=(7, 9, 6, 8), density: float = 0.45, b: int = 5,
             cap: float = float("inf"), scale: float = 0.8) -> Workload:
    """Small rectangular mixed-sign net for dense / finite-difference checks."""
    layers = [random_layer(seed * 100 + l, sizes[l + 1], sizes[l], density, scale=scale)
              for l in range(len(sizes) - 1)]
    x = normal_inputs(seed * 100 + 90, sizes[0], b)
    tg = uniform_targets(seed * 100 + 91, sizes[-1], b)
    return Workload(f"tiny-{seed}", layers, cap, x, b, "mse", 0.01, targets=tg)
