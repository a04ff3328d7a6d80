"""Workload descriptions and seeded synthetic input generators.

This module holds NO arithmetic of the training method: only shapes, hyper-parameters and
random input data.  It is the one module that both the GPU tests/benchmark and the CPU oracle's
tests may import, so that both sides see the same bytes.

The synthetic features stand in for the datasets of the paper's experiments (Madelon,
FashionMNIST, CIFAR10 and the artificial 65 536-feature binary task of the extreme-scale
section), copying only their shapes and value ranges; labels come from a seeded random linear
teacher.  Nothing here is real data.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

DEFAULT_SEED = 20210201


@dataclass(frozen=True)
class LayerSpec:
    n_in: int
    n_out: int
    nnz: int
    act_kind: int      # 0 identity (output layer), 1 All-ReLU
    act_parity: int    # (index of the receiving neuron layer, input layer = 1) % 2
    init_limit: float  # new weights ~ U(-init_limit, init_limit)
    layer_id: int


@dataclass(frozen=True)
class Workload:
    name: str
    dims: Tuple[int, ...]
    epsilon: float
    n_samples: int
    batch: int
    alpha: float
    feature_law: str            # "normal", "uniform01", "clipped_normal"
    init_rule: str              # "he_uniform_dense_fan_in" or "he_uniform_sparse_fan_in"
    lr: float = 0.01
    momentum: float = 0.9
    zeta: float = 0.3
    seed: int = DEFAULT_SEED
    layers: List[LayerSpec] = field(default_factory=list, compare=False)

    @property
    def n_classes(self) -> int:
        return self.dims[-1]

    @property
    def steps_per_epoch(self) -> int:
        return -(-self.n_samples // self.batch)


def er_nnz(n_in: int, n_out: int, epsilon: float) -> int:
    """Number of connections of an Erdos-Renyi layer with density parameter epsilon, capped at
    the size of the matrix (so narrow output layers come out fully dense)."""
    want = int(np.floor(float(epsilon) * float(n_in + n_out) + 0.5))
    return min(want, n_in * n_out)


def _layers(dims, epsilon, init_rule) -> List[LayerSpec]:
    out = []
    n_layers = len(dims) - 1
    for li in range(n_layers):
        n_in, n_out = dims[li], dims[li + 1]
        nnz = er_nnz(n_in, n_out, epsilon)
        last = li == n_layers - 1
        neuron_layer = li + 2                      # input neurons are layer 1
        if init_rule == "he_uniform_dense_fan_in":
            limit = np.sqrt(np.float32(6.0) / np.float32(n_in))
        else:
            limit = np.sqrt(np.float32(6.0) * np.float32(n_out) / np.float32(nnz))
        out.append(LayerSpec(n_in, n_out, nnz, 0 if last else 1, neuron_layer % 2, float(np.float32(limit)), li))
    return out


def make_workload(name: str, dims, epsilon, n_samples, batch, alpha, feature_law, init_rule, **kw) -> Workload:
    return Workload(name, tuple(dims), epsilon, n_samples, batch, alpha, feature_law, init_rule,
                    layers=_layers(dims, epsilon, init_rule), **kw)


WORKLOADS = {
    # small case the oracle finishes in seconds (Madelon-shaped)
    "set_mlp_madelon": make_workload("set_mlp_madelon", (500, 400, 100, 400, 2), 10, 4096, 128, 0.6,
                                     "normal", "he_uniform_sparse_fan_in"),
    # FashionMNIST-shaped
    "set_mlp_fmnist": make_workload("set_mlp_fmnist", (784, 1000, 1000, 1000, 10), 20, 60000, 128, 0.6,
                                    "uniform01", "he_uniform_dense_fan_in"),
    # CIFAR10-shaped
    "set_mlp_cifar": make_workload("set_mlp_cifar", (3072, 4000, 1000, 4000, 10), 20, 50000, 128, 0.75,
                                   "clipped_normal", "he_uniform_dense_fan_in"),
    # one-million-neuron-per-layer network of the extreme-scale section's kind
    "set_mlp_1m": make_workload("set_mlp_1m", (65536, 1000000, 1000000, 1000000, 2), 10, 16384, 128, 0.6,
                                "normal", "he_uniform_sparse_fan_in"),
}

# single-layer kernel sweep: n_in = n_out = 262 144
SWEEP_N = 262144
SWEEP_EPSILON = (1, 4, 16, 64)
SWEEP_BATCH = (32, 128, 512, 1024)


def sweep_layer(epsilon: float, n: int = SWEEP_N, alpha: float = 0.6) -> LayerSpec:
    nnz = er_nnz(n, n, epsilon)
    limit = float(np.float32(np.sqrt(np.float32(6.0) * np.float32(n) / np.float32(nnz))))
    return LayerSpec(n, n, nnz, 1, 0, limit, 0)


# ----------------------------------------------------------------------------------------------
# seeded data
# ----------------------------------------------------------------------------------------------
def features(law: str, n_samples: int, n_features: int, seed: int) -> np.ndarray:
    """[n_samples, n_features] float32, sample-major."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if law == "normal":
        x = rng.standard_normal((n_samples, n_features), dtype=np.float32)
    elif law == "uniform01":
        x = rng.random((n_samples, n_features), dtype=np.float32)
    elif law == "clipped_normal":
        x = rng.standard_normal((n_samples, n_features), dtype=np.float32) * np.float32(0.25) + np.float32(0.5)
        np.clip(x, 0.0, 1.0, out=x)
    else:
        raise ValueError(law)
    return x


def teacher_labels(x: np.ndarray, n_classes: int, seed: int, centre: float = 0.0) -> np.ndarray:
    """Labels from a seeded random linear teacher: argmax_c ((x - centre) . T_c), ties to the
    lowest class.  For two classes this is a random hyperplane through `centre`."""
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    if n_classes == 2:
        h = rng.standard_normal(x.shape[1])
        s = (x.astype(np.float64) - centre) @ h
        return (s > 0).astype(np.int32)
    T = rng.standard_normal((x.shape[1], n_classes))
    s = (x.astype(np.float64) - centre) @ T
    return np.argmax(s, axis=1).astype(np.int32)


def dataset(w: Workload, n_samples: int | None = None) -> Tuple[np.ndarray, np.ndarray]:
    """First `n_samples` samples of workload w (all of them if None): (X [n, n_in] f32, y [n] i32)."""
    n = w.n_samples if n_samples is None else min(n_samples, w.n_samples)
    x = features(w.feature_law, n, w.dims[0], w.seed)
    centre = 0.0 if w.feature_law == "normal" else 0.5
    y = teacher_labels(x, w.n_classes, w.seed, centre)
    return x, y


def to_batch_blocks(x: np.ndarray, batch: int, ld: int | None = None) -> np.ndarray:
    """Sample-major [n, f] -> feature-major minibatch blocks [n_batches, f, ld]: block k holds
    samples k*batch .. k*batch+batch-1 as columns (zero padding in the last block and beyond
    `batch` columns).  Pure layout change."""
    n, f = x.shape
    ld = batch if ld is None else ld
    nb = -(-n // batch)
    out = np.zeros((nb, f, ld), dtype=np.float32)
    for k in range(nb):
        blk = x[k * batch:(k + 1) * batch]
        out[k, :, : blk.shape[0]] = blk.T
    return out


def dense_operand(n: int, batch: int, seed: int, ld: int | None = None) -> np.ndarray:
    """[n, ld] float32 N(0,1) operand for single-kernel tests (columns >= batch are zero)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    ld = batch if ld is None else ld
    out = np.zeros((n, ld), dtype=np.float32)
    out[:, :batch] = rng.standard_normal((n, batch), dtype=np.float32)
    return out
