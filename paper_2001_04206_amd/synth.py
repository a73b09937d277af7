"""Seeded synthetic inputs for dense-network training runs.

This module only draws numbers: data sets, labels and initial parameters with
the shapes and value distributions of the workloads the library is exercised
on.  It holds none of the training arithmetic and is the single piece of code
that feeds both the device library and the independent CPU checker used by
the tests, so both sides see bit-identical fp32 inputs.

Draw order for one workload (numpy ``default_rng(seed)``): X, labels, then
W_1 ... W_L.  Biases start at zero.  The paper only says that weights and
biases are initialised before training (section "The Deep Netts Work-flow")
and names no distribution; the distributions here are the usual textbook ones.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

# Activation and loss identifiers (values match the C enums of the library
# and, independently, those of the CPU checker).
ACT_LINEAR, ACT_SIGMOID, ACT_TANH, ACT_RELU, ACT_SOFTMAX = 0, 1, 2, 3, 4
LOSS_MSE, LOSS_CROSS_ENTROPY = 0, 1


@dataclass
class Workload:
    name: str
    widths: List[int]
    acts: List[int]
    loss: int
    batch: int
    lr: float
    momentum: float
    epochs: int
    X: np.ndarray                       # [N, n0] float32
    labels: np.ndarray                  # [N] int32 class ids
    W: List[np.ndarray] = field(default_factory=list)   # W_l [n_l, n_{l-1}] float32
    b: List[np.ndarray] = field(default_factory=list)   # b_l [n_l] float32

    @property
    def n_samples(self) -> int:
        return int(self.X.shape[0])


def _features(rng, kind: str, n: int, d: int) -> np.ndarray:
    if kind == "uniform01":
        return rng.random((n, d), dtype=np.float32)
    if kind == "bytes255":
        k = rng.integers(0, 256, size=(n, d), dtype=np.int32)
        return (k.astype(np.float32) / np.float32(255.0)).astype(np.float32)
    if kind == "normal":
        return rng.standard_normal((n, d), dtype=np.float32)
    raise ValueError(kind)


def _init(rng, kind: str, n_out: int, n_in: int) -> np.ndarray:
    if kind == "uniform_half":           # U[-0.5, 0.5)
        return (rng.random((n_out, n_in), dtype=np.float32) - np.float32(0.5)).astype(np.float32)
    if kind == "xavier_uniform":         # U(-r, r), r = sqrt(6 / (fan_in + fan_out))
        r = np.float32(np.sqrt(6.0 / (n_in + n_out)))
        return ((rng.random((n_out, n_in), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)) * r).astype(np.float32)
    if kind == "he_normal":              # N(0, 2 / fan_in)
        s = np.float32(np.sqrt(2.0 / n_in))
        return (rng.standard_normal((n_out, n_in), dtype=np.float32) * s).astype(np.float32)
    raise ValueError(kind)


def make(name: str, widths: Sequence[int], acts: Sequence[int], loss: int, *,
         n_samples: int, features: str, init: str, batch: int, lr: float,
         momentum: float, epochs: int = 1, seed: int = 0) -> Workload:
    """Draw one workload.  ``features`` in {uniform01, bytes255, normal};
    ``init`` in {uniform_half, xavier_uniform, he_normal}."""
    widths = [int(w) for w in widths]
    rng = np.random.default_rng(seed)
    X = _features(rng, features, n_samples, widths[0])
    labels = rng.integers(0, widths[-1], size=n_samples, dtype=np.int32)
    W = [_init(rng, init, widths[l + 1], widths[l]) for l in range(len(widths) - 1)]
    b = [np.zeros(widths[l + 1], dtype=np.float32) for l in range(len(widths) - 1)]
    return Workload(name, widths, list(acts), loss, batch, float(lr), float(momentum),
                    epochs, np.ascontiguousarray(X), np.ascontiguousarray(labels), W, b)


# --- the five named workloads -------------------------------------------------

def iris_like(n_samples: int = 150, seed: int = 0) -> Workload:
    """4-16-3, sigmoid/sigmoid, MSE, online SGD: the shape of the 150x4,
    3-class set the paper's benchmark application loads (section "Benchmark
    Application"); values are synthetic."""
    return make("mlp_4_16_3_online", [4, 16, 3], [ACT_SIGMOID, ACT_SIGMOID], LOSS_MSE,
                n_samples=n_samples, features="uniform01", init="uniform_half",
                batch=1, lr=0.01, momentum=0.0, epochs=10, seed=seed)


def digits_like_online(n_samples: int = 60000, seed: int = 0) -> Workload:
    """784-128-10, ReLU / softmax + cross-entropy, online SGD; features have the
    shape and value grid of an 8-bit 28x28 image set, labels are random."""
    return make("mlp_784_128_10_online", [784, 128, 10], [ACT_RELU, ACT_SOFTMAX],
                LOSS_CROSS_ENTROPY, n_samples=n_samples, features="bytes255",
                init="xavier_uniform", batch=1, lr=0.01, momentum=0.0, seed=seed)


def digits_like_minibatch(n_samples: int = 60000, seed: int = 0) -> Workload:
    """Same network and data as ``digits_like_online``; minibatch 128 with momentum."""
    w = make("mlp_784_128_10_b128", [784, 128, 10], [ACT_RELU, ACT_SOFTMAX],
             LOSS_CROSS_ENTROPY, n_samples=n_samples, features="bytes255",
             init="xavier_uniform", batch=128, lr=0.05, momentum=0.9, seed=seed)
    return w


def wide_relu(n_samples: int = 65536, seed: int = 0, widths=(4096, 4096, 4096, 1000),
              batch: int = 256) -> Workload:
    """4096-4096-4096-1000, ReLU hidden, softmax + cross-entropy, He-normal
    init, minibatch 256 with momentum 0.9."""
    widths = list(widths)
    acts = [ACT_RELU] * (len(widths) - 2) + [ACT_SOFTMAX]
    return make("mlp_4096x3_1000_b%d" % batch, widths, acts, LOSS_CROSS_ENTROPY,
                n_samples=n_samples, features="normal", init="he_normal",
                batch=batch, lr=0.01, momentum=0.9, seed=seed)


def tanh_sweep(batch: int, n_samples: int = 16384, seed: int = 0,
               widths=(1024, 1024, 1024, 1024, 10)) -> Workload:
    """1024-1024-1024-1024-10 with tanh hidden layers, softmax + cross-entropy;
    one point of the batch-size sweep (plain SGD, lr 0.01, Xavier-uniform)."""
    widths = list(widths)
    acts = [ACT_TANH] * (len(widths) - 2) + [ACT_SOFTMAX]
    return make("mlp_1024x4_10_b%d" % batch, widths, acts, LOSS_CROSS_ENTROPY,
                n_samples=n_samples, features="normal", init="xavier_uniform",
                batch=batch, lr=0.01, momentum=0.0, seed=seed)


def paper_shape(n_samples: int = 64, seed: int = 0, hidden: int = 100000) -> Workload:
    """340 -> 100000 (tanh) -> 10 softmax + cross-entropy, online SGD: the
    network of the paper's evaluation (section "Benchmark Application") on
    synthetic features and labels."""
    return make("mlp_340_%d_10_online" % hidden, [340, hidden, 10], [ACT_TANH, ACT_SOFTMAX],
                LOSS_CROSS_ENTROPY, n_samples=n_samples, features="uniform01",
                init="xavier_uniform", batch=1, lr=0.01, momentum=0.0, seed=seed)


def learnable(widths: Sequence[int] = (20, 32, 4), n_samples: int = 400, batch: int = 8, lr: float = 0.1,
              momentum: float = 0.0, seed: int = 0) -> Workload:
    """A task with signal, for the loss-gated training loop and the held-out test: labels are the
    index of the largest of n_L fixed random projections of the features (all other workloads
    have random labels, on which the loss cannot fall).  Extra draw after the usual ones: the
    projection matrix."""
    acts = [ACT_TANH] * (len(widths) - 2) + [ACT_SOFTMAX]
    w = make("learnable", widths, acts, LOSS_CROSS_ENTROPY, n_samples=n_samples, features="normal",
             init="xavier_uniform", batch=batch, lr=lr, momentum=momentum, seed=seed)
    rng = np.random.default_rng(seed + 1000003)
    T = rng.standard_normal((w.widths[0], w.widths[-1]))
    w.labels = np.ascontiguousarray(np.argmax(w.X.astype(np.float64) @ T, axis=1).astype(np.int32))
    return w
