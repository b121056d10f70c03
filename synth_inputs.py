"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU tests.

This module holds NO arithmetic of the method (no similarity, no quota, no
greedy): it only draws feature matrices, labels and capacity vectors.  The
features stand in for the auto-encoder bottleneck features of CIFAR-10/100
that the paper partitions (Section 4); shapes follow those data sets' class
structure, values follow a Gaussian mixture per class.

Recipe (one numpy Generator per configuration, seeded):
  1. "cifar100" only: r = rng.integers(1, 5, size=K)   (capacities in {1..4})
  2. for each class in order:
        centers = rng.standard_normal((G, d))
        comp    = rng.integers(0, G, n_c)
        X_c     = centers[comp] + 0.5 * rng.standard_normal((n_c, d))
  3. cast to float32 (bf16 configurations: round to nearest even to bf16)
  4. one rng.permutation(N) shuffles rows and labels together
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    L: int            # classes
    n_c: int          # samples per class
    d: int            # feature dimension
    dtype: str        # "f32" | "bf16"
    K: int            # workers
    r: Optional[tuple]  # capacities; None = drawn from the generator (step 1)
    G: int            # mixture components per class
    seed: int

    @property
    def N(self) -> int:
        return self.L * self.n_c


WORKLOADS = {
    "tiny": Workload("tiny", 4, 250, 64, "f32", 2, (1, 1), 4, 0),
    "cifar10": Workload("cifar10", 10, 5000, 512, "f32", 4, (1, 1, 2, 4), 4, 1),
    "hetero8": Workload("hetero8", 10, 5000, 512, "f32", 8, (1, 1, 1, 2, 2, 3, 4, 6), 4, 2),
    "cifar100": Workload("cifar100", 100, 500, 512, "f32", 16, None, 4, 3),
    "large": Workload("large", 20, 50000, 2048, "bf16", 8, (1, 1, 2, 2, 3, 3, 4, 8), 8, 4),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


@dataclass
class Dataset:
    X: np.ndarray          # (N, d) float32, or uint16 bf16 bit patterns
    labels: np.ndarray     # (N,) int32
    r: np.ndarray          # (K,) int64 capacities
    L: int
    sigma2: float
    workload: Workload = field(repr=False)


def class_features(rng: np.random.Generator, n_c: int, d: int, G: int) -> np.ndarray:
    centers = rng.standard_normal((G, d))
    comp = rng.integers(0, G, n_c)
    return centers[comp] + 0.5 * rng.standard_normal((n_c, d))


def make_dataset(w: Workload, L: Optional[int] = None, n_c: Optional[int] = None,
                 d: Optional[int] = None, shuffle: bool = True) -> Dataset:
    """Draw the data set of a workload; L / n_c / d override its shape for
    scaled-down instances (same recipe, same seed)."""
    L = w.L if L is None else L
    n_c = w.n_c if n_c is None else n_c
    d = w.d if d is None else d
    rng = np.random.default_rng(w.seed)
    if w.r is None:
        r = rng.integers(1, 5, size=w.K).astype(np.int64)
    else:
        r = np.asarray(w.r, dtype=np.int64)
    blocks: List[np.ndarray] = []
    labels: List[np.ndarray] = []
    for c in range(L):
        blocks.append(class_features(rng, n_c, d, w.G).astype(np.float32))
        labels.append(np.full(n_c, c, dtype=np.int32))
    X = np.concatenate(blocks, axis=0) if blocks else np.zeros((0, d), np.float32)
    y = np.concatenate(labels, axis=0) if labels else np.zeros((0,), np.int32)
    if shuffle:
        perm = rng.permutation(X.shape[0])
        X = X[perm]
        y = y[perm]
    X = np.ascontiguousarray(X)
    if w.dtype == "bf16":
        X = f32_to_bf16_bits(X)
    return Dataset(X=X, labels=np.ascontiguousarray(y), r=r, L=L, sigma2=float(d), workload=w)


def make_class(seed: int, n: int, d: int, G: int = 4, dtype: str = "f32") -> np.ndarray:
    """One class worth of mixture features (no labels, no shuffle)."""
    rng = np.random.default_rng(seed)
    X = class_features(rng, n, d, G).astype(np.float32)
    return f32_to_bf16_bits(X) if dtype == "bf16" else X
