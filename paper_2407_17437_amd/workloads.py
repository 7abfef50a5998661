"""Seeded synthetic inputs for the sparse-MLP training path.

This module only *draws inputs*: sparsity patterns, initial values, batches and
labels.  It holds none of the arithmetic of the method (no products, no loss,
no update), so both the CPU oracle's tests and the HIP path's tests may use it
without sharing any computation.  Everything is numpy (PCG64 streams keyed by
the integer seeds given), fp32 values and int32 zero-based indices.

Shapes follow the paper's experiment (Section 5.1): an MLP 3072-1024-512-10 on
inputs with 3072 features, 10 classes, mini-batches of 100 examples stored one
example per column (Appendix B listing: ``Xtrain[:, batch]``).  The data set
itself is not available here; N(0,1) features and uniform labels stand in for
it.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

__all__ = [
    "round_half_up", "er_layer_densities", "er_layer_nnz", "uniform_layer_nnz",
    "uniform_pattern", "zipf_row_nnz", "pattern_from_row_nnz", "init_values",
    "make_batches", "SparseLayerData", "MLPData", "make_mlp", "make_zipf_matrix",
    "CIFAR_MLP", "WIDE_MLP",
]

CIFAR_MLP = (3072, 1024, 512, 10)      # Section 5.1
WIDE_MLP = (3072, 8192, 8192, 10)


def round_half_up(x: float) -> int:
    return int(math.floor(x + 0.5))


# --------------------------------------------------------------------------
# Per-layer densities
# --------------------------------------------------------------------------

def er_layer_densities(sizes: Sequence[int], global_density: float):
    """Erdos-Renyi split of a global density over the layers (Section 5.1).

    Layer l (n_in x n_out) gets density proportional to (n_in+n_out)/(n_in*n_out),
    so larger layers are sparser.  The factor eps is chosen so that the layer
    non-zero counts add up to round(global_density * total weights).  A layer
    whose density would exceed 1 is fixed fully dense and eps is solved again
    over the remaining layers.  Returns (densities, eps).
    """
    n_in = np.asarray(sizes[:-1], dtype=np.float64)
    n_out = np.asarray(sizes[1:], dtype=np.float64)
    size = n_in * n_out
    total = float(round_half_up(global_density * size.sum()))
    dense = np.zeros(len(size), dtype=bool)
    while True:
        free = ~dense
        remaining = total - size[dense].sum()
        # sum over free layers of eps*(n_in+n_out) = remaining
        eps = remaining / (n_in[free] + n_out[free]).sum()
        d = np.where(dense, 1.0, eps * (n_in + n_out) / size)
        over = (d > 1.0) & free
        if not over.any():
            return d, float(eps)
        dense |= over


def _apportion(targets: np.ndarray, total: int) -> List[int]:
    """Integers closest to `targets` that sum to `total` (largest remainder)."""
    base = np.floor(targets).astype(np.int64)
    short = int(total - base.sum())
    order = np.argsort(-(targets - base), kind="stable")
    base[order[:short]] += 1
    return [int(v) for v in base]


def er_layer_nnz(sizes: Sequence[int], global_density: float) -> List[int]:
    d, _ = er_layer_densities(sizes, global_density)
    size = np.asarray(sizes[:-1], dtype=np.float64) * np.asarray(sizes[1:], dtype=np.float64)
    total = round_half_up(global_density * size.sum())
    return _apportion(d * size, total)


def uniform_layer_nnz(sizes: Sequence[int], sparsity: float) -> List[int]:
    """Every layer at the same sparsity; nnz = round((1-s) * rows * cols)."""
    return [round_half_up((1.0 - sparsity) * a * b) for a, b in zip(sizes[:-1], sizes[1:])]


# --------------------------------------------------------------------------
# Patterns (canonical CSR: row pointers, column indices strictly ascending per row)
# --------------------------------------------------------------------------

def _csr_from_flat(flat_sorted: np.ndarray, rows: int, cols: int):
    r = flat_sorted // cols
    indices = (flat_sorted - r * cols).astype(np.int32)
    counts = np.bincount(r, minlength=rows)
    indptr = np.zeros(rows + 1, dtype=np.int32)
    np.cumsum(counts, out=indptr[1:])
    return indptr, indices


def uniform_pattern(rows: int, cols: int, nnz: int, seed: int):
    """`nnz` positions drawn uniformly without replacement from the rows x cols grid."""
    if not 0 <= nnz <= rows * cols:
        raise ValueError("nnz out of range")
    rng = np.random.default_rng(seed)
    n = rows * cols
    if nnz == n:
        flat = np.arange(n, dtype=np.int64)
    elif nnz * 4 >= n:
        flat = np.sort(rng.permutation(n)[:nnz].astype(np.int64))
    else:
        flat = np.sort(rng.choice(n, size=nnz, replace=False).astype(np.int64))
    return _csr_from_flat(flat, rows, cols)


def zipf_row_nnz(rows: int, cols: int, nnz: int, s: float, seed: int) -> np.ndarray:
    """Power-law row lengths: rank r gets weight r^-s, capped at `cols`.

    A scale is found by bisection so that sum(min(cols, scale*r^-s)) = nnz; the
    real-valued lengths are turned into integers by floor + largest remainder,
    and ranks are assigned to rows by a seeded permutation.
    """
    if not 0 <= nnz <= rows * cols:
        raise ValueError("nnz out of range")
    w = np.arange(1, rows + 1, dtype=np.float64) ** (-s)
    lo, hi = 0.0, float(cols) / w[-1]
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if np.minimum(cols, mid * w).sum() < nnz:
            lo = mid
        else:
            hi = mid
    t = np.minimum(cols, hi * w)
    t *= nnz / t.sum()
    t = np.minimum(t, cols)
    counts = np.floor(t).astype(np.int64)
    short = int(nnz - counts.sum())
    room = counts < cols
    order = np.argsort(-np.where(room, t - counts, -1.0), kind="stable")
    counts[order[:short]] += 1
    assert counts.sum() == nnz and counts.max() <= cols
    rng = np.random.default_rng(seed)
    out = np.empty(rows, dtype=np.int64)
    out[rng.permutation(rows)] = counts
    return out


def pattern_from_row_nnz(row_nnz: np.ndarray, cols: int, seed: int):
    """Columns uniform without replacement inside every row, ascending."""
    rng = np.random.default_rng(seed)
    rows = len(row_nnz)
    indptr = np.zeros(rows + 1, dtype=np.int64)
    np.cumsum(row_nnz, out=indptr[1:])
    indices = np.empty(int(indptr[-1]), dtype=np.int32)
    for i in range(rows):
        k = int(row_nnz[i])
        if k == 0:
            continue
        if k == cols:
            sel = np.arange(cols)
        elif k * 8 >= cols:
            sel = np.sort(rng.permutation(cols)[:k])
        else:
            sel = np.sort(rng.choice(cols, size=k, replace=False))
        indices[indptr[i]:indptr[i + 1]] = sel
    return indptr.astype(np.int32), indices


# --------------------------------------------------------------------------
# Values, batches
# --------------------------------------------------------------------------

def init_values(indptr: np.ndarray, seed: int) -> np.ndarray:
    """N(0, sqrt(2 / nnz of the row)) per stored weight, fp32."""
    rng = np.random.default_rng(seed)
    row_nnz = np.diff(indptr).astype(np.int64)
    std = np.sqrt(2.0 / np.maximum(1, row_nnz))
    z = rng.standard_normal(int(indptr[-1]))
    return (z * np.repeat(std, row_nnz)).astype(np.float32)


def make_batches(features: int, classes: int, batch: int, n_batches: int, seed: int):
    """`n_batches` blocks of N(0,1) inputs, shape (n_batches, features, batch), one
    example per column, and uniform integer labels, shape (n_batches, batch)."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n_batches, features, batch), dtype=np.float32)
    T = rng.integers(0, classes, size=(n_batches, batch), dtype=np.int32)
    return X, T


@dataclass
class SparseLayerData:
    rows: int                # n_out
    cols: int                # n_in
    indptr: np.ndarray       # int32[rows+1]
    indices: np.ndarray      # int32[nnz]
    values: np.ndarray       # float32[nnz]
    bias: np.ndarray         # float32[rows]
    relu: bool               # ReLU on the output (hidden layers) or none (last layer)

    @property
    def nnz(self) -> int:
        return int(self.indptr[-1])


@dataclass
class MLPData:
    sizes: Sequence[int]
    layers: List[SparseLayerData] = field(default_factory=list)

    @property
    def nnz(self) -> int:
        return sum(l.nnz for l in self.layers)


def make_mlp(sizes: Sequence[int], *, sparsity: float | None = None,
             er_density: float | None = None, layer_nnz: Sequence[int] | None = None,
             pattern_seed: int = 1000, value_seed: int = 2000,
             bias_std: float = 0.0) -> MLPData:
    """Static-sparse MLP: layer l is an (sizes[l+1] x sizes[l]) CSR matrix.

    Exactly one of `sparsity` (same for every layer), `er_density` (global density
    split by the Erdos-Renyi rule) or `layer_nnz` must be given.  Biases are dense
    and start at zero unless `bias_std` > 0 (used by tests so that bias terms matter).
    """
    given = [sparsity is not None, er_density is not None, layer_nnz is not None]
    if sum(given) != 1:
        raise ValueError("give exactly one of sparsity / er_density / layer_nnz")
    if sparsity is not None:
        nnzs = uniform_layer_nnz(sizes, sparsity)
    elif er_density is not None:
        nnzs = er_layer_nnz(sizes, er_density)
    else:
        nnzs = list(layer_nnz)
    mlp = MLPData(sizes=tuple(sizes))
    L = len(sizes) - 1
    for l in range(L):
        cols, rows = sizes[l], sizes[l + 1]
        indptr, indices = uniform_pattern(rows, cols, nnzs[l], pattern_seed + l + 1)
        values = init_values(indptr, value_seed + l + 1)
        if bias_std > 0:
            bias = (np.random.default_rng(value_seed + 500 + l).standard_normal(rows)
                    * bias_std).astype(np.float32)
        else:
            bias = np.zeros(rows, dtype=np.float32)
        mlp.layers.append(SparseLayerData(rows, cols, indptr, indices, values, bias, relu=(l < L - 1)))
    return mlp


def make_zipf_matrix(n: int, density: float, seed: int, s: float = 1.2) -> SparseLayerData:
    """Square n x n CSR with power-law row lengths and N(0,1) values."""
    nnz = round_half_up(density * n * n)
    rn = zipf_row_nnz(n, n, nnz, s, seed)
    indptr, indices = pattern_from_row_nnz(rn, n, seed + 1)
    rng = np.random.default_rng(seed + 2)
    values = rng.standard_normal(nnz, dtype=np.float32)
    bias = np.zeros(n, dtype=np.float32)
    return SparseLayerData(n, n, indptr, indices, values, bias, relu=False)
