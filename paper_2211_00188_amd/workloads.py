"""Seeded synthetic inputs shaped like the workloads AdaCGD is run on.

This module holds input generators only -- none of the method's arithmetic.
Everything is drawn on the host with NumPy's counter-based Philox bit
generator, so the same seed gives the same bytes everywhere; callers upload the
arrays to the device themselves.  The experiments of the paper (Section 6 and
its appendix) use logistic regression on LIBSVM data split evenly over n = 20
clients; those files are not redistributed here, so the logistic workloads
below are synthetic stand-ins with the same structure (equal shards, +-1
labels, dense or binary sparse features).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

TOPK = 0
QUANT = 1
QUANT_BLOCK = 2     # level (QUANT_BLOCK, (bits, block length))
RANK = 3            # level (RANK, (rank, columns))


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


@dataclass
class LogisticWorkload:
    name: str
    n: int
    d: int
    A: np.ndarray              # [sum N_i, d] float32 row-major
    labels: np.ndarray         # [sum N_i] float32 in {-1,+1}
    shard_offsets: np.ndarray  # [n+1] int64
    lam: float
    gamma: float
    worker_levels: list
    master_levels: list
    zeta_worker: float
    zeta_master: float
    T: int
    csr: tuple = None          # (row_ptr, col, val or None) when the features are kept as sparse rows

    def shards(self):
        o = self.shard_offsets
        return [(self.A[o[i]:o[i + 1]], self.labels[o[i]:o[i + 1]]) for i in range(self.n)]


@dataclass
class VectorWorkload:
    name: str
    n: int
    d: int
    worker_levels: list
    master_levels: list
    zeta_worker: float
    zeta_master: float
    T: int
    seed: int


def ratio_K(ratio: float, d: int) -> int:
    """K for a level given as a fraction of d: the ceiling, at least 1."""
    return max(1, min(d, math.ceil(ratio * d - 1e-9)))


def federated_levels(d: int) -> list:
    """Mixed level set of the federated configuration, listed in the order the cascade walks it at
    the configuration's full size d = 65536 (strongest compression first).  At other sizes the
    caller orders the set itself, or lets the library accept any order."""
    lv = [(TOPK, min(d, 16)), (TOPK, min(d, 256)), (QUANT, 4), (TOPK, min(d, 4096)), (QUANT, 8)]
    return list(dict.fromkeys(lv))


def kernel_stress_levels(d: int) -> list:
    """Mixed level set of the kernel-stress configuration, in the cascade's order at d = 2^20
    (see federated_levels for other sizes)."""
    lv = [(QUANT, 2), (TOPK, ratio_K(0.001, d)), (QUANT, 4), (TOPK, ratio_K(0.01, d)), (TOPK, ratio_K(0.1, d)),
          (QUANT, 8)]
    return list(dict.fromkeys(lv))


def _planted_labels(rng, A, w):
    z = A.astype(np.float64) @ w
    p = 1.0 / (1.0 + np.exp(-z))
    return np.where(p - rng.random(A.shape[0]) > 0, 1.0, -1.0).astype(np.float32)


def to_csr(A: np.ndarray, binary: bool = False):
    """Compressed-sparse-row arrays (row_ptr int64, col int32, val float32 or None) of the
    non-zero entries of a dense matrix, columns ascending inside every row.  `binary`: the
    matrix holds only 0 and 1 and no value array is returned."""
    rows, cols = np.nonzero(A)                      # row-major order: rows, then columns, ascending
    row_ptr = np.zeros(A.shape[0] + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=A.shape[0]), out=row_ptr[1:])
    val = None if binary else np.ascontiguousarray(A[rows, cols], dtype=np.float32)
    if binary:
        assert np.all(A[rows, cols] == 1)
    return row_ptr, cols.astype(np.int32), val


def tiny(seed=1, n=4, d=100, N=64, T=100, zeta=1.0) -> LogisticWorkload:
    """n=4 workers, d=100, 64 dense N(0,1) samples each, labels from a planted
    logistic model; Top-K levels {1,5,10,25,d}, master Top-25."""
    rng = _rng(seed)
    A = rng.standard_normal((n * N, d), dtype=np.float32)
    w = rng.standard_normal(d) / math.sqrt(d)
    labels = _planted_labels(rng, A, w)
    Ks = sorted({min(d, k) for k in (1, 5, 10, 25, d)})
    return LogisticWorkload("tiny", n, d, A, labels, np.arange(n + 1, dtype=np.int64) * N, 0.1, 0.1,
                            [(TOPK, k) for k in Ks], [(TOPK, min(d, 25))], zeta, 0.0, T)


def sparse_logreg(seed=2, n=20, d=300, N=2500, T=1000, zeta=1.0) -> LogisticWorkload:
    """n=20 equal shards of binary features at 4 % density (stored dense), labels
    from a planted weight vector thresholded at the median with 5 % flips."""
    rng = _rng(seed)
    A = (rng.random((n * N, d), dtype=np.float32) < 0.04).astype(np.float32)
    w = rng.standard_normal(d)
    z = A.astype(np.float64) @ w
    labels = np.where(z - np.median(z) > 0, 1.0, -1.0)
    flip = rng.random(n * N) < 0.05
    labels = np.where(flip, -labels, labels).astype(np.float32)
    Ks = sorted({min(d, k) for k in (1, 2, 5, 10, 30, d)})
    return LogisticWorkload("sparse_logreg", n, d, A, labels, np.arange(n + 1, dtype=np.int64) * N, 0.1, 0.1,
                            [(TOPK, k) for k in Ks], [(TOPK, min(d, 30))], zeta, 0.0, T)


def federated(seed=5, n=1000, d=65536, N=32, T=200, zeta=1.0, clusters=10) -> LogisticWorkload:
    """Many small shards; worker i's labels come from planted model i mod clusters.
    Mixed Top-K / b-bit level set, bidirectional with a Top-K master."""
    rng = _rng(seed)
    A = rng.standard_normal((n * N, d), dtype=np.float32)
    W = rng.standard_normal((clusters, d)) / math.sqrt(d)
    labels = np.empty(n * N, dtype=np.float32)
    for i in range(n):
        labels[i * N:(i + 1) * N] = _planted_labels(rng, A[i * N:(i + 1) * N], W[i % clusters])
    lv = federated_levels(d)
    return LogisticWorkload("federated", n, d, A, labels, np.arange(n + 1, dtype=np.int64) * N, 0.1, 0.1,
                            lv, [(TOPK, min(d, 4096))], zeta, 0.0, T)


def sparse_features(seed=6, n=200, d=65536, N=1000, per_row=64, T=50, zeta=1.0) -> LogisticWorkload:
    """Binary features kept as sparse rows only (no dense copy): every row stores `per_row` ones, one in
    each of `per_row` equal column strata (so the columns of a row are distinct and ascending); labels
    from a planted weight vector with 5 % flips.  Stands in for high-dimensional sparse LIBSVM-style
    data split over many workers."""
    rng = _rng(seed)
    rows = n * N
    stride = d // per_row
    col = (np.arange(per_row, dtype=np.int64)[None, :] * stride
           + rng.integers(0, stride, size=(rows, per_row))).astype(np.int32)
    w = rng.standard_normal(d)
    z = w[col].sum(axis=1)
    labels = np.where(z - np.median(z) > 0, 1.0, -1.0)
    labels = np.where(rng.random(rows) < 0.05, -labels, labels).astype(np.float32)
    row_ptr = np.arange(rows + 1, dtype=np.int64) * per_row
    lv = [(TOPK, ratio_K(r, d)) for r in (1e-3, 1e-2, 5e-2, 0.25)]
    return LogisticWorkload("sparse_features", n, d, None, labels, np.arange(n + 1, dtype=np.int64) * N, 0.1, 0.5,
                            lv, [(TOPK, ratio_K(0.05, d))], zeta, 0.0, T, csr=(row_ptr, col.reshape(-1), None))


def kernel_stress(seed=3, n=32, d=1 << 20, T=50, zeta=1.0) -> VectorWorkload:
    """Heavy-tailed difference vectors with a mixed Top-K / b-bit level set."""
    lv = kernel_stress_levels(d)
    return VectorWorkload("kernel_stress", n, d, lv, [(TOPK, ratio_K(0.01, d))], zeta, 0.0, T, seed)


def kernel_stress_diffs(wl: VectorWorkload, step: int):
    """Difference vectors v_i = exp(N(0,1)) * t_3 (Student-t, 3 degrees of freedom) and
    trigger right-hand sides D_i = ||v_i||^2 * 10^U(-3, 0.2) / zeta, so that every branch
    of the level cascade occurs.  Returns (v [n,d] float32, D [n] float64)."""
    rng = _rng([wl.seed, step])
    scale = np.exp(rng.standard_normal(wl.n)).astype(np.float32)
    v = rng.standard_t(3.0, size=(wl.n, wl.d)).astype(np.float32) * scale[:, None]
    S = np.sum(v.astype(np.float64) ** 2, axis=1)
    D = S * 10.0 ** rng.uniform(-3.0, 0.2, size=wl.n) / max(wl.zeta_worker, 1e-30)
    return v, D


def kernel_stress_blockwise(seed=3, n=32, d=1 << 20, T=50, zeta=1.0, block=256) -> VectorWorkload:
    """The kernel-stress vectors with block-wise quantisers (one scale per `block` coordinates) in place of
    the whole-vector ones, in the cascade's order at d = 2^20 and block = 256."""
    lv = [(TOPK, ratio_K(0.001, d)), (TOPK, ratio_K(0.01, d)), (QUANT_BLOCK, (2, block)), (TOPK, ratio_K(0.1, d)),
          (QUANT_BLOCK, (4, block)), (QUANT_BLOCK, (8, block))]
    return VectorWorkload("kernel_stress_blockwise", n, d, lv, [(TOPK, ratio_K(0.01, d))], zeta, 0.0, T, seed)


def matrix_shaped(seed=7, n=16, rows=16384, cols=64, T=20, zeta=1.0) -> VectorWorkload:
    """Matrix-shaped gradients (a layer's rows x cols weight gradient, flattened row-major) with Rank-K
    levels K in {1, 4, 16} next to the identity; master Top-K at 1 %."""
    d = rows * cols
    lv = [(RANK, (1, cols)), (RANK, (min(4, cols), cols)), (RANK, (min(16, cols), cols)), (TOPK, d)]
    lv = list(dict.fromkeys(lv))
    wl = VectorWorkload("matrix_shaped", n, d, lv, [(TOPK, ratio_K(0.01, d))], zeta, 0.0, T, seed)
    wl.rows, wl.cols = rows, cols
    return wl


class MatrixShapedGrads:
    """grad_i^t = L_i^t R + 0.3 E_i^t as a rows x cols matrix: R (8 x cols) is a fixed set of shared
    directions with weights 8, 4, 2, 1, 1/2, ...; the per-worker left factors follow an AR(1) drift
    L^t = 0.9 L^{t-1} + sqrt(1 - 0.81) xi^t; E is fresh N(0,1) noise.  Returns [n, d] float32."""

    def __init__(self, wl: VectorWorkload, k=8):
        self.wl, self.k = wl, k
        rng = _rng([wl.seed, 2_000_003])
        self.R = (rng.standard_normal((k, wl.cols)) * (8.0 * 0.5 ** np.arange(k))[:, None]).astype(np.float32)
        self.rng = _rng([wl.seed, 2_000_029])
        self.L = self.rng.standard_normal((wl.n, wl.rows, k), dtype=np.float32)

    def next(self):
        wl = self.wl
        out = (self.L @ self.R + np.float32(0.3) * self.rng.standard_normal((wl.n, wl.rows, wl.cols), dtype=np.float32))
        xi = self.rng.standard_normal(self.L.shape, dtype=np.float32)
        self.L = (np.float32(0.9) * self.L + np.float32(math.sqrt(1 - 0.81)) * xi).astype(np.float32)
        return np.ascontiguousarray(out.reshape(wl.n, wl.d), dtype=np.float32)


def model_sized(seed=4, n=16, d=11_200_000, T=20, zeta=1.0) -> VectorWorkload:
    """Model-sized gradient vectors; Top-K levels at fractions {1e-4,1e-3,1e-2,5e-2} of d."""
    lv = list(dict.fromkeys((TOPK, ratio_K(r, d)) for r in (1e-4, 1e-3, 1e-2, 5e-2)))    # ascending K
    return VectorWorkload("model_sized", n, d, lv, [(TOPK, ratio_K(1e-2, d))], zeta, 0.0, T, seed)


class ModelSizedGrads:
    """grad_i^t = z^t + 0.5 h_i with fixed per-worker offsets h_i ~ N(0,I) and a shared
    drift z^t = 0.95 z^{t-1} + sqrt(1 - 0.95^2) xi^t (unit marginal variance).  `out`, if
    given, is a preallocated [n,d] float32 array (for example pinned host memory)."""

    def __init__(self, wl: VectorWorkload, rho=0.95, sigma=0.5):
        self.wl, self.rho, self.sigma = wl, rho, sigma
        self.h = _rng([wl.seed, 1_000_003]).standard_normal((wl.n, wl.d), dtype=np.float32)
        self.rng = _rng([wl.seed, 1_000_033])
        self.z = self.rng.standard_normal(wl.d, dtype=np.float32)

    def next(self, out=None):
        if out is None:
            out = np.empty((self.wl.n, self.wl.d), dtype=np.float32)
        np.multiply(self.h, np.float32(self.sigma), out=out)
        out += self.z[None, :]
        xi = self.rng.standard_normal(self.wl.d, dtype=np.float32)
        self.z = (np.float32(self.rho) * self.z + np.float32(math.sqrt(1 - self.rho ** 2)) * xi).astype(np.float32)
        return out
