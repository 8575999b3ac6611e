"""Seeded synthetic inputs for the EF21 hot path.

This module holds input generators only: none of the method's arithmetic (no gradient, no
compressor, no update) lives here, so the same arrays can be fed to any implementation.
Everything is drawn on the host with ``numpy.random.default_rng(seed)`` in the order written
in each function, so a (function, arguments, seed) triple names one fixed input.

The shapes follow the experiments of the paper (Section 5 and Appendix A): a logistic
regression data set split evenly over n workers, and flat gradient vectors at the scale of a
small convolutional network.  The data sets themselves are not reproduced; only shape
classes and value scales are borrowed.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class DenseLogReg:
    A: np.ndarray        # [n][m][d] float32
    y: np.ndarray        # [n][m] float32, +1 / -1
    w_star: np.ndarray   # [d] float64 (the labelling vector; not an input of the method)


@dataclass
class CSRLogReg:
    rowptr: np.ndarray   # [n*m+1] int64
    col: np.ndarray      # [nnz] int32, ascending inside each row
    val: np.ndarray      # [nnz] float32
    y: np.ndarray        # [n][m] float32, +1 / -1
    n: int
    m: int
    d: int


def _labels(z: np.ndarray, rng, flip: float) -> np.ndarray:
    """sign(z) with sign(0) = +1, then each label flipped independently with probability `flip`."""
    y = np.where(z >= 0.0, 1.0, -1.0)
    y = np.where(rng.random(z.shape) < flip, -y, y)
    return y.astype(np.float32)


def logreg_dense(n: int, d: int, m: int, seed: int = 0, flip: float = 0.1) -> DenseLogReg:
    """Draw order: w* ~ N(0, I_d); then per worker i: A_i ~ N(0,1)[m][d] / sqrt(d) (float32),
    y_i = sign(A_i w*), flip mask U(0,1) < flip."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(d)
    A = np.empty((n, m, d), dtype=np.float32)
    y = np.empty((n, m), dtype=np.float32)
    scale = np.float32(1.0 / np.sqrt(d))
    for i in range(n):
        A[i] = rng.standard_normal((m, d), dtype=np.float32) * scale
        y[i] = _labels(A[i].astype(np.float64) @ w, rng, flip)
    return DenseLogReg(A, y, w)


def _distinct_sorted_columns(rng, rows: int, d: int, per_row: int) -> np.ndarray:
    """`per_row` distinct column indices per row, uniform without replacement, ascending.
    Drawn with replacement, then every repeated entry is redrawn until the row has no repeats;
    rejecting values already present is sequential sampling without replacement."""
    c = np.sort(rng.integers(0, d, size=(rows, per_row), dtype=np.int32), axis=1)
    while True:
        dup = np.zeros(c.shape, dtype=bool)
        dup[:, 1:] = c[:, 1:] == c[:, :-1]
        ndup = int(dup.sum())
        if ndup == 0:
            return c
        c[dup] = rng.integers(0, d, size=ndup, dtype=np.int32)
        c.sort(axis=1)


def logreg_csr(n: int, d: int, m: int, nnz_per_row: int, seed: int = 0, flip: float = 0.1) -> CSRLogReg:
    """Draw order: w* ~ N(0, I_d); then per worker i: column indices (see above), values
    U(0,1) float32, y_i = sign(A_i w*), flip mask.  One CSR over all n*m rows."""
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(d)
    col = np.empty((n * m, nnz_per_row), dtype=np.int32)
    val = np.empty((n * m, nnz_per_row), dtype=np.float32)
    y = np.empty((n, m), dtype=np.float32)
    for i in range(n):
        c = _distinct_sorted_columns(rng, m, d, nnz_per_row)
        v = rng.random((m, nnz_per_row), dtype=np.float32)
        z = np.einsum("lp,lp->l", v.astype(np.float64), w[c])
        y[i] = _labels(z, rng, flip)
        col[i * m:(i + 1) * m] = c
        val[i * m:(i + 1) * m] = v
    rowptr = np.arange(n * m + 1, dtype=np.int64) * nnz_per_row
    return CSRLogReg(rowptr, col.reshape(-1), val.reshape(-1), y, n, m, d)


def topk_rows(n: int, d: int, seed: int = 0, dup_frac: float = 0.01) -> np.ndarray:
    """[n][d] float32 ~ N(0,1); then per row a fraction `dup_frac` of positions (chosen without
    replacement) is overwritten with the value found at another uniformly drawn position, every
    second copy negated, so that exact magnitude ties (+a / -a included) exist."""
    rng = np.random.default_rng(seed)
    V = rng.standard_normal((n, d), dtype=np.float32)
    ndup = int(round(dup_frac * d))
    for i in range(n):
        if ndup == 0:
            break
        dst = rng.choice(d, size=ndup, replace=False)
        src = rng.integers(0, d, size=ndup)
        vals = V[i, src].copy()
        vals[1::2] = -vals[1::2]
        V[i, dst] = vals
    return V


def force_threshold_ties(V: np.ndarray, k: int, copies: int = 8, seed: int = 0) -> np.ndarray:
    """Copy of V in which, per row, the k-th largest magnitude is written into `copies` further
    random positions with alternating sign: the selection threshold itself is tied."""
    rng = np.random.default_rng(seed)
    W = V.copy()
    n, d = W.shape
    for i in range(n):
        mag = np.abs(W[i])
        kth = np.partition(mag, d - k)[d - k]
        pos = rng.choice(d, size=min(copies, d), replace=False)
        sign = np.where(np.arange(pos.size) % 2 == 0, 1.0, -1.0).astype(np.float32)
        W[i, pos] = kth * sign
    return W


def student_t_grads(n: int, d: int, seed: int = 0, nu: float = 3.0, scale: float = 1e-3) -> np.ndarray:
    """[n][d] float32 heavy-tailed stand-in for flat network gradients: scale * t_nu."""
    rng = np.random.default_rng(seed)
    out = np.empty((n, d), dtype=np.float32)
    for i in range(n):
        out[i] = (rng.standard_t(nu, size=d) * scale).astype(np.float32)
    return out


def student_t_grads_on_device(n: int, d: int, count: int, seed: int = 0, scale: float = 1e-3, device: str = "cuda"):
    """`count` independent [n][d] float32 draws of scale * t_3 made on the device (torch's generator, seeded):
    a standard normal over the root mean square of three others.  For timing runs that need a fresh
    gradient every step and cannot wait for the host generator; parity tests use student_t_grads."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    out = []
    for _ in range(count):
        z = torch.randn((n, d), device=device, generator=gen)
        chi = torch.randn((3, n, d), device=device, generator=gen).square_().sum(0).div_(3.0).sqrt_()
        out.append((z.div_(chi).mul_(scale)).contiguous())
        del chi
    return out


# The configurations the build is measured and tested on (sizes only; see each generator).
CONFIGS = {
    "C0": dict(kind="dense", n=4, d=100, m=250, k=1, gamma=0.1, lam=0.1, iters=100, seed=0),
    "C1": dict(kind="topk", n=20, d=1_000_000, ks=(1, 1000, 10000), seed=0),
    "C2": dict(kind="dense", n=20, d=2000, m=5000, k=20, gamma=0.5, lam=0.1, iters=1000, seed=0),
    "C3": dict(kind="csr", n=100, d=50_000, m=2000, nnz_per_row=500, k=500, gamma=0.5, lam=0.1, iters=500,
               seed=0),
    "C4": dict(kind="grads", n=8, d=11_200_000, k=112_000, gamma=0.01, iters=200, seed=0),
}
