"""Seeded synthetic inputs shaped like the workloads of the sparse-linear-model experiments.

This module only makes DATA (design matrices, labels, minibatch row ids, worker gradients).
It contains none of the method's arithmetic and is used by the tests, the smoke check and the
benchmark to feed the same bits to the GPU library and to the CPU checker.

The paper's linear-model experiments use LIBSVM news20 / rcv1 (Section 5.1, Table 1): very
high-dimensional, very sparse rows, +-1 labels, small minibatches per worker.  Those datasets
are not available here; the generators below are stand-ins of the same kind of shape and do
not reproduce any of their records.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


# --------------------------------------------------------------------------------------
# Data sets for the full training loop (local gradient -> ... -> update)
# --------------------------------------------------------------------------------------

@dataclass
class DenseProblem:
    A: np.ndarray          # f32 [n, d] row-major
    y: np.ndarray          # f32 [n] in {-1,+1}
    w_star: np.ndarray     # f32 [d]
    M: int                 # workers; worker m owns rows [m*n/M, (m+1)*n/M)


@dataclass
class CsrProblem:
    vals: np.ndarray       # f32 [nnz]
    indptr: np.ndarray     # i64 [n+1]
    indices: np.ndarray    # i32 [nnz], ascending within a row, distinct within a row
    y: np.ndarray          # f32 [n]
    w_star: np.ndarray     # f32 [d]
    n: int
    d: int
    M: int


def _labels(margin: np.ndarray, rng: np.random.Generator, noise: float) -> np.ndarray:
    m = margin + noise * rng.standard_normal(margin.shape)
    return np.where(m >= 0, 1.0, -1.0).astype(np.float32)


def dense_problem(n=4096, d=1000, M=4, frac_nonzero=0.10, noise=0.1, seed=0) -> DenseProblem:
    """Dense N(0,1) features, sparse ground-truth weights, sign labels with margin noise."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((n, d)).astype(np.float32)
    w = np.zeros(d, np.float32)
    nz = rng.choice(d, size=max(1, int(round(frac_nonzero * d))), replace=False)
    w[nz] = rng.standard_normal(nz.size).astype(np.float32)
    y = _labels(A.astype(np.float64) @ w.astype(np.float64), rng, noise)
    return DenseProblem(A, y, w, M)


def _zipf_cdf(d: int, s: float) -> np.ndarray:
    p = np.arange(1, d + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(p)
    return c / c[-1]


def csr_problem(n=1 << 18, d=1 << 20, nnz_per_row=100, zipf_s=1.1, M=16, frac_nonzero=0.01,
                noise=0.1, seed=1) -> CsrProblem:
    """CSR rows with `nnz_per_row` distinct column ids of Zipf(s) popularity, binary values
    scaled by 1/sqrt(nnz_per_row).  Popularity rank r is mapped to a column id through a fixed
    random permutation so that hot columns are spread over the index range."""
    rng = np.random.default_rng(seed)
    cdf = _zipf_cdf(d, zipf_s)
    perm = rng.permutation(d).astype(np.int32)
    k = nnz_per_row
    indices = np.empty((n, k), np.int32)
    chunk = 8192
    over = max(4 * k, k + 64)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        r = hi - lo
        draws = np.searchsorted(cdf, rng.random((r, over)), side="left").astype(np.int64)
        np.minimum(draws, d - 1, out=draws)
        order = np.argsort(draws, axis=1, kind="stable")
        sd = np.take_along_axis(draws, order, axis=1)
        first_sorted = np.ones_like(sd, dtype=bool)
        first_sorted[:, 1:] = sd[:, 1:] != sd[:, :-1]
        first = np.empty_like(first_sorted)
        np.put_along_axis(first, order, first_sorted, axis=1)   # first occurrence, draw order
        rank = np.cumsum(first, axis=1)
        keep = first & (rank <= k)
        for i in range(r):
            row = draws[i, keep[i]]
            while row.size < k:                                  # rare: too many duplicates
                extra = np.searchsorted(cdf, rng.random(over), side="left")
                row = np.concatenate([row, np.setdiff1d(np.minimum(extra, d - 1), row)])[:k]
            indices[lo + i] = np.sort(perm[row])
    vals = np.full(n * k, 1.0 / np.sqrt(k), np.float32)
    indptr = (np.arange(n + 1, dtype=np.int64) * k)
    w = np.zeros(d, np.float32)
    nz = rng.choice(d, size=max(1, int(round(frac_nonzero * d))), replace=False)
    w[nz] = rng.standard_normal(nz.size).astype(np.float32)
    margin = (w.astype(np.float64)[indices] * vals.reshape(n, k).astype(np.float64)).sum(axis=1)
    y = _labels(margin, rng, noise)
    return CsrProblem(vals, indptr, indices.reshape(-1), y, w, n, d, M)


def minibatch_rows(n: int, M: int, B: int, t: int, seed: int) -> np.ndarray:
    """Row ids of step t for all workers, i32 [M, B]: worker m draws B rows with replacement
    from its own shard [m*n/M, (m+1)*n/M)."""
    out = np.empty((M, B), np.int32)
    for m in range(M):
        rng = np.random.default_rng([seed, t, m])
        lo, hi = (m * n) // M, ((m + 1) * n) // M
        out[m] = rng.integers(lo, hi, size=B, dtype=np.int64).astype(np.int32)
    return out


# --------------------------------------------------------------------------------------
# Worker gradients for the optimizer-only workloads (any torch device)
# --------------------------------------------------------------------------------------

def _gen(device, seed, *stream):
    g = torch.Generator(device=device)
    s = int(seed)
    for v in stream:
        s = (s * 1000003 + int(v) + 12345) % (2 ** 62)
    g.manual_seed(s)
    return g


def grad_student_t_sparse(d, m, t, seed=2, scale=1e-2, keep=0.10, df=3, device="cpu",
                          out=None):
    """Heavy-tailed sparse gradient: Bernoulli(keep) mask times `scale` * Student-t(df)."""
    gen = _gen(device, seed, m, t)
    num = torch.randn(d, generator=gen, device=device, dtype=torch.float32)
    chi = torch.zeros(d, device=device, dtype=torch.float32)
    for _ in range(df):
        chi += torch.randn(d, generator=gen, device=device, dtype=torch.float32) ** 2
    num.div_(torch.sqrt(chi.div_(df))).mul_(scale)
    mask = torch.rand(d, generator=gen, device=device) < keep
    num.mul_(mask)
    if out is not None:
        out.copy_(num)
        return out
    return num


def grad_gaussian_biased(d, m, t, seed=3, var=1e-4, bias_var=1e-5, device="cpu", out=None):
    """Dense gradient N(beta_m, var) with a per-worker scalar bias beta_m ~ N(0, bias_var)."""
    gb = _gen("cpu", seed, m)
    beta = float(torch.randn(1, generator=gb).item()) * float(np.sqrt(bias_var))
    gen = _gen(device, seed, m, t, 7)
    g = torch.randn(d, generator=gen, device=device, dtype=torch.float32)
    g.mul_(float(np.sqrt(var))).add_(beta)
    if out is not None:
        out.copy_(g)
        return out
    return g


def grad_laplace_sparse(d, m, t, seed=4, b=1e-3, keep=0.05, device="cpu", out=None):
    """Sparse gradient: Bernoulli(keep) mask times Laplace(0, b) by inverse CDF."""
    gen = _gen(device, seed, m, t)
    u = torch.rand(d, generator=gen, device=device, dtype=torch.float32).sub_(0.5)
    mag = torch.log1p(-2.0 * u.abs().clamp_(max=0.49999997)).mul_(-b)
    g = torch.sign(u).mul_(mag)
    del mag
    mask = torch.rand(d, generator=gen, device=device) < keep
    g.mul_(mask)
    if out is not None:
        out.copy_(g)
        return out
    return g
