"""Seeded synthetic inputs for the TNG hot path.

This module only draws data (features, labels, start points, noise, reference vectors); it
contains none of the method's arithmetic and imports neither the HIP binding nor any
checker.  Everything is generated with torch on the device asked for, from an explicit
seed, so the same tensors can be handed to the library and, copied to the host, to a
checker.

Workloads mirror the paper's experiments (arXiv 1901.08227, section "Experiments"): all of
its data is synthetic -- Gaussian features with labels from a planted weight vector for
logistic regression ("Convex Problems"), and closed-form test functions whose stochastic
gradient is the exact gradient plus Gaussian noise ("Nonconvex Problems").  "N(0, v)"
is read as variance v throughout, as the paper writes N(0,1), N(0,I).
"""
from __future__ import annotations

import math

import torch


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def logreg_dense(M: int, n_rows: int, d: int, seed: int, device="cpu"):
    """Per-worker shards X[M][n_rows][d] ~ N(0,1), labels y in {0,1} from a planted w* ~ N(0, 1/d).

    Returns (X, y, w_star); y[m][i] ~ Bernoulli(sigmoid(x_i . w*)).
    """
    g = _gen(seed, device)
    w_star = torch.randn(d, generator=g, device=device, dtype=torch.float32) / math.sqrt(d)
    X = torch.empty((M, n_rows, d), device=device, dtype=torch.float32)
    y = torch.empty((M, n_rows), device=device, dtype=torch.float32)
    for m in range(M):
        X[m].normal_(generator=g)
        p = torch.sigmoid(X[m] @ w_star)
        y[m] = (torch.rand(n_rows, generator=g, device=device) < p).to(torch.float32)
    return X, y, w_star


def logreg_skewed(M: int, n_rows: int, d: int, c_sk: float, c_th: float, seed: int, device="cpu"):
    """Dense shards with a skewed feature scale (section "Convex Problems": D = 512, N = 2048 in all,
    M = 4, batch 8, c_th = 0.6, c_sk a power of 1/4).

    Normalised data a_bar ~ N(0,1); one magnitude vector B ~ U[0,1]^d shared by all rows, whose
    entries at or below c_th are shrunk by the factor c_sk; features a = a_bar * B; labels from a
    planted w_bar ~ N(0, I) as sign(a_bar . w_bar), stored as 0/1.  Returns (X[M][n_rows][d],
    y[M][n_rows], B).
    """
    g = _gen(seed, device)
    mag = torch.rand(d, generator=g, device=device, dtype=torch.float32)
    mag = torch.where(mag <= c_th, mag * c_sk, mag)
    w_bar = torch.randn(d, generator=g, device=device, dtype=torch.float32)
    X = torch.empty((M, n_rows, d), device=device, dtype=torch.float32)
    y = torch.empty((M, n_rows), device=device, dtype=torch.float32)
    for m in range(M):
        a_bar = torch.randn((n_rows, d), generator=g, device=device, dtype=torch.float32)
        y[m] = (a_bar @ w_bar > 0).to(torch.float32)
        X[m] = a_bar * mag
    return X, y, mag


def logreg_csr(M: int, n_rows: int, d: int, nnz_row: int, seed: int, device="cpu"):
    """Per-worker CSR shards: nnz_row distinct uniform columns per row (sorted), values ~ N(0,1).

    Labels from a planted w* ~ N(0, 1/nnz_row).  Returns lists (rowptr int64[n_rows+1],
    col int32[nnz], val float32[nnz], y float32[n_rows]) per worker, and w_star.
    """
    g = _gen(seed, device)
    w_star = torch.randn(d, generator=g, device=device, dtype=torch.float32) / math.sqrt(nnz_row)
    shards = []
    for _ in range(M):
        cols = torch.randint(0, d, (n_rows, nnz_row), generator=g, device=device, dtype=torch.int64)
        while True:
            cols, _ = torch.sort(cols, dim=1)
            dup = torch.zeros_like(cols, dtype=torch.bool)
            dup[:, 1:] = cols[:, 1:] == cols[:, :-1]
            n_dup = int(dup.sum())
            if n_dup == 0:
                break
            cols[dup] = torch.randint(0, d, (n_dup,), generator=g, device=device, dtype=torch.int64)
        val = torch.randn((n_rows, nnz_row), generator=g, device=device, dtype=torch.float32)
        z = (val * w_star[cols]).sum(dim=1)
        y = (torch.rand(n_rows, generator=g, device=device) < torch.sigmoid(z)).to(torch.float32)
        rowptr = torch.arange(0, n_rows + 1, device=device, dtype=torch.int64) * nnz_row
        shards.append((rowptr, cols.reshape(-1).to(torch.int32).contiguous(),
                       val.reshape(-1).contiguous(), y))
    return shards, w_star


def rosenbrock_start(d: int, seed: int, device="cpu"):
    """x0 ~ U(-2, 2)^d."""
    g = _gen(seed, device)
    return torch.rand(d, generator=g, device=device, dtype=torch.float32) * 4.0 - 2.0


def gradient_noise(M: int, d: int, seed: int, it: int, variance: float = 0.01, device="cpu"):
    """Per-worker additive gradient noise for iteration it: i.i.d. N(0, variance), shape [M][d]."""
    g = _gen(seed * 1_000_003 + it + 1, device)
    return torch.randn((M, d), generator=g, device=device, dtype=torch.float32) * math.sqrt(variance)


def codec_inputs(M: int, d: int, seed: int, rel_variance: float = 0.1, device="cpu"):
    """Reference g~ ~ N(0,1)^d and worker gradients g_m = g~ + eps_m (.) |g~|, eps ~ N(0, rel_variance)."""
    g = _gen(seed, device)
    gref = torch.randn(d, generator=g, device=device, dtype=torch.float32)
    grads = torch.empty((M, d), device=device, dtype=torch.float32)
    sd = math.sqrt(rel_variance)
    for m in range(M):
        grads[m].normal_(generator=g)
        grads[m].mul_(sd).mul_(gref.abs()).add_(gref)
    return grads, gref
