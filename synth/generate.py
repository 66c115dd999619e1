"""Seeded synthetic matrices and tensors shaped like the paper's workloads.

The paper measures on SuiteSparse matrices and FROSTT/BIGtensor tensors (Section
8.1, Table "Description of sparse tensors"); those are not available, so
power-law structured inputs of the same regime stand in: order 3, 1e7-1e8
nonzeros, very unequal mode sizes, skewed slices and fibers.

All draws come from `synth.rng` (counter based), so an input is a pure function
of its arguments and can be regenerated on the host or on a GPU.  Nothing here
performs any of the contractions.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np
import torch

from . import rng
from .formats import LevelTensor, pack_coo, pack_csf3, pack_csr, pack_dcsr

# stream ids (one per independent array)
ST_LEN, ST_COL, ST_VAL, ST_DENSE, ST_PERM, ST_THIN, ST_MODE, ST_MASK = 1, 2, 3, 4, 5, 6, 16, 7
ST_REDRAW = 1000


# ----------------------------------------------------------------------------------------------
# distributions
# ----------------------------------------------------------------------------------------------
def zipf_cdf(n: int, alpha: float, clamp_tail: bool = False) -> np.ndarray:
    """CDF table of P(rank k) proportional to k**-alpha on k = 1..n (host, float64).

    clamp_tail=False: the support is truncated at n (bounded Zipf).
    clamp_tail=True : the unbounded law is sampled and values above n are set to n,
                      i.e. rank n also carries the whole tail mass beyond n.
    """
    k = np.arange(1, n + 1, dtype=np.float64)
    w = k ** (-alpha)
    c = np.cumsum(w)
    if clamp_tail:
        from scipy.special import zeta
        c = c / float(zeta(alpha, 1))
    else:
        c = c / c[-1]
    c[-1] = 1.0
    return c


def sample_cdf(cdf: torch.Tensor, u: torch.Tensor) -> torch.Tensor:
    """Inverse-CDF sampling: the smallest rank r (0-based) with u < cdf[r]."""
    r = torch.searchsorted(cdf, u, right=True)
    return torch.clamp(r, max=cdf.numel() - 1)


def dense_operand(seed: int, which: int, shape: Sequence[int], device="cpu") -> torch.Tensor:
    """Row-major fp64 operand filled with U(-1,1); `which` separates operands of one config."""
    n = int(np.prod(shape))
    return rng.uniform_pm1(seed, ST_DENSE + 64 * which, n, device).reshape(*shape)


# ----------------------------------------------------------------------------------------------
# matrices
# ----------------------------------------------------------------------------------------------
def matrix_from_row_lengths(nrows: int, ncols: int, lengths: torch.Tensor, seed: int,
                            device="cpu") -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Rows with the given lengths, each holding distinct uniform-random columns, sorted.

    Collisions inside a row are redrawn (from a fresh stream per pass) until none remain,
    so every row has exactly its requested length.  Returns (rows, cols, vals) sorted by
    (row, col); vals[p] is U(-1,1) keyed by the final position p.
    """
    lengths = lengths.to(device=device, dtype=torch.int64)
    assert int(lengths.max()) <= ncols if lengths.numel() else True
    rows = torch.repeat_interleave(torch.arange(nrows, dtype=torch.int64, device=device), lengths)
    nnz = int(rows.numel())
    cols = rng.randint(seed, ST_COL, nnz, ncols, device)
    for it in range(1, 200):
        key, order = torch.sort(rows * ncols + cols, stable=True)
        rows, cols = rows[order], cols[order]
        dup = torch.zeros(nnz, dtype=torch.bool, device=device)
        if nnz > 1:
            dup[1:] = key[1:] == key[:-1]
        ndup = int(dup.sum())
        if ndup == 0:
            break
        fresh = rng.randint(seed, ST_REDRAW + it, nnz, ncols, device)
        cols = torch.where(dup, fresh, cols)
    else:
        raise RuntimeError("could not make row columns distinct")
    vals = rng.uniform_pm1(seed, ST_VAL, nnz, device)
    return rows, cols, vals


def bernoulli_matrix(nrows: int, ncols: int, density: float, seed: int, device="cpu"):
    """Every cell is a nonzero with probability `density` (tiny test matrices)."""
    u = rng.uniform01(seed, ST_MASK, nrows * ncols, device)
    idx = torch.nonzero(u < density).flatten()
    rows, cols = idx // ncols, idx % ncols
    vals = rng.uniform_pm1(seed, ST_VAL, int(idx.numel()), device)
    return rows, cols, vals


def zipf_row_lengths(nrows: int, alpha: float, cap: int, seed: int, device="cpu") -> torch.Tensor:
    """Row lengths min(Zipf(alpha) on 1,2,3,..., cap)."""
    cdf = torch.from_numpy(zipf_cdf(cap, alpha, clamp_tail=True)).to(device)
    return sample_cdf(cdf, rng.uniform01(seed, ST_LEN, nrows, device)) + 1


# ----------------------------------------------------------------------------------------------
# order-3 tensors
# ----------------------------------------------------------------------------------------------
def _mode_draws(seed: int, mode: int, n: int, size: int, alpha: Optional[float], permute: bool,
                device, offset: int) -> torch.Tensor:
    if alpha is None:
        return rng.randint(seed, ST_MODE + mode, n, size, device, offset)
    cdf = torch.from_numpy(zipf_cdf(size, alpha)).to(device)
    r = sample_cdf(cdf, rng.uniform01(seed, ST_MODE + mode, n, device, offset))
    if permute:
        r = rng.permutation(seed, ST_PERM + mode, size, device)[r]
    return r


def zipf_tensor3(dims: Sequence[int], alphas: Sequence[Optional[float]], target_nnz: int, seed: int,
                 device="cpu", permute: bool = True, chunk: int = 1 << 26, max_mult: float = 64.0,
                 margin: float = 0.02):
    """Distinct sorted coordinates of an order-3 tensor with independent per-mode laws.

    Each mode's index is Zipf(alpha) over ranks (alpha=None: uniform); ranks map to
    coordinates through a seeded permutation unless permute=False (which clusters the
    nonzeros at the low corner).  Draws are made in fixed-size chunks and merged into a
    sorted duplicate-free set until it holds at least target_nnz*(1+margin) keys (or
    max_mult*target_nnz draws were made); the set is then thinned to exactly target_nnz
    keys by keeping those with the smallest seeded hash.  Returns (i, j, k, vals, info).
    """
    I, J, K = (int(d) for d in dims)
    assert I * J * K < (1 << 62)
    want = int(target_nnz * (1.0 + margin)) + 1
    max_draws = int(max_mult * target_nnz)
    keys = torch.empty(0, dtype=torch.int64, device=device)
    drawn = 0
    while keys.numel() < want and drawn < max_draws:
        n = min(chunk, max_draws - drawn)
        ci = _mode_draws(seed, 0, n, I, alphas[0], permute, device, drawn)
        cj = _mode_draws(seed, 1, n, J, alphas[1], permute, device, drawn)
        ck = _mode_draws(seed, 2, n, K, alphas[2], permute, device, drawn)
        new = torch.unique((ci * J + cj) * K + ck)
        del ci, cj, ck
        keys = torch.unique(torch.cat([keys, new]))
        del new
        drawn += n
    distinct_before = int(keys.numel())
    if keys.numel() > target_nnz:
        h = rng.hash64(keys, seed, ST_THIN)
        thr = torch.sort(h).values[target_nnz - 1]
        keys = keys[h <= thr]
        del h
    k = keys % K
    ij = keys // K
    j = ij % J
    i = ij // J
    vals = rng.uniform_pm1(seed, ST_VAL, int(keys.numel()), device)
    info = {"draws": drawn, "distinct_before_thinning": distinct_before, "nnz": int(keys.numel())}
    return i, j, k, vals, info


def bernoulli_tensor3(dims: Sequence[int], density: float, seed: int, device="cpu"):
    """Every cell is a nonzero with probability `density` (tiny test tensors)."""
    I, J, K = (int(d) for d in dims)
    u = rng.uniform01(seed, ST_MASK, I * J * K, device)
    idx = torch.nonzero(u < density).flatten()
    k = idx % K
    j = (idx // K) % J
    i = idx // (J * K)
    vals = rng.uniform_pm1(seed, ST_VAL, int(idx.numel()), device)
    return i, j, k, vals


# ----------------------------------------------------------------------------------------------
# the five benchmark configurations (scale < 1 shrinks every size for tests)
# ----------------------------------------------------------------------------------------------
def _sc(x: int, scale: float, lo: int = 2) -> int:
    return max(lo, int(round(x * scale)))


def config_spmv(seed: int = 0, device="cpu", n: int = 4096, per_row: int = 10):
    """SpMV: CSR n x n, exactly `per_row` distinct uniform columns in every row; x U(-1,1)."""
    lengths = torch.full((n,), per_row, dtype=torch.int64, device=device)
    rows, cols, vals = matrix_from_row_lengths(n, n, lengths, seed, device)
    x = dense_operand(seed, 0, (n,), device)
    return {"coo": (rows, cols, vals), "dims": (n, n), "x": x}


def config_spmm(seed: int = 0, device="cpu", scale: float = 1.0, R: int = 32):
    """SpMM: CSR with Zipf(1.8) row lengths capped at 10,000, uniform columns; B dense n x R."""
    n = _sc(1_000_000, scale, 64)
    cap = min(10_000, max(1, n // 4))   # full-size: 10,000; shrunk configs keep rows well below n
    lengths = zipf_row_lengths(n, 1.8, cap, seed, device)
    rows, cols, vals = matrix_from_row_lengths(n, n, lengths, seed, device)
    B = dense_operand(seed, 0, (n, R), device)
    return {"coo": (rows, cols, vals), "dims": (n, n), "B": B, "R": R}


def _tensor_config(dims, alphas, nnz, seed, device, scale, **kw):
    dims = tuple(_sc(d, scale ** (1.0 / 3.0) if scale < 1 else 1.0, 4) for d in dims)
    nnz = _sc(nnz, scale, 16)
    i, j, k, vals, info = zipf_tensor3(dims, alphas, nnz, seed, device, **kw)
    return {"coo": (i, j, k, vals), "dims": dims, "info": info}


def config_ttv(seed: int = 0, device="cpu", scale: float = 1.0, **kw):
    """TTV: 20,000^3, 50M nonzeros, Zipf(1.3) on every mode; v dense."""
    c = _tensor_config((20_000, 20_000, 20_000), (1.3, 1.3, 1.3), 50_000_000, seed, device, scale, **kw)
    c["v"] = dense_operand(seed, 0, (c["dims"][2],), device)
    return c


def config_ttm(seed: int = 0, device="cpu", scale: float = 1.0, R: int = 16, **kw):
    """TTM: 200,000 x 100,000 x 5,000, 100M nonzeros, Zipf(1.5) on modes 1-2, uniform mode 3."""
    c = _tensor_config((200_000, 100_000, 5_000), (1.5, 1.5, None), 100_000_000, seed, device, scale, **kw)
    c["U"] = dense_operand(seed, 0, (c["dims"][2], R), device)
    c["R"] = R
    return c


def config_mttkrp(seed: int = 0, device="cpu", scale: float = 1.0, R: int = 16, **kw):
    """MTTKRP: 2,000,000 x 1,000,000 x 20,000, 150M nonzeros, Zipf(1.4) on every mode.

    The factor matrices are generated with 64 columns and cut to R, so a rank-16 run sees the
    first 16 columns of the rank-64 factors.
    """
    c = _tensor_config((2_000_000, 1_000_000, 20_000), (1.4, 1.4, 1.4), 150_000_000, seed, device, scale, **kw)
    full = max(R, 64)
    c["B"] = dense_operand(seed, 0, (c["dims"][1], full), device)[:, :R].contiguous()
    c["C"] = dense_operand(seed, 1, (c["dims"][2], full), device)[:, :R].contiguous()
    c["R"] = R
    return c


__all__ = [
    "zipf_cdf", "sample_cdf", "dense_operand", "matrix_from_row_lengths", "bernoulli_matrix",
    "zipf_row_lengths", "zipf_tensor3", "bernoulli_tensor3", "config_spmv", "config_spmm",
    "config_ttv", "config_ttm", "config_mttkrp", "LevelTensor", "pack_coo", "pack_csf3",
    "pack_csr", "pack_dcsr",
]
