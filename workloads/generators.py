"""Seeded synthetic workloads: sparsity patterns, values and dense operands.

Everything here is input preparation.  The five named configurations follow the
benchmark description this repository measures on (uniform random, two R-MAT
power-law graphs, a 5-point stencil and a lognormal-degree graph); they stand
in for the SuiteSparse matrices and GNN graphs of the paper's evaluation
(Section 4, "Datasets"), which are not available here.

Storage convention: every 16-bit floating tensor is carried as a numpy
``uint16`` array of raw bits plus a dtype tag (``"f16"`` or ``"bf16"``), so
that fp16 and bf16 travel the same way to both consumers.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

CONFIG_NAMES = ("cfg1_uniform", "cfg2_rmat16", "cfg3_stencil", "cfg4_rmat20", "cfg5_lognormal")


# --------------------------------------------------------------------------
# containers
# --------------------------------------------------------------------------
@dataclass
class Dense:
    """Row-major dense matrix of 16-bit floats, stored as raw bits."""

    bits: np.ndarray  # uint16, shape (rows, cols), C-contiguous
    dtype: str  # "f16" | "bf16"

    @property
    def shape(self):
        return self.bits.shape


@dataclass
class Csr:
    """CSR matrix; column indices strictly ascending inside each row."""

    M: int
    K: int
    rowptr: np.ndarray  # int32, M+1
    colidx: np.ndarray  # int32, nnz
    vals: np.ndarray  # uint16 raw bits, nnz
    dtype: str  # "f16" | "bf16"

    @property
    def nnz(self) -> int:
        return int(self.colidx.shape[0])


# --------------------------------------------------------------------------
# random streams and rounding to storage types
# --------------------------------------------------------------------------
def stream(seed: int, cfg: int, tensor_id: int) -> np.random.Generator:
    """Independent PCG64 stream per (seed, configuration, tensor)."""
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cfg, tensor_id])))


def round_to_bits(x32: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 draws to fp16 / bf16 (round-to-nearest-even); return raw bits."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "f16":
        return x32.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = x32.view(np.uint32)
        lsb = (u >> np.uint32(16)) & np.uint32(1)
        r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
        return r.astype(np.uint16)
    raise ValueError(dtype)


def bits_to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored bits to float64 (for test assertions on inputs)."""
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def _draw(rng: np.random.Generator, n, dist: str) -> np.ndarray:
    """float32 draws; dist in {"u01", "u11", "n01", "n0_8th"} (last: variance 1/8)."""
    if dist == "u01":
        return rng.random(n, dtype=np.float32)
    if dist == "u11":
        return rng.random(n, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    if dist == "n01":
        return rng.standard_normal(n, dtype=np.float32)
    if dist == "n0_8th":
        return rng.standard_normal(n, dtype=np.float32) * np.float32(np.sqrt(1.0 / 8.0))
    raise ValueError(dist)


def dense(rows: int, cols: int, dist: str, dtype: str, rng: np.random.Generator) -> Dense:
    return Dense(round_to_bits(_draw(rng, (rows, cols), dist), dtype), dtype)


# --------------------------------------------------------------------------
# pattern builders
# --------------------------------------------------------------------------
def csr_from_coo(M: int, K: int, rows: np.ndarray, cols: np.ndarray, dist: str, dtype: str,
                 rng: np.random.Generator) -> Csr:
    """Sort (row, col) pairs, drop duplicates, draw one value per stored entry."""
    key = rows.astype(np.int64) * np.int64(K) + cols.astype(np.int64)
    key = np.unique(key)
    r = (key // K).astype(np.int64)
    c = (key % K).astype(np.int32)
    rowptr = np.zeros(M + 1, dtype=np.int64)
    rowptr[1:] = np.bincount(r, minlength=M)
    rowptr = np.cumsum(rowptr).astype(np.int32)
    vals = round_to_bits(_draw(rng, key.shape[0], dist), dtype)
    return Csr(M, K, rowptr, c, vals, dtype)


def uniform_fixed_degree(M: int, K: int, deg: np.ndarray, rng: np.random.Generator):
    """Each row i gets exactly deg[i] distinct uniformly random columns.

    Draws with replacement, removes duplicates and tops the short rows up until
    every row holds its target count.  Returns (rows, cols) of the entries.
    """
    deg = np.minimum(np.asarray(deg, dtype=np.int64), K)
    have = np.zeros(0, dtype=np.int64)  # keys row*K+col, sorted unique
    need = deg.copy()
    for _ in range(200):
        tot = int(need.sum())
        if tot == 0:
            break
        r = np.repeat(np.arange(M, dtype=np.int64), need)
        c = rng.integers(0, K, size=tot, dtype=np.int64)
        have = np.unique(np.concatenate([have, r * K + c]))
        cnt = np.bincount(have // K, minlength=M)
        need = deg - cnt
    else:  # pragma: no cover
        raise RuntimeError("degree top-up did not converge")
    return (have // K), (have % K)


def rmat(scale: int, edge_factor: int, a: float, b: float, c: float, d: float,
         rng: np.random.Generator, chunk: int = 1 << 22):
    """Recursive-matrix edge draws: directed, self loops kept, no permutation, no noise.

    Each of ``edge_factor * 2**scale`` edges picks one quadrant per bit level
    with probabilities (a, b, c, d): the row bit is set in quadrants c and d,
    the column bit in quadrants b and d.  Duplicates are removed by the caller.
    """
    n_edges = edge_factor << scale
    rows = np.empty(n_edges, dtype=np.int64)
    cols = np.empty(n_edges, dtype=np.int64)
    ab, abc = np.float32(a + b), np.float32(a + b + c)
    a32 = np.float32(a)
    for s in range(0, n_edges, chunk):
        n = min(chunk, n_edges - s)
        r = np.zeros(n, dtype=np.int64)
        q = np.zeros(n, dtype=np.int64)
        for _level in range(scale):
            u = rng.random(n, dtype=np.float32)
            rbit = u >= ab  # quadrants c, d
            cbit = ((u >= a32) & (u < ab)) | (u >= abc)  # quadrants b, d
            r = (r << 1) | rbit
            q = (q << 1) | cbit
        rows[s:s + n] = r
        cols[s:s + n] = q
    return rows, cols


def stencil5(g: int):
    """5-point stencil on a g x g grid; row i = y*g + x couples to i, i+-1 (same grid row), i+-g."""
    i = np.arange(g * g, dtype=np.int64)
    x = i % g
    y = i // g
    rows = [i, i[x > 0], i[x < g - 1], i[y > 0], i[y < g - 1]]
    cols = [i, i[x > 0] - 1, i[x < g - 1] + 1, i[y > 0] - g, i[y < g - 1] + g]
    return np.concatenate(rows), np.concatenate(cols)


def lognormal_degree(M: int, mu: float, sigma: float, lo: int, hi: int, rng: np.random.Generator):
    """Per-row degree: exp(N(mu, sigma)) rounded to nearest integer and clipped to [lo, hi]."""
    z = rng.standard_normal(M)
    return np.clip(np.rint(np.exp(mu + sigma * z)), lo, hi).astype(np.int64)


def random_csr(M: int, K: int, density: float, dtype: str, seed: int, dist: str = "u11",
               empty_rows: float = 0.0) -> Csr:
    """Small Bernoulli-pattern matrix for unit tests (may contain empty rows and windows)."""
    rng = stream(seed, 99, 0)
    mask = rng.random((M, K)) < density
    if empty_rows > 0:
        mask[rng.random(M) < empty_rows, :] = False
    r, c = np.nonzero(mask)
    return csr_from_coo(M, K, r, c, dist, dtype, stream(seed, 99, 1))


# --------------------------------------------------------------------------
# the five named configurations
# --------------------------------------------------------------------------
def make_config(name: str, seed: int = 0, shrink: Optional[int] = None) -> Dict:
    """Build one named workload.

    ``shrink`` (a power-of-two divisor, optional) scales the problem down for
    CPU-only tests while keeping the structure: fewer rows for the uniform and
    lognormal graphs, a lower R-MAT scale, a smaller stencil grid.

    Returns a dict with key ``A`` (Csr) and, where the configuration has them,
    ``spmm`` = list of Dense B operands, ``sddmm`` = (X, Y), ``chain`` = H.
    """
    idx = CONFIG_NAMES.index(name) + 1
    sh = 1 if shrink is None else int(shrink)
    log_sh = sh.bit_length() - 1
    if sh & (sh - 1):
        raise ValueError("shrink must be a power of two")
    out: Dict = {"name": name, "seed": seed, "shrink": sh}
    if idx == 1:
        M = K = 4096 // sh
        r, c = uniform_fixed_degree(M, K, np.full(M, 16), stream(seed, 1, 0))
        out["A"] = csr_from_coo(M, K, r, c, "u11", "f16", stream(seed, 1, 1))
        out["spmm"] = [dense(K, 32, "u11", "f16", stream(seed, 1, 2))]
        out["sddmm"] = (dense(M, 32, "u11", "f16", stream(seed, 1, 3)),
                        dense(K, 32, "u11", "f16", stream(seed, 1, 4)))
    elif idx == 2:
        scale = 16 - log_sh
        M = K = 1 << scale
        r, c = rmat(scale, 16, 0.57, 0.19, 0.19, 0.05, stream(seed, 2, 0))
        out["A"] = csr_from_coo(M, K, r, c, "u01", "f16", stream(seed, 2, 1))
        out["spmm"] = [dense(K, 128, "n01", "f16", stream(seed, 2, 2))]
        out["sddmm"] = (dense(M, 32, "n01", "f16", stream(seed, 2, 3)),
                        dense(K, 32, "n01", "f16", stream(seed, 2, 4)))
    elif idx == 3:
        g = 1024 // sh
        M = K = g * g
        r, c = stencil5(g)
        out["A"] = csr_from_coo(M, K, r, c, "n01", "f16", stream(seed, 3, 1))
        out["spmm"] = [dense(K, 64, "n01", "f16", stream(seed, 3, 2)),
                       dense(K, 256, "n01", "f16", stream(seed, 3, 3))]
    elif idx == 4:
        scale = 20 - log_sh
        M = K = 1 << scale
        r, c = rmat(scale, 32, 0.57, 0.19, 0.19, 0.05, stream(seed, 4, 0))
        out["A"] = csr_from_coo(M, K, r, c, "u01", "bf16", stream(seed, 4, 1))
        del r, c
        out["spmm"] = [dense(K, 128, "n01", "bf16", stream(seed, 4, 2))]
    elif idx == 5:
        M = K = 262144 // sh
        deg = lognormal_degree(M, 2.5, 1.0, 1, 4096, stream(seed, 5, 0))
        r, c = uniform_fixed_degree(M, K, deg, stream(seed, 5, 5))
        # the stored values are placeholders: the SDDMM scores replace them in the chain
        out["A"] = csr_from_coo(M, K, r, c, "u01", "f16", stream(seed, 5, 1))
        out["sddmm"] = (dense(M, 64, "n0_8th", "f16", stream(seed, 5, 3)),
                        dense(K, 64, "n0_8th", "f16", stream(seed, 5, 4)))
        out["chain"] = dense(K, 256, "n01", "f16", stream(seed, 5, 2))
    return out
