"""Seeded synthetic inputs for the SpMM / SDDMM path.

This module only *draws* inputs (sparsity patterns, values, dense operands).
It contains none of the method's arithmetic: no planner, no multiplication.
Both the CPU oracle's tests and the GPU library's tests take their inputs
from here so that the two sides see bit-identical arrays.

The paper evaluates on SuiteSparse matrices and on GNN graphs (Section 5.1,
Table 4); neither is available offline, so the generators below stand in for
them: an R-MAT power-law graph, a block-community matrix that favours the
dense-tile path, a Zipf-degree irregular graph, and a tiny uniform case.

Every generator returns a ``Csr`` (M, Kc, rowptr int32, col int32, val
float16) with strictly increasing columns inside each row.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20250622


@dataclass
class Csr:
    M: int
    Kc: int
    rowptr: np.ndarray  # int32, M+1
    col: np.ndarray     # int32, nnz
    val: np.ndarray     # float16, nnz

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


def _csr_from_keys(keys: np.ndarray, M: int, Kc: int) -> tuple[np.ndarray, np.ndarray]:
    """keys = row*Kc + col, already unique and sorted."""
    rows = keys // Kc
    col = (keys - rows * Kc).astype(np.int32)
    counts = np.bincount(rows, minlength=M)
    rowptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2**31
    return rowptr.astype(np.int32), col


def uniform_values(rng: np.random.Generator, n: int) -> np.ndarray:
    """U(-1,1) rounded to fp16; entries that round to zero are drawn again."""
    v = rng.uniform(-1.0, 1.0, size=n).astype(np.float16)
    while True:
        z = np.flatnonzero(v == 0)
        if z.size == 0:
            return v
        v[z] = rng.uniform(-1.0, 1.0, size=z.size).astype(np.float16)


def unit_values(n: int) -> np.ndarray:
    return np.ones(n, dtype=np.float16)


def dense_normal(rows: int, cols: int, seed: int, dtype=np.float16) -> np.ndarray:
    """rows x cols N(0,1) drawn in fp32 and rounded once to ``dtype``."""
    rng = np.random.default_rng(seed)
    out = np.empty((rows, cols), dtype=dtype)
    step = max(1, (1 << 24) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        out[r0:r1] = rng.standard_normal((r1 - r0, cols), dtype=np.float32).astype(dtype)
    return out


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even; finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def dense_small_int(rows: int, cols: int, seed: int, lo=-4, hi=5, dtype=np.float16) -> np.ndarray:
    """Small integers: products and short sums are exact in fp16/fp32/fp64."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi, size=(rows, cols)).astype(dtype)


# ----------------------------------------------------------------------------
# Config 1: tiny uniform matrix
# ----------------------------------------------------------------------------
def tiny(M: int = 2048, per_row: int = 16, seed: int = BASE_SEED + 1) -> Csr:
    rng = np.random.default_rng(seed)
    per_row = min(per_row, M)
    # distinct columns per row: argpartition of random keys
    keys = rng.random((M, M), dtype=np.float32) if M <= 4096 else None
    if keys is not None:
        cols = np.argpartition(keys, per_row - 1, axis=1)[:, :per_row]
    else:
        cols = np.stack([rng.choice(M, per_row, replace=False) for _ in range(M)])
    cols = np.sort(cols, axis=1).astype(np.int32)
    rowptr = (np.arange(M + 1, dtype=np.int64) * per_row).astype(np.int32)
    val = uniform_values(rng, M * per_row)
    return Csr(M, M, rowptr, cols.reshape(-1), val)


# ----------------------------------------------------------------------------
# Configs 2 and 5: R-MAT power-law graph
# ----------------------------------------------------------------------------
def rmat(scale: int = 17, avg_degree: int = 16, seed: int = BASE_SEED + 2,
         abcd=(0.57, 0.19, 0.19, 0.05)) -> Csr:
    """avg_degree * 2**scale directed samples, then A <- A | A^T, then
    duplicates removed (self loops kept once); unit values."""
    n = 1 << scale
    ns = avg_degree * n
    rng = np.random.default_rng(seed)
    a, b, c, _d = abcd
    src = np.zeros(ns, dtype=np.int64)
    dst = np.zeros(ns, dtype=np.int64)
    for _level in range(scale):
        u = rng.random(ns, dtype=np.float32)
        row_bit = u >= (a + b)                      # quadrants c, d
        col_bit = ((u >= a) & (u < a + b)) | (u >= a + b + c)   # quadrants b, d
        src = (src << 1) | row_bit
        dst = (dst << 1) | col_bit
    keys = np.concatenate([src * n + dst, dst * n + src])
    del src, dst
    keys = np.unique(keys)
    rowptr, col = _csr_from_keys(keys, n, n)
    return Csr(n, n, rowptr, col, unit_values(col.size))


# ----------------------------------------------------------------------------
# Config 3: community-structured matrix
# ----------------------------------------------------------------------------
def community(n_blocks: int = 16384, block: int = 64, density: float = 0.3,
              off_block: int = 2, seed: int = BASE_SEED + 3) -> Csr:
    """Diagonal blocks of block x block with Bernoulli(density) entries plus
    ``off_block`` distinct uniform columns outside the row's own block."""
    rng = np.random.default_rng(seed)
    M = n_blocks * block
    key_parts = []
    chunk = max(1, (1 << 24) // (block * block))
    for b0 in range(0, n_blocks, chunk):
        b1 = min(n_blocks, b0 + chunk)
        mask = rng.random((b1 - b0, block, block), dtype=np.float32) < density
        bi, ri, ci = np.nonzero(mask)
        rows = (bi + b0).astype(np.int64) * block + ri
        cols = (bi + b0).astype(np.int64) * block + ci
        key_parts.append(rows * M + cols)
    if off_block > 0 and n_blocks > 1:
        rows = np.repeat(np.arange(M, dtype=np.int64), off_block)
        # a column outside the own block: draw in [0, M-block) and skip over it
        raw = rng.integers(0, M - block, size=rows.size, dtype=np.int64)
        start = (rows // block) * block
        cols = np.where(raw >= start, raw + block, raw)
        key_parts.append(rows * M + cols)
    keys = np.unique(np.concatenate(key_parts))
    rowptr, col = _csr_from_keys(keys, M, M)
    return Csr(M, M, rowptr, col, uniform_values(rng, col.size))


# ----------------------------------------------------------------------------
# Config 4: highly irregular graph, Zipf degrees
# ----------------------------------------------------------------------------
def zipf_degrees(rng: np.random.Generator, n: int, exponent: float = 2.1,
                 dmin: int = 1, dmax: int = 100_000, shift: float = 8.2003) -> np.ndarray:
    """P(d) ~ (d + shift)^-exponent on [dmin, dmax].  shift = 8.2003 makes the
    mean 50 with exponent 2.1 on [1, 1e5]; shift = 0 is the plain Zipf law."""
    d = np.arange(dmin, dmax + 1, dtype=np.float64)
    cdf = np.cumsum((d + shift) ** (-exponent))
    cdf /= cdf[-1]
    u = rng.random(n)
    return (np.searchsorted(cdf, u, side="left") + dmin).astype(np.int64)


def irregular(n: int = 2_400_000, seed: int = BASE_SEED + 4, shift: float = 8.2003,
              dmax: int = 100_000) -> Csr:
    rng = np.random.default_rng(seed)
    deg = zipf_degrees(rng, n, dmax=min(dmax, n), shift=shift)
    rows = np.repeat(np.arange(n, dtype=np.int64), deg)
    keys = rows * n
    del rows
    keys += rng.integers(0, n, size=keys.size, dtype=np.int64)
    keys = np.unique(keys)            # targets drawn with replacement; duplicates dropped
    rowptr, col = _csr_from_keys(keys, n, n)
    return Csr(n, n, rowptr, col, unit_values(col.size))


# ----------------------------------------------------------------------------
# Hand-shaped patterns used by unit tests
# ----------------------------------------------------------------------------
def from_dense(A: np.ndarray) -> Csr:
    """CSR of the nonzero pattern of a small dense array (values -> fp16)."""
    A = np.asarray(A)
    M, Kc = A.shape
    r, c = np.nonzero(A)
    counts = np.bincount(r, minlength=M)
    rowptr = np.zeros(M + 1, dtype=np.int32)
    np.cumsum(counts, out=rowptr[1:])
    return Csr(M, Kc, rowptr, c.astype(np.int32), A[r, c].astype(np.float16))


def random_pattern(M: int, Kc: int, density: float, seed: int, empty_rows: float = 0.0) -> Csr:
    """Bernoulli(density) pattern, U(-1,1) values, optionally some empty rows."""
    rng = np.random.default_rng(seed)
    mask = rng.random((M, Kc)) < density
    if empty_rows > 0:
        mask[rng.random(M) < empty_rows] = False
    r, c = np.nonzero(mask)
    counts = np.bincount(r, minlength=M)
    rowptr = np.zeros(M + 1, dtype=np.int32)
    np.cumsum(counts, out=rowptr[1:])
    return Csr(M, Kc, rowptr, c.astype(np.int32), uniform_values(rng, r.size))


def with_long_rows(base: Csr, rows: list[int], length: int, seed: int) -> Csr:
    """Replace the given rows of ``base`` by rows of ``length`` distinct
    uniform columns (stresses row splitting on small matrices)."""
    rng = np.random.default_rng(seed)
    new_cols, new_vals = [], []
    for i in range(base.M):
        if i in rows:
            c = np.sort(rng.choice(base.Kc, size=min(length, base.Kc), replace=False)).astype(np.int32)
            new_cols.append(c)
            new_vals.append(uniform_values(rng, c.size))
        else:
            s, e = base.rowptr[i], base.rowptr[i + 1]
            new_cols.append(base.col[s:e])
            new_vals.append(base.val[s:e])
    rowptr = np.zeros(base.M + 1, dtype=np.int32)
    np.cumsum([len(c) for c in new_cols], out=rowptr[1:])
    return Csr(base.M, base.Kc, rowptr, np.concatenate(new_cols).astype(np.int32),
               np.concatenate(new_vals).astype(np.float16))


# ----------------------------------------------------------------------------
# Named workloads (the five benchmark configurations) with a size knob for tests
# ----------------------------------------------------------------------------
def make(name: str, small: bool = False) -> Csr:
    """``small`` gives a reduced instance with the same structure, sized so the
    CPU oracle finishes in seconds."""
    if name == "tiny":
        return tiny()
    if name == "powerlaw":
        return rmat(scale=12 if small else 17, avg_degree=16, seed=BASE_SEED + 2)
    if name == "community":
        return community(n_blocks=96 if small else 16384, seed=BASE_SEED + 3)
    if name == "irregular":
        return irregular(n=40_000 if small else 2_400_000, seed=BASE_SEED + 4)
    if name == "irregular_plainzipf":
        return irregular(n=40_000 if small else 2_400_000, seed=BASE_SEED + 4, shift=0.0)
    if name == "gat":
        return rmat(scale=13 if small else 20, avg_degree=32, seed=BASE_SEED + 5)
    raise ValueError(name)
