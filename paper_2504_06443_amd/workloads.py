"""Seeded synthetic inputs shaped like the paper's SpMM workloads.

This module only *draws inputs* (CSR sparsity patterns, values, dense B).  It
contains none of the method's arithmetic: no brick building, no products, no
synergy model.  Both the CPU oracle's tests and the HIP path's tests/benchmarks
take their inputs from here so that the two sides see identical data.

The paper evaluates on SuiteSparse matrices with more than 10,000 rows
(Section 6.1, "Datasets"), which are not available offline.  The generators
below stand in for them: banded, clustered-structural (dense 3x3 blocks near
the diagonal, the shape and density of the structural matrix named in
Section 1), scattered power-law (the shape of the web graph named in
Section 1) and a brick-fill sweep that spans the three synergy classes of
Table 1.

Every generator returns sorted, duplicate-free CSR with int32 indices and
float32 values.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

__all__ = [
    "CSR", "csr_from_coo", "dense_b",
    "tiny_banded", "clustered_blocks", "power_law", "brick_sweep",
    "uniform_random", "paired_panels", "config", "CONFIG_NAMES",
]


@dataclass
class CSR:
    """Plain CSR container (host numpy arrays)."""
    M: int
    K: int
    rowptr: np.ndarray   # int32[M+1]
    colind: np.ndarray   # int32[nnz], strictly ascending inside each row
    vals: np.ndarray     # float32[nnz]

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def to_dense(self) -> np.ndarray:
        """Dense float64 copy; for tiny matrices in tests only."""
        A = np.zeros((self.M, self.K), dtype=np.float64)
        rows = np.repeat(np.arange(self.M), np.diff(self.rowptr))
        A[rows, self.colind] = self.vals.astype(np.float64)
        return A


def csr_from_coo(M: int, K: int, rows: np.ndarray, cols: np.ndarray,
                 vals: np.ndarray | None = None) -> CSR:
    """Sort (row, col) pairs, drop duplicates (first value wins), emit CSR."""
    rows = np.asarray(rows, dtype=np.int64)
    cols = np.asarray(cols, dtype=np.int64)
    key = rows * np.int64(K) + cols
    if vals is None:
        key = np.unique(key)
        v = None
    else:
        key, first = np.unique(key, return_index=True)
        v = np.asarray(vals, dtype=np.float32)[first]
    r = key // np.int64(K)
    c = (key - r * np.int64(K)).astype(np.int32)
    counts = np.bincount(r, minlength=M)
    rowptr = np.zeros(M + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    if rowptr[-1] >= 2**31:
        raise ValueError("nnz does not fit int32")
    if v is None:
        v = np.zeros(len(c), dtype=np.float32)
    return CSR(M, K, rowptr.astype(np.int32), c, v)


def _fill_uniform(csr: CSR, rng: np.random.Generator) -> CSR:
    csr.vals = rng.uniform(-1.0, 1.0, size=csr.nnz).astype(np.float32)
    return csr


def dense_b(K: int, N: int, seed: int) -> np.ndarray:
    """Dense right-hand side, float32 N(0,1), row-major K x N."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((K, N), dtype=np.float32)


# --------------------------------------------------------------------------
# config 1: tiny banded
# --------------------------------------------------------------------------
def tiny_banded(M: int = 4096, per_row: int = 10, half_width: int = 64,
                seed: int = 1001) -> CSR:
    """Each row draws `per_row` column offsets uniform in [-hw, hw] around the
    diagonal, clipped to the matrix and de-duplicated; values U(-1,1)."""
    rng = np.random.default_rng(seed)
    K = M
    off = rng.integers(-half_width, half_width + 1, size=(M, per_row))
    cols = np.clip(np.arange(M)[:, None] + off, 0, K - 1)
    rows = np.broadcast_to(np.arange(M)[:, None], cols.shape)
    csr = csr_from_coo(M, K, rows.ravel(), cols.ravel())
    return _fill_uniform(csr, rng)


# --------------------------------------------------------------------------
# configs 2 and 4: dense 3x3 blocks clustered around the diagonal
# --------------------------------------------------------------------------
def clustered_blocks(M: int, blocks_per_row: float, half_width: int,
                     block: int = 3, seed: int = 1002,
                     chunk_rows: int = 8192) -> CSR:
    """Rows are grouped in block rows of `block` rows (last one clipped).  Each
    block row holds floor/ceil(blocks_per_row) *distinct* dense block x block
    tiles at block-aligned columns within `half_width` columns of the
    diagonal; values U(-1,1)."""
    rng = np.random.default_rng(seed)
    K = M
    nbr = -(-M // block)                 # block rows
    nbc = -(-K // block)                 # block columns
    hwb = half_width // block            # half width in block columns
    width = 2 * hwb + 1
    base = int(np.floor(blocks_per_row))
    frac = float(blocks_per_row) - base
    all_rows, all_cols = [], []
    for r0 in range(0, nbr, chunk_rows):
        r1 = min(nbr, r0 + chunk_rows)
        br = np.arange(r0, r1)
        n = r1 - r0
        cnt = base + (rng.random(n) < frac).astype(np.int64)
        keys = rng.random((n, width), dtype=np.float32)
        bc = br[:, None] + np.arange(-hwb, hwb + 1)[None, :]
        keys[(bc < 0) | (bc >= nbc)] = np.inf
        kmax = base + 1
        pick = np.argpartition(keys, kmax - 1, axis=1)[:, :kmax]
        pk = np.take_along_axis(keys, pick, axis=1)
        order = np.argsort(pk, axis=1)
        pick = np.take_along_axis(pick, order, axis=1)
        pk = np.take_along_axis(pk, order, axis=1)
        keep = (np.arange(kmax)[None, :] < cnt[:, None]) & np.isfinite(pk)
        sel_br = np.broadcast_to(br[:, None], pick.shape)[keep]
        sel_bc = (sel_br - hwb) + pick[keep]
        # expand each block into block x block entries
        di, dj = np.meshgrid(np.arange(block), np.arange(block), indexing="ij")
        rr = sel_br[:, None] * block + di.ravel()[None, :]
        cc = sel_bc[:, None] * block + dj.ravel()[None, :]
        ok = (rr < M) & (cc < K)
        all_rows.append(rr[ok])
        all_cols.append(cc[ok])
    csr = csr_from_coo(M, K, np.concatenate(all_rows), np.concatenate(all_cols))
    return _fill_uniform(csr, rng)


# --------------------------------------------------------------------------
# config 3: scattered power-law graph
# --------------------------------------------------------------------------
def power_law(M: int = 325760, target_nnz: int | None = 929849,
              alpha: float = 2.1, cap: int = 3000, seed: int = 1003) -> CSR:
    """Row degree = min(Zipf(alpha) - 1, cap) (so empty rows exist), columns
    uniform over K, duplicates dropped, then thinned uniformly at random to
    `target_nnz` entries when more were drawn.  Unit values."""
    rng = np.random.default_rng(seed)
    K = M
    deg = np.minimum(rng.zipf(alpha, size=M) - 1, cap).astype(np.int64)
    rows = np.repeat(np.arange(M, dtype=np.int64), deg)
    cols = rng.integers(0, K, size=rows.size, dtype=np.int64)
    key = np.unique(rows * np.int64(K) + cols)
    if target_nnz is not None and key.size > target_nnz:
        keep = rng.choice(key.size, size=target_nnz, replace=False)
        key = np.sort(key[keep])
    r = key // np.int64(K)
    c = key - r * np.int64(K)
    csr = csr_from_coo(M, K, r, c)
    csr.vals = np.ones(csr.nnz, dtype=np.float32)
    return csr


# --------------------------------------------------------------------------
# config 5: brick-fill sweep
# --------------------------------------------------------------------------
def brick_sweep(fill: float, M: int = 65536, target_nnz: int = 2_000_000,
                seed: int = 1005, brick_m: int = 16, brick_k: int = 4) -> CSR:
    """Choose grid-aligned 16x4 cells of the index space uniformly at random
    (with replacement) and put round(64*fill) distinct entries in each;
    duplicates dropped; values U(-1,1)."""
    rng = np.random.default_rng(seed + int(round(fill * 1000)))
    K = M
    cells = brick_m * brick_k
    per = max(1, min(cells, int(round(cells * fill))))
    nbr = max(1, int(round(target_nnz / per)))
    gr = rng.integers(0, M // brick_m, size=nbr)
    gc = rng.integers(0, K // brick_k, size=nbr)
    keys = rng.random((nbr, cells), dtype=np.float32)
    pick = np.argpartition(keys, per - 1, axis=1)[:, :per] if per < cells else \
        np.broadcast_to(np.arange(cells), (nbr, cells))
    rr = gr[:, None] * brick_m + pick // brick_k
    cc = gc[:, None] * brick_k + pick % brick_k
    csr = csr_from_coo(M, K, rr.ravel(), cc.ravel())
    return _fill_uniform(csr, rng)


# --------------------------------------------------------------------------
# consecutive 16-row panels with (nearly) common active columns
# --------------------------------------------------------------------------
def paired_panels(M: int, cols_per_group: int = 240, half_width: int = 1024, row_fill: float = 0.19,
                  group_rows: int = 32, seed: int = 1006, chunk_groups: int = 2048) -> CSR:
    """Rows are grouped `group_rows` at a time.  Each group draws `cols_per_group` distinct
    columns within `half_width` of the diagonal, and every row of the group stores each of
    them with probability `row_fill`.  With 32-row groups both 16-row halves of a group see
    almost the same active columns (the first of the two extreme non-zero distributions of
    Section 4's discussion of the row-panel height), at a column density of about
    `row_fill`; values U(-1,1)."""
    rng = np.random.default_rng(seed)
    K = M
    ngroups = -(-M // group_rows)
    width = 2 * half_width + 1
    all_rows, all_cols = [], []
    for g0 in range(0, ngroups, chunk_groups):
        g1 = min(ngroups, g0 + chunk_groups)
        n = g1 - g0
        centre = (np.arange(g0, g1) * group_rows + group_rows // 2)
        keys = rng.random((n, width), dtype=np.float32)
        cand = centre[:, None] + np.arange(-half_width, half_width + 1)[None, :]
        keys[(cand < 0) | (cand >= K)] = np.inf
        pick = np.argpartition(keys, cols_per_group - 1, axis=1)[:, :cols_per_group]
        ok = np.isfinite(np.take_along_axis(keys, pick, axis=1))
        cols = np.take_along_axis(cand, pick, axis=1)                      # [n, cols_per_group]
        store = rng.random((n, group_rows, cols_per_group), dtype=np.float32) < row_fill
        store &= ok[:, None, :]
        rows = (np.arange(g0, g1) * group_rows)[:, None, None] + np.arange(group_rows)[None, :, None]
        store &= rows < M
        rr = np.broadcast_to(rows, store.shape)[store]
        cc = np.broadcast_to(cols[:, None, :], store.shape)[store]
        all_rows.append(rr)
        all_cols.append(cc)
    csr = csr_from_coo(M, K, np.concatenate(all_rows), np.concatenate(all_cols))
    return _fill_uniform(csr, rng)


# --------------------------------------------------------------------------
# small general-purpose matrices for tests
# --------------------------------------------------------------------------
def uniform_random(M: int, K: int, density: float, seed: int,
                   empty_row_frac: float = 0.0, integer_values: bool = False) -> CSR:
    """Bernoulli(density) pattern; optionally whole rows emptied; values either
    U(-1,1) or small non-zero integers (exactly representable products)."""
    rng = np.random.default_rng(seed)
    mask = rng.random((M, K)) < density if M * K else np.zeros((M, K), bool)
    if empty_row_frac > 0 and M:
        mask[rng.random(M) < empty_row_frac, :] = False
    rows, cols = np.nonzero(mask)
    csr = csr_from_coo(M, K, rows, cols)
    if integer_values:
        v = rng.integers(1, 8, size=csr.nnz) * rng.choice([-1, 1], size=csr.nnz)
        csr.vals = v.astype(np.float32)
    else:
        _fill_uniform(csr, rng)
    return csr


CONFIG_NAMES = ("tiny_banded", "clustered_262k", "powerlaw_326k", "fem_923k", "sweep_65k")


def config(index: int, **kw) -> tuple[CSR, list[int]]:
    """The five benchmark configurations.  Returns (A, list of N values).
    `index` is 1-based; config 5 takes fill=<f>."""
    if index == 1:
        return tiny_banded(seed=1001), [32]
    if index == 2:
        return clustered_blocks(262144, 10, 256, seed=1002), [128]
    if index == 3:
        return power_law(seed=1003), [128]
    if index == 4:
        return clustered_blocks(923136, 14.8, 1024, seed=1004), [32, 128]
    if index == 5:
        return brick_sweep(kw.get("fill", 0.4), seed=1005), [16, 32, 64, 128, 256, 512]
    raise ValueError("config index must be 1..5")
