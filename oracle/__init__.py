"""CPU oracle for the brick SpMM hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over `spmm_oracle.c` (plain C, fp64 accumulation) plus the
load-balance arithmetic of Section 5 written out in Python integers.  Only
tests, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may
import this package; the HIP library and its binding never do, and this
package imports nothing from them.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

SYNERGY_NAMES = ("Low", "Medium", "High")
HBM_BYTES_PER_S = 8.0e12        # MI355X published HBM3E bandwidth
MFMA_FP32_FLOPS = 157.3e12      # MI355X published dense fp32 matrix peak


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_num_threads.restype = C.c_int
        _lib.oracle_synergy.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def num_threads() -> int:
    return int(_L().oracle_num_threads())


def spmm_f64(rowptr, colind, vals, B, want_abs: bool = True):
    """C = A.B in fp64 (Section 3.1) and S = sum |a.b| (error normaliser)."""
    rowptr, colind, vals, B = _i32(rowptr), _i32(colind), _f32(vals), _f32(B)
    M = len(rowptr) - 1
    N = B.shape[1]
    Cout = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if want_abs else None
    _L().oracle_spmm_f64(C.c_int64(M), C.c_int64(N), _p(rowptr), _p(colind), _p(vals), _p(B),
                         _p(Cout), _p(S) if want_abs else None)
    return (Cout, S) if want_abs else Cout


def spmm_rows_f64(rows, rowptr, colind, vals, B):
    """Rows `rows` of C = A.B and of S, for sampled checks at full size."""
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    rowptr, colind, vals, B = _i32(rowptr), _i32(colind), _f32(vals), _f32(B)
    N = B.shape[1]
    Cout = np.empty((len(rows), N), dtype=np.float64)
    S = np.empty((len(rows), N), dtype=np.float64)
    _L().oracle_spmm_rows_f64(C.c_int64(len(rows)), _p(rows), C.c_int64(N), _p(rowptr),
                              _p(colind), _p(vals), _p(B), _p(Cout), _p(S))
    return Cout, S


def panel_active_cols(M, rowptr, colind):
    rowptr, colind = _i32(rowptr), _i32(colind)
    P = (M + 15) // 16
    ncols = np.zeros(P, dtype=np.int64)
    _L().oracle_panel_active_cols(C.c_int64(M), _p(rowptr), _p(colind), _p(ncols))
    return ncols


def build_bricks(M, rowptr, colind, vals) -> dict:
    """CSR -> brick format (Section 3.2).  Returns a dict of numpy arrays:
    panel_ptr u32[P+1], brick_cols u32[4 nb], brick_mask u64[nb],
    brick_valptr u32[nb+1], vals f32[nnz], ncols i64[P]."""
    rowptr, colind, vals = _i32(rowptr), _i32(colind), _f32(vals)
    P = (M + 15) // 16
    ncols = panel_active_cols(M, rowptr, colind)
    nb = int(((ncols + 3) // 4).sum())
    nnz = int(rowptr[M])
    out = dict(
        panel_ptr=np.zeros(P + 1, dtype=np.uint32),
        brick_cols=np.zeros(4 * nb, dtype=np.uint32),
        brick_mask=np.zeros(nb, dtype=np.uint64),
        brick_valptr=np.zeros(nb + 1, dtype=np.uint32),
        vals=np.zeros(nnz, dtype=np.float32),
        ncols=ncols,
    )
    _L().oracle_bricks_build(C.c_int64(M), _p(rowptr), _p(colind), _p(vals), _p(ncols),
                             _p(out["panel_ptr"]), _p(out["brick_cols"]), _p(out["brick_mask"]),
                             _p(out["brick_valptr"]), _p(out["vals"]))
    return out


def bricks_to_csr(M, fmt: dict):
    nnz = int(fmt["brick_valptr"][-1])
    rowptr = np.zeros(M + 1, dtype=np.int32)
    colind = np.zeros(nnz, dtype=np.int32)
    vals = np.zeros(nnz, dtype=np.float32)
    _L().oracle_bricks_to_csr(C.c_int64(M), _p(fmt["panel_ptr"]), _p(fmt["brick_cols"]),
                              _p(fmt["brick_mask"]), _p(fmt["brick_valptr"]), _p(fmt["vals"]),
                              _p(rowptr), _p(colind), _p(vals))
    return rowptr, colind, vals


def synergy(M, K, N, rowptr, colind, fmt: dict) -> dict:
    """Brick density alpha, OI_shmem = 512 alpha (Eq. 4), class per Table 1,
    per-panel class counts, and the HBM / MFMA roofline model."""
    rowptr, colind = _i32(rowptr), _i32(colind)
    icnt = np.zeros(82, dtype=np.int64)
    fval = np.zeros(10, dtype=np.float64)
    cls = _L().oracle_synergy(C.c_int64(M), C.c_int64(K), C.c_int64(N), _p(rowptr), _p(colind),
                              _p(fmt["panel_ptr"]), _p(fmt["brick_mask"]), _p(fmt["ncols"]),
                              C.c_double(HBM_BYTES_PER_S), C.c_double(MFMA_FP32_FLOPS),
                              _p(icnt), _p(fval))
    return dict(
        M=int(icnt[0]), K=int(icnt[1]), nnz=int(icnt[2]), n_panels=int(icnt[3]),
        n_nonempty_panels=int(icnt[4]), n_bricks=int(icnt[5]), n_active_cols=int(icnt[6]),
        n_distinct_cols=int(icnt[7]),
        panels_by_class=[int(x) for x in icnt[8:11]],
        bricks_by_class=[int(x) for x in icnt[11:14]],
        nnz_by_class=[int(x) for x in icnt[14:17]],
        brick_pop_hist=[int(x) for x in icnt[17:82]],
        synergy_class=int(cls),
        alpha_brick=float(fval[0]), alpha_col=float(fval[1]), beta=float(fval[2]),
        oi_shmem=float(fval[3]), bytes_min=float(fval[4]), bytes_noreuse=float(fval[5]),
        oi_hbm_min=float(fval[6]), oi_hbm_noreuse=float(fval[7]),
        roof_gflops_hbm=float(fval[8]), roof_gflops_mfma=float(fval[9]),
    )


# ---------------------------------------------------------------------------
# Section 4, Eq. 5: 32-row panels with up to two bricks per brick column
# ---------------------------------------------------------------------------
def build_tm32(M, rowptr, colind, vals, num: int = 6, den: int = 5) -> dict:
    """CSR -> 32-row panel format.  The two 16-row halves of a super-panel share one
    left-packed column list where |union| * den < num * max(|top|, |bottom|); elsewhere they
    keep their own lists (the bricks of the 16-row format).  Returns the arrays described in
    spmm_oracle.c plus the counts Q, nbc, nbr, n_merged and beta = nbr / nbc (Eq. 5)."""
    rowptr, colind, vals = _i32(rowptr), _i32(colind), _f32(vals)
    sizes = np.zeros(4, dtype=np.int64)
    _L().oracle_tm32_sizes(C.c_int64(M), _p(rowptr), _p(colind), C.c_int64(num), C.c_int64(den),
                           _p(sizes))
    Q, nbc, nbr, merged = (int(x) for x in sizes)
    nnz = int(rowptr[M])
    out = dict(
        sp_ptr=np.zeros(Q + 1, dtype=np.uint32),
        sp_merged=np.zeros(Q, dtype=np.uint8),
        bc_cols=np.zeros(4 * nbc, dtype=np.uint32),
        bc_brick=np.zeros(nbc + 1, dtype=np.uint32),
        br_row=np.zeros(nbr, dtype=np.uint8),
        br_mask=np.zeros(nbr, dtype=np.uint64),
        br_valptr=np.zeros(nbr + 1, dtype=np.uint32),
        vals=np.zeros(nnz, dtype=np.float32),
    )
    _L().oracle_tm32_build(C.c_int64(M), _p(rowptr), _p(colind), _p(vals), C.c_int64(num),
                           C.c_int64(den), _p(out["sp_ptr"]), _p(out["sp_merged"]),
                           _p(out["bc_cols"]), _p(out["bc_brick"]), _p(out["br_row"]),
                           _p(out["br_mask"]), _p(out["br_valptr"]), _p(out["vals"]))
    out.update(Q=Q, nbc=nbc, nbr=nbr, n_merged=merged, beta=(nbr / nbc if nbc else 0.0))
    return out


def tm32_to_csr(M, fmt: dict):
    nnz = int(fmt["br_valptr"][-1])
    rowptr = np.zeros(M + 1, dtype=np.int32)
    colind = np.zeros(nnz, dtype=np.int32)
    vals = np.zeros(nnz, dtype=np.float32)
    _L().oracle_tm32_to_csr(C.c_int64(M), _p(fmt["sp_ptr"]), _p(fmt["bc_cols"]),
                            _p(fmt["bc_brick"]), _p(fmt["br_row"]), _p(fmt["br_mask"]),
                            _p(fmt["br_valptr"]), _p(fmt["vals"]), _p(rowptr), _p(colind), _p(vals))
    return rowptr, colind, vals


# ---------------------------------------------------------------------------
# Section 5, Eq. 6-7: wave-aware split of heavy row panels along K
# ---------------------------------------------------------------------------
def _ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def partition_counts(nbricks_per_panel, total_work_items: int, num_cus: int,
                     resident_per_cu: int, policy: str = "from2"):
    """Number of virtual panels each row panel is split into.

    blocks_p = ceil(bricks_p / 4) (a block is TK/brick_k = 4 brick columns);
    num_waves = ceil(total_work_items / (num_cus * resident_per_cu)), at least 1;
    num_loads_p = blocks_p / average blocks over all panels (Eq. 6);
    partition_ratio_p = num_loads_p / num_waves (Eq. 7).
    The paper gives no rounding rule beyond "no partition if the ratio is 1".  Two readings,
    both evaluated in integers:
      "nearest"  parts_p = max(1, round-half-up(partition_ratio_p)): the literal one, a
                 panel is split once its ratio reaches 1.5;
      "from2"    parts_p = 1 while partition_ratio_p < 2, else round-half-up: a panel is
                 split once it carries two wave-adjusted average loads (the default of
                 the library, chosen there by measurement).
    Returns (parts list, num_waves)."""
    if policy not in ("from2", "nearest"):
        raise ValueError("policy must be 'from2' or 'nearest'")
    blocks = [_ceil_div(int(b), 4) for b in nbricks_per_panel]
    P = len(blocks)
    total = sum(blocks)
    waves = max(1, _ceil_div(int(total_work_items), int(num_cus) * int(resident_per_cu)))
    parts = []
    for b in blocks:
        if total == 0 or b == 0:
            parts.append(1)
        else:
            num, den = b * P, total * waves          # partition_ratio = num / den
            nearest = (2 * num + den) // (2 * den)
            if policy == "from2" and num < 2 * den:
                nearest = 1
            parts.append(max(1, nearest))
    return parts, waves


def partition_ranges(nbricks: int, parts: int):
    """Split one panel's bricks [0, nbricks) into `parts` contiguous K-ranges of
    whole blocks (4 bricks), each ceil(blocks/parts) blocks; empty tails dropped."""
    blocks = _ceil_div(nbricks, 4)
    per = _ceil_div(blocks, parts) if parts > 0 else blocks
    out = []
    for q in range(parts):
        lo = min(nbricks, q * per * 4)
        hi = min(nbricks, (q + 1) * per * 4)
        if hi > lo or (q == 0):
            out.append((lo, hi))
    return out
