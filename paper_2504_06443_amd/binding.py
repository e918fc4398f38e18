"""ctypes binding of libspmm_brick.so: same names as the C ABI in include/spmm.h.

Argument marshalling only -- every step of the path runs in the HIP library.
Device arrays are torch tensors (PyTorch is used for device memory and
streams); results of host-side queries come back as plain Python / numpy.
Importing this module raises if the library has not been built: there is no
fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # first: the library must bind to the HIP runtime torch has already loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspmm_brick.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} not found: build it with `python -m paper_2504_06443_amd.build` "
        "(or __graft_entry__.build()); there is no CPU fallback")

_lib = C.CDLL(LIB_PATH)

SPMM_OK, SPMM_EINVAL, SPMM_EFORMAT, SPMM_ENOMEM, SPMM_EHIP, SPMM_ELIMIT = 0, -1, -2, -3, -4, -5
ROUTE_AUTO, ROUTE_MFMA, ROUTE_VALU, ROUTE_CLASS = 0, 1, 2, 3
ORDER_PANEL, ORDER_HEAVY_FIRST = 0, 1
SPLIT_EQ7_NEAREST, SPLIT_EQ7_FROM2, SPLIT_NEVER = -1, 0, 1
PRECISION_FP32, PRECISION_BF16X3, PRECISION_BF16X6 = 0, 1, 2
SHARE_NONE, SHARE_WORKGROUP = 0, 1
PRECISIONS = {"fp32": PRECISION_FP32, "bf16x3": PRECISION_BF16X3, "bf16x6": PRECISION_BF16X6}
CLASS_NAMES = ("Low", "Medium", "High")

EXPORTED = (
    "spmm_plan", "spmm_plan_update_values", "spmm_exec", "spmm_exec_noalloc", "spmm_synergy",
    "spmm_plan_sizes",
    "spmm_plan_export",
    "spmm_plan_set_route", "spmm_plan_set_split", "spmm_plan_set_order", "spmm_plan_set_precision",
    "spmm_plan_set_tile_sharing", "spmm_plan_set_panel_height", "spmm_plan_tm32_sizes", "spmm_plan_tm32_export",
    "spmm_partition_counts",
    "spmm_plan_worklist", "spmm_plan_destroy", "spmm_last_error", "spmm_calibrate_gather",
)


class SpmmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"spmm status {code}: {msg}")
        self.code = code


class _Synergy(C.Structure):
    _fields_ = [
        ("M", C.c_int64), ("K", C.c_int64), ("nnz", C.c_int64),
        ("n_panels", C.c_int64), ("n_nonempty_panels", C.c_int64), ("n_bricks", C.c_int64),
        ("n_active_cols", C.c_int64), ("n_distinct_cols", C.c_int64),
        ("panels_by_class", C.c_int64 * 3), ("bricks_by_class", C.c_int64 * 3),
        ("nnz_by_class", C.c_int64 * 3), ("brick_pop_hist", C.c_int64 * 65),
        ("synergy_class", C.c_int32), ("reserved_", C.c_int32),
        ("alpha_brick", C.c_double), ("alpha_col", C.c_double), ("beta", C.c_double),
        ("oi_shmem", C.c_double), ("bytes_min", C.c_double), ("bytes_noreuse", C.c_double),
        ("oi_hbm_min", C.c_double), ("oi_hbm_noreuse", C.c_double),
        ("roof_gflops_hbm", C.c_double), ("roof_gflops_mfma", C.c_double),
    ]


class _Sizes(C.Structure):
    _fields_ = [("M", C.c_int64), ("K", C.c_int64), ("nnz", C.c_int64),
                ("n_panels", C.c_int64), ("n_bricks", C.c_int64)]


class _Tm32Sizes(C.Structure):
    _fields_ = [("n_super_panels", C.c_int64), ("n_brick_cols", C.c_int64),
                ("n_bricks", C.c_int64), ("n_merged", C.c_int64)]


class _WorkItem(C.Structure):
    _fields_ = [("panel", C.c_uint32), ("brick_begin", C.c_uint32), ("brick_end", C.c_uint32),
                ("part", C.c_uint32), ("nparts", C.c_uint32)]


class _WorklistInfo(C.Structure):
    _fields_ = [("n_mfma_items", C.c_int64), ("n_valu_panels", C.c_int64),
                ("n_split_panels", C.c_int64), ("num_waves", C.c_int64),
                ("n_tile", C.c_int32), ("n_tiles", C.c_int32),
                ("num_cus", C.c_int32), ("resident_waves_per_cu", C.c_int32)]


_vp = C.c_void_p
_lib.spmm_last_error.restype = C.c_char_p
_lib.spmm_plan.argtypes = [C.c_int64, C.c_int64, C.c_int64, _vp, _vp, _vp, _vp, C.POINTER(_vp)]
_lib.spmm_plan_update_values.argtypes = [_vp, _vp, _vp]
_lib.spmm_exec.argtypes = [_vp, _vp, C.c_int64, _vp, _vp]
_lib.spmm_exec_noalloc.argtypes = [_vp, _vp, C.c_int64, _vp, _vp]
_lib.spmm_synergy.argtypes = [_vp, C.c_int64, C.POINTER(_Synergy)]
_lib.spmm_plan_sizes.argtypes = [_vp, C.POINTER(_Sizes)]
_lib.spmm_plan_export.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp]
_lib.spmm_plan_set_route.argtypes = [_vp, C.c_int]
_lib.spmm_plan_set_split.argtypes = [_vp, C.c_int]
_lib.spmm_plan_set_order.argtypes = [_vp, C.c_int]
_lib.spmm_plan_set_precision.argtypes = [_vp, C.c_int]
_lib.spmm_plan_set_tile_sharing.argtypes = [_vp, C.c_int]
_lib.spmm_plan_set_panel_height.argtypes = [_vp, C.c_int, C.c_uint32, C.c_uint32, _vp]
_lib.spmm_plan_tm32_sizes.argtypes = [_vp, C.POINTER(_Tm32Sizes)]
_lib.spmm_plan_tm32_export.argtypes = [_vp] + [_vp] * 8
_lib.spmm_partition_counts.argtypes = [C.c_int64, _vp, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                       _vp, C.POINTER(C.c_int64)]
_lib.spmm_plan_worklist.argtypes = [_vp, C.c_int64, C.POINTER(_WorklistInfo), _vp, _vp]
_lib.spmm_plan_destroy.argtypes = [_vp]
_lib.spmm_calibrate_gather.argtypes = [_vp, C.c_int64, C.c_int64, C.c_int64, _vp, _vp]
_lib.spmm_plan_destroy.restype = None


def _check(status: int):
    if status != SPMM_OK:
        raise SpmmError(status, (_lib.spmm_last_error() or b"").decode())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(getattr(stream, "cuda_stream", stream))


def _dev(t, dtype):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("expected a CUDA/HIP torch tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"expected contiguous {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


class Plan:
    """Owner of an spmm_plan_t handle."""

    def __init__(self, handle, M, K, nnz):
        self._h = handle
        self.M, self.K, self.nnz = M, K, nnz

    def __del__(self):
        self.destroy()

    def destroy(self):
        if getattr(self, "_h", None):
            if _lib is not None:          # (None while the interpreter shuts down)
                _lib.spmm_plan_destroy(self._h)
            self._h = None


def spmm_plan(M: int, K: int, rowptr, colind, vals, stream=None) -> Plan:
    """CSR (device int32/int32/float32 tensors) -> plan holding the brick format."""
    nnz = int(colind.numel())
    if int(rowptr.numel()) != M + 1:
        raise ValueError("rowptr must have M + 1 entries")
    if int(vals.numel()) != nnz:
        raise ValueError("vals and colind must have the same length")
    out = _vp()
    _check(_lib.spmm_plan(M, K, nnz, _dev(rowptr, torch.int32),
                          _dev(colind, torch.int32) if nnz else None,
                          _dev(vals, torch.float32) if nnz else None,
                          _stream_ptr(stream), C.byref(out)))
    return Plan(out, M, K, nnz)


def spmm_plan_update_values(plan: Plan, vals, stream=None):
    """New values (device float32 [nnz], CSR order) for the plan's unchanged pattern."""
    if int(vals.numel()) != plan.nnz:
        raise ValueError("vals has the wrong length")
    _check(_lib.spmm_plan_update_values(plan._h, _dev(vals, torch.float32) if plan.nnz else None,
                                        _stream_ptr(stream)))


def spmm_exec(plan: Plan, B, C_out=None, stream=None, _entry=None):
    """C = A . B on the current (or given) stream.  B: device float32 [K, N]."""
    N = int(B.shape[1])
    if B.shape[0] != plan.K:
        raise ValueError("B has the wrong number of rows")
    if C_out is None:
        C_out = torch.empty((plan.M, N), dtype=torch.float32, device=B.device)
    elif tuple(C_out.shape) != (plan.M, N):
        raise ValueError("C has the wrong shape")
    entry = _entry or _lib.spmm_exec
    _check(entry(plan._h, _dev(B, torch.float32) if B.numel() else None, N,
                 _dev(C_out, torch.float32) if C_out.numel() else None, _stream_ptr(stream)))
    return C_out


def spmm_exec_noalloc(plan: Plan, B, C_out, stream=None):
    """Same product through the entry point that allocates no device memory; the caller
    provides C (allocating it here would defeat the purpose)."""
    return spmm_exec(plan, B, C_out, stream, _entry=_lib.spmm_exec_noalloc)


def spmm_synergy(plan: Plan, N: int) -> dict:
    s = _Synergy()
    _check(_lib.spmm_synergy(plan._h, N, C.byref(s)))
    out = {}
    for name, ctype in _Synergy._fields_:
        if name == "reserved_":
            continue
        v = getattr(s, name)
        out[name] = list(v) if hasattr(v, "__len__") else v
    return out


def spmm_plan_sizes(plan: Plan) -> dict:
    s = _Sizes()
    _check(_lib.spmm_plan_sizes(plan._h, C.byref(s)))
    return {n: getattr(s, n) for n, _ in _Sizes._fields_}


def spmm_plan_export(plan: Plan) -> dict:
    """Copy the brick format to host numpy arrays."""
    sz = spmm_plan_sizes(plan)
    P, nb, nnz = sz["n_panels"], sz["n_bricks"], sz["nnz"]
    out = dict(
        panel_ptr=np.zeros(P + 1, dtype=np.uint32),
        brick_cols=np.zeros(4 * nb, dtype=np.uint32),
        brick_mask=np.zeros(nb, dtype=np.uint64),
        brick_valptr=np.zeros(nb + 1, dtype=np.uint32),
        vals=np.zeros(nnz, dtype=np.float32),
    )
    _check(_lib.spmm_plan_export(plan._h, *[out[k].ctypes.data_as(_vp) for k in
                                            ("panel_ptr", "brick_cols", "brick_mask",
                                             "brick_valptr", "vals")]))
    return out


def spmm_plan_set_route(plan: Plan, route: int):
    _check(_lib.spmm_plan_set_route(plan._h, route))


def spmm_plan_set_split(plan: Plan, parts: int):
    _check(_lib.spmm_plan_set_split(plan._h, parts))


def spmm_plan_set_order(plan: Plan, order: int):
    _check(_lib.spmm_plan_set_order(plan._h, order))


def spmm_plan_set_precision(plan: Plan, precision: int):
    _check(_lib.spmm_plan_set_precision(plan._h, precision))


def spmm_calibrate_gather(buf, n_rows: int, loads_per_wave: int, n_waves: int, sink, stream=None):
    """Enqueue the random-row gather kernel (measurement aid); the caller times it."""
    if buf.numel() * buf.element_size() < n_rows * 512 or sink.numel() < 256:
        raise ValueError("buffer too small")
    status = _lib.spmm_calibrate_gather(_dev(buf, torch.float32), n_rows, loads_per_wave, n_waves,
                                        _dev(sink, torch.float32), _stream_ptr(stream))
    if status != SPMM_OK:
        raise SpmmError(status, "spmm_calibrate_gather: bad sizes")


def spmm_plan_set_tile_sharing(plan: Plan, mode: int):
    _check(_lib.spmm_plan_set_tile_sharing(plan._h, mode))


def spmm_plan_set_panel_height(plan: Plan, rows: int, merge_num: int = 6, merge_den: int = 5,
                               stream=None):
    """rows = 32: build the 32-row panel format and use it where it applies; 16: back."""
    _check(_lib.spmm_plan_set_panel_height(plan._h, rows, merge_num, merge_den, _stream_ptr(stream)))


def spmm_plan_tm32_sizes(plan: Plan) -> dict:
    s = _Tm32Sizes()
    _check(_lib.spmm_plan_tm32_sizes(plan._h, C.byref(s)))
    return {n: getattr(s, n) for n, _ in _Tm32Sizes._fields_}


def spmm_plan_tm32_export(plan: Plan) -> dict:
    """Copy the 32-row panel format to host numpy arrays."""
    sz = spmm_plan_tm32_sizes(plan)
    Q, nbc, nbr = sz["n_super_panels"], sz["n_brick_cols"], sz["n_bricks"]
    out = dict(
        sp_ptr=np.zeros(Q + 1, dtype=np.uint32), sp_merged=np.zeros(Q, dtype=np.uint8),
        bc_cols=np.zeros(4 * nbc, dtype=np.uint32), bc_brick=np.zeros(nbc + 1, dtype=np.uint32),
        br_row=np.zeros(nbr, dtype=np.uint8), br_mask=np.zeros(nbr, dtype=np.uint64),
        br_valptr=np.zeros(nbr + 1, dtype=np.uint32), vals=np.zeros(plan.nnz, dtype=np.float32),
    )
    _check(_lib.spmm_plan_tm32_export(plan._h, *[out[k].ctypes.data_as(_vp) for k in
                                                 ("sp_ptr", "sp_merged", "bc_cols", "bc_brick",
                                                  "br_row", "br_mask", "br_valptr", "vals")]))
    out.update(sz)
    return out


def spmm_partition_counts(nbricks, work_items: int, num_cus: int, resident_per_cu: int,
                          policy: int = SPLIT_EQ7_FROM2):
    """Eq. 6-7 on the host (no GPU needed). Returns (parts per panel, num_waves)."""
    nb = np.ascontiguousarray(nbricks, dtype=np.uint32)
    parts = np.zeros(len(nb), dtype=np.uint32)
    waves = C.c_int64(0)
    _check(_lib.spmm_partition_counts(len(nb), nb.ctypes.data_as(_vp), work_items, num_cus,
                                      resident_per_cu, policy, parts.ctypes.data_as(_vp),
                                      C.byref(waves)))
    return parts, waves.value


def spmm_plan_worklist(plan: Plan, N: int) -> dict:
    info = _WorklistInfo()
    _check(_lib.spmm_plan_worklist(plan._h, N, C.byref(info), None, None))
    items = (_WorkItem * max(1, info.n_mfma_items))()
    valu = np.zeros(max(1, info.n_valu_panels), dtype=np.uint32)
    _check(_lib.spmm_plan_worklist(plan._h, N, C.byref(info), items, valu.ctypes.data_as(_vp)))
    out = {n: getattr(info, n) for n, _ in _WorklistInfo._fields_}
    out["items"] = [(it.panel, it.brick_begin, it.brick_end, it.part, it.nparts)
                    for it in items[:info.n_mfma_items]]
    out["valu_panels"] = valu[:info.n_valu_panels].copy()
    return out


def spmm_plan_destroy(plan: Plan):
    plan.destroy()


def spmm_last_error() -> str:
    return (_lib.spmm_last_error() or b"").decode()
