"""Thin ctypes binding over libsparsert.so: argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels.  There is no
fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsparsert.so")

OK, EINVAL, ENOMEM, EHIP, EUNSUPPORTED, ECOMPILE = 0, -1, -2, -3, -4, -5
F32, F16, I8 = 0, 1, 2
_DTYPE_OF = {np.dtype(np.float32): F32, np.dtype(np.float16): F16, np.dtype(np.int8): I8}
_NP_OF = {F32: np.float32, F16: np.float16, I8: np.int8}
KERNEL_AUTO, KERNEL_ROWS, KERNEL_SPEC = 0, 1, 2
SPEC_AUTO, SPEC_DIRECT, SPEC_LDS = 0, 1, 2
(FIELD_INFO, FIELD_ROW_NNZ, FIELD_HIST, FIELD_PERM, FIELD_INV_PERM, FIELD_P_ROW_PTR,
 FIELD_P_COL_IDX, FIELD_P_VALS, FIELD_BINS, FIELD_STREAM, FIELD_CONV_SEG,
 FIELD_SEGMENTS, FIELD_SPEC_GROUPS, FIELD_SPEC_COLUMNS, FIELD_SPEC_CODE, FIELD_KERNEL_NAME) = range(16)
INFO_NAMES = ["M", "K", "N", "nnz", "dtype", "conv", "Cin", "H", "W", "kernel", "vec",
              "lanes_per_tile", "n_tiles", "gy", "split_threshold", "n_split", "n_wg_rows",
              "n_bins", "spec_rows", "spec_groups", "spec_depth", "spec_code_bytes",
              "spec_tiles", "spec_mode", "spec_lds_bytes", "spec_ksplit", "natural_order", "spec_lanes", "spec_swizzle", "batch", "spec_vec",
              "ldb", "ldc", "spec_prefetch"]
INFO_COUNT = 48

EXPORTED = ["sparsert_inspect", "sparsert_tune", "sparsert_spmm", "sparsert_conv3x3", "sparsert_compare_outputs", "sparsert_compare_outputs_static", "sparsert_plan_export",
            "sparsert_plan_save", "sparsert_plan_load", "sparsert_plan_destroy", "sparsert_last_error",
            "sparsert_version"]


class Options(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("kernel", ctypes.c_int32), ("conv", ctypes.c_int32),
                ("Cin", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("batch", ctypes.c_int32), ("host_only", ctypes.c_int32),
                ("vec", ctypes.c_int32), ("split_threshold", ctypes.c_int32),
                ("spec_rows", ctypes.c_int32), ("spec_depth", ctypes.c_int32),
                ("spec_tiles", ctypes.c_int32), ("spec_mode", ctypes.c_int32),
                ("spec_ksplit", ctypes.c_int32), ("natural_order", ctypes.c_int32),
                ("spec_lanes", ctypes.c_int32), ("spec_swizzle", ctypes.c_int32),
                ("spec_vec", ctypes.c_int32), ("ldb", ctypes.c_int32), ("ldc", ctypes.c_int32),
                ("tune_warm", ctypes.c_int32), ("spec_prefetch", ctypes.c_int32), ("reserved", ctypes.c_int32 * 2)]


TUNE_MAX = 64


class TuneEntry(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("vec", ctypes.c_int32), ("split_threshold", ctypes.c_int32),
                ("spec_mode", ctypes.c_int32), ("spec_rows", ctypes.c_int32),
                ("spec_tiles", ctypes.c_int32), ("spec_ksplit", ctypes.c_int32),
                ("spec_lanes", ctypes.c_int32), ("spec_swizzle", ctypes.c_int32),
                ("spec_vec", ctypes.c_int32), ("microseconds", ctypes.c_float),
                ("cold_microseconds", ctypes.c_float), ("agrees", ctypes.c_int32), ("spec_prefetch", ctypes.c_int32)]


class TuneReport(ctypes.Structure):
    _fields_ = [("count", ctypes.c_int32), ("best_microseconds", ctypes.c_float),
                ("best_cold_microseconds", ctypes.c_float), ("entries", TuneEntry * TUNE_MAX)]


class SparseRTError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"sparsert status {status}: {message}")
        self.status = status


# Load torch's HIP runtime first when torch is present: the library asks for
# libamdhip64.so.7 by soname, and a process must not end up with two HIP runtimes
# (the second one finds no device).  torch itself is used by callers for device
# memory and streams only.
try:
    import torch  # noqa: F401
except ImportError:  # pure ctypes / C callers use the system runtime
    torch = None

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` to build the HIP library")

_lib = ctypes.CDLL(LIB_PATH)
_vp, _i32 = ctypes.c_void_p, ctypes.c_int32
_lib.sparsert_inspect.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, ctypes.POINTER(Options),
                                  ctypes.POINTER(_vp)]
_lib.sparsert_inspect.restype = ctypes.c_int
_lib.sparsert_tune.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, ctypes.POINTER(Options), _vp, _vp, _vp,
                               ctypes.POINTER(_vp), ctypes.POINTER(TuneReport)]
_lib.sparsert_tune.restype = ctypes.c_int
_lib.sparsert_spmm.argtypes = [_vp, _vp, _vp, _vp]
_lib.sparsert_spmm.restype = ctypes.c_int
_lib.sparsert_conv3x3.argtypes = [_vp, _vp, _vp, _vp]
_lib.sparsert_conv3x3.restype = ctypes.c_int
_lib.sparsert_compare_outputs.argtypes = [_vp, _vp, _vp, _vp, _vp]
_lib.sparsert_compare_outputs.restype = ctypes.c_int
_lib.sparsert_compare_outputs_static.argtypes = [_vp, _vp, _vp, _vp, _vp]
_lib.sparsert_compare_outputs_static.restype = ctypes.c_int
_lib.sparsert_plan_export.argtypes = [_vp, _i32, _vp, ctypes.c_size_t,
                                      ctypes.POINTER(ctypes.c_size_t)]
_lib.sparsert_plan_export.restype = ctypes.c_int
_lib.sparsert_plan_save.argtypes = [_vp, _vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
_lib.sparsert_plan_save.restype = ctypes.c_int
_lib.sparsert_plan_load.argtypes = [_vp, ctypes.c_size_t, _i32, ctypes.POINTER(_vp)]
_lib.sparsert_plan_load.restype = ctypes.c_int
_lib.sparsert_plan_destroy.argtypes = [_vp]
_lib.sparsert_plan_destroy.restype = None
_lib.sparsert_last_error.restype = ctypes.c_char_p
_lib.sparsert_version.restype = _i32


def last_error() -> str:
    return _lib.sparsert_last_error().decode()


def version() -> int:
    return int(_lib.sparsert_version())


def _check(rc: int):
    if rc != OK:
        raise SparseRTError(rc, last_error())


_FIELD_DTYPE = {FIELD_STREAM: np.uint32, FIELD_SPEC_CODE: np.uint8, FIELD_KERNEL_NAME: np.uint8}


class Plan:
    """Owner of a sparsert_plan handle."""

    def __init__(self, handle: int, dtype: int):
        self.handle = handle
        self.dtype = dtype

    def export(self, field: int) -> np.ndarray:
        need = ctypes.c_size_t(0)
        _check(_lib.sparsert_plan_export(self.handle, field, None, 0, ctypes.byref(need)))
        if field == FIELD_P_VALS:
            dt = _NP_OF[self.dtype]
        else:
            dt = _FIELD_DTYPE.get(field, np.int32)
        out = np.empty(need.value // np.dtype(dt).itemsize, dtype=dt)
        _check(_lib.sparsert_plan_export(self.handle, field, out.ctypes.data_as(_vp),
                                         out.nbytes, None))
        return out

    def info(self) -> dict:
        raw = self.export(FIELD_INFO)
        return {k: int(raw[i]) for i, k in enumerate(INFO_NAMES)}

    def kernel_name(self) -> str:
        """The name a kernel trace shows for this plan's launches."""
        return self.export(FIELD_KERNEL_NAME).tobytes().decode()

    def save(self) -> bytes:
        """sparsert_plan_save: the whole plan (with its generated code, if any) as bytes."""
        need = ctypes.c_size_t(0)
        _check(_lib.sparsert_plan_save(self.handle, None, 0, ctypes.byref(need)))
        buf = ctypes.create_string_buffer(need.value)
        _check(_lib.sparsert_plan_save(self.handle, buf, need.value, None))
        return buf.raw

    def destroy(self):
        if self.handle:
            _lib.sparsert_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def inspect(row_ptr, col_idx, vals, M: int, K: int, N: int, *, dtype: Optional[int] = None,
            conv: Optional[Tuple[int, int, int]] = None, batch: int = 0, host_only: bool = False,
            vec: int = 0, split_threshold: int = 0, kernel: int = KERNEL_AUTO,
            spec_rows: int = 0, spec_depth: int = 0, spec_tiles: int = 0,
            spec_mode: int = 0, spec_ksplit: int = 0, natural_order: bool = False,
            spec_lanes: int = 0, spec_swizzle: bool = False, spec_vec: int = 0,
            ldb: int = 0, ldc: int = 0, spec_prefetch: int = 0) -> Plan:
    """sparsert_inspect.  `vals` must already be float32, float16 or int8; it is not converted."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    vals = np.ascontiguousarray(vals)
    if dtype is None:
        if vals.dtype not in _DTYPE_OF:
            raise TypeError("vals must be float32, float16 or int8")
        dtype = _DTYPE_OF[vals.dtype]
    opt = Options()
    opt.dtype, opt.kernel, opt.host_only = dtype, kernel, int(host_only)
    opt.vec, opt.split_threshold, opt.batch = vec, split_threshold, batch
    opt.spec_rows, opt.spec_depth, opt.spec_tiles = spec_rows, spec_depth, spec_tiles
    opt.spec_mode, opt.spec_ksplit, opt.natural_order = spec_mode, spec_ksplit, int(natural_order)
    opt.spec_lanes, opt.spec_swizzle, opt.spec_vec = spec_lanes, int(spec_swizzle), spec_vec
    opt.ldb, opt.ldc, opt.spec_prefetch = ldb, ldc, spec_prefetch
    if conv is not None:
        opt.conv, (opt.Cin, opt.H, opt.W) = 1, conv
    handle = _vp()
    _check(_lib.sparsert_inspect(row_ptr.ctypes.data_as(_vp), col_idx.ctypes.data_as(_vp),
                                 vals.ctypes.data_as(_vp), M, K, N, ctypes.byref(opt),
                                 ctypes.byref(handle)))
    return Plan(handle.value, dtype)


def tune(row_ptr, col_idx, vals, M: int, K: int, N: int, in_dev: int, out_dev: int, stream: int = 0, *,
         conv: Optional[Tuple[int, int, int]] = None, batch: int = 0, kernel: int = KERNEL_AUTO,
         natural_order: bool = False, ldb: int = 0, ldc: int = 0, tune_warm: bool = False):
    """sparsert_tune: returns (best plan, list of timed candidates as dicts).  `kernel` other
    than KERNEL_AUTO restricts the search to that executor family; tune_warm ranks by
    back-to-back launches instead of launches with displaced caches."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    vals = np.ascontiguousarray(vals)
    if vals.dtype not in _DTYPE_OF:
        raise TypeError("vals must be float32, float16 or int8")
    opt = Options()
    opt.dtype = _DTYPE_OF[vals.dtype]
    opt.kernel, opt.natural_order, opt.batch = kernel, int(natural_order), batch
    opt.ldb, opt.ldc, opt.tune_warm = ldb, ldc, int(tune_warm)
    if conv is not None:
        opt.conv, (opt.Cin, opt.H, opt.W) = 1, conv
    handle, rep = _vp(), TuneReport()
    _check(_lib.sparsert_tune(row_ptr.ctypes.data_as(_vp), col_idx.ctypes.data_as(_vp),
                              vals.ctypes.data_as(_vp), M, K, N, ctypes.byref(opt), in_dev, out_dev,
                              stream, ctypes.byref(handle), ctypes.byref(rep)))
    names = [f[0] for f in TuneEntry._fields_]
    entries = [{n: getattr(rep.entries[i], n) for n in names} for i in range(rep.count)]
    return Plan(handle.value, opt.dtype), entries


def load(blob: bytes, host_only: bool = False) -> Plan:
    """sparsert_plan_load: a plan from bytes written by Plan.save; nothing is analysed or assembled."""
    handle = _vp()
    _check(_lib.sparsert_plan_load(blob, len(blob), int(host_only), ctypes.byref(handle)))
    plan = Plan(handle.value, F32)
    plan.dtype = plan.info()["dtype"]
    return plan


def spmm(plan: Plan, B_dev: int, C_dev: int, stream: int = 0):
    """sparsert_spmm: device addresses and a hipStream_t as integers."""
    _check(_lib.sparsert_spmm(plan.handle, B_dev, C_dev, stream))


def conv3x3(plan: Plan, X_dev: int, Y_dev: int, stream: int = 0):
    """sparsert_conv3x3: device addresses and a hipStream_t as integers."""
    _check(_lib.sparsert_conv3x3(plan.handle, X_dev, Y_dev, stream))


def compare_outputs(plan: Plan, a_dev: int, b_dev: int, result_dev: int, stream: int = 0):
    """sparsert_compare_outputs: result_dev receives four 32-bit words (see the header)."""
    _check(_lib.sparsert_compare_outputs(plan.handle, a_dev, b_dev, result_dev, stream))


def compare_outputs_static(plan: Plan, a_dev: int, b_dev: int, result_dev: int, stream: int = 0):
    """sparsert_compare_outputs_static: the same comparison without any allocation (static scratch, no synchronisation)."""
    _check(_lib.sparsert_compare_outputs_static(plan.handle, a_dev, b_dev, result_dev, stream))


# Raw entry points for callers that time launches without Python argument handling.
raw = _lib
