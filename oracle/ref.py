"""NumPy-facing wrappers of the C oracle (TEST INFRASTRUCTURE ONLY).

Inputs of any storage type (float32, float16) are converted to float64 first,
which is exact, so the oracle consumes exactly the values the HIP path is
given and computes in double precision.
"""
from __future__ import annotations

import ctypes
from typing import Tuple

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        i32, ptr = ctypes.c_int32, ctypes.c_void_p
        lib.oracle_spmm.argtypes = [i32, i32, i32, ptr, ptr, ptr, ptr, ptr, ptr, i32]
        lib.oracle_spmm.restype = None
        lib.oracle_conv3x3.argtypes = [i32, i32, i32, i32, i32, ptr, ptr, ptr, ptr, i32]
        lib.oracle_conv3x3.restype = None
        lib.oracle_im2col3x3.argtypes = [i32, i32, i32, ptr, ptr]
        lib.oracle_im2col3x3.restype = None
        lib.oracle_max_threads.restype = i32
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def spmm(M, K, N, row_ptr, col_idx, vals, B, want_scale=True, threads=0
         ) -> Tuple[np.ndarray, np.ndarray]:
    """C = A*B of Section 3.2 in float64, and the scale S = |A|*|B| (or None)."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    assert row_ptr.shape == (M + 1,) and B.shape == (K, N)
    assert col_idx.shape == vals.shape == (int(row_ptr[-1]),)
    assert col_idx.size == 0 or (col_idx.min() >= 0 and col_idx.max() < K)
    C = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if want_scale else None
    _load().oracle_spmm(M, K, N, _p(row_ptr), _p(col_idx), _p(vals), _p(B), _p(C),
                        _p(S) if want_scale else None, threads)
    return C, S


def conv3x3(Wdense, X, want_scale=True, threads=0) -> Tuple[np.ndarray, np.ndarray]:
    """Direct 3x3 / pad 1 / stride 1 cross-correlation of Section 3.6 in float64."""
    Wd = np.ascontiguousarray(Wdense, dtype=np.float64)
    Xd = np.ascontiguousarray(X, dtype=np.float64)
    Cout, Cin, kh, kw = Wd.shape
    batch, Cin2, H, W = Xd.shape
    assert (kh, kw) == (3, 3) and Cin2 == Cin
    Y = np.empty((batch, Cout, H, W), dtype=np.float64)
    S = np.empty_like(Y) if want_scale else None
    _load().oracle_conv3x3(batch, Cin, Cout, H, W, _p(Wd), _p(Xd), _p(Y),
                           _p(S) if want_scale else None, threads)
    return Y, S


def im2col3x3(X) -> np.ndarray:
    """Explicit im2col matrix [9*Cin, H*W] of a [Cin,H,W] input (cross-check only)."""
    Xd = np.ascontiguousarray(X, dtype=np.float64)
    Cin, H, W = Xd.shape
    Bcol = np.empty((9 * Cin, H * W), dtype=np.float64)
    _load().oracle_im2col3x3(Cin, H, W, _p(Xd), _p(Bcol))
    return Bcol


HALF_STORE_ROUNDING = 2.0 ** -25   # half of the spacing of binary16 below 2^-14


def error_metrics(got, ref, scale, abs_floor=0.0) -> dict:
    """The three error figures the parity gate uses.

    abs_floor: an absolute error every element is allowed before the figures are formed.  Half
    storage passes HALF_STORE_ROUNDING: binary16 has the fixed spacing 2^-24 below 2^-14, so the
    one rounding at the store costs up to 2^-25 whatever the size of the sum, which no bound
    relative to |A|*|B| can express for results that small.

    componentwise: max |got-ref| / S   with S = |A|*|B| (Higham-style bound; the
                   gate), entries with S == 0 must match exactly;
    normwise:      max |got-ref| / max |ref|;
    relative:      max |got-ref| / |ref| over entries with |ref| >= 1e-2 * rms(ref)
                   (below that floor cancellation makes |ref| arbitrarily small and even a
                   correctly rounded fp32 sum exceeds any fixed relative bound);
                   relative_excluded_fraction is the share of entries below the floor.
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.asarray(scale, dtype=np.float64)
    diff = np.maximum(np.abs(got - ref) - abs_floor, 0.0)
    zero = scale == 0.0
    exact_on_zero = bool(np.all(diff[zero] == 0.0)) if zero.any() else True
    comp = float(np.max(diff[~zero] / scale[~zero])) if (~zero).any() else 0.0
    ref_max = float(np.max(np.abs(ref))) if ref.size else 0.0
    normwise = float(np.max(diff) / ref_max) if ref_max > 0 else float(np.max(diff, initial=0.0))
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    big = np.abs(ref) >= 1e-2 * rms
    rel = float(np.max(diff[big] / np.abs(ref[big]))) if (rms > 0 and big.any()) else 0.0
    return {"componentwise": comp, "normwise": normwise, "relative": rel,
            "relative_excluded_fraction": float(1.0 - np.mean(big)) if ref.size else 0.0,
            "exact_on_zero_scale": exact_on_zero}
