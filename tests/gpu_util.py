"""Helpers for the GPU parity tests: device buffers through torch, calls through the C ABI."""
import numpy as np
import torch

from oracle import ref
from paper_2008_11849_amd import sparsert as sp

TOL = {np.dtype(np.float32): 1e-4, np.dtype(np.float16): 2e-2}


def _tdtype(dt):
    return {np.dtype(np.float16): torch.float16, np.dtype(np.int8): torch.int8}.get(np.dtype(dt), torch.float32)


def _poisoned(shape, in_dtype, dev):
    """Output buffer pre-filled with a value no correct result has: NaN, or for int8 plans
    (int32 output) an integer beyond any reachable sum."""
    if np.dtype(in_dtype) == np.int8:
        return torch.full(shape, -(2 ** 31) + 12345, dtype=torch.int32, device=dev)
    return torch.full(shape, float("nan"), dtype=_tdtype(in_dtype), device=dev)


def run_spmm(csr, B, **opts):
    """B is [K, N], or [batch, K, N] for a batched plan."""
    dev = torch.device("cuda:0")
    if B.ndim == 3:
        opts = dict(opts, batch=B.shape[0])
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, B.shape[-1], **opts)
    Bd = torch.from_numpy(np.ascontiguousarray(B)).to(dev)
    # poison the output so unwritten elements are caught
    Cd = _poisoned(B.shape[:-2] + (csr.M, B.shape[-1]), B.dtype, dev)
    sp.spmm(plan, Bd.data_ptr(), Cd.data_ptr(), torch.cuda.current_stream(dev).cuda_stream)
    torch.cuda.synchronize()
    out = Cd.cpu().numpy()
    info = plan.info()
    plan.destroy()
    return out, info


def run_spmm_strided(csr, B, ldb, ldc, **opts):
    """B [K, N] (or [batch, K, N]) handed over at a row pitch of ldb elements, C received at a
    pitch of ldc.  The unused columns of the operand hold NaN (or a large integer) and those of
    the result a poison value: returns (C [.., M, N], whether the poison columns of the result
    buffer are untouched, plan info)."""
    dev = torch.device("cuda:0")
    N = B.shape[-1]
    lead = B.shape[:-2]
    if B.ndim == 3:
        opts = dict(opts, batch=B.shape[0])
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, N, ldb=ldb, ldc=ldc, **opts)
    wide = np.full(lead + (csr.K, ldb), 100 if B.dtype == np.int8 else np.nan, dtype=B.dtype)
    wide[..., :N] = B
    Bd = torch.from_numpy(wide).to(dev)
    Cd = _poisoned(lead + (csr.M, ldc), B.dtype, dev)
    before = Cd.clone()
    sp.spmm(plan, Bd.data_ptr(), Cd.data_ptr(), torch.cuda.current_stream(dev).cuda_stream)
    torch.cuda.synchronize()
    # the poison of the floating types is NaN, which equals nothing: compare the bytes
    pad_ok = Cd[..., N:].contiguous().cpu().numpy().tobytes() == before[..., N:].contiguous().cpu().numpy().tobytes()
    out = Cd[..., :N].contiguous().cpu().numpy()
    info = plan.info()
    plan.destroy()
    return out, pad_ok, info


def run_conv(csr, X, Cout, **opts):
    dev = torch.device("cuda:0")
    batch, Cin, H, W = X.shape
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, Cout, 9 * Cin, H * W,
                      conv=(Cin, H, W), batch=batch, **opts)
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to(dev)
    Yd = _poisoned((batch, Cout, H, W), X.dtype, dev)
    sp.conv3x3(plan, Xd.data_ptr(), Yd.data_ptr(), torch.cuda.current_stream(dev).cuda_stream)
    torch.cuda.synchronize()
    out = Yd.cpu().numpy()
    info = plan.info()
    plan.destroy()
    return out, info


def check(got, ref_c, scale, dtype, gate_relative=False):
    """Error figures must be under the tolerance of the storage type: max relative error
    1e-4 for fp32, 2e-2 for fp16 (fp32 accumulation).  The componentwise and normwise
    figures gate every case; the plain element-wise relative error (entries above 1e-2 rms)
    gates the named configurations only, since with several hundred terms per output even a
    correctly rounded sequential fp32 sum reaches 1e-4 on entries that nearly cancel."""
    tol = TOL[np.dtype(dtype)]
    assert not np.isnan(got).any(), "unwritten or NaN outputs"
    # half results: the rounding at the store has an absolute part (binary16 spacing near zero)
    m = ref.error_metrics(got, ref_c, scale, ref.HALF_STORE_ROUNDING if np.dtype(dtype) == np.float16 else 0.0)
    assert m["exact_on_zero_scale"], m
    assert m["componentwise"] <= tol, m
    assert m["normwise"] <= tol, m
    if gate_relative:
        assert m["relative"] <= tol, m
    return m
