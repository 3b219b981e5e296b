"""sparsert_compare_outputs on the GPU against the same figures formed with NumPy on the host."""
import numpy as np
import pytest

from paper_2008_11849_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():  # pragma: no cover
    pytest.skip("no GPU", allow_module_level=True)

from paper_2008_11849_amd import sparsert as sp  # noqa: E402


def expected(a, b, N):
    """The four result words for outputs a, b of shape [.., rows, ld] with N valid columns."""
    a, b = a[..., :N], b[..., :N]
    if a.dtype.kind == "i":
        return 0.0, 0.0, int((a != b).sum())
    a32, b32 = a.astype(np.float32), b.astype(np.float32)
    fa, fb = np.isfinite(a32), np.isfinite(b32)
    both = fa & fb
    dmax = float(np.abs(a32[both] - b32[both]).max()) if both.any() else 0.0
    bmax = float(np.abs(b32[both]).max()) if both.any() else 0.0
    rest = ~both
    bad = (fa != fb) | (np.isnan(a32) != np.isnan(b32)) | (~np.isnan(a32) & (a32 != b32))
    return dmax, bmax, int((bad & rest).sum())


def run(plan, a, b, fn=None):
    dev = torch.device("cuda:0")
    ad, bd = torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)
    res = torch.full((4,), 0x7fffffff, dtype=torch.int32, device=dev)
    (fn or sp.compare_outputs)(plan, ad.data_ptr(), bd.data_ptr(), res.data_ptr(), torch.cuda.current_stream(dev).cuda_stream)
    torch.cuda.synchronize()
    w = res.cpu().numpy().view(np.uint32)
    return float(w[:1].view(np.float32)[0]), float(w[1:2].view(np.float32)[0]), int(w[2]), int(w[3])


CASES = [(np.float32, 70, 130, 130, 1), (np.float32, 300, 1000, 1024, 1), (np.float16, 64, 196, 200, 3), (np.int8, 50, 100, 128, 2),
         (np.float32, 1, 1, 1, 1), (np.float32, 3000, 1024, 1024, 1)]


@pytest.mark.parametrize("dtype,M,N,ldc,batch", CASES)
def test_compare_outputs_matches_numpy(dtype, M, N, ldc, batch):
    csr = synth.int8_csr(M, 40, 0.8, 1) if dtype == np.int8 else synth.uniform_csr(M, 40, 0.8, 1, dtype=dtype)
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, M, 40, N, ldc=ldc, batch=batch, kernel=sp.KERNEL_ROWS)
    rng = np.random.default_rng(M + N)
    out_dt = np.int32 if dtype == np.int8 else dtype
    shape = (batch, M, ldc)
    if dtype == np.int8:
        a = rng.integers(-1000, 1000, size=shape).astype(np.int32)
    else:
        a = rng.standard_normal(shape).astype(out_dt)
    assert run(plan, a, a.copy())[:3] == (0.0, float(np.abs(a[..., :N].astype(np.float32)).max()) if dtype != np.int8 else 0.0, 0)
    b = a.copy()
    # differences in the valid columns: small ones, one large one, and special values
    idx = rng.choice(batch * M * N, size=min(40, batch * M * N), replace=False)
    bi, mi, ni = np.unravel_index(idx, (batch, M, N))
    if dtype == np.int8:
        b[bi, mi, ni] += 1
    else:
        b[bi, mi, ni] += (rng.standard_normal(len(idx)) * 1e-3).astype(out_dt)
        b[bi[0], mi[0], ni[0]] = out_dt(7.5)
        if len(idx) > 4:
            b[bi[1], mi[1], ni[1]] = np.nan
            a[bi[2], mi[2], ni[2]] = np.inf
            a[bi[3], mi[3], ni[3]] = b[bi[3], mi[3], ni[3]] = np.nan      # NaN in both: same kind
    if ldc > N:   # the padding columns are no part of a result
        b[..., N:] = 99
    got = run(plan, a, b)
    want = expected(a, b, N)
    assert got[:3] == want, (got, want)
    assert got[3] == -(-(batch * M * N) // 16384)
    plan.destroy()


def test_compare_outputs_argument_errors():
    csr = synth.uniform_csr(8, 8, 0.5, 1)
    host = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 8, 8, 8, host_only=True)
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 8, 8, 8)
    t = torch.zeros(64, device="cuda:0")
    r = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    for args in ((host, t.data_ptr(), t.data_ptr(), r.data_ptr()), (plan, 0, t.data_ptr(), r.data_ptr()),
                 (plan, t.data_ptr(), t.data_ptr(), 0), (plan, t.data_ptr() + 4, t.data_ptr(), r.data_ptr())):
        with pytest.raises(sp.SparseRTError) as e:
            sp.compare_outputs(*args)
        assert e.value.status == sp.EINVAL
