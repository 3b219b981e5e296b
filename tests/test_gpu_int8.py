"""GPU parity of int8 plans (int8 weights and activations, exact int32 sums) against the CPU
oracle: integer work, so every output must match bit for bit."""
import numpy as np
import pytest

from oracle import ref
from paper_2008_11849_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():  # pragma: no cover
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import run_conv, run_spmm  # noqa: E402
from paper_2008_11849_amd import sparsert as sp  # noqa: E402

POISON = -(2 ** 31) + 12345


def _want(csr, B):
    C, _ = ref.spmm(csr.M, csr.K, B.shape[1], csr.row_ptr, csr.col_idx, csr.vals, B, want_scale=False)
    assert np.abs(C).max() < 2 ** 31
    return C.astype(np.int64)


@pytest.mark.parametrize("N", [1, 3, 4, 64, 100, 196, 260, 1024])
def test_int8_spmm_is_exact(N):
    csr = synth.int8_csr(77, 130, 0.85, N)
    B = synth.int8_dense(130, N, N + 1)
    want = _want(csr, B)
    variants = [dict(), dict(vec=1), dict(vec=1, split_threshold=1), dict(split_threshold=7),
                dict(kernel=sp.KERNEL_SPEC, spec_rows=1), dict(kernel=sp.KERNEL_SPEC, spec_rows=9),
                dict(kernel=sp.KERNEL_SPEC, spec_rows=20, spec_ksplit=4, spec_swizzle=True),
                dict(kernel=sp.KERNEL_SPEC, spec_rows=77, spec_ksplit=8, spec_depth=3)]
    if N % 4 == 0:
        variants += [dict(vec=4), dict(vec=4, split_threshold=1), dict(vec=4, split_threshold=9),
                     dict(kernel=sp.KERNEL_SPEC, spec_vec=4, spec_rows=1), dict(kernel=sp.KERNEL_SPEC, spec_vec=4, spec_rows=9),
                     dict(kernel=sp.KERNEL_SPEC, spec_vec=4, spec_rows=20, spec_ksplit=4, spec_swizzle=True),
                     dict(kernel=sp.KERNEL_SPEC, spec_vec=4, spec_rows=48, spec_ksplit=8, spec_depth=3)]
    for opts in variants:
        got, info = run_spmm(csr, B, **opts)
        assert got.dtype == np.int32 and info["dtype"] == sp.I8
        assert not (got == POISON).any(), "unwritten outputs"
        assert np.array_equal(got.astype(np.int64), want), (N, opts)


def test_int8_extreme_values_and_empty_rows():
    K = 3000
    vals = np.full((3, K), -128, dtype=np.int8)
    mask = np.ones((3, K), dtype=bool)
    mask[1] = False                                     # an empty row gives 0
    csr = synth.csr_from_mask(vals, mask)
    B = np.full((K, 68), -128, dtype=np.int8)
    B[:, 1] = 127
    for opts in (dict(vec=1), dict(vec=4), dict(vec=4, split_threshold=100), dict(kernel=sp.KERNEL_SPEC, spec_rows=3),
                 dict(kernel=sp.KERNEL_SPEC, spec_rows=3, spec_ksplit=8), dict(kernel=sp.KERNEL_SPEC, spec_rows=3, spec_vec=4),
                 dict(kernel=sp.KERNEL_SPEC, spec_rows=3, spec_vec=4, spec_ksplit=8)):
        got, _ = run_spmm(csr, B, **opts)
        assert np.all(got[1] == 0)
        assert np.all(got[0, 0] == K * 16384) and np.all(got[2, 1] == -K * 128 * 127)
        assert np.array_equal(got.astype(np.int64), _want(csr, B))


@pytest.mark.parametrize("M,K,N,s", [(256, 512, 196, 0.95), (512, 1024, 784, 0.9), (1024, 256, 64, 0.8)])
def test_int8_skewed_rows(M, K, N, s):
    """Zipf-like row lengths (long rows are split over waves, many rows are empty)."""
    f = synth.skewed_csr(M, K, s, 17)
    q = np.clip(np.rint(f.vals / np.abs(f.vals).max() * 127.0), -127, 127).astype(np.int8)
    q[q == 0] = 1
    csr = synth.CSR(M, K, f.row_ptr, f.col_idx, q)
    B = synth.int8_dense(K, N, 18)
    for opts in (dict(), dict(kernel=sp.KERNEL_SPEC, spec_rows=16, spec_ksplit=4)):
        got, info = run_spmm(csr, B, **opts)
        assert np.array_equal(got.astype(np.int64), _want(csr, B)), info


@pytest.mark.parametrize("Cin,Cout,H,W,batch", [(3, 5, 1, 1, 1), (4, 6, 2, 3, 2), (2, 3, 9, 1, 1), (16, 24, 14, 14, 3),
                                                (64, 64, 28, 28, 1)])
def test_int8_conv_is_exact(Cin, Cout, H, W, batch):
    rng = np.random.default_rng(Cin * 100 + H)
    Wd = (rng.integers(-128, 128, size=(Cout, Cin, 3, 3)) * (rng.random((Cout, Cin, 3, 3)) < 0.2)).astype(np.int8)
    csr = synth.csr_from_mask(Wd.reshape(Cout, -1), Wd.reshape(Cout, -1) != 0)
    X = rng.integers(-128, 128, size=(batch, Cin, H, W)).astype(np.int8)
    want = ref.conv3x3(Wd, X, want_scale=False)[0].astype(np.int64)
    for opts in (dict(), dict(split_threshold=1), dict(kernel=sp.KERNEL_SPEC, spec_rows=3),
                 dict(kernel=sp.KERNEL_SPEC, spec_rows=4, spec_ksplit=2)):
        got, info = run_conv(csr, X, Cout, **opts)
        assert got.dtype == np.int32 and info["batch"] == batch
        assert np.array_equal(got.astype(np.int64), want), opts


def test_int8_batched_spmm_and_tune():
    csr = synth.int8_csr(300, 256, 0.9, 5)
    B = np.stack([synth.int8_dense(256, 512, 6 + i) for i in range(2)])
    want = np.stack([_want(csr, B[i]) for i in range(2)])
    for opts in (dict(), dict(kernel=sp.KERNEL_SPEC, spec_rows=24, spec_ksplit=4),
                 dict(kernel=sp.KERNEL_SPEC, spec_rows=24, spec_ksplit=4, spec_vec=4)):
        got, info = run_spmm(csr, B, **opts)
        assert info["batch"] == 2 and np.array_equal(got.astype(np.int64), want)
    dev = torch.device("cuda:0")
    Bd = torch.from_numpy(B[0]).to(dev)
    Cd = torch.zeros((300, 512), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    plan, report = sp.tune(csr.row_ptr, csr.col_idx, csr.vals, 300, 256, 512, Bd.data_ptr(), Cd.data_ptr(), stream)
    assert len(report) >= 4 and {r["kernel"] for r in report} == {sp.KERNEL_ROWS, sp.KERNEL_SPEC}
    Cd.fill_(POISON)
    sp.spmm(plan, Bd.data_ptr(), Cd.data_ptr(), stream)
    torch.cuda.synchronize()
    assert np.array_equal(Cd.cpu().numpy().astype(np.int64), want[0])
    plan.destroy()
