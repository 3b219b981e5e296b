"""GPU parity of the per-matrix generated kernel (values of A as instruction constants,
Section 3.5) against the CPU oracle, through the same C-ABI calls as the row-walk path."""
import numpy as np
import pytest

from oracle import ref
from paper_2008_11849_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():  # pragma: no cover
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import check, run_spmm  # noqa: E402
from paper_2008_11849_amd import sparsert as sp  # noqa: E402


def _oracle(csr, B):
    return ref.spmm(csr.M, csr.K, B.shape[1], csr.row_ptr, csr.col_idx, csr.vals, B)


@pytest.mark.parametrize("N", [1, 3, 49, 63, 64, 65, 196, 256, 300])
@pytest.mark.parametrize("rows", [0, 1, 5, 64])
def test_spec_small_integers_bit_exact(N, rows):
    csr = synth.small_int_csr(77, 130, 0.85, N)
    B = synth.small_int_dense(130, N, N + 1)
    Cref, _ = _oracle(csr, B)
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_rows=rows)
    assert info["kernel"] == sp.KERNEL_SPEC and info["spec_code_bytes"] > 0
    assert np.array_equal(got.astype(np.float64), Cref), (N, rows)


def test_spec_empty_rows_dense_row_and_empty_matrix():
    M, K, N = 40, 64, 130
    A = np.zeros((M, K), dtype=np.float32)
    A[5] = np.arange(1, K + 1)
    A[17, 3] = -2.0
    csr = synth.csr_from_mask(A, A != 0)
    B = synth.small_int_dense(K, N, 9)
    got, _ = run_spmm(csr, B, kernel=sp.KERNEL_SPEC)
    Cref, _ = _oracle(csr, B)
    assert np.array_equal(got.astype(np.float64), Cref)
    assert not np.signbit(got[0]).any()
    empty = synth.csr_from_mask(np.zeros((M, K), np.float32), np.zeros((M, K), bool))
    got, _ = run_spmm(empty, B, kernel=sp.KERNEL_SPEC)
    assert np.array_equal(got, np.zeros((M, N), np.float32)) and not np.signbit(got).any()


def test_spec_identity_returns_B():
    K, N = 300, 196
    B = synth.normal_dense(K, N, 3)
    eye = synth.csr_from_mask(np.eye(K, dtype=np.float32), np.eye(K, dtype=bool))
    got, _ = run_spmm(eye, B, kernel=sp.KERNEL_SPEC)
    assert got.tobytes() == B.tobytes()


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c3t"])
def test_spec_configs(name):
    case = synth.config(name)
    got, info = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC)
    Cref, S = _oracle(case.csr, case.B)
    m = check(got, Cref, S, np.float32, gate_relative=True)
    print(name, info, m)


@pytest.mark.parametrize("M,K,N,s,kind", [(512, 1024, 784, 0.95, "skewed"), (1024, 512, 196, 0.9, "magnitude"),
                                         (256, 4096, 196, 0.8, "uniform"), (2048, 2048, 64, 0.98, "skewed")])
def test_spec_sweep_subset(M, K, N, s, kind):
    case = synth.sweep_case(M, K, N, s, kind, np.float32)
    got, _ = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC)
    Cref, S = _oracle(case.csr, case.B)
    check(got, Cref, S, np.float32)


def test_spec_rejects_what_it_does_not_cover():
    csr = synth.uniform_csr(16, 18, 0.5, 1, dtype=np.float16)
    with pytest.raises(sp.SparseRTError) as e:
        sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 16, 18, 8, kernel=sp.KERNEL_SPEC, host_only=True)
    assert e.value.status == sp.EUNSUPPORTED
