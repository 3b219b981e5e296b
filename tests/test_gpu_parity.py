"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerances: max relative error 1e-4 (fp32) and 2e-2 (fp16 storage, fp32 accumulation),
measured three ways (see oracle.ref.error_metrics).  Integer-valued inputs must match
bit for bit under any summation order.
"""
import numpy as np
import pytest

from oracle import ref
from paper_2008_11849_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():  # pragma: no cover
    pytest.skip("no GPU", allow_module_level=True)

from gpu_util import check, run_conv, run_spmm  # noqa: E402
from paper_2008_11849_amd import sparsert as sp  # noqa: E402

# Every case runs with the always-available row-walk kernel and with what the inspector picks
# when the caller leaves the choice to it (the generated kernel for these sizes).
FAMILIES = [pytest.param(sp.KERNEL_ROWS, id="rows"), pytest.param(sp.KERNEL_AUTO, id="auto")]


def _oracle(csr, B):
    return ref.spmm(csr.M, csr.K, B.shape[1], csr.row_ptr, csr.col_idx, csr.vals, B)


@pytest.mark.parametrize("family", FAMILIES)
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c3t"])
def test_spmm_configs(name, dtype, family):
    case = synth.config(name, dtype)
    got, info = run_spmm(case.csr, case.B, kernel=family)
    assert info["kernel"] == (sp.KERNEL_ROWS if family == sp.KERNEL_ROWS else sp.KERNEL_SPEC)
    Cref, S = _oracle(case.csr, case.B)
    m = check(got, Cref, S, dtype, gate_relative=True)
    print(name, np.dtype(dtype).name, info, m)


@pytest.mark.parametrize("family", FAMILIES)
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_conv_config_c4(dtype, family):
    case = synth.config("c4", dtype)
    got, info = run_conv(case.csr, case.X, 256, kernel=family)
    Yref, S = ref.conv3x3(case.Wdense, case.X)
    m = check(got, Yref, S, dtype, gate_relative=True)
    print("c4", np.dtype(dtype).name, info, m)


EDGE_N = [1, 2, 3, 4, 49, 63, 64, 65, 100, 196, 255, 256, 257, 784]


@pytest.mark.parametrize("N", EDGE_N)
def test_small_integers_are_bit_exact_any_order(N):
    # |sum| stays far below 2^24: every order of summation gives the same bits
    csr = synth.small_int_csr(77, 130, 0.85, N)
    B = synth.small_int_dense(130, N, N + 1)
    Cref, _ = _oracle(csr, B)
    for opts in ({}, {"kernel": sp.KERNEL_ROWS}, {"vec": 1}, {"split_threshold": 1}, {"split_threshold": 7, "vec": 1}):
        if opts and "vec" not in opts and N % 2 == 0:
            for v in (2, 4):
                if N % v == 0:
                    got, _ = run_spmm(csr, B, vec=v, **opts)
                    assert np.array_equal(got.astype(np.float64), Cref), (N, v, opts)
        got, _ = run_spmm(csr, B, **opts)
        assert np.array_equal(got.astype(np.float64), Cref), (N, opts)


@pytest.mark.parametrize("N", [8, 64, 200, 520])
def test_small_integers_half(N):
    csr = synth.small_int_csr(50, 90, 0.9, N, dtype=np.float16, vmax=3)
    B = synth.small_int_dense(90, N, N + 1, dtype=np.float16, bmax=4)
    Cref, _ = _oracle(csr, B)
    assert np.abs(Cref).max() <= 2048
    for opts in ({}, {"kernel": sp.KERNEL_ROWS}, {"vec": 1}, {"vec": 8, "split_threshold": 2}, {"vec": 2}):
        got, _ = run_spmm(csr, B, **opts)
        assert np.array_equal(got.astype(np.float64), Cref), (N, opts)


def test_identity_and_permutation_return_B_bit_for_bit():
    K, N = 300, 196
    B = synth.normal_dense(K, N, 3)
    eye = synth.csr_from_mask(np.eye(K, dtype=np.float32), np.eye(K, dtype=bool))
    perm = np.random.default_rng(0).permutation(K)
    P = np.zeros((K, K), dtype=np.float32)
    P[np.arange(K), perm] = 1.0
    for family in (sp.KERNEL_ROWS, sp.KERNEL_AUTO):
        got, _ = run_spmm(eye, B, kernel=family)
        assert got.tobytes() == B.tobytes()
        got, _ = run_spmm(synth.csr_from_mask(P, P != 0), B, kernel=family)
        assert got.tobytes() == B[perm].tobytes()


def test_empty_rows_empty_matrix_and_dense_row():
    M, K, N = 40, 64, 130
    A = np.zeros((M, K), dtype=np.float32)
    A[5] = np.arange(1, K + 1)          # one dense row
    A[17, 3] = -2.0                     # one single-nonzero row; all others empty
    csr = synth.csr_from_mask(A, A != 0)
    B = synth.small_int_dense(K, N, 9)
    Cref, _ = _oracle(csr, B)
    for family in (sp.KERNEL_ROWS, sp.KERNEL_AUTO):
        got, info = run_spmm(csr, B, kernel=family)
        assert np.array_equal(got.astype(np.float64), Cref)
        assert not np.signbit(got[0]).any()  # empty row: +0.0
    for thr in (1, 16):
        got, _ = run_spmm(csr, B, split_threshold=thr)
        assert np.array_equal(got.astype(np.float64), Cref)
    empty = synth.csr_from_mask(np.zeros((M, K), np.float32), np.zeros((M, K), bool))
    for family in (sp.KERNEL_ROWS, sp.KERNEL_AUTO):
        got, _ = run_spmm(empty, B, kernel=family)
        assert np.array_equal(got, np.zeros((M, N), np.float32)) and not np.signbit(got).any()


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_skewed_rows_at_98_percent(dtype):
    csr = synth.skewed_csr(512, 2048, 0.98, 13, dtype=dtype)
    assert (np.diff(csr.row_ptr) == 0).any()
    B = synth.normal_dense(2048, 784, 14, dtype=dtype)
    Cref, S = _oracle(csr, B)
    for family in (sp.KERNEL_ROWS, sp.KERNEL_AUTO):
        got, info = run_spmm(csr, B, kernel=family)
        assert info["n_split"] > 0
        check(got, Cref, S, dtype)


def test_run_to_run_determinism_and_two_streams():
    import torch
    from paper_2008_11849_amd import sparsert as sp
    case = synth.config("c2")
    csr = case.csr
    a, _ = run_spmm(csr, case.B, split_threshold=8)
    b, _ = run_spmm(csr, case.B, split_threshold=8)
    assert a.tobytes() == b.tobytes()
    dev = torch.device("cuda:0")
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N)
    Bd = torch.from_numpy(case.B).to(dev)
    s1, s2 = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
    C1 = torch.empty((csr.M, case.N), device=dev)
    C2 = torch.empty((csr.M, case.N), device=dev)
    torch.cuda.synchronize()
    for _ in range(5):
        sp.spmm(plan, Bd.data_ptr(), C1.data_ptr(), s1.cuda_stream)
        sp.spmm(plan, Bd.data_ptr(), C2.data_ptr(), s2.cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(C1, C2)
    plan.destroy()


CONV_SHAPES = [(3, 5, 1, 1), (4, 6, 2, 3), (8, 8, 7, 7), (16, 24, 14, 14), (6, 10, 9, 13),
               (64, 64, 56, 56), (128, 128, 28, 28), (512, 512, 7, 7)]


@pytest.mark.parametrize("Cin,Cout,H,W", CONV_SHAPES)
def test_conv_shapes(Cin, Cout, H, W):
    for dtype, sparsity in ((np.float32, 0.9), (np.float16, 0.95)):
        csr, Wd = synth.conv_weights_csr(Cout, Cin, sparsity, Cin + H, dtype=dtype)
        X = synth.normal_dense(Cin, H * W, Cout + W, dtype=dtype).reshape(1, Cin, H, W)
        Yref, S = ref.conv3x3(Wd, X)
        for family in (sp.KERNEL_ROWS, sp.KERNEL_AUTO):
            got, _ = run_conv(csr, X, Cout, kernel=family)
            check(got, Yref, S, dtype)


def test_conv_integer_taps_bit_exact():
    Cin, Cout, H, W = 7, 9, 11, 6
    rng = np.random.default_rng(4)
    Wd = (rng.integers(-3, 4, size=(Cout, Cin, 3, 3)) * (rng.random((Cout, Cin, 3, 3)) < 0.3)).astype(np.float32)
    X = rng.integers(-5, 6, size=(1, Cin, H, W)).astype(np.float32)
    csr = synth.csr_from_mask(Wd.reshape(Cout, -1), Wd.reshape(Cout, -1) != 0)
    Yref, _ = ref.conv3x3(Wd, X)
    for opts in ({}, {"kernel": sp.KERNEL_ROWS}, {"split_threshold": 1}, {"split_threshold": 5}):
        got, _ = run_conv(csr, X, Cout, **opts)
        assert np.array_equal(got.astype(np.float64), Yref)
    # one tap at a time: a zero-filled shift of the input, bit for bit
    for t in range(9):
        W1 = np.zeros((1, 1, 3, 3), dtype=np.float32)
        W1[0, 0, t // 3, t % 3] = 1.0
        X1 = synth.normal_dense(1, H * W, t).reshape(1, 1, H, W)
        Yr, _ = ref.conv3x3(W1, X1)
        for family in (sp.KERNEL_ROWS, sp.KERNEL_AUTO):
            got, _ = run_conv(synth.csr_from_mask(W1.reshape(1, 9), W1.reshape(1, 9) != 0), X1, 1, kernel=family)
            assert np.array_equal(got.astype(np.float64), Yr)


SWEEP = [(256, 256, 64, 0.8, "uniform"), (1024, 512, 196, 0.9, "magnitude"),
         (512, 1024, 784, 0.95, "skewed"), (2048, 2048, 64, 0.98, "skewed"),
         (256, 4096, 196, 0.8, "uniform")]


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("M,K,N,s,kind", SWEEP)
def test_sweep_subset_full_check(M, K, N, s, kind, dtype):
    case = synth.sweep_case(M, K, N, s, kind, dtype)
    Cref, S = _oracle(case.csr, case.B)
    for family in (sp.KERNEL_ROWS, sp.KERNEL_AUTO):
        got, _ = run_spmm(case.csr, case.B, kernel=family)
        check(got, Cref, S, dtype)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_largest_sweep_shape_on_sampled_rows(dtype):
    # 4096 x 4096 x 4096 at 80 %: the oracle computes a sample of rows one by one
    case = synth.sweep_case(4096, 4096, 4096, 0.8, "uniform", dtype)
    got, info = run_spmm(case.csr, case.B)
    assert not np.isnan(got).any()
    rows = np.random.default_rng(1).choice(4096, size=48, replace=False)
    rp = case.csr.row_ptr
    sub_ptr = np.zeros(len(rows) + 1, dtype=np.int32)
    cols, vals = [], []
    for i, r in enumerate(rows):
        cols.append(case.csr.col_idx[rp[r]:rp[r + 1]])
        vals.append(case.csr.vals[rp[r]:rp[r + 1]])
        sub_ptr[i + 1] = sub_ptr[i] + (rp[r + 1] - rp[r])
    Cref, S = ref.spmm(len(rows), 4096, 4096, sub_ptr, np.concatenate(cols), np.concatenate(vals), case.B)
    check(got[rows], Cref, S, dtype)
