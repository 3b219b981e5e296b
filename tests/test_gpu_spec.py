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

from gpu_util import check, run_conv, run_spmm  # noqa: E402
from paper_2008_11849_amd import sparsert as sp  # noqa: E402


def _oracle(csr, B):
    return ref.spmm(csr.M, csr.K, B.shape[1], csr.row_ptr, csr.col_idx, csr.vals, B)


MODES = [sp.SPEC_DIRECT, sp.SPEC_LDS]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("N", [1, 3, 49, 63, 64, 65, 196, 256, 300])
@pytest.mark.parametrize("rows", [0, 1, 5, 64])
def test_spec_small_integers_bit_exact(N, rows, mode):
    csr = synth.small_int_csr(77, 130, 0.85, N)
    B = synth.small_int_dense(130, N, N + 1)
    Cref, _ = _oracle(csr, B)
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_rows=rows, spec_mode=mode)
    assert info["kernel"] == sp.KERNEL_SPEC and info["spec_code_bytes"] > 0 and info["spec_mode"] == mode
    assert np.array_equal(got.astype(np.float64), Cref), (N, rows)


@pytest.mark.parametrize("K", [1, 4, 127, 128, 129, 255, 257, 300, 515])
@pytest.mark.parametrize("waves", [1, 2, 8, 16])
def test_spec_lds_chunk_edges_and_wave_counts(K, waves):
    # K around the 128-row staging chunk, with every workgroup width
    csr = synth.small_int_csr(37, K, 0.5 if K < 16 else 0.9, K + waves)
    B = synth.small_int_dense(K, 70, K)
    Cref, _ = _oracle(csr, B)
    got, _ = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_mode=sp.SPEC_LDS, spec_rows=3, spec_tiles=waves)
    assert np.array_equal(got.astype(np.float64), Cref), (K, waves)
    got, _ = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_mode=sp.SPEC_DIRECT, spec_rows=3, spec_tiles=waves)
    assert np.array_equal(got.astype(np.float64), Cref), (K, waves)


@pytest.mark.parametrize("mode", MODES)
def test_spec_empty_rows_dense_row_and_empty_matrix(mode):
    M, K, N = 40, 64, 130
    A = np.zeros((M, K), dtype=np.float32)
    A[5] = np.arange(1, K + 1)
    A[17, 3] = -2.0
    csr = synth.csr_from_mask(A, A != 0)
    B = synth.small_int_dense(K, N, 9)
    got, _ = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_mode=mode)
    Cref, _ = _oracle(csr, B)
    assert np.array_equal(got.astype(np.float64), Cref)
    assert not np.signbit(got[0]).any()
    empty = synth.csr_from_mask(np.zeros((M, K), np.float32), np.zeros((M, K), bool))
    got, _ = run_spmm(empty, B, kernel=sp.KERNEL_SPEC, spec_mode=mode)
    assert np.array_equal(got, np.zeros((M, N), np.float32)) and not np.signbit(got).any()


@pytest.mark.parametrize("mode", MODES)
def test_spec_identity_returns_B(mode):
    K, N = 300, 196
    B = synth.normal_dense(K, N, 3)
    eye = synth.csr_from_mask(np.eye(K, dtype=np.float32), np.eye(K, dtype=bool))
    got, _ = run_spmm(eye, B, kernel=sp.KERNEL_SPEC, spec_mode=mode)
    assert got.tobytes() == B.tobytes()


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c3t"])
def test_spec_configs(name, mode):
    case = synth.config(name)
    got, info = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_mode=mode)
    Cref, S = _oracle(case.csr, case.B)
    m = check(got, Cref, S, np.float32, gate_relative=True)
    print(name, info, m)


@pytest.mark.parametrize("M,K,N,s,kind", [(512, 1024, 784, 0.95, "skewed"), (1024, 512, 196, 0.9, "magnitude"),
                                         (256, 4096, 196, 0.8, "uniform"), (2048, 2048, 64, 0.98, "skewed")])
@pytest.mark.parametrize("mode", MODES)
def test_spec_sweep_subset(M, K, N, s, kind, mode):
    case = synth.sweep_case(M, K, N, s, kind, np.float32)
    got, _ = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_mode=mode)
    Cref, S = _oracle(case.csr, case.B)
    check(got, Cref, S, np.float32)


@pytest.mark.parametrize("ks", [2, 4, 8])
@pytest.mark.parametrize("N", [1, 65, 196, 300])
def test_spec_ksplit_small_integers_bit_exact(N, ks):
    csr = synth.small_int_csr(77, 130, 0.85, N)
    B = synth.small_int_dense(130, N, N + 1)
    Cref, _ = _oracle(csr, B)
    for rows in (0, 1, 7, 36, 77):   # 77 rows x 8 waves: the exchange area spans three 64 KiB windows
        got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_rows=rows, spec_ksplit=ks)
        assert info["spec_ksplit"] == ks and info["spec_tiles"] == ks
        assert np.array_equal(got.astype(np.float64), Cref), (N, rows, ks)


@pytest.mark.parametrize("depth", [1, 2, 3, 5, 48])
def test_spec_depth_small_integers_bit_exact(depth):
    csr = synth.small_int_csr(40, 90, 0.8, depth)
    B = synth.small_int_dense(90, 100, depth + 1)
    Cref, _ = _oracle(csr, B)
    for ks in (0, 2):
        got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_rows=9, spec_depth=depth, spec_ksplit=ks)
        assert info["spec_depth"] == depth
        assert np.array_equal(got.astype(np.float64), Cref), (depth, ks)


def test_spec_ksplit_largest_block():
    csr = synth.small_int_csr(200, 96, 0.9, 5)
    B = synth.small_int_dense(96, 130, 6)
    Cref, _ = _oracle(csr, B)
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_rows=200, spec_ksplit=4, spec_depth=24)
    assert info["spec_lds_bytes"] == 3 * 200 * 256
    assert np.array_equal(got.astype(np.float64), Cref)
    # 7 x 200 rows of partial sums do not fit the LDS at once: exchanged in phases of 91 rows
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_rows=200, spec_ksplit=8)
    assert info["spec_lds_bytes"] == 7 * 91 * 256
    assert np.array_equal(got.astype(np.float64), Cref)
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_rows=130, spec_ksplit=8, spec_swizzle=True)
    assert np.array_equal(got.astype(np.float64), Cref)


@pytest.mark.parametrize("name,opts", [("c3", dict(spec_rows=96, spec_ksplit=4)),
                                       ("c3", dict(spec_rows=96, spec_ksplit=4, spec_swizzle=True)),
                                       ("c3t", dict(spec_rows=48, spec_ksplit=8)),
                                       ("c3t", dict(spec_rows=48, spec_ksplit=8, spec_swizzle=True))])
def test_headline_layers_in_the_plans_the_tuner_picks(name, opts):
    """Full-size c3 / c3t in the launch configurations the benchmark ends up timing."""
    case = synth.config(name)
    got, info = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, **opts)
    assert info["spec_ksplit"] == opts["spec_ksplit"] and info["spec_rows"] == opts["spec_rows"]
    Cref, S = _oracle(case.csr, case.B)
    check(got, Cref, S, np.float32, gate_relative=True)


def test_spec_ksplit_configs_and_skew():
    for name in ("c2", "c3t"):
        case = synth.config(name)
        got, info = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_rows=48, spec_ksplit=4)
        Cref, S = _oracle(case.csr, case.B)
        check(got, Cref, S, np.float32, gate_relative=True)
    case = synth.sweep_case(512, 1024, 784, 0.95, "skewed", np.float32)  # empty rows, empty K parts
    got, _ = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_rows=16, spec_ksplit=8)
    Cref, S = _oracle(case.csr, case.B)
    check(got, Cref, S, np.float32)


@pytest.mark.parametrize("lanes", [16, 32, 64])
@pytest.mark.parametrize("N", [1, 17, 65, 196, 300])
def test_spec_narrow_tiles_small_integers_bit_exact(N, lanes):
    csr = synth.small_int_csr(77, 130, 0.85, N + lanes)
    B = synth.small_int_dense(130, N, N + 1)
    Cref, _ = _oracle(csr, B)
    for opts in (dict(spec_rows=7), dict(spec_rows=20, spec_ksplit=4), dict(spec_rows=77, spec_ksplit=8)):
        got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_lanes=lanes, **opts)
        assert 1 <= info["spec_lanes"] <= lanes and info["n_tiles"] >= 1
        assert np.array_equal(got.astype(np.float64), Cref), (N, lanes, opts)


def test_spec_narrow_tiles_config_and_conv():
    case = synth.config("c2")
    Cref, S = _oracle(case.csr, case.B)
    for lanes in (16, 32):
        got, info = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_rows=16, spec_ksplit=2, spec_lanes=lanes)
        check(got, Cref, S, np.float32, gate_relative=True)
    csr, Wd = synth.conv_weights_csr(24, 16, 0.8, 5)
    X = synth.normal_dense(16, 9 * 13, 6).reshape(1, 16, 9, 13)
    Yref, S = ref.conv3x3(Wd, X)
    for lanes in (16, 32):
        got, info = run_conv(csr, X, 24, kernel=sp.KERNEL_SPEC, spec_rows=3, spec_lanes=lanes)
        check(got, Yref, S, np.float32)


@pytest.mark.parametrize("opts", [dict(spec_rows=8), dict(spec_rows=16, spec_ksplit=4),
                                  dict(spec_rows=12, spec_tiles=4, spec_mode=sp.SPEC_LDS)])
def test_row_swizzle_results(opts):
    csr = synth.clustered_csr(256, 512, 0.9, 3, clusters=8)
    B = synth.normal_dense(512, 196, 4)
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_swizzle=True, **opts)
    assert info["spec_swizzle"] == 1
    Cref, S = _oracle(csr, B)
    check(got, Cref, S, np.float32)
    csr = synth.small_int_csr(77, 130, 0.85, 21)
    B = synth.small_int_dense(130, 65, 22)
    got, _ = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_swizzle=True, **opts)
    assert np.array_equal(got.astype(np.float64), _oracle(csr, B)[0])


def test_row_swizzle_conv():
    csr, Wd = synth.conv_weights_csr(24, 16, 0.8, 5)
    X = synth.normal_dense(16, 14 * 14, 6).reshape(1, 16, 14, 14)
    Yref, S = ref.conv3x3(Wd, X)
    got, info = run_conv(csr, X, 24, kernel=sp.KERNEL_SPEC, spec_rows=4, spec_swizzle=True)
    assert info["spec_swizzle"] == 1
    check(got, Yref, S, np.float32)


@pytest.mark.parametrize("batch", [2, 3, 8])
def test_conv_batch_generated_and_row_walk(batch):
    """Images of a batch are independent convolutions with the same filters (grid z / grid y)."""
    Cin, Cout, H, W = 16, 24, 9, 13
    csr, Wd = synth.conv_weights_csr(Cout, Cin, 0.8, 5)
    X = synth.normal_dense(batch * Cin, H * W, 6).reshape(batch, Cin, H, W)
    Yref, S = ref.conv3x3(Wd, X)
    for opts in (dict(), dict(kernel=sp.KERNEL_SPEC, spec_rows=3), dict(kernel=sp.KERNEL_SPEC, spec_rows=6, spec_ksplit=4)):
        got, info = run_conv(csr, X, Cout, **opts)
        assert info["batch"] == batch and got.shape == (batch, Cout, H, W)
        check(got, Yref, S, np.float32)
    # half storage, row-walk kernel
    csr16, W16 = synth.conv_weights_csr(Cout, Cin, 0.8, 5, dtype=np.float16)
    X16 = X.astype(np.float16)
    Yref, S = ref.conv3x3(W16, X16)
    got, _ = run_conv(csr16, X16, Cout)
    check(got, Yref, S, np.float16)
    # small integers: every image bit-exact, and image i equals the batch-1 result of image i
    Wi = np.zeros((Cout, Cin, 3, 3), dtype=np.float32)
    ci = synth.small_int_csr(Cout, 9 * Cin, 0.8, 11)
    Wi.reshape(Cout, -1)[np.repeat(np.arange(Cout), np.diff(ci.row_ptr)), ci.col_idx] = ci.vals
    Xi = synth.small_int_dense(batch * Cin, H * W, 12).reshape(batch, Cin, H, W)
    Yi, _ = ref.conv3x3(Wi, Xi)
    for opts in (dict(), dict(kernel=sp.KERNEL_SPEC, spec_rows=5)):
        got, _ = run_conv(ci, Xi, Cout, **opts)
        assert np.array_equal(got.astype(np.float64), Yi)
        one, _ = run_conv(ci, Xi[batch - 1:batch], Cout, **opts)
        assert np.array_equal(one[0], got[batch - 1])


HALF_OPTS = [dict(spec_rows=1), dict(spec_rows=7), dict(spec_rows=20, spec_ksplit=4), dict(spec_rows=9, spec_swizzle=True),
             dict(spec_rows=50, spec_ksplit=8, spec_depth=3)]
HALF_PAIRS = [dict(spec_vec=2, spec_rows=1), dict(spec_vec=2, spec_rows=7), dict(spec_vec=2, spec_rows=20, spec_ksplit=4),
              dict(spec_vec=2, spec_rows=50, spec_ksplit=8, spec_depth=3, spec_swizzle=True)]


@pytest.mark.parametrize("N", [1, 8, 65, 200, 520])
def test_spec_half_small_integers_bit_exact(N):
    """Half storage in the generated kernel: sums in fp32, exact on small integers in any order."""
    csr = synth.small_int_csr(50, 90, 0.9, N, dtype=np.float16, vmax=3)
    B = synth.small_int_dense(90, N, N + 1, dtype=np.float16, bmax=4)
    Cref, _ = _oracle(csr, B)
    assert np.abs(Cref).max() <= 2048
    for opts in HALF_OPTS + (HALF_PAIRS if N % 2 == 0 else []):   # pairs: two halves per lane in one dword
        got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, **opts)
        assert info["kernel"] == sp.KERNEL_SPEC and info["dtype"] == sp.F16 and got.dtype == np.float16
        assert info["spec_vec"] == opts.get("spec_vec", 1)
        assert np.array_equal(got.astype(np.float64), Cref), (N, opts)


def test_spec_half_rounds_once_at_the_store():
    """fp32 accumulation, one rounding to nearest even: identity returns B bit for bit; rows of
    2049 and 2051 ones times a column of ones sum exactly in fp32 and round to the even
    neighbours 2048 and 2052 (a half-precision running sum would stall at 2048)."""
    K, N = 130, 70
    B = synth.normal_dense(K, N, 3, dtype=np.float16)
    eye = synth.csr_from_mask(np.eye(K, dtype=np.float16), np.eye(K, dtype=bool))
    got, _ = run_spmm(eye, B, kernel=sp.KERNEL_SPEC, spec_rows=5)
    assert got.tobytes() == B.tobytes()
    mask = np.ones((2, 2051), dtype=bool)
    mask[0, 2049:] = False
    ones = synth.csr_from_mask(np.ones((2, 2051), dtype=np.float16), mask)
    Bx = np.ones((2051, 66), dtype=np.float16)
    Bx[:, 1] = 2.0 ** -14
    want = _oracle(ones, Bx)[0].astype(np.float16)
    assert want[0, 0] == 2048 and want[1, 0] == 2052
    for opts in (dict(spec_rows=2), dict(spec_rows=2, spec_ksplit=8), dict(kernel=sp.KERNEL_ROWS),
                 dict(spec_rows=2, spec_vec=2), dict(spec_rows=2, spec_vec=2, spec_ksplit=4)):
        got, _ = run_spmm(ones, Bx, **{"kernel": sp.KERNEL_SPEC, **opts})
        assert got.tobytes() == want.tobytes(), opts


def test_half_subnormals_are_kept():
    """Half subnormals in B and in A are operands like any other (no flush to zero on the way in),
    and a result in the subnormal range is rounded to the nearest subnormal, not to zero."""
    tiny = np.float16(2.0 ** -24)          # smallest positive half subnormal
    K, N = 6, 70
    B = np.full((K, N), tiny, dtype=np.float16)
    B[1, :] = np.float16(3 * 2.0 ** -24)
    B[:, 1] = -B[:, 1]
    A = np.zeros((3, K), dtype=np.float16)
    A[0, 0] = 1024.0                       # 2^10 * 2^-24 = 2^-14: smallest normal half
    A[1, 1] = 1.0                          # subnormal in, same subnormal out
    A[1, 2] = 1.0                          # 3*2^-24 + 2^-24 = 2^-22
    A[2, 3] = tiny                         # subnormal value of A times a subnormal of B: 2^-48, rounds to +-0
    A[2, 4] = 0.5                          # 2^-25: a tie, rounds to even = 0; together with 2^-48 just above the tie -> 2^-24
    csr = synth.csr_from_mask(A, A != 0)
    want = _oracle(csr, B)[0].astype(np.float16)
    assert want[0, 0] == np.float16(2.0 ** -14) and want[1, 0] == np.float16(2.0 ** -22) and want[2, 0] == tiny
    assert want[2, 1] == -tiny
    for opts in (dict(kernel=sp.KERNEL_ROWS), dict(spec_rows=3), dict(spec_rows=1), dict(spec_rows=3, spec_vec=2)):
        got, _ = run_spmm(csr, B, **{"kernel": sp.KERNEL_SPEC, **opts})
        assert got.tobytes() == want.tobytes(), opts


def test_single_precision_subnormals_are_kept():
    """fp32 subnormals as operands, as values of A (literals of the generated code) and as results."""
    K, N = 5, 67
    B = np.full((K, N), np.float32(2.0 ** -149), dtype=np.float32)
    B[2, :] = 1024.0
    B[:, 1] = -B[:, 1]
    A = np.zeros((3, K), dtype=np.float32)
    A[0, 0] = 2.0 ** 20                    # 2^-129: subnormal result from a subnormal operand
    A[1, 2] = 2.0 ** -140                  # subnormal value of A: 2^-130
    A[2, 1] = 3.0                          # 3 * 2^-149 ...
    A[2, 3] = 1.0                          # ... + 2^-149 = 2^-147
    csr = synth.csr_from_mask(A, A != 0)
    want = _oracle(csr, B)[0].astype(np.float32)
    assert want[0, 0] == np.float32(2.0 ** -129) and want[1, 0] == np.float32(2.0 ** -130)
    assert want[2, 0] == np.float32(2.0 ** -147) and want[2, 1] == -want[2, 0]
    for opts in (dict(kernel=sp.KERNEL_ROWS), dict(spec_rows=3), dict(spec_rows=1),
                 dict(spec_rows=3, spec_mode=sp.SPEC_LDS)):
        got, _ = run_spmm(csr, B, **{"kernel": sp.KERNEL_SPEC, **opts})
        assert got.tobytes() == want.tobytes(), opts


@pytest.mark.parametrize("name", ["c1", "c2", "c3t"])
def test_spec_half_configs(name):
    case = synth.config(name, np.float16)
    opts = dict(spec_rows=48, spec_ksplit=8) if name == "c3t" else dict(spec_rows=4)
    Cref, S = _oracle(case.csr, case.B)
    for extra in (dict(), dict(spec_vec=2)):
        got, _ = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, **opts, **extra)
        check(got, Cref, S, np.float16, gate_relative=True)


def test_spec_half_skewed_and_conv():
    case = synth.sweep_case(256, 512, 196, 0.95, "skewed", np.float16)
    got, _ = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_rows=16, spec_ksplit=4)
    Cref, S = _oracle(case.csr, case.B)
    check(got, Cref, S, np.float16)
    for (Cin, Cout, H, W, batch) in ((16, 24, 14, 14, 1), (5, 7, 9, 13, 3), (3, 4, 1, 9, 2)):
        csr, Wd = synth.conv_weights_csr(Cout, Cin, 0.8, 5, dtype=np.float16)
        X = synth.normal_dense(batch * Cin, H * W, 6, dtype=np.float16).reshape(batch, Cin, H, W)
        Yref, S = ref.conv3x3(Wd, X)
        for opts in (dict(spec_rows=3), dict(spec_rows=4, spec_ksplit=2)):
            got, info = run_conv(csr, X, Cout, kernel=sp.KERNEL_SPEC, **opts)
            assert info["dtype"] == sp.F16
            check(got, Yref, S, np.float16)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_spmm_batch_of_matrices(dtype):
    """opt->batch on an SpMM plan: [b, K, N] times the same A in one launch."""
    half = dtype == np.float16
    csr = synth.small_int_csr(40, 90, 0.8, 31, dtype=dtype, vmax=3)
    B = np.stack([synth.small_int_dense(90, 130, 40 + i, dtype=dtype, bmax=4) for i in range(3)])
    Cref = np.stack([_oracle(csr, B[i])[0] for i in range(3)])
    assert np.abs(Cref).max() <= 2048
    for opts in (dict(), dict(vec=2), dict(split_threshold=4), dict(kernel=sp.KERNEL_SPEC, spec_rows=7),
                 dict(kernel=sp.KERNEL_SPEC, spec_rows=10, spec_ksplit=4)) + \
            (() if half else (dict(kernel=sp.KERNEL_SPEC, spec_rows=5, spec_tiles=2, spec_mode=sp.SPEC_LDS),)):
        got, info = run_spmm(csr, B, **opts)
        assert info["batch"] == 3 and got.shape == (3, 40, 130)
        assert np.array_equal(got.astype(np.float64), Cref), opts


def test_launches_replay_from_a_hip_graph():
    """The executors allocate nothing and only enqueue a kernel, so they can be captured; every
    replay, with eager work on the same buffers in between, must give the eager result."""
    dev = torch.device("cuda:0")
    case = synth.config("c2")
    csr = case.csr
    ccsr, Wd = synth.conv_weights_csr(24, 16, 0.8, 5)
    X = synth.normal_dense(2 * 16, 14 * 14, 6).reshape(2, 16, 14, 14)
    plans = [sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N),
             sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N, kernel=sp.KERNEL_SPEC,
                        spec_rows=16, spec_ksplit=4),
             sp.inspect(ccsr.row_ptr, ccsr.col_idx, ccsr.vals, 24, 144, 196, conv=(16, 14, 14), batch=2,
                        kernel=sp.KERNEL_SPEC)]
    Bd = torch.from_numpy(case.B).to(dev)
    Xd = torch.from_numpy(X).to(dev)
    outs = [torch.zeros((csr.M, case.N), device=dev), torch.zeros((csr.M, case.N), device=dev),
            torch.zeros((2, 24, 14, 14), device=dev)]

    def launch_all():
        st = torch.cuda.current_stream(dev).cuda_stream
        sp.spmm(plans[0], Bd.data_ptr(), outs[0].data_ptr(), st)
        sp.spmm(plans[1], Bd.data_ptr(), outs[1].data_ptr(), st)
        sp.conv3x3(plans[2], Xd.data_ptr(), outs[2].data_ptr(), st)

    launch_all()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    Cref, S = _oracle(csr, case.B)
    check(eager[1].cpu().numpy(), Cref, S, np.float32, gate_relative=True)
    side = torch.cuda.Stream(dev)
    with torch.cuda.stream(side):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            launch_all()
    for rep in range(4):
        for o in outs:
            o.fill_(float(rep) - 7.0)      # eager work between replays, on the buffers the graph writes
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, e in zip(outs, eager):
            assert torch.equal(o, e), rep
    for p in plans:
        p.destroy()


@pytest.mark.parametrize("seed", range(12))
def test_random_small_cases_all_executors(seed):
    """Seeded random shapes, densities, storage types and plan options; small integers, so every
    executor must reproduce the oracle bit for bit whatever its summation order."""
    rng = np.random.default_rng(1000 + seed)
    for _ in range(6):
        M, K, N = int(rng.integers(1, 90)), int(rng.integers(1, 200)), int(rng.integers(1, 300))
        dtype = [np.float32, np.float16, np.int8][int(rng.integers(0, 3))]
        density = float(rng.choice([0.02, 0.1, 0.4, 1.0]))
        mask = rng.random((M, K)) < density
        vals = (rng.integers(1, 4, size=(M, K)) * rng.choice([-1, 1], size=(M, K))).astype(dtype)
        csr = synth.csr_from_mask(vals, mask)
        B = rng.integers(-4, 5, size=(K, N)).astype(dtype)
        want = _oracle(csr, B)[0]
        assert np.abs(want).max() <= 2048
        rows = int(rng.integers(1, 60))
        ks = int(rng.choice([0, 2, 4, 8]))
        variants = [dict(), dict(split_threshold=int(rng.integers(1, 9))),
                    dict(kernel=sp.KERNEL_SPEC, spec_rows=rows, spec_ksplit=ks, spec_swizzle=bool(rng.integers(0, 2)),
                         spec_depth=int(rng.integers(1, 20)), natural_order=bool(rng.integers(0, 2)))]
        if dtype == np.float32:
            variants.append(dict(kernel=sp.KERNEL_SPEC, spec_rows=rows, spec_mode=sp.SPEC_LDS,
                                 spec_tiles=int(rng.choice([1, 2, 4, 8]))))
        for opts in variants:
            got, _ = run_spmm(csr, B, **opts)
            assert np.array_equal(got.astype(np.float64), want), (M, K, N, np.dtype(dtype).name, density, opts)


def test_loaded_plans_execute_like_the_saved_ones():
    """A tuned plan saved by one process and loaded by another must run the same kernel."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream(dev).cuda_stream
    case = synth.config("c2")
    csr = case.csr
    Bd = torch.from_numpy(case.B).to(dev)
    for opts in (dict(), dict(kernel=sp.KERNEL_SPEC, spec_rows=16, spec_ksplit=4, spec_swizzle=True),
                 dict(kernel=sp.KERNEL_SPEC, spec_rows=12, spec_mode=sp.SPEC_LDS)):
        plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N, **opts)
        again = sp.load(plan.save())
        outs = []
        for p in (plan, again):
            Cd = torch.full((csr.M, case.N), float("nan"), device=dev)
            sp.spmm(p, Bd.data_ptr(), Cd.data_ptr(), stream)
            torch.cuda.synchronize()
            outs.append(Cd)
        assert torch.equal(outs[0], outs[1]), opts
        Cref, S = _oracle(csr, case.B)
        check(outs[1].cpu().numpy(), Cref, S, np.float32, gate_relative=True)
        plan.destroy()
        again.destroy()
    ccsr, Wd = synth.conv_weights_csr(24, 16, 0.8, 5, dtype=np.float16)
    X = synth.normal_dense(2 * 16, 14 * 14, 6, dtype=np.float16).reshape(2, 16, 14, 14)
    plan = sp.inspect(ccsr.row_ptr, ccsr.col_idx, ccsr.vals, 24, 144, 196, conv=(16, 14, 14), batch=2,
                      kernel=sp.KERNEL_SPEC, spec_rows=3)
    again = sp.load(plan.save())
    plan.destroy()
    Xd = torch.from_numpy(X).to(dev)
    Yd = torch.full((2, 24, 14, 14), float("nan"), dtype=torch.float16, device=dev)
    sp.conv3x3(again, Xd.data_ptr(), Yd.data_ptr(), stream)
    torch.cuda.synchronize()
    Yref, S = ref.conv3x3(Wd, X)
    check(Yd.cpu().numpy(), Yref, S, np.float16)
    again.destroy()


@pytest.mark.parametrize("seed", range(8))
def test_random_small_convolutions_all_executors(seed):
    """Seeded random convolution shapes, batches, storage types and plan options on small
    integers: bit-exact against the direct-loop oracle whatever the executor."""
    rng = np.random.default_rng(5000 + seed)
    for _ in range(4):
        Cin, Cout = int(rng.integers(1, 12)), int(rng.integers(1, 40))
        H, W, batch = int(rng.integers(1, 12)), int(rng.integers(1, 12)), int(rng.integers(1, 4))
        dtype = [np.float32, np.float16, np.int8][int(rng.integers(0, 3))]
        Wd = (rng.integers(1, 4, size=(Cout, Cin, 3, 3)) * rng.choice([-1, 1], size=(Cout, Cin, 3, 3))
              * (rng.random((Cout, Cin, 3, 3)) < float(rng.choice([0.05, 0.3, 1.0])))).astype(dtype)
        csr = synth.csr_from_mask(Wd.reshape(Cout, -1), Wd.reshape(Cout, -1) != 0)
        X = rng.integers(-4, 5, size=(batch, Cin, H, W)).astype(dtype)
        want = ref.conv3x3(Wd, X, want_scale=False)[0]
        assert np.abs(want).max() <= 2048
        variants = [dict(), dict(split_threshold=int(rng.integers(1, 9))),
                    dict(kernel=sp.KERNEL_SPEC, spec_rows=int(rng.integers(1, 30)), spec_ksplit=int(rng.choice([0, 2, 4, 8])),
                         spec_swizzle=bool(rng.integers(0, 2)), spec_depth=int(rng.integers(1, 20)),
                         natural_order=bool(rng.integers(0, 2)), spec_lanes=int(rng.choice([0, 16, 32])))]
        for opts in variants:
            got, _ = run_conv(csr, X, Cout, **opts)
            assert np.array_equal(got.astype(np.float64), want), (Cin, Cout, H, W, batch, np.dtype(dtype).name, opts)


NATURAL = [dict(), dict(kernel=sp.KERNEL_SPEC, spec_rows=9), dict(kernel=sp.KERNEL_SPEC, spec_rows=12, spec_mode=sp.SPEC_LDS),
           dict(kernel=sp.KERNEL_SPEC, spec_rows=20, spec_ksplit=4)]


@pytest.mark.parametrize("opts", NATURAL)
def test_natural_order_ablation_is_still_exact(opts):
    """Rows in input order, unsplit, contiguous code blocks: slower on skewed matrices, same result."""
    case = synth.sweep_case(256, 512, 196, 0.95, "skewed", np.float32)   # long and empty rows side by side
    got, info = run_spmm(case.csr, case.B, natural_order=True, **opts)
    assert info["natural_order"] == 1 and info["n_split"] == 0
    Cref, S = _oracle(case.csr, case.B)
    check(got, Cref, S, np.float32)
    csr = synth.small_int_csr(77, 130, 0.85, 9)
    B = synth.small_int_dense(130, 65, 10)
    got, _ = run_spmm(csr, B, natural_order=True, **opts)
    assert np.array_equal(got.astype(np.float64), _oracle(csr, B)[0])


def test_natural_order_conv():
    csr, Wd = synth.conv_weights_csr(24, 16, 0.8, 5)
    X = synth.normal_dense(16, 14 * 14, 6).reshape(1, 16, 14, 14)
    Yref, S = ref.conv3x3(Wd, X)
    for opts in (dict(), dict(kernel=sp.KERNEL_SPEC, spec_rows=3)):
        got, info = run_conv(csr, X, 24, natural_order=True, **opts)
        assert info["natural_order"] == 1
        check(got, Yref, S, np.float32)


CONV_SHAPES = [(3, 5, 1, 1), (4, 6, 2, 3), (2, 3, 1, 9), (2, 3, 9, 1), (8, 8, 7, 7), (16, 24, 14, 14),
               (6, 10, 9, 13), (64, 64, 56, 56), (128, 128, 28, 28), (256, 256, 14, 14), (512, 512, 7, 7)]


@pytest.mark.parametrize("Cin,Cout,H,W", CONV_SHAPES)
def test_spec_conv_shapes(Cin, Cout, H, W):
    from gpu_util import run_conv
    csr, Wd = synth.conv_weights_csr(Cout, Cin, 0.9 if Cin > 4 else 0.5, Cin + H)
    X = synth.normal_dense(Cin, H * W, Cout + W).reshape(1, Cin, H, W)
    Yref, S = ref.conv3x3(Wd, X)
    for rows in (0, 1, 5):
        got, info = run_conv(csr, X, Cout, kernel=sp.KERNEL_SPEC, spec_rows=rows)
        assert info["kernel"] == sp.KERNEL_SPEC and info["conv"] == 1
        check(got, Yref, S, np.float32)


def test_spec_conv_integer_taps_bit_exact():
    from gpu_util import run_conv
    Cin, Cout, H, W = 7, 9, 11, 6
    rng = np.random.default_rng(4)
    Wd = (rng.integers(-3, 4, size=(Cout, Cin, 3, 3)) * (rng.random((Cout, Cin, 3, 3)) < 0.3)).astype(np.float32)
    X = rng.integers(-5, 6, size=(1, Cin, H, W)).astype(np.float32)
    csr = synth.csr_from_mask(Wd.reshape(Cout, -1), Wd.reshape(Cout, -1) != 0)
    Yref, _ = ref.conv3x3(Wd, X)
    for rows, tiles in ((0, 0), (1, 1), (3, 2), (9, 16)):
        got, _ = run_conv(csr, X, Cout, kernel=sp.KERNEL_SPEC, spec_rows=rows, spec_tiles=tiles)
        assert np.array_equal(got.astype(np.float64), Yref)
    for ks in (2, 4):
        got, _ = run_conv(csr, X, Cout, kernel=sp.KERNEL_SPEC, spec_rows=3, spec_ksplit=ks)
        assert np.array_equal(got.astype(np.float64), Yref)
    for t in range(9):  # one tap at a time: a zero-filled shift of the input, bit for bit
        W1 = np.zeros((1, 1, 3, 3), dtype=np.float32)
        W1[0, 0, t // 3, t % 3] = 1.0
        X1 = synth.normal_dense(1, H * W, t).reshape(1, 1, H, W)
        got, _ = run_conv(synth.csr_from_mask(W1.reshape(1, 9), W1.reshape(1, 9) != 0), X1, 1,
                          kernel=sp.KERNEL_SPEC)
        Yr, _ = ref.conv3x3(W1, X1)
        assert np.array_equal(got.astype(np.float64), Yr)


def test_spec_rejects_what_it_does_not_cover():
    ccsr, _ = synth.conv_weights_csr(4, 2, 0.5, 1)
    with pytest.raises(sp.SparseRTError) as e:   # the LDS-staged variant is for SpMM plans
        sp.inspect(ccsr.row_ptr, ccsr.col_idx, ccsr.vals, 4, 18, 16, conv=(2, 4, 4), kernel=sp.KERNEL_SPEC, host_only=True,
                   spec_mode=sp.SPEC_LDS)
    assert e.value.status == sp.EUNSUPPORTED


@pytest.mark.parametrize("dtype", [np.float16, np.int8])
@pytest.mark.parametrize("N,waves", [(1, 1), (65, 4), (196, 8), (300, 16)])
def test_lds_staged_variant_half_and_int8_bit_exact(N, waves, dtype):
    """Operands of the narrow storage types are widened to 32 bits on their way into LDS."""
    if dtype == np.int8:
        csr, B = synth.int8_csr(70, 270, 0.85, N), synth.int8_dense(270, N, N + 1)
    else:
        csr = synth.small_int_csr(70, 270, 0.85, N, dtype=np.float16, vmax=3)
        B = synth.small_int_dense(270, N, N + 1, dtype=np.float16, bmax=4)
    Cref, _ = _oracle(csr, B)
    for rows in (1, 5, 24):
        got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_mode=sp.SPEC_LDS, spec_rows=rows, spec_tiles=waves)
        assert info["spec_mode"] == sp.SPEC_LDS
        assert np.array_equal(got.astype(np.float64), Cref), (rows, info)


def test_lds_staged_variant_half_config_and_batch():
    case = synth.config("c2", np.float16)
    got, _ = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_mode=sp.SPEC_LDS, spec_rows=12, spec_tiles=8)
    Cref, S = _oracle(case.csr, case.B)
    check(got, Cref, S, np.float16, gate_relative=True)
    B3 = np.stack([case.B, case.B[::-1].copy(), case.B * np.float16(0.5)])
    got, _ = run_spmm(case.csr, B3, kernel=sp.KERNEL_SPEC, spec_mode=sp.SPEC_LDS, spec_rows=12, spec_tiles=4)
    for i in range(3):
        Cref, S = _oracle(case.csr, B3[i])
        check(got[i], Cref, S, np.float16)


def test_tune_returns_a_correct_plan_and_a_report():
    case = synth.config("c2")
    csr = case.csr
    dev = torch.device("cuda:0")
    Bd = torch.from_numpy(case.B).to(dev)
    Cd = torch.full((csr.M, case.N), float("nan"), device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    plan, report = sp.tune(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N,
                           Bd.data_ptr(), Cd.data_ptr(), stream)
    assert len(report) >= 4 and all(r["microseconds"] > 0 for r in report)
    assert {r["kernel"] for r in report} == {sp.KERNEL_ROWS, sp.KERNEL_SPEC}
    Cd.fill_(float("nan"))
    sp.spmm(plan, Bd.data_ptr(), Cd.data_ptr(), stream)
    torch.cuda.synchronize()
    Cref, S = _oracle(csr, case.B)
    check(Cd.cpu().numpy(), Cref, S, np.float32, gate_relative=True)
    print(plan.info(), sorted(report, key=lambda r: r["microseconds"])[:3])
    plan.destroy()


def test_tune_covers_half_and_conv():
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream(dev).cuda_stream
    csr, Wd = synth.conv_weights_csr(24, 16, 0.9, 3, dtype=np.float16)
    X = synth.normal_dense(16, 14 * 14, 4, dtype=np.float16).reshape(1, 16, 14, 14)
    Xd = torch.from_numpy(X).to(dev)
    Yd = torch.empty((1, 24, 14, 14), dtype=torch.float16, device=dev)
    plan, report = sp.tune(csr.row_ptr, csr.col_idx, csr.vals, 24, 144, 196, Xd.data_ptr(), Yd.data_ptr(),
                           stream, conv=(16, 14, 14))
    assert len(report) >= 2
    sp.conv3x3(plan, Xd.data_ptr(), Yd.data_ptr(), stream)
    torch.cuda.synchronize()
    Yref, S = ref.conv3x3(Wd, X)
    check(Yd.cpu().numpy(), Yref, S, np.float16)
    plan.destroy()


# ---------------------------------------------------------------- leading dimensions (strided N)
@pytest.mark.parametrize("opts", [dict(kernel=sp.KERNEL_ROWS), dict(kernel=sp.KERNEL_ROWS, split_threshold=3),
                                  dict(kernel=sp.KERNEL_SPEC, spec_rows=5), dict(kernel=sp.KERNEL_SPEC, spec_rows=16, spec_ksplit=4),
                                  dict(kernel=sp.KERNEL_SPEC, spec_rows=7, spec_mode=sp.SPEC_LDS, spec_tiles=4), dict()])
@pytest.mark.parametrize("N,ldb,ldc", [(1, 5, 3), (64, 64, 80), (65, 130, 65), (196, 1024, 3136), (256, 260, 264), (300, 304, 512)])
def test_leading_dimensions_small_integers_bit_exact(N, ldb, ldc, opts):
    """A column slice of wider activation matrices (Section 4.3: more columns make N larger):
    only the N columns are read and written, at the given pitches; sums are exact integers."""
    from gpu_util import run_spmm_strided
    csr = synth.small_int_csr(60, 140, 0.85, N + ldb)
    B = synth.small_int_dense(140, N, N + ldc)
    Cref, _ = ref.spmm(csr.M, csr.K, N, csr.row_ptr, csr.col_idx, csr.vals, B)
    got, pad_ok, info = run_spmm_strided(csr, B, ldb, ldc, **opts)
    assert np.array_equal(got.astype(np.float64), Cref), info
    assert pad_ok, "columns beyond N of the result buffer were written"


@pytest.mark.parametrize("dtype", [np.float32, np.float16, np.int8])
def test_leading_dimensions_batch_and_storage_types(dtype):
    from gpu_util import run_spmm_strided
    N, ldb, ldc, batch = 200, 208, 256, 3
    if dtype == np.int8:
        csr = synth.int8_csr(90, 300, 0.9, 1)
        B = synth.int8_dense(batch * 300, N, 2).reshape(batch, 300, N)
    else:
        csr = synth.small_int_csr(90, 300, 0.9, 1, dtype=dtype, vmax=3)
        B = synth.small_int_dense(batch * 300, N, 2, dtype=dtype, bmax=4).reshape(batch, 300, N)
    want = np.stack([ref.spmm(90, 300, N, csr.row_ptr, csr.col_idx, csr.vals, B[i])[0] for i in range(batch)])
    for opts in (dict(kernel=sp.KERNEL_ROWS), dict(kernel=sp.KERNEL_SPEC, spec_rows=8, spec_ksplit=2),
                 dict(kernel=sp.KERNEL_SPEC, spec_rows=6, spec_vec=2 if dtype == np.float16 else 4 if dtype == np.int8 else 1)):
        got, pad_ok, info = run_spmm_strided(csr, B, ldb, ldc, **opts)
        assert np.array_equal(got.astype(np.float64), want), (opts, info)
        assert pad_ok


def test_leading_dimensions_headline_layer_slice():
    """c3 on a 1024-column slice of 4096-column activations, in the plan the inspector picks."""
    from gpu_util import run_spmm_strided
    case = synth.config("c3")
    got, pad_ok, info = run_spmm_strided(case.csr, case.B, 4096, 4096)
    Cref, S = ref.spmm(case.csr.M, case.csr.K, case.N, case.csr.row_ptr, case.csr.col_idx, case.csr.vals, case.B)
    check(got, Cref, S, np.float32, gate_relative=True)
    assert pad_ok and info["kernel"] == sp.KERNEL_SPEC


# ---------------------------------------------------------------- code prefetch
@pytest.mark.parametrize("opts", [dict(spec_rows=1), dict(spec_rows=96, spec_ksplit=2), dict(spec_rows=24, spec_ksplit=8),
                                  dict(spec_rows=200, spec_ksplit=8), dict(spec_rows=12, spec_mode=sp.SPEC_LDS, spec_tiles=8)])
@pytest.mark.parametrize("N", [1, 65, 196])
def test_code_prefetch_changes_no_result(N, opts):
    """Waves that touch their block's code ahead (blocks from a few hundred bytes to several
    prefetch lines per lane) compute exactly what they compute without."""
    csr = synth.small_int_csr(300, 500, 0.8, N)
    B = synth.small_int_dense(500, N, N + 1)
    Cref, _ = _oracle(csr, B)
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_prefetch=1, **opts)
    assert info["spec_prefetch"] >= 1
    assert np.array_equal(got.astype(np.float64), Cref), info


def test_code_prefetch_headline_layers_half_int8_and_conv():
    for name, opts in (("c3", dict(spec_rows=96, spec_ksplit=4, spec_swizzle=True)), ("c3t", dict(spec_rows=48, spec_ksplit=8))):
        case = synth.config(name)
        got, info = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_prefetch=1, **opts)
        Cref, S = _oracle(case.csr, case.B)
        check(got, Cref, S, np.float32, gate_relative=True)
    case = synth.config("c2", np.float16)
    got, _ = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_prefetch=1, spec_vec=2, spec_rows=8)
    Cref, S = _oracle(case.csr, case.B)
    check(got, Cref, S, np.float16, gate_relative=True)
    case = synth.config("c1", np.int8)
    got, _ = run_spmm(case.csr, case.B, kernel=sp.KERNEL_SPEC, spec_prefetch=1, spec_vec=4, spec_rows=8, spec_ksplit=2)
    Cref, _ = _oracle(case.csr, case.B)
    assert np.array_equal(got.astype(np.float64), Cref)
    case = synth.config("c4")
    got, _ = run_conv(case.csr, case.X, 256, kernel=sp.KERNEL_SPEC, spec_prefetch=1)
    Yref, S = ref.conv3x3(case.Wdense, case.X)
    check(got, Yref, S, np.float32, gate_relative=True)


@pytest.mark.parametrize("M,K,N,rows", [(1024, 512, 784, 54), (256, 128, 3136, 14), (1024, 600, 3136, 103)])
def test_default_rows_that_avoid_a_thin_last_round(M, K, N, rows):
    """Shapes whose default row count is raised so that the workgroups fit a whole number of
    rounds over the compute units (54 rows: 19 blocks x 13 tiles = 247 workgroups, not 260)."""
    csr = synth.small_int_csr(M, K, 0.95, N)
    B = synth.small_int_dense(K, N, N + 1)
    Cref, _ = _oracle(csr, B)
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC)
    assert info["spec_rows"] == rows, info
    assert np.array_equal(got.astype(np.float64), Cref)


@pytest.mark.parametrize("N", [49, 130])
def test_blocks_of_the_most_rows_the_registers_hold(N):
    """232 rows per block with the reduction axis split over eight waves: the partial sums are
    exchanged in several phases through all of the LDS."""
    csr = synth.small_int_csr(464, 300, 0.9, N)
    B = synth.small_int_dense(300, N, N + 1)
    Cref, _ = _oracle(csr, B)
    got, info = run_spmm(csr, B, kernel=sp.KERNEL_SPEC, spec_rows=232, spec_ksplit=8)
    assert info["spec_rows"] == 232 and info["spec_lds_bytes"] > 150 * 1024
    assert np.array_equal(got.astype(np.float64), Cref)
