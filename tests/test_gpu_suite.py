"""GPU parity at the paper's own problem sizes, in the plans the autotuner picks.

Table 1 (twenty SpMM shapes, Section 4.1; problems 1-11 also at 95 %) and Table 3 (four 3x3
convolutions, Section 4.2) with synthetic magnitude-pruned weights, and a seeded sample of the
shape / sparsity sweep that reaches the smallest and the largest sizes, every N, both storage
types and both mask kinds.  Every element of every result is compared with the CPU oracle (for
the largest sweep cases: every element of a seeded sample of rows)."""
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


def _tuned_run(case, dtype):
    """sparsert_tune on the case's own operands, then one fresh launch of the returned plan into
    a poisoned buffer.  Returns (result, plan info, report entries)."""
    dev = torch.device("cuda:0")
    csr = case.csr
    stream = torch.cuda.current_stream(dev).cuda_stream
    tdt = torch.float16 if np.dtype(dtype) == np.float16 else torch.float32
    if case.conv is not None:
        inp = torch.from_numpy(case.X).to(dev)
        shape = (case.X.shape[0], csr.M, case.conv[1], case.conv[2])
    else:
        inp = torch.from_numpy(case.B).to(dev)
        shape = (csr.M, case.N)
    out = torch.empty(shape, dtype=tdt, device=dev)
    plan, entries = sp.tune(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N, inp.data_ptr(), out.data_ptr(),
                            stream, conv=case.conv, batch=case.X.shape[0] if case.conv is not None else 0)
    out.fill_(float("nan"))
    (sp.conv3x3 if case.conv is not None else sp.spmm)(plan, inp.data_ptr(), out.data_ptr(), stream)
    torch.cuda.synchronize()
    info = plan.info()
    plan.destroy()
    return out.cpu().numpy(), info, entries


@pytest.mark.parametrize("tag,i,sparsity", synth.table1_problems())
def test_table1_problem_in_its_tuned_plan(tag, i, sparsity):
    case = synth.table1_case(i, sparsity)
    got, info, entries = _tuned_run(case, np.float32)
    csr = case.csr
    Cref, S = ref.spmm(csr.M, csr.K, case.N, csr.row_ptr, csr.col_idx, csr.vals, case.B)
    m = check(got, Cref, S, np.float32)
    assert all(e["agrees"] for e in entries), [e for e in entries if not e["agrees"]]
    print(tag, {k: info[k] for k in ("kernel", "vec", "spec_rows", "spec_ksplit", "spec_tiles", "spec_swizzle")}, m)


@pytest.mark.parametrize("i", range(4))
@pytest.mark.parametrize("sparsity", [0.90, 0.95])
def test_table3_convolution_in_its_tuned_plan(i, sparsity):
    case = synth.table3_case(i, sparsity)
    got, info, entries = _tuned_run(case, np.float32)
    Yref, S = ref.conv3x3(case.Wdense, case.X)
    m = check(got, Yref, S, np.float32)
    assert all(e["agrees"] for e in entries), [e for e in entries if not e["agrees"]]
    print(case.name, {k: info[k] for k in ("kernel", "spec_rows", "spec_ksplit", "spec_tiles")}, m)


def test_table1_half_precision_problems_in_their_tuned_plans():
    # the two extremes of N (ResNet-50's 49 columns, MobileNetV1's 12544)
    for i, sparsity in ((7, 0.95), (11, 0.90)):
        case = synth.table1_case(i, sparsity, np.float16)
        got, info, _ = _tuned_run(case, np.float16)
        csr = case.csr
        Cref, S = ref.spmm(csr.M, csr.K, case.N, csr.row_ptr, csr.col_idx, csr.vals, case.B)
        check(got, Cref, S, np.float16)


SAMPLE = synth.sweep_sample(16)


def _rows_sample(csr, rows):
    rp = csr.row_ptr
    sub_ptr = np.zeros(len(rows) + 1, dtype=np.int32)
    cols, vals = [], []
    for j, r in enumerate(rows):
        cols.append(csr.col_idx[rp[r]:rp[r + 1]])
        vals.append(csr.vals[rp[r]:rp[r + 1]])
        sub_ptr[j + 1] = sub_ptr[j] + (rp[r + 1] - rp[r])
    return sub_ptr, np.concatenate(cols), np.concatenate(vals)


@pytest.mark.parametrize("M,K,N,sparsity,kind,dtype", SAMPLE,
                         ids=[f"{m}x{k}x{n}_{int(s * 100)}_{kind}_{np.dtype(dt).name}" for m, k, n, s, kind, dt in SAMPLE])
def test_sweep_sample(M, K, N, sparsity, kind, dtype):
    """The plan a caller gets without options (the generated kernel up to 4194304 nonzeros, the
    row-walk kernel beyond) and, for the smaller matrices, the tuned plan."""
    case = synth.sweep_case(M, K, N, sparsity, kind, dtype)
    csr = case.csr
    work = csr.nnz * N
    if work <= 400e6:
        rows = np.arange(M)
        Cref, S = ref.spmm(M, K, N, csr.row_ptr, csr.col_idx, csr.vals, case.B)
    else:   # the oracle computes a seeded sample of rows, every column of each
        rows = np.sort(np.random.default_rng(synth.sweep_seed(M, K, N, sparsity, kind, dtype)).choice(M, size=64, replace=False))
        sub_ptr, cols, vals = _rows_sample(csr, rows)
        Cref, S = ref.spmm(len(rows), K, N, sub_ptr, cols, vals, case.B)
    got, info = run_spmm(csr, case.B)
    assert info["kernel"] == (sp.KERNEL_SPEC if csr.nnz <= 4194304 else sp.KERNEL_ROWS)
    check(got[rows], Cref, S, dtype)
    if csr.nnz <= 60000:
        got, info, entries = _tuned_run(case, dtype)
        check(got[rows], Cref, S, dtype)
        assert all(e["agrees"] for e in entries)
