"""The allocation-free comparison entry point against the allocating one, through the C ABI."""
import numpy as np
import pytest

from paper_2008_11849_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():  # pragma: no cover
    pytest.skip("no GPU", allow_module_level=True)

from paper_2008_11849_amd import sparsert as sp  # noqa: E402


def _words(plan, fn, a, b):
    dev = torch.device("cuda:0")
    res = torch.full((4,), 0x7fffffff, dtype=torch.int32, device=dev)
    fn(plan, a.data_ptr(), b.data_ptr(), res.data_ptr(), torch.cuda.current_stream(dev).cuda_stream)
    torch.cuda.synchronize()
    return res.cpu().numpy().view(np.uint32).tolist()


def _pair(M, N, batch, dtype, seed):
    """Two results of a real plan: the row-walk kernel's and the generated kernel's, the second
    with a few planted differences (a large one, a NaN)."""
    dev = torch.device("cuda:0")
    csr = synth.uniform_csr(M, 96, 0.9, seed, dtype=dtype)
    B = torch.from_numpy(synth.normal_dense(batch * 96, N, seed + 1, dtype).reshape(batch, 96, N)).to(dev)
    tdt = torch.float16 if dtype == np.float16 else torch.float32
    outs, plans = [], []
    for kernel in (sp.KERNEL_ROWS, sp.KERNEL_SPEC):
        plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, M, 96, N, batch=batch, kernel=kernel)
        C = torch.empty((batch, M, N), dtype=tdt, device=dev)
        sp.spmm(plan, B.data_ptr(), C.data_ptr(), torch.cuda.current_stream(dev).cuda_stream)
        outs.append(C)
        plans.append(plan)
    torch.cuda.synchronize()
    outs[1][0, M // 2, N // 3] += 3.0
    outs[1][batch - 1, M - 1, N - 1] = float("nan")
    return plans, outs


def test_static_comparison_equals_the_allocating_one_on_two_calls_in_a_row():
    # first a large output (1024 blocks of partials), then a small one (3 blocks): the second call
    # finds the first call's partials in the static array and must not read them
    big_plans, big = _pair(4096, 4096, 1, np.float32, 3)
    small_plans, small = _pair(150, 300, 1, np.float16, 4)
    want_big = _words(big_plans[0], sp.compare_outputs, big[0], big[1])
    want_small = _words(small_plans[0], sp.compare_outputs, small[0], small[1])
    got_big = _words(big_plans[0], sp.compare_outputs_static, big[0], big[1])
    got_small = _words(small_plans[0], sp.compare_outputs_static, small[0], small[1])
    assert got_big == want_big and got_small == want_small
    assert want_big[2] == 1 and want_big[3] == 1024 and want_small[2] == 1 and want_small[3] == 3
    assert np.array([want_big[0]], dtype=np.uint32).view(np.float32)[0] >= 2.9     # the planted difference is what it found
    # and once more the other way round, with a batch
    plans3, outs3 = _pair(64, 64, 5, np.float32, 5)
    assert _words(plans3[1], sp.compare_outputs_static, outs3[0], outs3[1]) == _words(plans3[1], sp.compare_outputs, outs3[0], outs3[1])
    assert _words(big_plans[1], sp.compare_outputs_static, big[1], big[0]) == _words(big_plans[1], sp.compare_outputs, big[1], big[0])
    for p in big_plans + small_plans + plans3:
        p.destroy()


def test_static_comparison_refuses_what_its_array_does_not_cover():
    csr = synth.uniform_csr(8192, 16, 0.9, 1)
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 8192, 16, 4104, kernel=sp.KERNEL_ROWS)   # 33.6 M elements
    t = torch.zeros(16, device="cuda:0")
    r = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    with pytest.raises(sp.SparseRTError) as e:
        sp.compare_outputs_static(plan, t.data_ptr(), t.data_ptr(), r.data_ptr())
    assert e.value.status == sp.EUNSUPPORTED and "33554432" in str(e.value)
    plan.destroy()
