"""Host-side tests: the C-ABI library loads and exports what include/sparsert.h declares,
argument validation returns error codes, and the exported plan equals the NumPy statement
of the plan specification byte for byte.  No GPU is touched (host_only plans)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import plan_ref
from paper_2008_11849_amd import sparsert as sp
from paper_2008_11849_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

FIELDS = {"row_nnz": sp.FIELD_ROW_NNZ, "hist": sp.FIELD_HIST, "perm": sp.FIELD_PERM,
          "inv_perm": sp.FIELD_INV_PERM, "p_row_ptr": sp.FIELD_P_ROW_PTR,
          "p_col_idx": sp.FIELD_P_COL_IDX, "p_vals": sp.FIELD_P_VALS, "bins": sp.FIELD_BINS,
          "stream": sp.FIELD_STREAM, "conv_seg": sp.FIELD_CONV_SEG,
          "segments": sp.FIELD_SEGMENTS}


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sparsert.h")).read()
    declared = set(re.findall(r"\b(sparsert_[a-z0-9_]+)\s*\(", header))
    assert declared == set(sp.EXPORTED)
    lib = ctypes.CDLL(sp.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert sp.version() >= 100


def test_boundary_from_plain_c99(tmp_path):
    """include/sparsert.h is strict C99 and the library can be driven without Python."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    exe = tmp_path / "c_abi_check"
    libdir = os.path.dirname(sp.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", str(exe), "-L", libdir, "-lsparsert",
           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and "c abi ok" in run.stdout, run.stdout + run.stderr


def _header_struct_fields(name):
    """(field, element count) of a header struct whose members are all int32_t / float."""
    text = open(os.path.join(os.path.dirname(sp.LIB_PATH), "..", "include", "sparsert.h")).read()
    body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (name, name), text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    out = []
    for decl in re.findall(r"(?:int32_t|float)\s+([^;]+);", body):
        for item in decl.split(","):
            m = re.match(r"\s*(\w+)(?:\[(\d+)\])?\s*$", item)
            out.append((m.group(1), int(m.group(2) or 1)))
    return out


def test_options_struct_matches_header_layout():
    want = _header_struct_fields("sparsert_options")
    got = [(n, getattr(t, "_length_", 1)) for n, t in sp.Options._fields_]
    assert got == want
    assert ctypes.sizeof(sp.Options) == 4 * sum(c for _, c in want) == 25 * 4
    assert [n for n, _ in sp.TuneEntry._fields_] == [n for n, _ in _header_struct_fields("sparsert_tune_entry")]


def _host_plan(csr, N, **kw):
    return sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, N, host_only=True, **kw)


def _assert_plan_equal(plan, refp):
    info = plan.info()
    for k, v in refp["info"].items():
        assert info[k] == v, (k, info[k], v)
    for name, fid in FIELDS.items():
        got, want = plan.export(fid), refp[name]
        assert got.dtype == want.dtype, name
        assert got.tobytes() == want.tobytes(), name


CASES = [
    ("uniform", 64, 48, 100, 0.9, np.float32),
    ("uniform", 33, 17, 49, 0.5, np.float32),
    ("uniform", 256, 256, 1024, 0.9, np.float32),
    ("magnitude", 512, 512, 196, 0.9, np.float32),
    ("skewed", 300, 700, 64, 0.9, np.float32),
    ("skewed", 256, 2048, 784, 0.98, np.float16),
    ("uniform", 128, 96, 3136, 0.8, np.float16),
    ("uniform", 1, 1, 1, 0.0, np.float32),
]


@pytest.mark.parametrize("kind,M,K,N,sp_,dt", CASES)
def test_plan_is_bit_exact_against_numpy_spec(kind, M, K, N, sp_, dt):
    csr = {"uniform": synth.uniform_csr, "skewed": synth.skewed_csr,
           "magnitude": lambda *a, **k: synth.magnitude_csr(a[0], a[1], a[2], a[3], 1.0, **k)}[kind](
        M, K, sp_, 7, dtype=dt)
    plan = _host_plan(csr, N)
    _assert_plan_equal(plan, plan_ref.plan(csr.row_ptr, csr.col_idx, csr.vals, M, K, N))
    plan.destroy()


@pytest.mark.parametrize("vec,thr", [(1, 1), (2, 8), (4, 100000)])
def test_plan_overrides(vec, thr):
    csr = synth.skewed_csr(100, 200, 0.8, 3)
    plan = _host_plan(csr, 64, vec=vec, split_threshold=thr)
    _assert_plan_equal(plan, plan_ref.plan(csr.row_ptr, csr.col_idx, csr.vals, 100, 200, 64,
                                           vec=vec, split_threshold=thr))


@pytest.mark.parametrize("N,ldb,ldc,dt", [(100, 128, 0, np.float32), (64, 64, 200, np.float32), (96, 98, 102, np.float16),
                                          (196, 1024, 4096, np.float32), (64, 68, 64, np.int8)])
def test_leading_dimensions_in_the_plan(N, ldb, ldc, dt):
    """A wider row pitch of B changes the operand offsets and which vector widths are legal; nothing else."""
    csr = synth.int8_csr(70, 50, 0.8, 4) if dt == np.int8 else synth.uniform_csr(70, 50, 0.8, 4, dtype=dt)
    plan = _host_plan(csr, N, ldb=ldb, ldc=ldc)
    refp = plan_ref.plan(csr.row_ptr, csr.col_idx, csr.vals, 70, 50, N, ldb=ldb, ldc=ldc)
    _assert_plan_equal(plan, refp)
    info = plan.info()
    assert info["ldb"] == (ldb or N) and info["ldc"] == (ldc or N)
    assert info["ldb"] % info["vec"] == 0 and info["ldc"] % info["vec"] == 0
    plan.destroy()
    for bad in (dict(ldb=N - 1), dict(ldc=N - 1), dict(ldb=-4), dict(ldb=N + 1, vec=2), dict(ldc=N + 2, vec=4)):
        if N % bad.get("vec", 1):
            continue
        with pytest.raises(sp.SparseRTError) as e:
            _host_plan(csr, N, **bad)
        assert e.value.status == sp.EINVAL, bad
    ccsr, _ = synth.conv_weights_csr(4, 2, 0.5, 1)
    with pytest.raises(sp.SparseRTError) as e:
        sp.inspect(ccsr.row_ptr, ccsr.col_idx, ccsr.vals, 4, 18, 16, conv=(2, 4, 4), host_only=True, ldb=32)
    assert e.value.status == sp.EINVAL
    # the 2 GiB limit of the 32-bit operand offsets counts the pitch, not N
    with pytest.raises(sp.SparseRTError) as e:
        _host_plan(synth.uniform_csr(4, 1 << 16, 0.999, 1), 64, ldb=1 << 13)
    assert e.value.status == sp.EUNSUPPORTED


@pytest.mark.parametrize("N,conv", [(64, None), (63, None), (100, None), (1024, None), (42, (4, 6, 7))])
def test_int8_plan_is_bit_exact(N, conv):
    if conv:
        rng = np.random.default_rng(2)
        Wd = (rng.integers(-128, 128, size=(9, 4, 3, 3)) * (rng.random((9, 4, 3, 3)) < 0.3)).astype(np.int8)
        csr = synth.csr_from_mask(Wd.reshape(9, 36), Wd.reshape(9, 36) != 0)
    else:
        csr = synth.int8_csr(600 if N == 1024 else 50, 36, 0.8, 5)
    plan = _host_plan(csr, N, conv=conv)
    refp = plan_ref.plan(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, N, conv=conv)
    _assert_plan_equal(plan, refp)
    info = plan.info()
    assert info["dtype"] == sp.I8 and info["vec"] == (4 if N == 1024 else 1)   # four packed columns once there is enough work
    assert plan.export(sp.FIELD_P_VALS).dtype == np.int8
    # the stream carries the sign-extended value
    stream = plan.export(sp.FIELD_STREAM).reshape(-1, 2)
    if not conv:
        assert np.array_equal(stream[:, 1].view(np.int32), plan.export(sp.FIELD_P_VALS).astype(np.int32))
    plan.destroy()
    for bad in ({"vec": 2},) + (({"kernel": sp.KERNEL_SPEC, "spec_mode": sp.SPEC_LDS},) if conv else ()):
        with pytest.raises(sp.SparseRTError):
            _host_plan(csr, 64 if not conv else N, conv=conv, **bad)


def test_int8_rejects_a_reduction_axis_that_could_overflow():
    rp = np.array([0, 1], dtype=np.int32)
    ci = np.array([0], dtype=np.int32)
    v = np.ones(1, dtype=np.int8)
    assert _inspect_rc(rp, ci, v, 1, (1 << 17) - 1, 4) == sp.OK
    assert _inspect_rc(rp, ci, v, 1, 1 << 17, 4) == sp.EUNSUPPORTED


def test_natural_order_plan_is_bit_exact():
    """Load-balance ablation: identity permutation, no split rows, contiguous code blocks."""
    csr = synth.skewed_csr(100, 200, 0.8, 3)
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 100, 200, 64, host_only=True, natural_order=True)
    ref = plan_ref.plan(csr.row_ptr, csr.col_idx, csr.vals, 100, 200, 64, natural_order=True)
    _assert_plan_equal(plan, ref)
    info = plan.info()
    assert info["natural_order"] == 1 and info["n_split"] == 0
    assert np.array_equal(plan.export(sp.FIELD_PERM), np.arange(100))
    assert np.array_equal(plan.export(sp.FIELD_P_COL_IDX), csr.col_idx)
    plan.destroy()
    spec = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 100, 200, 64, host_only=True, natural_order=True,
                      kernel=sp.KERNEL_SPEC, spec_rows=7)
    assert spec.export(sp.FIELD_SPEC_GROUPS).tobytes() == plan_ref.spec_groups(100, 7, natural_order=True).tobytes()
    spec.destroy()
    with pytest.raises(sp.SparseRTError):
        opt = sp.Options()
        opt.natural_order = 2
        h = ctypes.c_void_p()
        sp._check(sp.raw.sparsert_inspect(csr.row_ptr.ctypes.data_as(ctypes.c_void_p), csr.col_idx.ctypes.data_as(ctypes.c_void_p),
                                       csr.vals.ctypes.data_as(ctypes.c_void_p), 100, 200, 64, ctypes.byref(opt), ctypes.byref(h)))


@pytest.mark.parametrize("Cin,Cout,H,W,dt", [(5, 7, 6, 9, np.float32), (16, 24, 14, 14, np.float16),
                                            (64, 64, 7, 7, np.float32)])
def test_conv_plan_is_bit_exact(Cin, Cout, H, W, dt):
    csr, _ = synth.conv_weights_csr(Cout, Cin, 0.8, 11, dtype=dt)
    plan = _host_plan(csr, H * W, conv=(Cin, H, W))
    _assert_plan_equal(plan, plan_ref.plan(csr.row_ptr, csr.col_idx, csr.vals, Cout, 9 * Cin, H * W,
                                           conv=(Cin, H, W)))


def test_plan_invariants_and_round_trip():
    csr = synth.skewed_csr(257, 300, 0.95, 5)
    # plant special bit patterns: they must come back untouched
    bits = csr.vals.view(np.uint32)
    bits[0], bits[1], bits[2] = 0x80000000, 0x7FC12345, 0x00000000  # -0.0, NaN payload, +0.0
    plan = _host_plan(csr, 128)
    perm, inv = plan.export(sp.FIELD_PERM), plan.export(sp.FIELD_INV_PERM)
    assert sorted(perm.tolist()) == list(range(257))
    assert np.array_equal(inv[perm], np.arange(257))
    prp, pci = plan.export(sp.FIELD_P_ROW_PTR), plan.export(sp.FIELD_P_COL_IDX)
    pv = plan.export(sp.FIELD_P_VALS)
    nn = np.diff(prp)
    assert np.all(nn[:-1] >= nn[1:])  # descending nnz
    bins = plan.export(sp.FIELD_BINS).reshape(-1, 4)
    assert bins[:, 2].sum() == 257 and bins[:, 3].sum() == csr.nnz
    assert np.array_equal(bins[:, 1], np.concatenate([[0], np.cumsum(bins[:, 2])[:-1]]))
    assert plan.export(sp.FIELD_HIST).sum() == 257
    # un-permuting reproduces the input CSR byte for byte
    rp = np.zeros(258, dtype=np.int32)
    rp[1:] = np.cumsum(nn[inv])
    assert rp.tobytes() == csr.row_ptr.tobytes()
    cols = np.concatenate([pci[prp[inv[m]]:prp[inv[m] + 1]] for m in range(257)])
    vals = np.concatenate([pv[prp[inv[m]]:prp[inv[m] + 1]] for m in range(257)])
    assert cols.tobytes() == csr.col_idx.tobytes()
    assert vals.tobytes() == csr.vals.tobytes()
    # split segments: every wave but the last gets the same share (Section 3.4)
    info = plan.info()
    seg = plan.export(sp.FIELD_SEGMENTS).reshape(info["n_split"], info["gy"] + 1)
    for s in range(info["n_split"]):
        assert seg[s, 0] == prp[s] and seg[s, -1] == prp[s + 1]
        d = np.diff(seg[s])
        assert np.all(d[:-1] == d[0]) or np.all(np.diff(d) <= 0)
        assert np.all(d >= 0)


def test_tiling_example_shares(golden):
    # Section 3.3 worked example: an extent divided into equal parts; the plan's
    # per-wave share of a split row uses the same ceil-division.
    for extent, parts, share in golden("tiling_example.txt")["split"].astype(int):
        assert -(-extent // parts) == share
    rp = np.array([0, 3056], dtype=np.int32)
    cols = np.arange(3056, dtype=np.int32)
    plan = sp.inspect(rp, cols, np.ones(3056, np.float32), 1, 3056, 512, host_only=True)
    seg = plan.export(sp.FIELD_SEGMENTS)
    assert np.array_equal(np.diff(seg), [764] * 4)  # 3056 / 4 waves


def _inspect_rc(row_ptr, col_idx, vals, M, K, N, **kw):
    try:
        sp.inspect(row_ptr, col_idx, vals, M, K, N, host_only=True, **kw).destroy()
        return 0
    except sp.SparseRTError as e:
        assert str(e)
        return e.status


def test_validation_errors():
    rp = np.array([0, 2, 3], dtype=np.int32)
    ci = np.array([0, 2, 1], dtype=np.int32)
    v = np.ones(3, dtype=np.float32)
    assert _inspect_rc(rp, ci, v, 2, 3, 8) == 0
    assert _inspect_rc(rp, ci, v, 0, 3, 8) == sp.EINVAL
    assert _inspect_rc(rp, ci, v, 2, 3, 0) == sp.EINVAL
    assert _inspect_rc(np.array([1, 2, 3], np.int32), ci, v, 2, 3, 8) == sp.EINVAL  # row_ptr[0]
    assert _inspect_rc(np.array([0, 3, 2], np.int32), ci, v, 2, 3, 8) == sp.EINVAL  # decreasing
    assert _inspect_rc(rp, np.array([0, 3, 1], np.int32), v, 2, 3, 8) == sp.EINVAL  # col >= K
    assert _inspect_rc(rp, np.array([0, -1, 1], np.int32), v, 2, 3, 8) == sp.EINVAL
    assert _inspect_rc(rp, np.array([2, 0, 1], np.int32), v, 2, 3, 8) == sp.EINVAL  # unsorted
    assert _inspect_rc(rp, np.array([1, 1, 1], np.int32), v, 2, 3, 8) == sp.EINVAL  # duplicate
    assert _inspect_rc(rp, ci, v, 2, 3, 8, vec=3) == sp.EINVAL
    assert _inspect_rc(rp, ci, v, 2, 3, 9, vec=2) == sp.EINVAL
    assert _inspect_rc(rp, ci, v, 2, 3, 8, vec=8) == sp.EINVAL  # 8 is f16 only
    assert _inspect_rc(rp, ci, v, 2, 3, 8, dtype=7) == sp.EINVAL
    assert _inspect_rc(rp, ci, v, 2, 3, 8, conv=(1, 2, 4)) == sp.EINVAL  # K != 9*Cin
    assert _inspect_rc(rp, ci, v, 2, 9, 8, conv=(1, 2, 4)) == 0
    assert _inspect_rc(rp, ci, v, 2, 9, 8, conv=(1, 2, 4), batch=2) == sp.OK
    assert _inspect_rc(rp, ci, v, 2, 9, 8, conv=(1, 2, 4), batch=70000) == sp.EINVAL
    assert _inspect_rc(rp, ci, v, 2, 9, 8, conv=(1, 2, 4), batch=-1) == sp.EINVAL
    assert _inspect_rc(rp, ci, v, 2, 9, 7, conv=(1, 2, 4)) == sp.EINVAL  # N != H*W
    assert _inspect_rc(rp, ci, v, 2, 70000, 70000) == sp.EUNSUPPORTED  # >= 2 GiB operands


def test_null_pointers_and_host_only_execution_are_rejected():
    lib = sp.raw
    out = ctypes.c_void_p(123)
    assert lib.sparsert_inspect(None, None, None, 1, 1, 1, None, ctypes.byref(out)) == sp.EINVAL
    assert out.value is None
    assert lib.sparsert_inspect(None, None, None, 1, 1, 1, None, None) == sp.EINVAL
    assert lib.sparsert_spmm(None, 16, 16, None) == sp.EINVAL
    csr = synth.uniform_csr(8, 8, 0.5, 1)
    plan = _host_plan(csr, 8)
    assert lib.sparsert_spmm(plan.handle, 4096, 8192, None) == sp.EINVAL  # host-only plan
    assert "host_only" in sp.last_error()
    assert lib.sparsert_spmm(plan.handle, 4097, 8192, None) == sp.EINVAL  # misaligned
    assert lib.sparsert_spmm(plan.handle, None, 8192, None) == sp.EINVAL
    assert lib.sparsert_conv3x3(plan.handle, 4096, 8192, None) == sp.EINVAL
    need = ctypes.c_size_t()
    assert lib.sparsert_plan_export(plan.handle, 99, None, 0, ctypes.byref(need)) == sp.EINVAL
    assert lib.sparsert_plan_export(plan.handle, sp.FIELD_PERM, None, 0, ctypes.byref(need)) == 0
    assert need.value == 32
    buf = (ctypes.c_int32 * 4)()
    assert lib.sparsert_plan_export(plan.handle, sp.FIELD_PERM, buf, 16, None) == sp.EINVAL
    lib.sparsert_plan_destroy(None)


def test_inspect_from_several_threads_at_once():
    """Plans made concurrently (code generation and assembling included) equal the ones made alone."""
    import threading
    cases = [synth.magnitude_csr(150 + 10 * i, 200, 0.9, i) for i in range(6)]

    def code_of(a):
        p = sp.inspect(a.row_ptr, a.col_idx, a.vals, a.M, a.K, 196, kernel=sp.KERNEL_SPEC, spec_rows=8,
                       spec_ksplit=2, host_only=True)
        code = p.export(sp.FIELD_SPEC_CODE).tobytes()
        p.destroy()
        return code

    alone = [code_of(a) for a in cases]
    together, errors = [None] * len(cases), []

    def work(i):
        try:
            for _ in range(3):
                together[i] = code_of(cases[i])
        except Exception as ex:   # reported by the asserting thread
            errors.append((i, repr(ex)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(len(cases))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors
    assert together == alone


@pytest.mark.parametrize("M,K,N,batch,rows,ksplit", [
    (3072, 768, 1024, 1, 96, 4),     # c3: rows capped at 96, four parts already give 2048 waves
    (768, 3072, 1024, 1, 48, 8),     # c3t: 16 blocks x 16 tiles x 8 parts = 2048 waves
    (256, 128, 784, 1, 3, 1),        # short reduction axis: no split, about 1024 waves
    (512, 512, 196, 1, 8, 8),
    (512, 512, 196, 4, 32, 8),       # the problems of a batch bring their own waves
    (64, 1024, 64, 1, 1, 8),         # tiny: one row per block, everything else from the split
    (1024, 4096, 784, 1, 54, 8),     # 52 rows would make 20 blocks x 13 tiles = 260 workgroups for 256 compute units; 54 make 247
    (256, 256, 3136, 1, 14, 1),      # 12 rows: 22 x 13 = 286 workgroups of four tiles; 14 rows: 19 x 13 = 247
    (1024, 1024, 3136, 1, 103, 4),   # 96 rows: 11 blocks x 49 tiles = 539 workgroups, a thin third round; 103 rows: 10 x 49 = 490
    (2048, 1000, 4096, 1, 96, 2),    # 22 x 64 = 1408 workgroups: the last round is half full, nothing to gain
    (2048, 2048, 4096, 1, 64, 1),    # large and 98 % sparse with a long reduction axis: the LDS-staged variant, eight waves of 64 rows
    (64, 256, 3136, 1, 3, 1),        # blocks of a few rows are left alone
])
def test_untuned_defaults_of_the_generated_kernel(M, K, N, batch, rows, ksplit):
    """spec_rows = spec_ksplit = 0: as many rows per block as leave about two waves per SIMD
    (2048 waves), the reduction axis split over up to eight waves where K >= 512."""
    csr = synth.uniform_csr(M, K, 0.98, 11)
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, M, K, N, host_only=True, kernel=sp.KERNEL_SPEC, batch=batch)
    info = plan.info()
    assert (info["spec_rows"], info["spec_ksplit"]) == (rows, ksplit)
    # an explicit row count keeps the split off unless it is asked for
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, M, K, N, host_only=True, kernel=sp.KERNEL_SPEC, spec_rows=2)
    assert plan.info()["spec_ksplit"] == 1


@pytest.mark.parametrize("mode", [sp.SPEC_DIRECT, sp.SPEC_LDS])
@pytest.mark.parametrize("rows", [1, 7, 24])
def test_generated_kernel_plan_assembles_on_the_host(rows, mode):
    csr = synth.magnitude_csr(100, 300, 0.9, 3)
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 100, 300, 196, host_only=True,
                      kernel=sp.KERNEL_SPEC, spec_rows=rows, spec_mode=mode)
    info = plan.info()
    assert info["kernel"] == sp.KERNEL_SPEC and info["spec_rows"] == rows and info["spec_mode"] == mode
    groups = plan.export(sp.FIELD_SPEC_GROUPS)
    assert groups.tobytes() == plan_ref.spec_groups(100, rows).tobytes()
    assert np.bincount(groups).max() <= rows
    code = plan.export(sp.FIELD_SPEC_CODE)
    assert code[:4].tobytes() == b"\x7fELF" and code.size == info["spec_code_bytes"]
    # block balance: nonzeros per block within one row's worth of each other
    nn = np.diff(plan.export(sp.FIELD_P_ROW_PTR))
    per_block = np.bincount(groups, weights=nn)
    assert per_block.max() - per_block.min() <= nn.max()
    cols = plan.export(sp.FIELD_SPEC_COLUMNS)
    assert cols[:info["spec_groups"]].sum() >= len(np.unique(csr.col_idx))
    # the row-walk plan arrays are unaffected by the choice of executor
    _assert_plan_equal(plan, {**plan_ref.plan(csr.row_ptr, csr.col_idx, csr.vals, 100, 300, 196),
                              "info": {"M": 100, "nnz": csr.nnz}})


@pytest.mark.parametrize("rows", [2, 8, 16, 200])
def test_row_swizzle_groups_are_bit_exact_and_balanced(rows):
    M, K = 256, 512
    csr = synth.clustered_csr(M, K, 0.9, 3, clusters=8)
    args = (csr.row_ptr, csr.col_idx, csr.vals, M, K, 196)
    plan = sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, spec_rows=rows, spec_swizzle=True, spec_depth=4)
    info = plan.info()
    assert info["spec_swizzle"] == 1
    groups = plan.export(sp.FIELD_SPEC_GROUPS)
    prp, pci = plan.export(sp.FIELD_P_ROW_PTR), plan.export(sp.FIELD_P_COL_IDX)
    assert groups.tobytes() == plan_ref.spec_groups_swizzled(prp, pci, M, K, rows).tobytes()
    assert np.bincount(groups).max() <= rows
    nn = np.diff(prp)
    per_block = np.bincount(groups, weights=nn)
    assert per_block.max() - per_block.min() <= nn.max()          # same balance bound as the serpentine deal
    plain = sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, spec_rows=rows, spec_depth=4)
    fetched = lambda p: int(p.export(sp.FIELD_SPEC_COLUMNS)[:p.info()["spec_groups"]].sum())
    if rows in (8, 16):   # eight hidden clusters: a swizzled block fetches far fewer rows of B
        assert fetched(plan) < 0.65 * fetched(plain), (fetched(plan), fetched(plain))
    else:
        assert fetched(plan) <= fetched(plain)
    plan.destroy()
    plain.destroy()


def test_generated_kernel_ksplit_lds_budget():
    """(KS-1) x rows x 4 x lanes bytes of exchange area: within the 160 KiB of a compute unit in
    one phase, else as many rows per phase as fit."""
    csr = synth.uniform_csr(200, 64, 0.9, 2)
    args = (csr.row_ptr, csr.col_idx, csr.vals, 200, 64, 100)
    plan = sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, spec_rows=200, spec_ksplit=8)
    assert plan.info()["spec_lds_bytes"] == 7 * 91 * 256 <= 160 * 1024 < 7 * 92 * 256   # three phases of 91, 91, 18 rows
    plan.destroy()
    plan = sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, spec_rows=200, spec_ksplit=8, spec_lanes=16)
    info = plan.info()
    assert info["spec_lds_bytes"] == 7 * 200 * 64 and info["spec_lanes"] == 15   # 100 columns in 7 balanced tiles
    plan.destroy()


def test_workgroups_whose_registers_do_not_fit_a_compute_unit_are_refused():
    """Sixteen waves are four per SIMD: at most 128 registers each.  The hardware queue rejects a
    dispatch that does not fit (and the process with it), so the inspector must."""
    csr = synth.uniform_csr(480, 600, 0.9, 1)
    args = (csr.row_ptr, csr.col_idx, csr.vals, 480, 600, 130)
    for kw in (dict(spec_mode=sp.SPEC_LDS, spec_rows=103, spec_tiles=16), dict(spec_rows=120, spec_tiles=16),
               dict(spec_mode=sp.SPEC_LDS, spec_rows=128, spec_tiles=16)):
        with pytest.raises(sp.SparseRTError) as e:
            sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, **kw)
        assert e.value.status == sp.EINVAL and "fit a compute unit" in str(e.value), kw
    for kw in (dict(spec_mode=sp.SPEC_LDS, spec_rows=60, spec_tiles=16), dict(spec_rows=96, spec_tiles=16),
               dict(spec_rows=200, spec_ksplit=8), dict(spec_mode=sp.SPEC_LDS, spec_rows=128, spec_tiles=8)):
        plan = sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, **kw)
        info = plan.info()
        plan.destroy()
    # eight waves are two per SIMD, 256 registers each: two blocks of 232 rows, the fetch ring of 20 and 4 more
    csr = synth.uniform_csr(464, 300, 0.9, 1)
    args = (csr.row_ptr, csr.col_idx, csr.vals, 464, 300, 130)
    sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, spec_rows=232, spec_ksplit=8).destroy()
    for kw in (dict(spec_rows=233, spec_ksplit=8), dict(spec_rows=232, spec_ksplit=8, spec_depth=32)):
        with pytest.raises(sp.SparseRTError) as e:
            sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, **kw)
        assert e.value.status == sp.EINVAL, kw


def test_generated_kernel_option_errors():
    csr = synth.uniform_csr(16, 18, 0.5, 1)
    args = (csr.row_ptr, csr.col_idx, csr.vals, 16, 18, 8)
    for kw in ({"spec_tiles": 3}, {"spec_mode": 9}, {"spec_depth": 99}, {"spec_rows": 500}, {"spec_lanes": 48},
               {"spec_ksplit": 3}, {"spec_ksplit": 2, "spec_mode": sp.SPEC_LDS}, {"spec_lanes": 32, "spec_mode": sp.SPEC_LDS},
               {"spec_vec": 2}, {"spec_vec": 4}, {"spec_vec": 3}):   # packed columns are for half / int8 plans
        with pytest.raises(sp.SparseRTError) as e:
            sp.inspect(*args, host_only=True, kernel=sp.KERNEL_SPEC, **kw)
        assert e.value.status == sp.EINVAL, kw
    ccsr, _ = synth.conv_weights_csr(4, 2, 0.5, 1)
    with pytest.raises(sp.SparseRTError) as e:
        sp.inspect(ccsr.row_ptr, ccsr.col_idx, ccsr.vals, 4, 18, 16, conv=(2, 4, 4), host_only=True,
                   kernel=sp.KERNEL_SPEC, spec_mode=sp.SPEC_LDS)
    assert e.value.status == sp.EUNSUPPORTED
    sp.inspect(ccsr.row_ptr, ccsr.col_idx, ccsr.vals, 4, 18, 16, conv=(2, 4, 4), host_only=True,
               kernel=sp.KERNEL_SPEC).destroy()
    # tune validates before it touches the GPU
    out, rep = ctypes.c_void_p(1), sp.TuneReport()
    rc = sp.raw.sparsert_tune(None, None, None, 1, 1, 1, None, 16, 16, None, ctypes.byref(out), ctypes.byref(rep))
    assert rc == sp.EINVAL and out.value is None


ALL_FIELDS = dict(FIELDS, spec_groups=sp.FIELD_SPEC_GROUPS, spec_columns=sp.FIELD_SPEC_COLUMNS,
                  spec_code=sp.FIELD_SPEC_CODE, info=sp.FIELD_INFO)


@pytest.mark.parametrize("opts", [dict(), dict(vec=2, split_threshold=3), dict(kernel=sp.KERNEL_SPEC, spec_rows=7, spec_ksplit=4),
                                  dict(kernel=sp.KERNEL_SPEC, spec_rows=12, spec_mode=sp.SPEC_LDS, spec_tiles=2),
                                  dict(natural_order=True, batch=3)])
def test_saved_plan_loads_to_the_same_plan(opts):
    """Plan persistence: every exported array, the info block and the generated code survive."""
    csr = synth.skewed_csr(60, 300, 0.9, 4)
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 60, 300, 196, host_only=True, **opts)
    blob = plan.save()
    again = sp.load(blob, host_only=True)
    for name, fid in ALL_FIELDS.items():
        assert again.export(fid).tobytes() == plan.export(fid).tobytes(), name
    assert again.save() == blob
    plan.destroy()
    again.destroy()


def test_saved_conv_half_and_int8_plans_round_trip():
    ccsr, _ = synth.conv_weights_csr(8, 6, 0.7, 2, dtype=np.float16)
    for csr, kw in ((ccsr, dict(conv=(6, 5, 7), batch=2, kernel=sp.KERNEL_SPEC, spec_rows=3)),
                    (synth.int8_csr(30, 64, 0.8, 3), dict(kernel=sp.KERNEL_SPEC, spec_rows=5, spec_vec=4))):
        N = 35 if "conv" in kw else 64
        plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, N, host_only=True, **kw)
        again = sp.load(plan.save(), host_only=True)
        assert again.dtype == plan.dtype
        for name, fid in ALL_FIELDS.items():
            assert again.export(fid).tobytes() == plan.export(fid).tobytes(), name
        plan.destroy()
        again.destroy()


def test_load_rejects_damaged_blobs():
    csr = synth.uniform_csr(20, 30, 0.8, 1)
    plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 20, 30, 64, host_only=True, kernel=sp.KERNEL_SPEC, spec_rows=4)
    blob = plan.save()
    plan.destroy()

    def status(b):
        try:
            sp.load(b, host_only=True).destroy()
            return sp.OK
        except sp.SparseRTError as e:
            assert str(e)
            return e.status

    assert status(blob) == sp.OK
    assert status(blob[:10]) == sp.EINVAL                                   # too short for a header
    assert status(blob[:-1]) == sp.EINVAL and status(blob + b"x") == sp.EINVAL   # truncated, padded
    assert status(b"XXXX" + blob[4:]) == sp.EINVAL                          # not ours
    flipped = bytearray(blob)
    flipped[len(blob) // 2] ^= 0x40
    assert status(bytes(flipped)) == sp.EINVAL                              # checksum
    other = bytearray(blob)
    other[4] = 99
    assert status(bytes(other)) == sp.EUNSUPPORTED                          # another format version
    h = ctypes.c_void_p()
    assert sp.raw.sparsert_plan_load(None, 100, 1, ctypes.byref(h)) == sp.EINVAL
    assert sp.raw.sparsert_plan_save(None, None, 0, None) == sp.EINVAL


def test_staged_default_for_large_and_very_sparse_products():
    """With no tiling option set, a large fp32 SpMM with a long reduction axis and at least 94.5 %
    zeros takes the LDS-staged variant with eight waves; anything else keeps DIRECT."""
    def default_mode(M, K, N, sparsity, dtype=np.float32, **kw):
        csr = synth.uniform_csr(M, K, sparsity, 5, dtype=dtype)
        plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, M, K, N, host_only=True, kernel=sp.KERNEL_SPEC, **kw)
        info = plan.info()
        plan.destroy()
        return info["spec_mode"], info["spec_tiles"], info["spec_rows"]
    assert default_mode(2048, 1024, 4096, 0.97) == (sp.SPEC_LDS, 8, 64)      # 2048 x 64 tiles = 131072
    assert default_mode(4096, 1024, 3136, 0.96)[:2] == (sp.SPEC_LDS, 8)
    assert default_mode(2048, 1024, 4096, 0.90)[0] == sp.SPEC_DIRECT          # too dense: the multiply-adds dominate
    assert default_mode(2048, 512, 4096, 0.97)[0] == sp.SPEC_DIRECT           # short reduction axis
    assert default_mode(2048, 1024, 3136, 0.97)[0] == sp.SPEC_DIRECT          # 2048 x 49 tiles: under 512 per compute unit
    assert default_mode(2048, 1024, 4096, 0.97, dtype=np.float16)[0] == sp.SPEC_DIRECT
    assert default_mode(2048, 1024, 4096, 0.97, spec_rows=48)[0] == sp.SPEC_DIRECT   # any tiling option: the caller's call
    assert default_mode(2048, 1024, 4096, 0.97, spec_mode=sp.SPEC_DIRECT)[0] == sp.SPEC_DIRECT
    assert default_mode(2048, 1024, 2048, 0.97, batch=2)[:2] == (sp.SPEC_LDS, 8)      # the problems of a batch count
    assert default_mode(512, 1024, 4096, 0.97, batch=4)[0] == sp.SPEC_DIRECT          # few rows: not what was measured


def test_kernel_name_of_row_walk_plans_is_a_symbol_of_the_library():
    """SPARSERT_FIELD_KERNEL_NAME is what a kernel trace shows: the demangled instantiation of
    rows_kernel, or - for half storage, whose type the profiler's demangler does not know - the
    symbol itself.  Either way it must name a kernel this library holds."""
    import shutil
    import subprocess
    if shutil.which("nm") is None:
        pytest.skip("nm is not installed")
    lib = os.path.join(os.path.dirname(sp.__file__), "libsparsert.so")
    mangled = {l.split()[-1] for l in subprocess.run(["nm", "-D", lib], capture_output=True, text=True, check=True).stdout.splitlines() if l.split()}
    demangled = {l.split(None, 2)[-1] for l in subprocess.run(["nm", "-D", "-C", lib], capture_output=True, text=True, check=True).stdout.splitlines() if "rows_kernel" in l}
    seen = set()
    for dtype in (np.float32, np.float16, np.int8):
        csr = synth.int8_csr(24, 40, 0.8, 2) if dtype == np.int8 else synth.uniform_csr(24, 40, 0.8, 2, dtype=dtype)
        for vec in (1, 4) if dtype == np.int8 else (1, 2, 4):
            plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, 24, 40, 64, host_only=True, kernel=sp.KERNEL_ROWS, vec=vec)
            name = plan.kernel_name()
            plan.destroy()
            assert name in (mangled if dtype == np.float16 else demangled), name
            seen.add(name)
    ccsr, _ = synth.conv_weights_csr(4, 2, 0.5, 1, dtype=np.float16)
    plan = sp.inspect(ccsr.row_ptr, ccsr.col_idx, ccsr.vals, 4, 18, 16, conv=(2, 4, 4), host_only=True, kernel=sp.KERNEL_ROWS)
    assert plan.kernel_name() in mangled
    plan.destroy()
    assert len(seen) == 8
