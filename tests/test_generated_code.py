"""The code generator's output, checked statically on the host: every memory access of every
generated block stays inside its buffer, no register is used before its load has been waited
for (see asm_check.py).  Runs over the executor variants, storage types, convolution, batch,
leading dimensions and a randomised grid - with no GPU."""
import os

import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

import asm_check
from paper_2008_11849_amd import sparsert as sp, synth

ESZ = {np.dtype(np.float32): (4, 4), np.dtype(np.float16): (2, 2), np.dtype(np.int8): (1, 4)}


def _generated(csr, N, tmp_path, **opts):
    """Host-only plan with the generated kernel; returns (assembly text, plan info)."""
    path = os.path.join(str(tmp_path), "kernel.s")
    os.environ["SPARSERT_DUMP_ASM"] = path
    try:
        plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, N, host_only=True, kernel=sp.KERNEL_SPEC, **opts)
    finally:
        del os.environ["SPARSERT_DUMP_ASM"]
    info = plan.info()
    plan.destroy()
    return open(path).read(), info


def _clean(csr, N, tmp_path, **opts):
    text, info = _generated(csr, N, tmp_path, **opts)
    esz, osz = ESZ[csr.vals.dtype]
    problems, stats = asm_check.check(text, info, esz, osz)
    assert not problems, problems[:5]
    return info, stats


def _csr(dtype, M, K, sparsity, seed):
    return synth.int8_csr(M, K, sparsity, seed) if dtype == np.int8 else synth.uniform_csr(M, K, sparsity, seed, dtype=dtype)


@pytest.mark.parametrize("dtype", [np.float32, np.float16, np.int8])
@pytest.mark.parametrize("opts", [dict(spec_rows=1), dict(spec_rows=7, spec_tiles=2), dict(spec_rows=16, spec_ksplit=2),
                                  dict(spec_rows=24, spec_ksplit=8), dict(spec_rows=200, spec_ksplit=8), dict(spec_rows=210, spec_ksplit=8), dict(spec_rows=9, spec_depth=3),
                                  dict(spec_rows=5, spec_swizzle=True), dict(spec_rows=8, spec_lanes=16, spec_ksplit=4), dict()])
@pytest.mark.parametrize("N", [1, 49, 64, 196, 300])
def test_direct_and_k_split_blocks_stay_in_bounds(dtype, opts, N, tmp_path):
    csr = _csr(dtype, 210, 333, 0.9, N)
    info, stats = _clean(csr, N, tmp_path, **opts)
    esz, osz = ESZ[np.dtype(dtype)]
    # the checker saw the far corner of both matrices: the last row of B and of C are reached
    assert stats["max_out_end"] == 210 * N * osz
    assert stats["max_in_end"] <= 333 * N * esz and stats["loads"] > 0 and stats["stores"] >= 210



def test_code_prefetch_is_checked(tmp_path):
    csr = synth.uniform_csr(300, 500, 0.8, 2)
    text, info = _generated(csr, 130, tmp_path, spec_rows=96, spec_ksplit=2, spec_prefetch=1)
    problems, stats = asm_check.check(text, info, 4, 4)
    assert not problems and stats["prefetch_loads"] >= 2 and info["spec_prefetch"] == stats["prefetch_loads"]   # blocks of more than 8 KiB
    off, info2 = _generated(csr, 130, tmp_path, spec_rows=96, spec_ksplit=2)
    assert asm_check.check(off, info2, 4, 4) == ([], dict(stats, prefetch_loads=0)) and info2["spec_prefetch"] == 0
    # a prefetch whose offset runs ahead of its mask would read past the block: the checker sees it
    bad = text.replace("global_load_dword v2, v4, s[18:19] offset:128", "global_load_dword v2, v4, s[18:19] offset:256", 1)
    assert any("not covered by its length mask" in p for p in asm_check.check(bad, info, 4, 4)[0])


@pytest.mark.parametrize("N,vec,dtype", [(64, 2, np.float16), (130, 2, np.float16), (64, 4, np.int8), (260, 4, np.int8)])
@pytest.mark.parametrize("ks", [1, 4])
def test_packed_columns_stay_in_bounds(N, vec, dtype, ks, tmp_path):
    _clean(_csr(dtype, 100, 200, 0.85, 5), N, tmp_path, spec_rows=12, spec_vec=vec, spec_ksplit=ks)


@pytest.mark.parametrize("dtype", [np.float32, np.float16, np.int8])
@pytest.mark.parametrize("waves", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("K", [5, 128, 129, 515])
def test_lds_staged_blocks_stay_in_bounds(waves, K, dtype, tmp_path):
    csr = _csr(dtype, 90, K, 0.8, K)
    info, stats = _clean(csr, 130, tmp_path, spec_rows=6, spec_mode=sp.SPEC_LDS, spec_tiles=waves)
    assert stats["lds"] > 0 and stats["max_lds_end"] <= info["spec_lds_bytes"]


@pytest.mark.parametrize("ldb,ldc,batch", [(0, 0, 3), (136, 0, 1), (0, 4096, 1), (200, 264, 2)])
def test_leading_dimensions_and_batches_stay_in_bounds(ldb, ldc, batch, tmp_path):
    N = 130
    csr = synth.uniform_csr(77, 150, 0.9, 2)
    for opts in (dict(spec_rows=8), dict(spec_rows=16, spec_ksplit=4), dict(spec_rows=8, spec_mode=sp.SPEC_LDS, spec_tiles=4)):
        info, stats = _clean(csr, N, tmp_path, ldb=ldb, ldc=ldc, batch=batch, **opts)
        assert stats["max_out_end"] == (76 * (ldc or N) + N) * 4      # the extent of one matrix of the batch
        assert stats["max_in_end"] <= (149 * (ldb or N) + N) * 4


@pytest.mark.parametrize("Cin,Cout,H,W", [(3, 5, 1, 1), (4, 6, 2, 3), (16, 24, 14, 14), (6, 10, 9, 13), (8, 4, 56, 56)])
@pytest.mark.parametrize("dtype", [np.float32, np.float16, np.int8])
def test_convolution_blocks_stay_in_bounds(Cin, Cout, H, W, dtype, tmp_path):
    csr, _ = synth.conv_weights_csr(Cout, Cin, 0.7, H + W)
    if dtype == np.int8:
        csr = synth.CSR(csr.M, csr.K, csr.row_ptr, csr.col_idx, synth.quantise_weights(csr.vals))
    else:
        csr = synth.CSR(csr.M, csr.K, csr.row_ptr, csr.col_idx, csr.vals.astype(dtype))
    for opts in (dict(spec_rows=3), dict(spec_rows=4, spec_ksplit=4), dict(batch=4)):
        info, stats = _clean(csr, H * W, tmp_path, conv=(Cin, H, W), **opts)
        esz = ESZ[np.dtype(dtype)][0]
        # a tap at the bottom right of the last channel reaches the end of the padded descriptor, never beyond
        assert stats["max_in_end"] <= (Cin * H * W + 2 * (W + 1)) * esz


def test_the_checker_catches_planted_mistakes(tmp_path):
    """The checker itself: one edit of a clean kernel per property it guards."""
    csr = synth.uniform_csr(64, 200, 0.9, 1)
    text, info = _generated(csr, 100, tmp_path, spec_rows=16, spec_ksplit=4)
    assert asm_check.check(text, info, 4, 4)[0] == []
    lines = text.splitlines()

    def edited(find, replace_with, nth=0):
        idx = [i for i, l in enumerate(lines) if find(l)][nth]
        out = list(lines)
        out[idx] = replace_with(out[idx])
        return "\n".join(out)

    import re
    # a row offset one row past the end of B
    t = edited(lambda l: l.startswith("\ts_mov_b32 s62, "), lambda l: "\ts_mov_b32 s62, 0x%x" % (200 * 100 * 4))
    assert any("operand" in p for p in asm_check.check(t, info, 4, 4)[0])
    # a wait that lets one more load stay in flight than the code assumes
    t = edited(lambda l: "s_waitcnt vmcnt(" in l, lambda l: re.sub(r"vmcnt\((\d+)\)", lambda m: "vmcnt(%d)" % (int(m.group(1)) + 1), l))
    assert any("in flight" in p for p in asm_check.check(t, info, 4, 4)[0])
    # an LDS offset beyond the exchange area
    t = edited(lambda l: l.startswith("\tds_write_"), lambda l: re.sub(r"offset:\d+", "offset:%d" % info["spec_lds_bytes"], l))
    assert any("group segment" in p for p in asm_check.check(t, info, 4, 4)[0])
    # a register above the allocation
    t = edited(lambda l: l.startswith("\tv_fmac_f32"), lambda l: re.sub(r"v_fmac_f32_e32 v\d+", "v_fmac_f32_e32 v255", l))
    assert any("next_free_vgpr" in p for p in asm_check.check(t, info, 4, 4)[0])
    # a store below the start of C's last row ... moved past the end of C
    t = edited(lambda l: l.startswith("\tbuffer_store_dword"), lambda l: l, 0)
    idx = [i for i, l in enumerate(lines) if l.startswith("\tbuffer_store_dword")][0]
    out = list(lines)
    out[idx - 1] = re.sub(r"0x[0-9a-f]+", "0x%x" % (64 * 100 * 4), out[idx - 1])
    assert any("result" in p for p in asm_check.check("\n".join(out), info, 4, 4)[0])
    # a block that runs into the next one
    idx = [i for i, l in enumerate(lines) if l.strip() == "s_endpgm"][2]
    out = list(lines)
    out[idx] = "\ts_nop 0"
    assert any("does not end" in p for p in asm_check.check("\n".join(out), info, 4, 4)[0])


@settings(max_examples=60, deadline=None, suppress_health_check=[HealthCheck.function_scoped_fixture])
@given(M=st.integers(1, 130), K=st.integers(1, 400), N=st.integers(1, 330), sparsity=st.sampled_from([0.0, 0.5, 0.9, 0.99]),
       rows=st.sampled_from([0, 1, 3, 8, 31, 96]), ks=st.sampled_from([0, 1, 2, 4, 8]), mode=st.sampled_from([1, 1, 2]),
       dtype=st.sampled_from([np.float32, np.float16, np.int8]), swizzle=st.booleans(), seed=st.integers(0, 99), prefetch=st.booleans())
def test_random_generated_kernels_are_clean(M, K, N, sparsity, rows, ks, mode, dtype, swizzle, seed, prefetch, tmp_path):
    csr = _csr(dtype, M, K, sparsity, seed)
    opts = dict(spec_rows=rows, spec_ksplit=ks, spec_mode=mode, spec_swizzle=swizzle, spec_prefetch=int(prefetch))
    if mode == sp.SPEC_LDS:
        opts["spec_ksplit"] = 0
    try:
        text, info = _generated(csr, N, tmp_path, **opts)
    except sp.SparseRTError as e:
        assert e.status in (sp.EINVAL, sp.EUNSUPPORTED)   # a refusal is fine, a broken kernel is not
        return
    problems, _ = asm_check.check(text, info, *ESZ[np.dtype(dtype)])
    assert not problems, (opts, problems[:5])
