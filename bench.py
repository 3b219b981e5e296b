#!/usr/bin/env python3
"""Benchmark of the SpMM / sparse-conv hot path on one MI355X.

A "step" is one pass of the hot path over one batch of synthetic input for the chosen
workload.  Default workload c3 = the Transformer FC pair at 95 % sparsity: the 3072x768
projection and its transposed 768x3072 partner, both against N = 1024 activation columns
(batch 8 x 128 tokens).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: effective GFLOP/s (2*nnz*N / time), the speedup over a dense GEMM of
the same shape on the same GPU, the roofline position of the dominant kernel (timed live
with HIP events on the launch stream) and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
FP32_VECTOR_PEAK_TF = 157.3  # MI355X vector fp32


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--dtype", default="f32", choices=["f32", "f16", "i8"],
                    help="storage type; i8: int8 weights and activations, exact int32 results")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cases", action="store_true", help="skip the side table of the other configs")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-operand timing of every layer")
    ap.add_argument("--kernel", default="tune", choices=["tune", "rows", "spec"],
                    help="tune: sparsert_tune picks the executor per layer (default); rows/spec: fixed family")
    ap.add_argument("--plan-file", default=None,
                    help="JSON of tuned per-layer options: read if it exists (no tuning in this process, so a "
                         "profile sees only the chosen kernels), else written after tuning")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured copy / multiply-add / operand-fetch ceilings")
    ap.add_argument("--no-traffic", action="store_true",
                    help="skip the two rocprofv3 --pmc child runs (FETCH_SIZE, WRITE_SIZE) that measure the bytes leaving the L2 caches")
    ap.add_argument("--pmc-mode", action="store_true",
                    help="for rocprofv3 --pmc runs: a 256 MiB copy (counter calibration), then 20 launches "
                         "of every layer of the workload, nothing else")
    return ap.parse_args()


class Layer:
    """One sparse layer resident on the GPU: plan, input, output and its dense twin."""

    PLAN_KEYS = ("kernel", "vec", "split_threshold", "spec_mode", "spec_rows", "spec_tiles", "spec_ksplit",
                 "spec_swizzle", "spec_vec", "spec_prefetch")

    def __init__(self, case, torch, sp, kernel="tune", fixed=None):
        import numpy as np
        self.case, self.torch, self.sp = case, torch, sp
        csr = case.csr
        dev = torch.device("cuda:0")
        self.is_conv = case.conv is not None
        self.M, self.K, self.N, self.nnz = csr.M, csr.K, case.N, csr.nnz
        self.int8 = csr.vals.dtype == np.int8
        tdt = torch.float16 if csr.vals.dtype == np.float16 else torch.int32 if self.int8 else torch.float32
        self.esize = 2 if tdt == torch.float16 else 1 if self.int8 else 4       # bytes of an input element
        self.osize = 2 if tdt == torch.float16 else 4                           # bytes of an output element
        # dense twin: same storage type; int8 has no dense convolution here and int8 GEMM only through
        # torch._int_mm, so int8 layers are compared with the half-precision dense kernels (values exact in half)
        ddt = torch.float16 if self.int8 else tdt
        self.dense_kind = "f16 (int8 operands widened)" if self.int8 else str(ddt).replace("torch.", "")
        if self.is_conv:
            self.inp = torch.from_numpy(case.X).to(dev)
            self.out = torch.empty((1, csr.M, case.conv[1], case.conv[2]), dtype=tdt, device=dev)
            self.Wd = torch.from_numpy(case.Wdense).to(dev).to(ddt)
            self.dense_in = self.inp.to(ddt)
            self.fn = sp.raw.sparsert_conv3x3
        else:
            self.inp = torch.from_numpy(case.B).to(dev)
            self.out = torch.empty((csr.M, case.N), dtype=tdt, device=dev)
            self.Ad = torch.from_numpy(csr.todense(np.float32)).to(dev).to(ddt)
            self.dense_in = self.inp.to(ddt)
            self.fn = sp.raw.sparsert_spmm
            if self.int8:
                try:   # the int8 GEMM of the BLAS library, where this build of torch has it
                    A8 = torch.from_numpy(csr.todense(np.int8)).to(dev)
                    torch._int_mm(A8, self.inp)
                    torch.cuda.synchronize()
                    self.Ad, self.dense_in, self.dense_kind = A8, self.inp, "int8 (torch._int_mm)"
                except Exception:
                    pass
        self.tuned = None
        if fixed is not None:
            fixed = dict(fixed, spec_prefetch=1 if fixed.get("spec_prefetch") else 0)   # the plan reports lines, the option is a switch
            self.plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N, conv=case.conv, **fixed)
        elif kernel == "tune":
            # offline, once per matrix (Section 3.7); not part of the timed region
            self.plan, self.tuned = sp.tune(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N,
                                            self.inp.data_ptr(), self.out.data_ptr(),
                                            torch.cuda.current_stream().cuda_stream, conv=case.conv)
        else:
            self.plan = sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N, conv=case.conv,
                                   kernel={"rows": sp.KERNEL_ROWS, "spec": sp.KERNEL_SPEC}[kernel])
        self.info = self.plan.info()
        self.args = (ctypes.c_void_p(self.plan.handle), ctypes.c_void_p(self.inp.data_ptr()),
                     ctypes.c_void_p(self.out.data_ptr()))

    def set_plan(self, plan):
        self.plan = plan
        self.info = plan.info()
        self.args = (ctypes.c_void_p(plan.handle), self.args[1], self.args[2])

    def variant(self, **changes):
        """A new plan with this plan's options and `changes` on top (generated-kernel plans)."""
        csr, case = self.case.csr, self.case
        opts = {k: self.info[k] for k in self.PLAN_KEYS}
        opts["spec_prefetch"] = 1 if opts.get("spec_prefetch") else 0   # the plan reports lines, the option is a switch
        opts.update(changes)
        return self.sp.inspect(csr.row_ptr, csr.col_idx, csr.vals, csr.M, csr.K, case.N, conv=case.conv, **opts)

    @property
    def flops(self):
        return 2.0 * self.nnz * self.N

    @property
    def algorithmic_bytes(self):
        """Compulsory HBM traffic of one launch: the dense operand read once, the output
        written once, the nonzero stream (8 B per nonzero) and the row pointers read once."""
        e = self.esize
        dense_in = (self.case.conv[0] * self.N if self.is_conv else self.K * self.N) * e
        return dense_in + self.M * self.N * self.osize + 8 * self.nnz + 4 * (self.M + 1)

    def launch(self, stream):
        rc = self.fn(self.args[0], self.args[1], self.args[2], stream)
        if rc != 0:
            raise RuntimeError(self.sp.last_error())

    def cold_us(self, iters=200, footprint=640 << 20):
        """Microseconds per launch when every launch works on operands no cache holds: the input
        and output rotate through enough copies to exceed twice the 256 MB memory-side cache
        (the plan - weights, code - stays warm, as it does in an inference loop)."""
        torch = self.torch
        per_set = self.inp.numel() * self.inp.element_size() + self.out.numel() * self.out.element_size()
        n = max(2, -(-footprint // per_set))
        ins = [self.inp.clone() for _ in range(n)]
        outs = [torch.empty_like(self.out) for _ in range(n)]
        args = [(ctypes.c_void_p(i.data_ptr()), ctypes.c_void_p(o.data_ptr())) for i, o in zip(ins, outs)]
        st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        for a, b in args:
            self.fn(self.args[0], a, b, st)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for k in range(iters):
            a, b = args[k % n]
            if self.fn(self.args[0], a, b, st) != 0:
                raise RuntimeError(self.sp.last_error())
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e3, n

    def dense(self):
        if self.is_conv:
            return self.torch.nn.functional.conv2d(self.dense_in, self.Wd, padding=1)
        if self.Ad.dtype == self.torch.int8:
            return self.torch._int_mm(self.Ad, self.dense_in)
        return self.torch.matmul(self.Ad, self.dense_in)

    def dense_candidates(self):
        """Dense baselines of the same product on operands prepared ahead of time (the paper took the
        vendor library's best algorithm with the weight stored transposed, Section 4): the fastest counts."""
        c = {"A@B" if not self.is_conv else "conv2d": self.dense}
        if not self.is_conv and self.Ad.dtype != self.torch.int8:
            if not hasattr(self, "At"):
                self.At, self.Bt = self.Ad.t().contiguous(), self.dense_in.t().contiguous()
            c["(B^T@A^T)"] = lambda: self.torch.matmul(self.Bt, self.At)
            c["A(col-major)@B"] = lambda: self.torch.matmul(self.At.t(), self.dense_in)
        return c


def time_loop(torch, fn, iters, warmup):
    """Average milliseconds per call of fn, HIP events on torch's current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def time_repeats(torch, fn, iters, warmup, repeats=5):
    """(median, min, max) milliseconds per call over `repeats` timed loops of `iters` calls."""
    t = sorted(time_loop(torch, fn, iters, warmup if r == 0 else 0) for r in range(repeats))
    return t[len(t) // 2], t[0], t[-1]


def best_dense(torch, L, iters):
    """(milliseconds, how) of the fastest dense baseline of layer L: every candidate formulation,
    each under the event loop and as 20 launches per HIP graph (without PyTorch's per-call host
    time, which a short dense kernel would otherwise be charged)."""
    best, how = None, None
    for name, fn in L.dense_candidates().items():
        t = time_loop(torch, fn, iters, 10)
        h = "event loop"
        try:
            g = graph_us(torch, fn) / 1e3
            if g < t:
                t, h = g, "20 launches per HIP graph"
        except Exception:   # a library call that cannot be captured
            torch.cuda.synchronize()
        if best is None or t < best:
            best, how = t, f"{h}, {name}"
    return best, how


def device_clocks():
    """Current shader / memory clocks as rocm-smi prints them, or None (clocks are left at their defaults)."""
    import subprocess
    try:
        r = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20)
        card = next(iter(json.loads(r.stdout).values()))
        return {k: v for k, v in card.items() if "sclk" in k or "mclk" in k}
    except Exception:
        return None


def graph_us(torch, fn, inner=20, replays=20):
    """Microseconds per call of fn with `inner` calls captured in one HIP graph and replayed:
    neither side pays per-call host overhead (what matters for the few-microsecond configurations)."""
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for _ in range(inner):
                fn()
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (replays * inner)


def measure_traffic(args, layers, plan_path):
    """Bytes that leave the L2 caches per launch of every layer, from two rocprofv3 --pmc child
    runs of this script in --pmc-mode (FETCH_SIZE, then WRITE_SIZE; one counter set per run) with
    the plans of this run.  Each counter is scaled by what it reads for the 256 MiB device copy
    that --pmc-mode issues first.  FETCH_SIZE counts 128-byte data requests as 64 bytes (the copy
    factor is 2) but 64-byte instruction fetches in full, so the plainly scaled figure counts the
    generated code twice; `refined` takes the code (once per XCD, eight XCDs) out before scaling.
    Returns None where the profiler is not available or a child run fails."""
    import csv
    import glob
    import shutil
    import subprocess
    import tempfile
    if shutil.which("rocprofv3") is None or any("ROCPROF" in k for k in os.environ):
        return None
    out = tempfile.mkdtemp(prefix="sparsert_pmc_", dir="/tmp")
    env = dict(os.environ, TMPDIR="/tmp")
    counted = {}
    try:
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            cmd = ["timeout", "-s", "KILL", "150", "rocprofv3", "--pmc", counter, "-d", out, "-o", counter,
                   "--output-format", "csv", "--", sys.executable, os.path.join(ROOT, "bench.py"), "--pmc-mode",
                   "--plan-file", plan_path, "--workload", args.workload, "--dtype", args.dtype]
            r = subprocess.run(cmd, cwd="/tmp", env=env, capture_output=True, text=True)
            files = glob.glob(os.path.join(out, "**", f"{counter}_counter_collection.csv"), recursive=True)
            if r.returncode != 0 or not files:
                return None
            per_kernel = {}
            for row in csv.DictReader(open(files[0])):
                if row["Counter_Name"] == counter:
                    per_kernel.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
            counted[counter] = per_kernel
        copy_bytes = 64 * 1024 * 1024 * 4
        factor = {}
        for counter, per_kernel in counted.items():
            copies = [v for k, v in per_kernel.items() if "copyBuffer" in k]
            if not copies:
                return None
            factor[counter] = copy_bytes / (copies[0][-1] * 1024.0)
        res = {"copy_factor": factor, "layers": []}
        for L in layers:
            name = L.plan.kernel_name()
            vals = {c: [v for k, v in counted[c].items() if name in k] for c in counted}
            if not all(vals.values()):
                return None
            kib = {c: sum(vals[c][0][-10:]) / len(vals[c][0][-10:]) for c in counted}   # the last launches: steady state
            fetch, write = kib["FETCH_SIZE"] * 1024.0, kib["WRITE_SIZE"] * 1024.0
            code = 8.0 * L.info["spec_code_bytes"]
            # waves that prefetch their code bring most of it in through data requests, which the counter
            # halves like any other: there the plain scaling is the estimate (an upper one: what still
            # arrives as instruction fetches is counted in full)
            split = code > 0 and fetch > code and not L.info.get("spec_prefetch")
            refined = (code + (fetch - code) * factor["FETCH_SIZE"]) if split else fetch * factor["FETCH_SIZE"]
            res["layers"].append({"layer": L.case.name, "kernel": name,
                                  "refined_how": "instruction fetches (8 x code, counted in full) taken out before scaling" if split
                                                 else "scaled plainly",

                                  "fetch_counted_bytes": fetch, "write_counted_bytes": write,
                                  "plain_scaled_bytes": fetch * factor["FETCH_SIZE"] + write * factor["WRITE_SIZE"],
                                  "refined_bytes": refined + write * factor["WRITE_SIZE"]})
        return res
    except Exception as e:   # a profiler that is missing a counter, an unreadable file: no figure rather than no benchmark
        print(f"bench.py: traffic measurement skipped: {e}", file=sys.stderr)
        return None
    finally:
        shutil.rmtree(out, ignore_errors=True)


def measure_ceilings(torch, footprint_bytes, stream):
    """What this GPU delivers, measured in this run with the three kernels of
    libsparsert_ceilings.so (HIP events on the launch stream): a copy far larger than the caches
    (HBM), a copy at the step's own footprint (L2 / memory-side cache), independent fp32
    multiply-adds without packed instructions, and 256-byte row fetches into registers from a
    cache-resident matrix (operand delivery through the vector-memory path)."""
    path = os.path.join(ROOT, "paper_2008_11849_amd", "libsparsert_ceilings.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: run `python __graft_entry__.py`")
    lib = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    lib.sparsert_ceiling_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.sparsert_ceiling_fma.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp]
    lib.sparsert_ceiling_loads.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp]
    dev = "cuda:0"

    def timed(fn, iters, warm=3):
        for _ in range(warm):
            assert fn() == 0
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / iters
            best = t if best is None else min(best, t)
        return best

    res = {}
    big = 512 << 20
    src = torch.empty(big // 4, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    t = timed(lambda: lib.sparsert_ceiling_copy(src.data_ptr(), dst.data_ptr(), big, stream), 5, 2)
    res["copy_cold_GBs"] = 2.0 * big / t / 1e9
    res["copy_cold_what"] = "512 MiB read + 512 MiB written per pass (four times the memory-side cache)"
    half = max(1 << 20, (int(footprint_bytes) // 2) // 4096 * 4096)
    t = timed(lambda: lib.sparsert_ceiling_copy(src.data_ptr(), dst.data_ptr(), half, stream), 200, 20)
    res["copy_warm_GBs"] = 2.0 * half / t / 1e9
    res["copy_warm_what"] = "%d bytes read + as many written per pass, the same buffers every pass (the footprint of one launch of the step)" % half
    del src, dst
    wgs, iters = 4096, 2000
    out = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
    t = timed(lambda: lib.sparsert_ceiling_fma(out.data_ptr(), wgs, iters, stream), 5, 2)
    res["fma_TFLOPs"] = wgs * 256.0 * iters * lib.sparsert_ceiling_fma_flops_per_thread_iter() / t / 1e12
    res["fma_what"] = "independent v_fma_f32 on registers, 16 waves per compute unit and more; no packed instructions"
    rows, pitch, tiles, wg2, reps = 3072, 1024, 16, 512, 4
    m = torch.empty(rows * pitch, dtype=torch.float32, device=dev).normal_()
    out2 = torch.empty(wg2 * 256, dtype=torch.float32, device=dev)
    t = timed(lambda: lib.sparsert_ceiling_loads(m.data_ptr(), rows, pitch, tiles, wg2, reps, out2.data_ptr(), stream), 20, 3)
    res["operand_fetch_GBs"] = wg2 * 4.0 * reps * rows * 256 / t / 1e9
    res["operand_fetch_what"] = ("2048 waves, each pulling the 3072 rows of one 64-column tile of a 12.6 MB matrix into registers "
                                 "four times, one dword per lane, eight rows in flight (as the generated kernel fetches B)")
    return res


def cpu_baseline(cases, gpu_outputs):
    """The CPU oracle as it stands, on the host cores, on the same workload: whole steps are
    repeated for about 10 s of wall time and the mean pass is reported.  The oracle's result
    is also held against what the timed plans left in their output buffers (every element);
    a mismatch beyond the storage type's tolerance ends the run with an error."""
    from oracle import ref
    threads = min(ref.max_threads(), len(os.sched_getaffinity(0)))
    flops = sum(2.0 * c.csr.nnz * c.N for c in cases)

    def one_pass():
        for case in cases:
            csr = case.csr
            if case.conv is not None:
                ref.conv3x3(case.Wdense, case.X, want_scale=False, threads=threads)
            else:
                ref.spmm(csr.M, csr.K, case.N, csr.row_ptr, csr.col_idx, csr.vals, case.B,
                         want_scale=False, threads=threads)

    one_pass()  # page in, start the thread pool
    passes, t0 = 0, time.perf_counter()
    while passes < 3 or time.perf_counter() - t0 < 10.0:
        one_pass()
        passes += 1
    per_pass = (time.perf_counter() - t0) / passes
    threads_all, threads = threads, 1          # the same pass on one core, three times
    one_pass()
    t1 = time.perf_counter()
    for _ in range(3):
        one_pass()
    per_pass_1 = (time.perf_counter() - t1) / 3
    threads = threads_all
    worst, worst_rel, excluded = 0.0, 0.0, 0.0
    for case, got in zip(cases, gpu_outputs):
        csr = case.csr
        if case.conv is not None:
            want, scale = ref.conv3x3(case.Wdense, case.X, threads=threads)
        else:
            want, scale = ref.spmm(csr.M, csr.K, case.N, csr.row_ptr, csr.col_idx, csr.vals, case.B, threads=threads)
        m = ref.error_metrics(got.reshape(want.shape), want, scale, ref.HALF_STORE_ROUNDING if got.dtype.itemsize == 2 else 0.0)
        tol = 2e-2 if got.dtype.itemsize == 2 else 0.0 if got.dtype.kind == "i" else 1e-4   # integer work: exact
        if not (m["componentwise"] <= tol and m["normwise"] <= tol and m["relative"] <= tol and m["exact_on_zero_scale"]):
            print(f"bench.py: the timed plan of {case.name} disagrees with the oracle: {m}", file=sys.stderr)
            sys.exit(1)
        worst = max(worst, m["componentwise"])
        worst_rel = max(worst_rel, m["relative"])
        excluded = max(excluded, m["relative_excluded_fraction"])
    return {"value": flops / per_pass / 1e9, "unit": "GFLOP/s", "cores": threads, "kind": "oracle",
            "value_one_core": flops / per_pass_1 / 1e9,
            "parity_max_componentwise_error": worst,
            "parity_max_relative_error": worst_rel,
            "parity_relative_error_what": "max |got-ref|/|ref| over entries with |ref| >= 1e-2 rms(ref); "
                                          "share of entries below that floor: %.4f" % excluded,
            "sample": "every layer of the step, all rows, float64 oracle with OpenMP over rows; "
                      "%d passes in %.1f s, %.4f s per pass" % (passes, per_pass * passes, per_pass)}


def refine_in_context(torch, sp, layers, stream, steps=400, repeats=4):
    """Offline, after every layer has been tuned on its own (Section 3.7 tunes each problem once,
    off the inference path): whether a generated kernel's waves should prefetch their code depends
    on what the other layers of the step leave in the L2 caches, which a layer timed alone cannot
    see - so each layer's plan is tried with the switch flipped inside the whole step, and the
    variant is kept if the step gets at least 1 % shorter (best of `repeats` loops of `steps` steps
    for both, alternating).  Returns what was tried, for the report."""
    def step_us():
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            for L in layers:
                L.launch(stream)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / steps
    for _ in range(2):
        step_us()   # clocks up
    tried = []
    for L in layers:
        if L.info["kernel"] != sp.KERNEL_SPEC:
            continue
        had = 1 if L.info["spec_prefetch"] else 0
        try:
            other = L.variant(spec_prefetch=1 - had)
        except sp.SparseRTError:
            continue
        mine = L.plan
        best = {True: 1e30, False: 1e30}
        for _ in range(repeats):
            for alt in (False, True):
                L.set_plan(other if alt else mine)
                best[alt] = min(best[alt], step_us())
        keep_other = best[True] < 0.99 * best[False]
        L.set_plan(other if keep_other else mine)
        (mine if keep_other else other).destroy()
        tried.append({"layer": L.case.name, "code_prefetch_from_tuner": bool(had), "code_prefetch_kept": bool(L.info["spec_prefetch"]),
                      "step_us_with_tuner_choice": best[False], "step_us_with_the_switch_flipped": best[True]})
    return tried


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); nothing here uses a second GPU",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2008_11849_amd import sparsert as sp, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.backends.cuda.matmul.allow_tf32 = False
    torch.backends.cudnn.allow_tf32 = False
    dt = {"f16": np.float16, "i8": np.int8}.get(args.dtype, np.float32)
    kernel = args.kernel
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    names = {"c1": ["c1"], "c2": ["c2"], "c3": ["c3", "c3t"], "c4": ["c4"]}[args.workload]
    cases = [synth.config(n, dt) for n in names]
    saved = {}
    if args.plan_file and os.path.exists(args.plan_file):
        saved = json.load(open(args.plan_file))
    layers = [Layer(c, torch, sp, kernel, saved.get(f"{c.name}_{args.dtype}")) for c in cases]
    in_context = None
    if kernel == "tune" and not saved and len(layers) > 1:
        in_context = refine_in_context(torch, sp, layers, stream)
    if args.plan_file and not saved:
        with open(args.plan_file, "w") as f:
            json.dump({f"{L.case.name}_{args.dtype}": {k: L.info[k] for k in Layer.PLAN_KEYS} for L in layers}, f)

    if args.pmc_mode:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        for L in layers:
            for _ in range(20):
                L.launch(stream)
            torch.cuda.synchronize()
        print(json.dumps({"pmc_mode": True, "copy_bytes": src.numel() * 4,
                          "layers": [{"layer": L.case.name, "plan": L.info} for L in layers]}))
        return

    def step():
        for L in layers:
            L.launch(stream)

    # ---- the timed region: exactly --steps steps between two synchronisations.  Before the
    # --warmup steps the step runs 300 times untimed: planning and tuning leave the GPU idle for
    # seconds, and a short run (--steps 20) would otherwise time the clocks ramping up
    for _ in range(300):
        step()
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    r0.record()
    for _ in range(args.steps):
        step()
    r1.record()
    # the host watches the closing event before it synchronises: a blocking wait alone wakes up
    # tens of microseconds after the GPU is done, which a short run (--steps 20) would count as step time
    while not r1.query():
        pass
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    region_us_per_launch = r0.elapsed_time(r1) * 1e3 / (args.steps * len(layers))   # HIP events around the timed region
    ms_per_step = wall * 1e3 / args.steps
    flops_step = sum(L.flops for L in layers)

    # ---- per-kernel durations, live, HIP events on the launch stream
    iters = max(200, min(args.steps, 2000))
    per_layer = []
    for L in layers:
        ms, ms_min, ms_max = time_repeats(torch, lambda L=L: L.launch(stream), iters, 50)
        ms_dense, dense_how = best_dense(torch, L, max(50, iters // 10))
        cold, n_sets = (ms * 1e3, 0) if args.no_cold else L.cold_us()
        per_layer.append({"layer": L.case.name, "M": L.M, "K": L.K, "N": L.N, "nnz": L.nnz,
                          "kernel_name": L.plan.kernel_name(),
                          "us": ms * 1e3, "us_min": ms_min * 1e3, "us_max": ms_max * 1e3, "repeats": 5,
                          "launches_per_repeat": iters, "gflops": L.flops / ms / 1e6,
                          "cold_us": cold, "cold_operand_sets": n_sets,
                          "dense_us": ms_dense * 1e3, "speedup_vs_dense": ms_dense / ms, "dense_kind": L.dense_kind,
                          "dense_timing": dense_how,
                          "plan": {k: L.info[k] for k in ("kernel", "vec", "n_split", "spec_mode", "spec_rows",
                                                          "spec_tiles", "spec_ksplit", "spec_swizzle", "spec_vec",
                                                          "spec_prefetch", "spec_code_bytes")},
                          "tuned_candidates": len(L.tuned) if L.tuned else 0,
                          # the tuner's six fastest candidates (ranked with displaced caches), for the record
                          "tuned_top": sorted(({k: (round(v, 2) if isinstance(v, float) else v) for k, v in e.items()
                                                if k in ("kernel", "vec", "spec_mode", "spec_rows", "spec_tiles", "spec_ksplit",
                                                         "spec_swizzle", "spec_vec", "spec_prefetch", "microseconds", "cold_microseconds", "agrees")}
                                               for e in (L.tuned or []) if e["cold_microseconds"] > 0),
                                              key=lambda e: e["cold_microseconds"])[:6]})
    # ---- every layer's launch duration inside the step.  The HIP events around the timed region
    # give the time of a whole step (kernels and the gaps between them); it is apportioned to the
    # layers in the ratio of their back-to-back durations.  (Event pairs around single launches
    # inside the step were tried: each pair adds about 3 us of its own, 29.6 against 23.8 us per
    # step, so they measure the markers.)
    total_b2b = sum(p["us"] for p in per_layer)
    for p in per_layer:
        p["in_step_us"] = region_us_per_launch * len(layers) * p["us"] / total_b2b

    # ---- roofline of the dominant kernel (the layer that takes longest inside the step)
    dom = max(range(len(layers)), key=lambda i: per_layer[i]["in_step_us"])
    D, dom_row = layers[dom], per_layer[dom]
    ceilings = None if args.no_ceilings else measure_ceilings(
        torch, sum(L.algorithmic_bytes for L in layers) / len(layers), stream)
    peak_tf = {"f32": FP32_VECTOR_PEAK_TF}.get(args.dtype, FP32_VECTOR_PEAK_TF)   # sums are fp32 multiply-adds in every storage type but int8
    intensity = D.flops / D.algorithmic_bytes
    ridge_published = peak_tf * 1e12 / (HBM_PEAK_GBS * 1e9)
    # the ridge this build can reach: packed fp32 instructions are never emitted, so the ALU side
    # is what the multiply-add ceiling kernel measures
    ridge_reachable = (ceilings["fma_TFLOPs"] * 1e12 / (HBM_PEAK_GBS * 1e9)) if ceilings else ridge_published
    bound = "alu" if intensity >= ridge_reachable else "hbm"
    t_dom = dom_row["in_step_us"] * 1e-6
    hbm_achieved = D.algorithmic_bytes / t_dom / 1e9
    alu_achieved = D.flops / t_dom / 1e12
    traffic = None
    traffic_detail = None
    if not args.no_traffic:
        import tempfile
        with tempfile.NamedTemporaryFile("w", suffix=".json", dir="/tmp", delete=False) as f:
            json.dump({f"{L.case.name}_{args.dtype}": {k: L.info[k] for k in Layer.PLAN_KEYS} for L in layers}, f)
        try:
            traffic_detail = measure_traffic(args, layers, f.name)
        finally:
            os.unlink(f.name)
        if traffic_detail:
            traffic = traffic_detail["layers"][dom]["refined_bytes"]
    alg_all = sum(L.algorithmic_bytes for L in layers) / len(layers)
    roofline = {
        "bound": bound,
        "achieved": alu_achieved if bound == "alu" else hbm_achieved,
        "peak": peak_tf if bound == "alu" else HBM_PEAK_GBS,
        "unit": "TFLOP/s" if bound == "alu" else "GB/s",
        "frac": (alu_achieved / peak_tf) if bound == "alu" else (hbm_achieved / HBM_PEAK_GBS),
        "traffic": traffic,
        "kernel": D.plan.kernel_name(),
        "kernel_layer": D.case.name,
        "kernel_avg_us": dom_row["in_step_us"],
        "kernel_avg_us_what": "HIP events around the timed region (kernels and the gaps between them), apportioned to the "
                              "step's layers in the ratio of their back-to-back durations",
        "kernel_back_to_back_us": dom_row["us"],
        "algorithmic_bytes_per_launch": D.algorithmic_bytes,
        "flops_per_launch": D.flops,
        "arithmetic_intensity_flop_per_byte": intensity,
        "ridge_published_flop_per_byte": ridge_published,
        "ridge_reachable_flop_per_byte": ridge_reachable,
        "bound_rule": "alu if the intensity is at or above the reachable ridge (measured unpacked multiply-add ceiling / 8 TB/s), else hbm",
        "hbm_frac": hbm_achieved / HBM_PEAK_GBS,
        "alu_frac": alu_achieved / peak_tf,
        "frac_back_to_back": (D.flops / (dom_row["us"] * 1e-6) / 1e12 / peak_tf) if bound == "alu"
                             else (D.algorithmic_bytes / (dom_row["us"] * 1e-6) / 1e9 / HBM_PEAK_GBS),
        "all_launches": {"avg_us_timed_region": region_us_per_launch,
                         "hbm_frac_timed_region": alg_all / (region_us_per_launch * 1e-6) / 1e9 / HBM_PEAK_GBS,
                         "avg_us_back_to_back": sum(p["us"] for p in per_layer) / len(per_layer),
                         "avg_us_cold_operands": sum(p["cold_us"] for p in per_layer) / len(per_layer)},
        "traffic_detail": traffic_detail,
        "traffic_over_algorithmic": (traffic / D.algorithmic_bytes) if traffic else None,
    }
    if ceilings:
        # the same kernel against what this GPU was measured to deliver in this run
        roofline["measured_ceilings"] = ceilings
        roofline["frac_of_measured"] = {
            "hbm_cold_copy": hbm_achieved / ceilings["copy_cold_GBs"],
            "warm_copy_at_step_footprint": hbm_achieved / ceilings["copy_warm_GBs"],
            "fma_unpacked": alu_achieved / ceilings["fma_TFLOPs"]}
        if D.info["kernel"] == sp.KERNEL_SPEC:
            # third ceiling: bytes of B a launch pulls into registers (one 256-byte row per code
            # block, column tile and column the block touches) at the measured fetch rate
            vcols = max(1, D.info["spec_vec"])
            tiles = -(-(D.N // vcols) // 64)
            fetched = (float(D.plan.export(sp.FIELD_SPEC_COLUMNS).astype("int64").sum()) * tiles
                       * D.info["spec_lanes"] * vcols * D.esize)
            roofline["operand_delivery"] = {"register_ingest_bytes_per_launch": fetched,
                                            "floor_us_at_measured_fetch_rate": fetched / ceilings["operand_fetch_GBs"] / 1e3,
                                            "frac": fetched / ceilings["operand_fetch_GBs"] / 1e3 / dom_row["in_step_us"]}
    dense_ms = sum(p["dense_us"] for p in per_layer) / 1e3
    sparse_ms = sum(p["us"] for p in per_layer) / 1e3
    out = {
        "metric": "effective GFLOP/s (2*nnz*N)",
        "value": flops_step / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": {
            "c1": "c1: 256x256 @ 90% uniform, N=1024",
            "c2": "c2: MobileNet-like 1x1 conv 512x512 @ 90% magnitude-pruned, N=196",
            "c3": "c3: Transformer FC 3072x768 and transposed 768x3072 @ 95% magnitude-pruned, N=1024",
            "c4": "c4: 3x3 conv 256->256 @ 90%, 14x14, pad 1, implicit im2col"}[args.workload],
            "layers_per_step": len(layers), "kernel": args.kernel},
        "speedup_vs_dense": dense_ms / sparse_ms,
        "dense_ms_per_step": dense_ms,
        "kernel_ms_per_step": sparse_ms,
        "layers": per_layer,
        "clocks": device_clocks(),
        "roofline": roofline,
    }
    if in_context is not None:
        out["in_context_refinement"] = {"what": "after sparsert_tune, before the timed region: each generated plan's code prefetch "
                                                "switched on / off inside the whole step, kept if the step is at least 1 % shorter",
                                        "layers": in_context}

    if not args.no_cases:
        side = []
        for n in ["c1", "c2", "c3", "c3t", "c4"]:
            if n in names:
                continue
            L = Layer(synth.config(n, dt), torch, sp, kernel)
            ms = time_loop(torch, lambda L=L: L.launch(stream), 500, 50)
            msd = min(time_loop(torch, fn, 100, 10) for fn in L.dense_candidates().values())
            cur = lambda: ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
            g_sparse = graph_us(torch, lambda L=L: L.launch(cur()))
            g_dense = None
            for fn in L.dense_candidates().values():
                try:
                    g = graph_us(torch, fn)
                    g_dense = g if g_dense is None else min(g_dense, g)
                except Exception:   # a library call that cannot be captured
                    torch.cuda.synchronize()
            side.append({"layer": n, "us": ms * 1e3, "gflops": L.flops / ms / 1e6,
                         "dense_us": msd * 1e3, "speedup_vs_dense": msd / ms,
                         "graph_us": g_sparse, "dense_graph_us": g_dense,
                         "speedup_vs_dense_graph": (g_dense / g_sparse) if g_dense else None,
                         "plan": {k: L.info[k] for k in ("kernel", "vec", "n_split", "spec_mode", "spec_rows",
                                                         "spec_tiles", "spec_ksplit", "spec_swizzle", "spec_vec")}})
            L.plan.destroy()
        out["other_configs"] = side

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cases, [L.out.cpu().numpy() for L in layers])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
