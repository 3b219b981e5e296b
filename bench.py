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
    ap.add_argument("--pmc-mode", action="store_true",
                    help="for rocprofv3 --pmc runs: a 256 MiB copy (counter calibration), then 20 launches "
                         "of every layer of the workload, nothing else")
    return ap.parse_args()


class Layer:
    """One sparse layer resident on the GPU: plan, input, output and its dense twin."""

    PLAN_KEYS = ("kernel", "vec", "split_threshold", "spec_mode", "spec_rows", "spec_tiles", "spec_ksplit",
                 "spec_swizzle", "spec_vec")

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


def load_traffic(kernel_tag):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_pmc.txt")
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


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
    worst = 0.0
    for case, got in zip(cases, gpu_outputs):
        csr = case.csr
        if case.conv is not None:
            want, scale = ref.conv3x3(case.Wdense, case.X, threads=threads)
        else:
            want, scale = ref.spmm(csr.M, csr.K, case.N, csr.row_ptr, csr.col_idx, csr.vals, case.B, threads=threads)
        m = ref.error_metrics(got.reshape(want.shape), want, scale)
        tol = 2e-2 if got.dtype.itemsize == 2 else 0.0 if got.dtype.kind == "i" else 1e-4   # integer work: exact
        if not (m["componentwise"] <= tol and m["normwise"] <= tol and m["exact_on_zero_scale"]):
            print(f"bench.py: the timed plan of {case.name} disagrees with the oracle: {m}", file=sys.stderr)
            sys.exit(1)
        worst = max(worst, m["componentwise"])
    return {"value": flops / per_pass / 1e9, "unit": "GFLOP/s", "cores": threads, "kind": "oracle",
            "value_one_core": flops / per_pass_1 / 1e9,
            "parity_max_componentwise_error": worst,
            "sample": "every layer of the step, all rows, float64 oracle with OpenMP over rows; "
                      "%d passes in %.1f s, %.4f s per pass" % (passes, per_pass * passes, per_pass)}


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

    # ---- the timed region: exactly --steps steps between two synchronisations
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    r0.record()
    for _ in range(args.steps):
        step()
    r1.record()
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
        ms_dense = time_loop(torch, L.dense, max(50, iters // 10), 10)
        dense_how = "event loop"
        try:   # without PyTorch's per-call host time, which a short dense kernel would otherwise be charged
            g = graph_us(torch, L.dense) / 1e3
            if g < ms_dense:
                ms_dense, dense_how = g, "20 launches per HIP graph"
        except Exception:   # a library call that cannot be captured
            torch.cuda.synchronize()
        cold, n_sets = (ms * 1e3, 0) if args.no_cold else L.cold_us()
        per_layer.append({"layer": L.case.name, "M": L.M, "K": L.K, "N": L.N, "nnz": L.nnz,
                          "us": ms * 1e3, "us_min": ms_min * 1e3, "us_max": ms_max * 1e3, "repeats": 5,
                          "launches_per_repeat": iters, "gflops": L.flops / ms / 1e6,
                          "cold_us": cold, "cold_operand_sets": n_sets,
                          "dense_us": ms_dense * 1e3, "speedup_vs_dense": ms_dense / ms, "dense_kind": L.dense_kind,
                          "dense_timing": dense_how,
                          "plan": {k: L.info[k] for k in ("kernel", "vec", "n_split", "spec_mode", "spec_rows",
                                                          "spec_tiles", "spec_ksplit", "spec_swizzle", "spec_vec",
                                                          "spec_code_bytes")},
                          "tuned_candidates": len(L.tuned) if L.tuned else 0})
    kernel_ms = sum(p["us"] for p in per_layer) / 1e3 / len(layers)       # average launch
    alg_bytes = sum(L.algorithmic_bytes for L in layers) / len(layers)    # average launch
    achieved = alg_bytes / (kernel_ms * 1e-3) / 1e9
    dense_ms = sum(p["dense_us"] for p in per_layer) / 1e3
    sparse_ms = sum(p["us"] for p in per_layer) / 1e3
    tag = f"spmm_{args.workload}_{args.dtype}"
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
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": load_traffic(tag),
                     "kernel": "sparsert_spec_<M>x<K>x<N> (generated per layer) / sparsert::rows_kernel; see layers[].plan.kernel: 2 / 1",
                     "avg_launch_us": kernel_ms * 1e3,
                     "avg_launch_us_timed_region": region_us_per_launch,
                     "frac_timed_region": alg_bytes / (region_us_per_launch * 1e-6) / 1e9 / HBM_PEAK_GBS,
                     "avg_launch_us_cold_operands": sum(p["cold_us"] for p in per_layer) / len(per_layer),
                     "frac_cold_operands": alg_bytes / (sum(p["cold_us"] for p in per_layer) / len(per_layer) * 1e-6) / 1e9
                                           / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "alu_frac_of_fp32_vector_peak":
                         flops_step / len(layers) / (kernel_ms * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TF},
    }

    if not args.no_cases:
        side = []
        for n in ["c1", "c2", "c3", "c3t", "c4"]:
            if n in names:
                continue
            L = Layer(synth.config(n, dt), torch, sp, kernel)
            ms = time_loop(torch, lambda L=L: L.launch(stream), 500, 50)
            msd = time_loop(torch, L.dense, 100, 10)
            cur = lambda: ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
            g_sparse = graph_us(torch, lambda L=L: L.launch(cur()))
            try:
                g_dense = graph_us(torch, L.dense)
            except Exception:   # a library call that cannot be captured
                torch.cuda.synchronize()
                g_dense = None
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
