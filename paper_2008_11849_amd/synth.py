"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *draws* inputs (masks, weights, activations) and converts a
dense array with zeros into CSR.  It holds none of the method's arithmetic (no
products, no sums over nonzeros, no plan logic), so that the CPU oracle and the
HIP path can both be fed from it without sharing any code of the method.

The paper measures on pruned ResNet-50 / Transformer / MobileNetV1 weights
(Evaluation section, Table 1 and Table 3).  Those checkpoints are not available
here; the generators below reproduce their shapes, sparsity levels and the
"quite uniform" nonzero statistics of magnitude pruning, plus a deliberately
skewed (Zipf-like) variant that stresses load balancing.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 200811849


@dataclass
class CSR:
    """Canonical CSR of the sparse matrix A (M x K): ascending columns per row."""

    M: int
    K: int
    row_ptr: np.ndarray  # int32 [M+1]
    col_idx: np.ndarray  # int32 [nnz]
    vals: np.ndarray  # float32 or float16 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.col_idx.shape[0])

    def todense(self, dtype=np.float64) -> np.ndarray:
        """Zero-filled dense A.  Duplicate-free CSR only (pure scatter, no adds)."""
        A = np.zeros((self.M, self.K), dtype=dtype)
        rows = np.repeat(np.arange(self.M), np.diff(self.row_ptr))
        A[rows, self.col_idx] = self.vals.astype(dtype)
        return A


def exact_nnz(M: int, K: int, sparsity: float) -> int:
    """Number of kept weights for a nominal sparsity: round(density * M * K)."""
    return int(round((1.0 - sparsity) * M * K))


def csr_from_mask(values: np.ndarray, mask: np.ndarray) -> CSR:
    """CSR of `values` restricted to the True positions of `mask` (row-major scan)."""
    M, K = values.shape
    rows, cols = np.nonzero(mask)  # row-major order => ascending columns per row
    row_ptr = np.zeros(M + 1, dtype=np.int64)
    np.add.at(row_ptr, rows + 1, 1)
    row_ptr = np.cumsum(row_ptr)
    return CSR(M, K, row_ptr.astype(np.int32), cols.astype(np.int32),
               np.ascontiguousarray(values[rows, cols]))


def uniform_mask(M: int, K: int, sparsity: float, rng: np.random.Generator) -> np.ndarray:
    """Exactly exact_nnz positions, drawn uniformly without replacement."""
    nnz = exact_nnz(M, K, sparsity)
    flat = rng.choice(M * K, size=nnz, replace=False)
    mask = np.zeros(M * K, dtype=bool)
    mask[flat] = True
    return mask.reshape(M, K)


def magnitude_mask(W: np.ndarray, sparsity: float) -> np.ndarray:
    """Global magnitude pruning: keep the exact_nnz largest |W| (ties: lower flat index)."""
    M, K = W.shape[0], int(np.prod(W.shape[1:]))
    nnz = exact_nnz(M, K, sparsity)
    flat = np.abs(W.reshape(-1))
    order = np.argsort(-flat, kind="stable")
    mask = np.zeros(M * K, dtype=bool)
    mask[order[:nnz]] = True
    return mask.reshape(M, K)


def _as_dtype(x: np.ndarray, dtype) -> np.ndarray:
    return np.ascontiguousarray(x.astype(np.float32).astype(dtype))


def uniform_csr(M, K, sparsity, seed, dtype=np.float32) -> CSR:
    """Uniform random mask, nonzeros ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    mask = uniform_mask(M, K, sparsity, rng)
    W = rng.standard_normal((M, K))
    W[W == 0.0] = 1.0
    return csr_from_mask(_as_dtype(W, dtype), mask)


def magnitude_csr(M, K, sparsity, seed, std=1.0, dtype=np.float32) -> CSR:
    """Magnitude-pruned N(0, std) weights: per-row nnz varies binomially."""
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((M, K)) * std
    return csr_from_mask(_as_dtype(W, dtype), magnitude_mask(W, sparsity))


def skewed_csr(M, K, sparsity, seed, dtype=np.float32) -> CSR:
    """Magnitude pruning of rows with Zipf-like scales.

    Row r is scaled by (1 + pi(r))**-0.5 with pi a seeded permutation, so after
    global pruning a few rows stay nearly dense and many become (almost) empty.
    """
    rng = np.random.default_rng(seed)
    sigma = (1.0 + rng.permutation(M)) ** -0.5
    W = rng.standard_normal((M, K)) * sigma[:, None]
    return csr_from_mask(_as_dtype(W, dtype), magnitude_mask(W, sparsity))


def clustered_csr(M, K, sparsity, seed, clusters=8, dtype=np.float32) -> CSR:
    """Rows fall into `clusters` hidden groups, scattered over the matrix by a seeded
    permutation; a row only uses the K/clusters columns of its group (a second seeded
    permutation), uniformly at `clusters` times the overall density.  A stand-in for the
    block structure pruned layers can show (heads, channel groups): rows of one group share
    their columns, rows of different groups share none - the case a row swizzle is for.
    """
    rng = np.random.default_rng(seed)
    group_of_row = rng.permutation(M) % clusters
    col_group = rng.permutation(K) % clusters
    W = rng.standard_normal((M, K))
    allowed = group_of_row[:, None] == col_group[None, :]
    nnz = int(round((1.0 - sparsity) * M * K))
    assert nnz <= int(allowed.sum()), "density x clusters must stay below 1"
    score = np.where(allowed, rng.random((M, K)), -1.0)
    keep = np.argsort(-score.reshape(-1), kind="stable")[:nnz]
    mask = np.zeros(M * K, dtype=bool)
    mask[keep] = True
    return csr_from_mask(_as_dtype(W, dtype), mask.reshape(M, K))


def small_int_csr(M, K, sparsity, seed, dtype=np.float32, vmax=4) -> CSR:
    """Uniform mask with nonzeros in {-vmax..vmax} minus {0}.

    Together with small_int_dense every partial sum is an exactly representable
    integer, so any summation order gives the same bits.
    """
    rng = np.random.default_rng(seed)
    mask = uniform_mask(M, K, sparsity, rng)
    W = rng.integers(1, vmax + 1, size=(M, K)) * rng.choice([-1, 1], size=(M, K))
    return csr_from_mask(W.astype(dtype), mask)


def int8_csr(M, K, sparsity, seed) -> CSR:
    """Uniform mask, values uniform over the int8 range without zero (a quantised weight matrix)."""
    rng = np.random.default_rng(seed)
    mask = uniform_mask(M, K, sparsity, rng)
    W = rng.integers(1, 128, size=(M, K)) * rng.choice([-1, 1], size=(M, K))
    W[rng.random((M, K)) < 0.01] = -128          # the asymmetric end of the range shows up too
    return csr_from_mask(W.astype(np.int8), mask)


def int8_dense(K, N, seed) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(-128, 128, size=(K, N)).astype(np.int8)


def small_int_dense(K, N, seed, dtype=np.float32, bmax=8) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(-bmax, bmax + 1, size=(K, N)).astype(dtype)


def normal_dense(K, N, seed, dtype=np.float32, relu=False) -> np.ndarray:
    rng = np.random.default_rng(seed)
    B = rng.standard_normal((K, N))
    if relu:
        B = np.maximum(B, 0.0)
    return _as_dtype(B, dtype)


def conv_weights_csr(Cout, Cin, sparsity, seed, dtype=np.float32) -> Tuple[CSR, np.ndarray]:
    """Magnitude-pruned 3x3 filters.

    Returns the CSR of the [Cout, Cin*9] flattening (k = c*9 + r*3 + s, the
    C-order flattening of [Cout, Cin, 3, 3]) and the dense zero-filled
    [Cout, Cin, 3, 3] tensor holding the same values.
    """
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((Cout, Cin, 3, 3))
    mask = magnitude_mask(W, sparsity)
    Wd = _as_dtype(W, dtype).reshape(Cout, Cin * 9)
    csr = csr_from_mask(Wd, mask)
    dense = np.where(mask, Wd, np.zeros_like(Wd)).reshape(Cout, Cin, 3, 3)
    return csr, np.ascontiguousarray(dense)


@dataclass
class Case:
    """One synthetic problem instance."""

    name: str
    csr: CSR
    N: int
    B: Optional[np.ndarray] = None  # [K, N] for SpMM
    X: Optional[np.ndarray] = None  # [1, Cin, H, W] for conv
    Wdense: Optional[np.ndarray] = None  # [Cout, Cin, 3, 3] for conv
    conv: Optional[Tuple[int, int, int]] = None  # (Cin, H, W)
    sparsity: float = 0.0


def config(name: str, dtype=np.float32) -> Case:
    """The named configurations of the headline benchmark.

    c1  : 256x256 @ 90 % uniform mask, N(0,1) values, B 256x1024 N(0,1)
    c2  : MobileNet-like 1x1 conv: 512x512 @ 90 % magnitude-pruned N(0,1),
          B = ReLU(N(0,1)) of shape 512 x 196 (batch 1, 14x14)
    c3  : Transformer FC: 3072x768 @ 95 % magnitude-pruned N(0, std 0.02), B 768x1024
    c3t : the transposed projection 768x3072 (independent draw), B 3072x1024
    c4  : 3x3 conv, 256 -> 256 channels, 14x14, pad 1, @ 90 % magnitude-pruned

    dtype int8: the float32 case quantised - weights symmetric per tensor to -127..127 (kept
    weights that round to zero become +-1, so the pattern is unchanged), activations times 32
    and clipped to -128..127 (four standard deviations).
    """
    if np.dtype(dtype) == np.int8:
        return _quantised(config(name, np.float32))
    if name == "c1":
        s = BASE_SEED + 0
        return Case("c1", uniform_csr(256, 256, 0.90, s, dtype), 1024,
                    B=normal_dense(256, 1024, s + 1000, dtype), sparsity=0.90)
    if name == "c2":
        s = BASE_SEED + 1
        return Case("c2", magnitude_csr(512, 512, 0.90, s, 1.0, dtype), 196,
                    B=normal_dense(512, 196, s + 1000, dtype, relu=True), sparsity=0.90)
    if name == "c3":
        s = BASE_SEED + 2
        return Case("c3", magnitude_csr(3072, 768, 0.95, s, 0.02, dtype), 1024,
                    B=normal_dense(768, 1024, s + 1000, dtype), sparsity=0.95)
    if name == "c3t":
        s = BASE_SEED + 3
        return Case("c3t", magnitude_csr(768, 3072, 0.95, s, 0.02, dtype), 1024,
                    B=normal_dense(3072, 1024, s + 1000, dtype), sparsity=0.95)
    if name == "c4":
        s = BASE_SEED + 4
        csr, Wd = conv_weights_csr(256, 256, 0.90, s, dtype)
        X = normal_dense(256, 14 * 14, s + 1000, dtype).reshape(1, 256, 14, 14)
        return Case("c4", csr, 196, X=X, Wdense=Wd, conv=(256, 14, 14), sparsity=0.90)
    raise KeyError(name)


def quantise_weights(w: np.ndarray) -> np.ndarray:
    """Symmetric per-tensor int8; nonzero inputs stay nonzero."""
    top = float(np.abs(w).max()) if w.size else 1.0
    q = np.clip(np.rint(w / (top if top > 0 else 1.0) * 127.0), -127, 127).astype(np.int8)
    lost = (q == 0) & (w != 0)
    q[lost] = np.where(w[lost] > 0, 1, -1).astype(np.int8)
    return q


def quantise_activations(x: np.ndarray) -> np.ndarray:
    return np.clip(np.rint(x * 32.0), -128, 127).astype(np.int8)


def _quantised(case: Case) -> Case:
    csr = case.csr
    top = np.abs(case.Wdense).max() if case.Wdense is not None else None
    q = CSR(csr.M, csr.K, csr.row_ptr, csr.col_idx, quantise_weights(csr.vals))
    Wq = None
    if case.Wdense is not None:   # same scale as the CSR values: both come from the same tensor
        assert top == np.abs(csr.vals).max()
        Wq = quantise_weights(case.Wdense)
    return Case(case.name, q, case.N,
                B=None if case.B is None else quantise_activations(case.B),
                X=None if case.X is None else quantise_activations(case.X),
                Wdense=Wq, conv=case.conv, sparsity=case.sparsity)


def sweep_seed(M, K, N, sparsity, mask_kind, dtype) -> int:
    """Seed of a sweep case, derived from the case tuple alone."""
    kind = {"uniform": 1, "magnitude": 2, "skewed": 3}[mask_kind]
    half = 1 if np.dtype(dtype) == np.float16 else 0
    h = (M * 1000003 + K * 10007 + N * 101 + int(round(sparsity * 1000)) * 7 + kind * 3 + half)
    return BASE_SEED + 5 + (h % 1000000007)


def sweep_case(M, K, N, sparsity, mask_kind="uniform", dtype=np.float32) -> Case:
    """A case of the shape/sparsity sweep (config 5)."""
    s = sweep_seed(M, K, N, sparsity, mask_kind, dtype)
    if mask_kind == "uniform":
        csr = uniform_csr(M, K, sparsity, s, dtype)
    elif mask_kind == "magnitude":
        csr = magnitude_csr(M, K, sparsity, s, 1.0, dtype)
    elif mask_kind == "skewed":
        csr = skewed_csr(M, K, sparsity, s, dtype)
    else:
        raise KeyError(mask_kind)
    name = f"sweep_{M}x{K}x{N}_s{sparsity}_{mask_kind}_{np.dtype(dtype).name}"
    return Case(name, csr, N, B=normal_dense(K, N, s + 1000, dtype), sparsity=sparsity)


# ---------------------------------------------------------------- the paper's problem lists
# Shapes only (Table 1: twenty SpMM problems from ResNet-50, Transformer and MobileNetV1, at 90 %
# and, for problems 1-11, 95 % sparsity; Table 3: four 3x3 convolutions as (image, Cin, Cout)).
# The pruned checkpoints behind them are not available; weights are magnitude-pruned N(0,1) draws.
TABLE1 = [(64, 256, 3136), (256, 64, 3136), (128, 512, 784), (512, 128, 784), (256, 1024, 196),
          (1024, 256, 196), (512, 2048, 49), (2048, 512, 49), (2048, 512, 256), (512, 2048, 256),
          (512, 512, 256), (64, 32, 12544), (128, 64, 3136), (128, 128, 3136), (256, 128, 784),
          (256, 256, 784), (512, 256, 196), (512, 512, 196), (1024, 512, 49), (1024, 1024, 49)]
TABLE3 = [(56, 64, 64), (28, 128, 128), (14, 256, 256), (7, 512, 512)]


def table1_problems():
    """(tag, index, sparsity) of every Table 1 instance: problems 1-20 at 90 %, 1-11 at 95 %."""
    out = [(f"t1_p{i + 1}_90", i, 0.90) for i in range(len(TABLE1))]
    out += [(f"t1_p{i + 1}_95", i, 0.95) for i in range(11)]
    return out


def table1_case(i: int, sparsity: float, dtype=np.float32) -> Case:
    M, K, N = TABLE1[i]
    pct = int(round(sparsity * 100))
    seed = BASE_SEED + 1000 + 100 * i + pct
    return Case(f"t1_p{i + 1}_{pct}", magnitude_csr(M, K, sparsity, seed, 1.0, dtype), N,
                B=normal_dense(K, N, seed + 1, dtype), sparsity=sparsity)


def table3_case(i: int, sparsity: float, dtype=np.float32, batch: int = 1) -> Case:
    img, Cin, Cout = TABLE3[i]
    pct = int(round(sparsity * 100))
    seed = BASE_SEED + 5000 + 100 * i + pct
    csr, Wd = conv_weights_csr(Cout, Cin, sparsity, seed, dtype)
    X = normal_dense(batch * Cin, img * img, seed + 1, dtype).reshape(batch, Cin, img, img)
    return Case(f"t3_p{i + 1}_{pct}", csr, img * img, X=X, Wdense=Wd, conv=(Cin, img, img), sparsity=sparsity)


# ---------------------------------------------------------------- the shape / sparsity sweep
SWEEP_MK = [256, 512, 1024, 2048, 4096]
SWEEP_N = [64, 196, 784, 3136, 4096]
SWEEP_SPARSITY = [0.80, 0.90, 0.95, 0.98]
# The measured subset of the M x K cross product: the squares and two 4:1 rectangles.
SWEEP_SHAPES = [(m, m) for m in SWEEP_MK] + [(4096, 1024), (1024, 4096)]


def sweep_sample(count: int, seed: int = BASE_SEED + 77):
    """A seeded sample of the full sweep grid as (M, K, N, sparsity, mask kind, dtype) tuples:
    independent uniform draws per axis, except that on every axis the first len(axis) positions
    (in a seeded rotation) run through all of the axis' values, so that each size, each N, each
    sparsity, both mask kinds and both storage types occur (count >= 5)."""
    rng = np.random.default_rng(seed)
    axes = [SWEEP_MK, SWEEP_MK, SWEEP_N, SWEEP_SPARSITY, ["uniform", "skewed"], [np.float32, np.float16]]
    cols = []
    for a in axes:
        idx = rng.integers(0, len(a), size=count)
        forced = (int(rng.integers(0, count)) + np.arange(len(a))) % count
        idx[forced] = rng.permutation(len(a))
        cols.append([a[i] for i in idx])
    return list(zip(*cols))
