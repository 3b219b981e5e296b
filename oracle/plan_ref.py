"""NumPy statement of the inspector's plan specification (TEST INFRASTRUCTURE ONLY).

Written from the specification, not from the C++ inspector; the two share no
code.  Everything here is integer work on the sparsity pattern (Sections 2.3,
3.4 of the paper: offline analysis, load balance over blocks and thread
groups); values are only moved.

Specification
  row_nnz[m]  = row_ptr[m+1] - row_ptr[m]
  bin(x)      = 0 if x == 0 else 1 + floor(log2 x);  hist[b] = rows with bin == b (33 bins)
  perm        = rows in stable order of descending row_nnz (ties: ascending row)
  permuted CSR= rows gathered by perm; columns stay ascending; values bit-copied
  bins        = maximal runs of slots with equal bin: (bin, first slot, rows, nonzeros)
  V           = columns of C per lane.  Candidates 1,2,4 (and 8 for half) dividing N;
                work(V) = ceil((N/V)/64) * V; keep those with work <= 1.07 * least work;
                take the largest with M * tiles(V) >= 2048, else the smallest kept
  tiles       = ceil((N/V)/64); lanes_per_tile = ceil((N/V)/tiles)
  threshold   = 64 if M*tiles < 2048 else 512 (unless given); slots with row_nnz >= threshold
                are split rows (they are the first n_split slots)
  segments    = for a split slot with n nonzeros starting at s: share = ceil(n/Gy), bounds
                s + min(g*share, n), g = 0..Gy  (all waves but the last get `share`)
  stream      = per nonzero {int32 byte offset, float32 bits of the value}
                SpMM: offset = col*ldb*itemsize (ldb = row pitch of B, N unless given), permuted-CSR order
                conv: k = c*9 + r*3 + s  ->  word = tap << 28 | (displacement & 0x0fffffff) with
                tap = r*3+s and displacement = (c*H*W + (r-1)*W + (s-1))*itemsize; each slot
                stably reordered by tap; conv_seg[slot] holds the ten stream positions where
                the taps start/end
  kernel      = executor family when the caller leaves the choice to the inspector: 2 (per-matrix
                generated code) if nnz <= 4194304 and neither vec nor split_threshold is given,
                else 1 (row-walk).  (Stated for a process that can load the code object manager.)
"""
from __future__ import annotations

import numpy as np

GY = 4
WAVE = 64
FULL_TASKS = 2048
AUTO_SPEC_NNZ = 4 * 1024 * 1024


def _bin(x: np.ndarray) -> np.ndarray:
    out = np.zeros(x.shape, dtype=np.int64)
    nz = x > 0
    out[nz] = 1 + np.floor(np.log2(x[nz].astype(np.float64))).astype(np.int64)
    # guard the float log2 at exact powers of two
    for b in range(1, 33):
        out[(x >= (1 << (b - 1))) & (x < (1 << b))] = b
    return out


def choose_vec(M, N, vmax, skip=0, ldb=0, ldc=0):
    # a lane's V columns are one aligned vector access: V divides N and both row pitches
    cands = [v for v in (1, 2, 4, 8) if v <= vmax and N % v == 0 and ldb % v == 0 and ldc % v == 0 and v != skip]
    tiles = {v: -(-(N // v) // WAVE) for v in cands}
    work = {v: tiles[v] * v for v in cands}
    wmin = min(work.values())
    kept = [v for v in cands if work[v] * 100 <= wmin * 107]
    full = [v for v in kept if M * tiles[v] >= FULL_TASKS]
    return max(full) if full else min(kept)


def plan(row_ptr, col_idx, vals, M, K, N, conv=None, vec=0, split_threshold=0, natural_order=False, ldb=0, ldc=0):
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    col_idx = np.asarray(col_idx, dtype=np.int64)
    vals = np.asarray(vals)
    half = vals.dtype == np.float16
    int8 = vals.dtype == np.int8
    item = 2 if half else 1 if int8 else 4
    nnz = int(row_ptr[M])
    row_nnz = np.diff(row_ptr)
    bins_of = _bin(row_nnz)
    hist = np.bincount(bins_of, minlength=33)
    # natural order (load-balance ablation): identity permutation and no split rows
    perm = np.arange(M) if natural_order else np.argsort(-row_nnz, kind="stable")
    inv_perm = np.empty(M, dtype=np.int64)
    inv_perm[perm] = np.arange(M)
    p_nnz = row_nnz[perm]
    p_row_ptr = np.concatenate([[0], np.cumsum(p_nnz)])
    gather = np.concatenate([np.arange(row_ptr[r], row_ptr[r + 1]) for r in perm]) if nnz else np.zeros(0, np.int64)
    gather = gather.astype(np.int64)
    p_col = col_idx[gather]
    p_vals = vals[gather]

    pb = bins_of[perm]
    bins = []
    i = 0
    while i < M:
        j = i
        while j < M and pb[j] == pb[i]:
            j += 1
        bins.append((pb[i], i, j - i, p_row_ptr[j] - p_row_ptr[i]))
        i = j

    vmax = 1 if conv else (8 if half else 4)
    ldb, ldc = ldb or N, ldc or N   # elements between consecutive rows of B and of C
    V = vec if vec else choose_vec(M, N, vmax, skip=2 if int8 else 0, ldb=ldb, ldc=ldc)   # int8: one column or a packed dword of four
    nvc = N // V
    n_tiles = -(-nvc // WAVE)
    lanes_per_tile = -(-nvc // n_tiles)
    thr = split_threshold if split_threshold else (64 if M * n_tiles < FULL_TASKS else 512)
    if natural_order:
        thr = 2**31 - 1
    n_split = int(np.sum(p_nnz >= thr))
    n_wg_rows = n_split + -(-(M - n_split) // GY)
    segments = np.zeros((n_split, GY + 1), dtype=np.int64)
    for s in range(n_split):
        n = int(p_nnz[s])
        share = -(-n // GY)
        segments[s] = p_row_ptr[s] + np.minimum(np.arange(GY + 1) * share, n)

    if int8:
        val_bits = p_vals.astype(np.int32).view(np.uint32)    # sign-extended
    else:
        val_bits = p_vals.astype(np.float32).view(np.uint32)  # half -> float is exact
    stream = np.zeros((nnz, 2), dtype=np.uint32)
    conv_seg = np.zeros((0,), dtype=np.int64)
    if not conv:
        stream[:, 0] = (p_col * ldb * item).astype(np.int64).astype(np.uint32)
        stream[:, 1] = val_bits
    else:
        Cin, H, W = conv
        c, t = p_col // 9, p_col % 9
        r, s = t // 3, t % 3
        off = ((c * H * W + (r - 1) * W + (s - 1)) * item).astype(np.int64)
        off32 = ((off & 0x0FFFFFFF) | (t << 28)).astype(np.uint32)
        conv_seg = np.zeros((M, 10), dtype=np.int64)
        for slot in range(M):
            a, b = int(p_row_ptr[slot]), int(p_row_ptr[slot + 1])
            order = np.argsort(t[a:b], kind="stable") + a
            stream[a:b, 0] = off32[order]
            stream[a:b, 1] = val_bits[order]
            conv_seg[slot] = a + np.concatenate([[0], np.cumsum(np.bincount(t[a:b], minlength=9))])

    info = dict(M=M, K=K, N=N, nnz=nnz, dtype=1 if half else 2 if int8 else 0, conv=1 if conv else 0,
                Cin=conv[0] if conv else 0, H=conv[1] if conv else 0, W=conv[2] if conv else 0,
                kernel=2 if (nnz <= AUTO_SPEC_NNZ and not vec and not split_threshold) else 1, vec=V, lanes_per_tile=lanes_per_tile, n_tiles=n_tiles, gy=GY,
                split_threshold=thr, n_split=n_split, n_wg_rows=n_wg_rows, n_bins=len(bins),
                ldb=ldb, ldc=ldc)
    i32 = lambda a: np.ascontiguousarray(np.asarray(a, dtype=np.int64).astype(np.int32))
    return dict(info=info, row_nnz=i32(row_nnz), hist=i32(hist), perm=i32(perm),
                inv_perm=i32(inv_perm), p_row_ptr=i32(p_row_ptr), p_col_idx=i32(p_col),
                p_vals=np.ascontiguousarray(p_vals), bins=i32(np.array(bins).reshape(-1)),
                stream=stream.reshape(-1), conv_seg=i32(conv_seg.reshape(-1)),
                segments=i32(segments.reshape(-1)))


def spec_groups(M, rows_per_group, natural_order=False):
    """Code block of every slot in the generated kernel: serpentine dealing of the
    nnz-descending slots over G = ceil(M/R) blocks (block-level balance, Section 3.4);
    in natural order, contiguous ranges of R rows."""
    R = min(rows_per_group, M)
    G = -(-M // R)
    i = np.arange(M)
    if natural_order:
        return (i // R).astype(np.int32)
    rnd, pos = i // G, i % G
    return np.where(rnd % 2 == 1, G - 1 - pos, pos).astype(np.int32)


def spec_groups_swizzled(p_row_ptr, p_col_idx, M, K, rows_per_group):
    """Row swizzle (Section 5 names it as a preprocessing step that would help): the
    nnz-descending slots are handed out in rounds of G = ceil(M/R); round 0 seeds block i
    with slot i; in every later round the blocks, visited in serpentine direction, each take
    the candidate of the round that shares the most columns with the union of the rows the
    block already holds (ties: the lowest slot)."""
    R = min(rows_per_group, M)
    G = -(-M // R)
    pat = np.zeros((M, K), dtype=bool)
    for i in range(M):
        pat[i, p_col_idx[p_row_ptr[i]:p_row_ptr[i + 1]]] = True
    union = np.zeros((G, K), dtype=bool)
    group = np.full(M, -1, dtype=np.int32)
    rnd = 0
    for first in range(0, M, G):
        cand = list(range(first, min(M, first + G)))
        for step in range(len(cand)):
            g = G - 1 - step if rnd % 2 else step
            free = [c for c in range(first, min(M, first + G)) if group[c] < 0]
            if rnd == 0:
                pick = free[0]
            else:
                shared = [(int(np.count_nonzero(pat[c] & union[g])), -c) for c in free]
                pick = -max(shared)[1]
            group[pick] = g
            union[g] |= pat[pick]
        rnd += 1
    return group
