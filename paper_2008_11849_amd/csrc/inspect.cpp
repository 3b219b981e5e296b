// Host-side inspector (Sections 2.3 and 3.4): integer analysis of the fixed
// sparsity pattern.  Nothing here touches a value arithmetically.
#include <algorithm>
#include <climits>
#include <cstring>
#include <numeric>

#include "plan.h"

namespace sparsert {

static inline int bin_of(int32_t x) {
    int b = 0;
    while (x > 0) { ++b; x >>= 1; }
    return b;  // 0 for x == 0, else 1 + floor(log2 x)
}

static int validate(const int32_t *row_ptr, const int32_t *col_idx, const void *vals,
                    int32_t M, int32_t K, int32_t N, const sparsert_options &opt,
                    std::string &err) {
    if (!row_ptr) { err = "row_ptr is NULL"; return SPARSERT_EINVAL; }
    if (M <= 0 || K <= 0 || N <= 0) { err = "M, K and N must be positive"; return SPARSERT_EINVAL; }
    if (opt.dtype != SPARSERT_F32 && opt.dtype != SPARSERT_F16 && opt.dtype != SPARSERT_I8) { err = "unknown dtype"; return SPARSERT_EINVAL; }
    if (opt.kernel < SPARSERT_KERNEL_AUTO || opt.kernel > SPARSERT_KERNEL_SPEC) { err = "unknown kernel family"; return SPARSERT_EINVAL; }
    if (opt.natural_order != 0 && opt.natural_order != 1) { err = "natural_order must be 0 or 1"; return SPARSERT_EINVAL; }
    if (opt.spec_lanes != 0 && opt.spec_lanes != 16 && opt.spec_lanes != 32 && opt.spec_lanes != 64) { err = "spec_lanes must be 0,16,32,64"; return SPARSERT_EINVAL; }
    if (opt.spec_swizzle != 0 && opt.spec_swizzle != 1) { err = "spec_swizzle must be 0 or 1"; return SPARSERT_EINVAL; }
    if (opt.spec_vec != 0 && opt.spec_vec != 1 && opt.spec_vec != 2 && opt.spec_vec != 4) { err = "spec_vec must be 0,1,2,4"; return SPARSERT_EINVAL; }
    if (opt.spec_prefetch != 0 && opt.spec_prefetch != 1) { err = "spec_prefetch must be 0 or 1"; return SPARSERT_EINVAL; }
    for (int i = 0; i < 2; ++i)
        if (opt.reserved[i] != 0) { err = "reserved option fields must be zero"; return SPARSERT_EINVAL; }
    if (row_ptr[0] != 0) { err = "row_ptr[0] must be 0"; return SPARSERT_EINVAL; }
    for (int32_t m = 0; m < M; ++m)
        if (row_ptr[m + 1] < row_ptr[m]) { err = "row_ptr must be non-decreasing"; return SPARSERT_EINVAL; }
    const int32_t nnz = row_ptr[M];
    if (nnz > 0 && (!col_idx || !vals)) { err = "col_idx / vals is NULL"; return SPARSERT_EINVAL; }
    for (int32_t m = 0; m < M; ++m) {
        for (int32_t p = row_ptr[m]; p < row_ptr[m + 1]; ++p) {
            const int32_t c = col_idx[p];
            if (c < 0 || c >= K) { err = "column index out of range"; return SPARSERT_EINVAL; }
            if (p > row_ptr[m] && c <= col_idx[p - 1]) {
                err = "columns must be strictly ascending inside a row";
                return SPARSERT_EINVAL;
            }
        }
    }
    const int vmax = opt.dtype == SPARSERT_F16 ? 8 : 4;
    if (opt.vec != 0) {
        const int v = opt.vec;
        if (!(v == 1 || v == 2 || v == 4 || v == 8) || v > vmax || (opt.dtype == SPARSERT_I8 && v == 2)) {
            err = "vec must be 0,1,2,4 (8 for f16; 1 or 4 for int8)"; return SPARSERT_EINVAL;
        }
        if (N % v != 0) { err = "N must be a multiple of vec"; return SPARSERT_EINVAL; }
        if ((opt.ldb && opt.ldb % v) || (opt.ldc && opt.ldc % v)) { err = "ldb and ldc must be multiples of vec"; return SPARSERT_EINVAL; }
        if (opt.conv && v != 1) { err = "conv plans use vec = 1"; return SPARSERT_EINVAL; }
    }
    if (opt.spec_depth < 0 || opt.spec_depth > 48) { err = "spec_depth must be in 0..48"; return SPARSERT_EINVAL; }
    if (opt.spec_tiles != 0 && opt.spec_tiles != 1 && opt.spec_tiles != 2 && opt.spec_tiles != 4 &&
        opt.spec_tiles != 8 && opt.spec_tiles != 16) { err = "spec_tiles must be 0,1,2,4,8,16"; return SPARSERT_EINVAL; }
    if (opt.spec_mode < SPARSERT_SPEC_AUTO || opt.spec_mode > SPARSERT_SPEC_LDS) { err = "unknown spec_mode"; return SPARSERT_EINVAL; }
    if (opt.spec_rows < 0) { err = "spec_rows must be >= 0"; return SPARSERT_EINVAL; }
    if (opt.split_threshold < 0) { err = "split_threshold must be >= 0"; return SPARSERT_EINVAL; }
    const int64_t esz = opt.dtype == SPARSERT_F16 ? 2 : opt.dtype == SPARSERT_I8 ? 1 : 4;
    const int64_t osz = opt.dtype == SPARSERT_F16 ? 2 : 4;
    // int8: |sum| <= K * 128 * 128 must stay below 2^31
    if (opt.dtype == SPARSERT_I8 && K >= (1 << 17)) { err = "K too long for exact 32-bit sums of int8 products"; return SPARSERT_EUNSUPPORTED; }
    if (opt.batch < 0 || opt.batch > 65535) { err = "batch must be in 0..65535"; return SPARSERT_EINVAL; }
    if (opt.tune_warm != 0 && opt.tune_warm != 1) { err = "tune_warm must be 0 or 1"; return SPARSERT_EINVAL; }
    if ((opt.ldb != 0 && opt.ldb < N) || (opt.ldc != 0 && opt.ldc < N)) { err = "ldb and ldc must be 0 or at least N"; return SPARSERT_EINVAL; }
    if (opt.conv && (opt.ldb || opt.ldc)) { err = "convolution plans take no leading dimensions"; return SPARSERT_EINVAL; }
    const int64_t ldb = opt.ldb ? opt.ldb : N, ldc = opt.ldc ? opt.ldc : N;
    if (opt.conv) {
        if (opt.conv != 1) { err = "conv must be 0 or 1"; return SPARSERT_EINVAL; }
        if (opt.Cin <= 0 || opt.H <= 0 || opt.W <= 0) { err = "conv needs Cin, H, W > 0"; return SPARSERT_EINVAL; }
        if ((int64_t)K != 9ll * opt.Cin) { err = "conv needs K == 9*Cin"; return SPARSERT_EINVAL; }
        if ((int64_t)N != (int64_t)opt.H * opt.W) { err = "conv needs N == H*W"; return SPARSERT_EINVAL; }
        if (((int64_t)opt.Cin * opt.H * opt.W + opt.W + 1) * esz >= (1ll << 27)) {
            err = "conv input too large for 28-bit operand displacements"; return SPARSERT_EUNSUPPORTED;
        }
        if ((int64_t)M * N * osz >= (1ll << 31)) { err = "one image of Y reaches 2 GiB"; return SPARSERT_EUNSUPPORTED; }
    } else if ((int64_t)K * ldb * esz >= (1ll << 31) || (int64_t)M * ldc * osz >= (1ll << 31)) {
        err = "B or C reaches 2 GiB: operand offsets are 32-bit"; return SPARSERT_EUNSUPPORTED;
    }
    return SPARSERT_OK;
}

// Columns of C per lane.  A wave covers n_tiles(V) = ceil(N/(64 V)) tiles and
// issues V multiply-adds per nonzero per tile, so work(V) = n_tiles(V) * V.
// Among the V dividing N whose work is within 7 % of the least, take the
// largest that still leaves kFullTasks wave tasks; if none does, the smallest.
// `skip` names a V the storage type has no kernel for (2 for int8), or 0.  V also has to divide
// the row pitches of B and C.
static int choose_vec(int32_t M, int32_t N, int32_t ldb, int32_t ldc, int vmax, int skip) {
    int cand[4], nc = 0;
    int64_t work[4], wmin = INT64_MAX;
    for (int v = 1; v <= vmax; v *= 2) {
        if (N % v || ldb % v || ldc % v || v == skip) continue;   // a lane's V columns are one aligned vector access
        const int64_t tiles = ((int64_t)N / v + kWave - 1) / kWave;
        cand[nc] = v; work[nc] = tiles * v; wmin = std::min(wmin, work[nc]); ++nc;
    }
    int best = -1, smallest = -1;
    for (int i = 0; i < nc; ++i) {
        if (work[i] * 100 > wmin * 107) continue;
        if (smallest < 0) smallest = cand[i];
        const int64_t tiles = ((int64_t)N / cand[i] + kWave - 1) / kWave;
        if ((int64_t)M * tiles >= kFullTasks) best = cand[i];
    }
    return best > 0 ? best : smallest;
}

int build_host_plan(const int32_t *row_ptr, const int32_t *col_idx, const void *vals,
                    int32_t M, int32_t K, int32_t N, const sparsert_options &opt,
                    HostPlan &h, std::string &err) {
    if (int rc = validate(row_ptr, col_idx, vals, M, K, N, opt, err)) return rc;
    h.M = M; h.K = K; h.N = N; h.nnz = row_ptr[M];
    h.dtype = opt.dtype; h.conv = opt.conv ? 1 : 0;
    h.Cin = h.conv ? opt.Cin : 0; h.H = h.conv ? opt.H : 0; h.W = h.conv ? opt.W : 0;
    h.batch = std::max(1, opt.batch);
    h.ldb = opt.ldb ? opt.ldb : N;
    h.ldc = opt.ldc ? opt.ldc : N;
    // AUTO: the per-matrix generated kernel with the inspector's shape defaults where it can be
    // built in a few seconds (the inspector is off the latency path, Section 2.3), else the
    // row-walk kernel, whose inspector generates nothing.  Options that only the row-walk kernel
    // reads (vec, split_threshold) select it as well.
    if (opt.kernel != SPARSERT_KERNEL_AUTO) h.kernel = opt.kernel;
    else h.kernel = (opt.vec == 0 && opt.split_threshold == 0 && h.nnz <= kAutoSpecNnz && spec_available())
                        ? SPARSERT_KERNEL_SPEC : SPARSERT_KERNEL_ROWS;
    h.kernel_auto = opt.kernel == SPARSERT_KERNEL_AUTO;
    const int esz = h.elem_size();

    // Row histogram and the nnz-descending stable row order.
    h.row_nnz.resize(M);
    h.hist.assign(kBins, 0);
    for (int32_t m = 0; m < M; ++m) {
        h.row_nnz[m] = row_ptr[m + 1] - row_ptr[m];
        ++h.hist[bin_of(h.row_nnz[m])];
    }
    h.perm.resize(M);
    std::iota(h.perm.begin(), h.perm.end(), 0);
    h.natural_order = opt.natural_order;
    if (!h.natural_order)
        std::stable_sort(h.perm.begin(), h.perm.end(),
                         [&](int32_t a, int32_t b) { return h.row_nnz[a] > h.row_nnz[b]; });
    h.inv_perm.resize(M);
    for (int32_t i = 0; i < M; ++i) h.inv_perm[h.perm[i]] = i;

    // Permuted CSR: rows gathered by perm, values copied bit for bit.
    h.p_row_ptr.resize(M + 1);
    h.p_col_idx.resize(h.nnz);
    h.p_vals.resize((size_t)h.nnz * esz);
    h.p_row_ptr[0] = 0;
    const uint8_t *vsrc = static_cast<const uint8_t *>(vals);
    for (int32_t i = 0; i < M; ++i) {
        const int32_t r = h.perm[i], n = h.row_nnz[r], dst = h.p_row_ptr[i];
        if (n) {
            std::memcpy(&h.p_col_idx[dst], col_idx + row_ptr[r], (size_t)n * sizeof(int32_t));
            std::memcpy(&h.p_vals[(size_t)dst * esz], vsrc + (size_t)row_ptr[r] * esz, (size_t)n * esz);
        }
        h.p_row_ptr[i + 1] = dst + n;
    }

    // Bins: maximal runs of slots whose rows share a bin id.
    h.bins.clear();
    for (int32_t i = 0; i < M;) {
        const int b = bin_of(h.row_nnz[h.perm[i]]);
        int32_t j = i;
        while (j < M && bin_of(h.row_nnz[h.perm[j]]) == b) ++j;
        h.bins.insert(h.bins.end(), {b, i, j - i, h.p_row_ptr[j] - h.p_row_ptr[i]});
        i = j;
    }

    // Column tiling.
    const int vmax = h.conv ? 1 : (h.dtype == SPARSERT_F16 ? 8 : 4);
    h.vec = opt.vec ? opt.vec : choose_vec(M, N, h.ldb, h.ldc, vmax, h.dtype == SPARSERT_I8 ? 2 : 0);
    const int32_t nvc = N / h.vec;  // vector columns
    h.n_tiles = (nvc + kWave - 1) / kWave;
    h.lanes_per_tile = (nvc + h.n_tiles - 1) / h.n_tiles;
    h.gy = kGy;

    // Long rows are split over the waves of one workgroup.
    if (opt.split_threshold) h.split_threshold = opt.split_threshold;
    else h.split_threshold = ((int64_t)M * h.n_tiles < kFullTasks) ? 64 : 512;
    h.n_split = 0;
    if (h.natural_order) h.split_threshold = INT32_MAX;   // split rows are a prefix of the sorted order only
    while (h.n_split < M && h.row_nnz[h.perm[h.n_split]] >= h.split_threshold) ++h.n_split;
    h.n_wg_rows = h.n_split + (M - h.n_split + h.gy - 1) / h.gy;
    h.segments.resize((size_t)h.n_split * (h.gy + 1));
    for (int32_t i = 0; i < h.n_split; ++i) {
        const int32_t start = h.p_row_ptr[i], n = h.p_row_ptr[i + 1] - start;
        const int32_t share = (n + h.gy - 1) / h.gy;  // every wave but the last gets `share`
        for (int g = 0; g <= h.gy; ++g)
            h.segments[(size_t)i * (h.gy + 1) + g] = start + std::min<int64_t>((int64_t)g * share, n);
    }

    // The nonzero stream the executor reads: {operand byte offset, value as binary32 bits};
    // int8 plans: the value sign-extended to 32 bits.
    h.stream.resize((size_t)h.nnz * 2);
    auto value_bits = [&](int32_t p) -> uint32_t {
        if (h.dtype == SPARSERT_F16) {
            uint16_t hb; std::memcpy(&hb, &h.p_vals[(size_t)p * 2], 2);
            return half_bits_to_float_bits(hb);
        }
        if (h.dtype == SPARSERT_I8) return (uint32_t)(int32_t)(int8_t)h.p_vals[(size_t)p];
        uint32_t fb; std::memcpy(&fb, &h.p_vals[(size_t)p * 4], 4);
        return fb;
    };
    if (!h.conv) {
        for (int32_t p = 0; p < h.nnz; ++p) {
            h.stream[2 * (size_t)p] = (uint32_t)((uint64_t)h.p_col_idx[p] * (uint64_t)h.ldb * esz);
            h.stream[2 * (size_t)p + 1] = value_bits(p);
        }
    } else {
        // Section 3.6: each reference to B[k, oh*W+ow], k = c*9 + r*3 + s, is the input
        // element X[c, oh+r-1, ow+s-1].  Relative to pixel (oh,ow) of channel 0 that is the
        // fixed (possibly negative) displacement c*H*W + (r-1)*W + (s-1).  The stream word holds
        // the tap r*3+s in its top 4 bits and the byte displacement in the low 28 (two's complement).
        // Inside a slot the nonzeros are grouped by tap (r,s) so that the padding test is
        // made once per group instead of once per multiply-add.
        h.conv_seg.resize((size_t)M * 10);
        const int32_t HW = h.H * h.W;
        for (int32_t i = 0; i < M; ++i) {
            const int32_t s0 = h.p_row_ptr[i], s1 = h.p_row_ptr[i + 1];
            int32_t count[9] = {0};
            for (int32_t p = s0; p < s1; ++p) ++count[h.p_col_idx[p] % 9];
            int32_t pos[10];
            pos[0] = s0;
            for (int t = 0; t < 9; ++t) pos[t + 1] = pos[t] + count[t];
            for (int t = 0; t < 10; ++t) h.conv_seg[(size_t)i * 10 + t] = pos[t];
            for (int32_t p = s0; p < s1; ++p) {  // ascending k => ascending c inside a group
                const int32_t k = h.p_col_idx[p], c = k / 9, rs = k % 9, r = rs / 3, s = rs % 3;
                const int32_t q = pos[rs]++;
                const int64_t off = (int64_t)c * HW + (r - 1) * h.W + (s - 1);
                h.stream[2 * (size_t)q] = ((uint32_t)(int32_t)(off * esz) & 0x0fffffffu) | ((uint32_t)rs << 28);
                h.stream[2 * (size_t)q + 1] = value_bits(p);
            }
        }
    }
    return SPARSERT_OK;
}

}  // namespace sparsert
