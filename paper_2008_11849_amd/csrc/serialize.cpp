// Plan persistence: a tuned plan is built once, offline (the inspector of Section 2.3, the
// autotuner of Section 3.7), and an inference process only needs to load it.  The blob is the
// host plan field by field, little endian, behind a header with a magic word, a format
// version and an FNV-1a checksum of the payload.  The checksum guards against truncation and
// bit rot, not against a crafted blob: load only what sparsert_plan_save wrote.
#include <cstring>
#include <exception>
#include <new>
#include <string>
#include <vector>

#include "plan.h"

namespace {

constexpr uint32_t kMagic = 0x54525053u;   // "SPRT"
constexpr uint32_t kFormat = 3;   // bumped whenever the field list below changes

struct Writer {
    std::vector<uint8_t> out;
    void raw(const void *p, size_t n) { const uint8_t *b = static_cast<const uint8_t *>(p); out.insert(out.end(), b, b + n); }
    void i32(int32_t v) { raw(&v, 4); }
    void i64(int64_t v) { raw(&v, 8); }
    template <typename T> void vec(const std::vector<T> &v) { i64((int64_t)v.size()); if (!v.empty()) raw(v.data(), v.size() * sizeof(T)); }
    void str(const std::string &s) { i64((int64_t)s.size()); raw(s.data(), s.size()); }
};

struct Reader {
    const uint8_t *p, *end;
    bool ok = true;
    bool raw(void *dst, size_t n) {
        if (!ok || (size_t)(end - p) < n) { ok = false; return false; }
        std::memcpy(dst, p, n); p += n; return true;
    }
    int32_t i32() { int32_t v = 0; raw(&v, 4); return v; }
    int64_t i64() { int64_t v = 0; raw(&v, 8); return v; }
    template <typename T> void vec(std::vector<T> &v) {
        const int64_t n = i64();
        if (!ok || n < 0 || (uint64_t)n > (uint64_t)(end - p) / sizeof(T)) { ok = false; return; }
        v.resize((size_t)n);
        if (n) raw(v.data(), (size_t)n * sizeof(T));
    }
    void str(std::string &s) {
        const int64_t n = i64();
        if (!ok || n < 0 || n > end - p || n > 4096) { ok = false; return; }
        s.assign(reinterpret_cast<const char *>(p), (size_t)n); p += n;
    }
};

uint64_t fnv1a(const uint8_t *p, size_t n) {
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < n; ++i) { h ^= p[i]; h *= 1099511628211ull; }
    return h;
}

inline void field(Writer &w, int32_t &x) { w.i32(x); }
inline void field(Reader &r, int32_t &x) { x = r.i32(); }

template <typename IO> void scalars(IO &io, sparsert::HostPlan &h) {
    int32_t *f[] = {&h.M, &h.K, &h.N, &h.nnz, &h.dtype, &h.conv, &h.Cin, &h.H, &h.W, &h.kernel, &h.vec,
                    &h.lanes_per_tile, &h.n_tiles, &h.gy, &h.split_threshold, &h.n_split, &h.n_wg_rows,
                    &h.natural_order, &h.batch, &h.ldb, &h.ldc,
                    &h.spec.rows_per_group, &h.spec.n_groups, &h.spec.depth, &h.spec.n_tiles, &h.spec.lanes_per_tile,
                    &h.spec.tiles_per_wg, &h.spec.swizzle, &h.spec.vec, &h.spec.mode, &h.spec.n_blocks,
                    &h.spec.lds_bytes, &h.spec.ksplit, &h.spec.prefetch_lines};
    for (int32_t *x : f) field(io, *x);
}

// The relations every executor launch relies on, checked once more on what was read.
bool consistent(const sparsert::HostPlan &h) {
    if (h.M <= 0 || h.K <= 0 || h.N <= 0 || h.nnz < 0) return false;
    if (h.dtype < SPARSERT_F32 || h.dtype > SPARSERT_I8) return false;
    if (h.kernel != SPARSERT_KERNEL_ROWS && h.kernel != SPARSERT_KERNEL_SPEC) return false;
    const size_t M = (size_t)h.M, nnz = (size_t)h.nnz;
    if (h.row_nnz.size() != M || h.perm.size() != M || h.inv_perm.size() != M || h.p_row_ptr.size() != M + 1) return false;
    if (h.p_col_idx.size() != nnz || h.p_vals.size() != nnz * (size_t)h.elem_size() || h.stream.size() != 2 * nnz) return false;
    if (h.p_row_ptr[0] != 0 || h.p_row_ptr[M] != h.nnz) return false;
    for (size_t i = 0; i < M; ++i)
        if (h.p_row_ptr[i + 1] < h.p_row_ptr[i] || h.perm[i] < 0 || h.perm[i] >= h.M) return false;
    for (int32_t c : h.p_col_idx)
        if (c < 0 || c >= h.K) return false;
    if (h.n_split < 0 || h.n_split > h.M || h.segments.size() != (size_t)h.n_split * (size_t)(h.gy + 1)) return false;
    if (h.conv && h.conv_seg.size() != M * 10) return false;
    if (h.batch < 1 || h.batch > 65535) return false;
    if (h.ldb < h.N || h.ldc < h.N || (h.conv && (h.ldb != h.N || h.ldc != h.N))) return false;
    const int64_t esz = h.elem_size(), osz = h.out_elem_size();
    // Row-walk geometry: what launch_rows and rows_kernel index with.
    if (h.gy != sparsert::kGy || h.vec < 1 || h.vec > 8 || h.N % h.vec || h.ldb % h.vec || h.ldc % h.vec) return false;
    if (h.lanes_per_tile < 1 || h.lanes_per_tile > sparsert::kWave || h.n_tiles < 1) return false;
    if (h.n_wg_rows != h.n_split + (h.M - h.n_split + h.gy - 1) / h.gy) return false;
    // Split rows: the shares of slot i are ascending positions inside the slot's own nonzeros.
    for (int32_t i = 0; i < h.n_split; ++i) {
        const int32_t *sg = &h.segments[(size_t)i * (h.gy + 1)];
        if (sg[0] != h.p_row_ptr[i] || sg[h.gy] != h.p_row_ptr[i + 1]) return false;
        for (int g = 0; g < h.gy; ++g)
            if (sg[g + 1] < sg[g]) return false;
    }
    // The operand words the row-walk kernel turns into addresses.
    if (!h.conv) {
        if ((int64_t)h.K * h.ldb * esz >= (1ll << 31) || (int64_t)h.M * h.ldc * osz >= (1ll << 31)) return false;
        const uint64_t row_bytes = (uint64_t)h.ldb * (uint64_t)esz, limit = (uint64_t)h.K * row_bytes;
        for (size_t p = 0; p < nnz; ++p) {
            const uint64_t off = h.stream[2 * p];
            if (off >= limit || off % row_bytes) return false;
        }
    } else {
        if (h.Cin <= 0 || h.H <= 0 || h.W <= 0 || (int64_t)h.K != 9ll * h.Cin || (int64_t)h.N != (int64_t)h.H * h.W) return false;
        if (((int64_t)h.Cin * h.H * h.W + h.W + 1) * esz >= (1ll << 27)) return false;
        for (size_t i = 0; i < M; ++i) {
            const int32_t *cs = &h.conv_seg[i * 10];
            if (cs[0] != h.p_row_ptr[i] || cs[9] != h.p_row_ptr[i + 1]) return false;
            for (int t = 0; t < 9; ++t) {
                if (cs[t + 1] < cs[t]) return false;
                for (int32_t p = cs[t]; p < cs[t + 1]; ++p) {
                    // the word names tap t and a displacement (c*H*W + (r-1)*W + (s-1)) * esz with c < Cin
                    const uint32_t w = h.stream[2 * (size_t)p];
                    if ((int)(w >> 28) != t) return false;
                    const int64_t d = (int32_t)(w << 4) >> 4;
                    const int64_t rel = d - ((int64_t)(t / 3 - 1) * h.W + (t % 3 - 1)) * esz;
                    if (rel < 0 || rel % ((int64_t)h.H * h.W * esz) || rel / ((int64_t)h.H * h.W * esz) >= h.Cin) return false;
                }
            }
        }
    }
    if (h.kernel == SPARSERT_KERNEL_SPEC) {
        const sparsert::SpecPlan &sp = h.spec;
        if (sp.code.size() < 64 || sp.symbol.empty() || sp.group_of_slot.size() != M) return false;
        if (sp.n_groups < 1 || sp.n_blocks < sp.n_groups || sp.n_tiles < 1) return false;
        // what launch_spec turns into a grid, and what the generated prologue assumes of it
        const int tpw = sp.tiles_per_wg;
        if (tpw < 1 || tpw > 16 || (tpw & (tpw - 1))) return false;
        if (sp.mode != SPARSERT_SPEC_DIRECT && sp.mode != SPARSERT_SPEC_LDS) return false;
        if (sp.vec < 1 || h.N % sp.vec || sp.lanes_per_tile < 1 || sp.lanes_per_tile > sparsert::kWave) return false;
        const int64_t nvc = h.N / sp.vec;
        if ((int64_t)sp.n_tiles * sp.lanes_per_tile < nvc || (int64_t)(sp.n_tiles - 1) * sp.lanes_per_tile >= nvc) return false;
        if (sp.rows_per_group < 1 || (int64_t)sp.n_groups * sp.rows_per_group < h.M) return false;
        if (sp.lds_bytes < 0 || sp.lds_bytes > 160 * 1024) return false;
        const bool lds = sp.mode == SPARSERT_SPEC_LDS;
        if (lds && (sp.ksplit != 1 || sp.n_blocks % tpw)) return false;
        if (!lds && (sp.ksplit < 1 || sp.n_blocks != sp.n_groups * sp.ksplit || (sp.ksplit > 1 && sp.ksplit != tpw))) return false;
        if (sp.group_columns.size() != (size_t)sp.n_blocks) return false;
        for (int32_t g : sp.group_of_slot)
            if (g < 0 || g >= sp.n_groups) return false;
    }
    return true;
}

int save_impl(const sparsert_plan *plan, void *buf, size_t cap, size_t *need) {
    if (!plan) return sparsert::set_error(SPARSERT_EINVAL, "plan is NULL");
    sparsert::HostPlan &h = const_cast<sparsert::HostPlan &>(plan->host);   // the writer only reads
    Writer w;
    scalars(w, h);
    w.i64(h.spec.asm_bytes);
    w.str(h.spec.symbol);
    w.vec(h.row_nnz); w.vec(h.hist); w.vec(h.perm); w.vec(h.inv_perm); w.vec(h.p_row_ptr); w.vec(h.p_col_idx);
    w.vec(h.p_vals); w.vec(h.bins); w.vec(h.stream); w.vec(h.conv_seg); w.vec(h.segments);
    w.vec(h.spec.group_of_slot); w.vec(h.spec.group_columns); w.vec(h.spec.code);
    const size_t total = 24 + w.out.size();
    if (need) *need = total;
    if (!buf) return SPARSERT_OK;
    if (cap < total) return sparsert::set_error(SPARSERT_EINVAL, "buffer too small for the serialised plan");
    uint8_t *o = static_cast<uint8_t *>(buf);
    const uint64_t sum = fnv1a(w.out.data(), w.out.size()), len = w.out.size();
    std::memcpy(o, &kMagic, 4); std::memcpy(o + 4, &kFormat, 4);
    std::memcpy(o + 8, &len, 8); std::memcpy(o + 16, &sum, 8);
    std::memcpy(o + 24, w.out.data(), w.out.size());
    return SPARSERT_OK;
}

int load_impl(const void *buf, size_t size, int32_t host_only, sparsert_plan **out) {
    if (!out) return sparsert::set_error(SPARSERT_EINVAL, "out is NULL");
    *out = nullptr;
    if (!buf || size < 24) return sparsert::set_error(SPARSERT_EINVAL, "not a serialised plan: too short");
    const uint8_t *b = static_cast<const uint8_t *>(buf);
    uint32_t magic, format; uint64_t len, sum;
    std::memcpy(&magic, b, 4); std::memcpy(&format, b + 4, 4); std::memcpy(&len, b + 8, 8); std::memcpy(&sum, b + 16, 8);
    if (magic != kMagic) return sparsert::set_error(SPARSERT_EINVAL, "not a serialised plan: bad magic word");
    if (format != kFormat) return sparsert::set_error(SPARSERT_EUNSUPPORTED, "serialised plan has another format version");
    if (len != size - 24) return sparsert::set_error(SPARSERT_EINVAL, "serialised plan is truncated or padded");
    if (fnv1a(b + 24, (size_t)len) != sum) return sparsert::set_error(SPARSERT_EINVAL, "serialised plan fails its checksum");
    sparsert_plan *plan = new (std::nothrow) sparsert_plan();
    if (!plan) return sparsert::set_error(SPARSERT_ENOMEM, "out of host memory");
    sparsert::HostPlan &h = plan->host;
    Reader r{b + 24, b + size};
    scalars(r, h);
    h.spec.asm_bytes = r.i64();
    r.str(h.spec.symbol);
    r.vec(h.row_nnz); r.vec(h.hist); r.vec(h.perm); r.vec(h.inv_perm); r.vec(h.p_row_ptr); r.vec(h.p_col_idx);
    r.vec(h.p_vals); r.vec(h.bins); r.vec(h.stream); r.vec(h.conv_seg); r.vec(h.segments);
    r.vec(h.spec.group_of_slot); r.vec(h.spec.group_columns); r.vec(h.spec.code);
    if (!r.ok || r.p != r.end || !consistent(h)) {
        delete plan;
        return sparsert::set_error(SPARSERT_EINVAL, "serialised plan is inconsistent");
    }
    if (!host_only) {
        std::string err;
        const int rc = sparsert::upload_plan(h, plan->dev, err);
        if (rc != SPARSERT_OK) {
            sparsert::free_device_plan(plan->dev);
            delete plan;
            return sparsert::set_error(rc, err);
        }
        plan->on_device = true;
    }
    *out = plan;
    return SPARSERT_OK;
}

template <typename F> int guarded(F f) {
    try {   // no exception may cross the C boundary
        return f();
    } catch (const std::bad_alloc &) {
        return sparsert::set_error(SPARSERT_ENOMEM, "out of host memory");
    } catch (const std::exception &ex) {
        return sparsert::set_error(SPARSERT_EINVAL, std::string("internal error: ") + ex.what());
    }
}

}  // namespace

extern "C" int sparsert_plan_save(const sparsert_plan *plan, void *buf, size_t cap, size_t *need) {
    return guarded([&] { return save_impl(plan, buf, cap, need); });
}

extern "C" int sparsert_plan_load(const void *buf, size_t size, int32_t host_only, sparsert_plan **out) {
    return guarded([&] { return load_impl(buf, size, host_only, out); });
}
