// Autotuner (Section 3.7 of the paper): exhaustive search over a short, hand-picked list
// of executor configurations for one problem, each built by the inspector and timed on
// the GPU; the fastest plan is kept.  The paper tunes (M_blocks, N_blocks, Gy); the knobs
// here are the executor family, columns per lane, rows per generated code block, waves
// per workgroup and the staging variant.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstring>
#include <exception>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "plan.h"

namespace {

// Times plans on one stream.  "Warm": back-to-back launches of the same plan, whose code and
// operands then sit in the L2 caches.  "Cold": a fill of more scratch memory than the L2 caches
// hold runs before every launch, as the other layers of a model would displace this one's code
// and operands; the fill's own time, measured the same way once, is subtracted.
struct Bench {
    hipStream_t s = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    void *scratch = nullptr;
    size_t scratch_bytes = 0;
    float fill_us = 0.0f;
    bool conv = false;
    const void *in = nullptr;
    void *out = nullptr;
    int launches = 30, repeats = 3;

    int run(sparsert_plan *p) const { return conv ? sparsert_conv3x3(p, in, out, s) : sparsert_spmm(p, in, out, s); }
    bool fill() const {
        std::string err;
        return sparsert::displace_caches(scratch, scratch_bytes, s, err) == SPARSERT_OK;
    }
    // best-of-repeats microseconds per iteration of `body`, which returns false on failure
    template <typename F> float loop(F body) const {
        float best = -1.0f;
        for (int r = 0; r < repeats; ++r) {
            if (hipEventRecord(e0, s) != hipSuccess) return -1.0f;
            for (int i = 0; i < launches; ++i)
                if (!body()) return -1.0f;
            if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -1.0f;
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1.0f;
            const float us = ms * 1000.0f / launches;
            if (best < 0.0f || us < best) best = us;
        }
        return best;
    }
    float warm(sparsert_plan *p) const {
        for (int i = 0; i < 5; ++i)
            if (run(p) != SPARSERT_OK) return -1.0f;
        return loop([&] { return run(p) == SPARSERT_OK; });
    }
    float cold(sparsert_plan *p) const {
        if (!scratch) return -1.0f;
        const float both = loop([&] { return fill() && run(p) == SPARSERT_OK; });
        return both < 0.0f ? -1.0f : std::max(0.01f, both - fill_us);
    }
};

}  // namespace

static int tune_impl(const int32_t *row_ptr, const int32_t *col_idx, const void *vals,
                     int32_t M, int32_t K, int32_t N, const sparsert_options *base,
                     const void *in_dev, void *out_dev, void *stream,
                     sparsert_plan **out, sparsert_tune_report *report) {
    if (out) *out = nullptr;
    if (report) std::memset(report, 0, sizeof(*report));
    sparsert_options b;
    if (base) b = *base; else std::memset(&b, 0, sizeof(b));
    b.host_only = 0;
    b.vec = b.split_threshold = b.spec_rows = b.spec_depth = b.spec_tiles = b.spec_mode = b.spec_ksplit = b.spec_lanes = b.spec_swizzle = b.spec_vec = 0;
    const int32_t tune_warm = b.tune_warm;
    b.spec_prefetch = 0;   // tried on the winner at the end
    b.tune_warm = 0;   // a tuner flag, not a property of the plans
    // First candidate: the inspector's own choice.  It also validates every argument.
    sparsert_plan *best = nullptr;
    {
        sparsert_options o = b;
        o.kernel = b.kernel == SPARSERT_KERNEL_SPEC ? SPARSERT_KERNEL_SPEC : SPARSERT_KERNEL_ROWS;
        if (int rc = sparsert_inspect(row_ptr, col_idx, vals, M, K, N, &o, &best)) return rc;
    }
    if (!out || !in_dev || !out_dev || (((uintptr_t)in_dev | (uintptr_t)out_dev) & 15u)) {
        sparsert_plan_destroy(best);
        return sparsert::set_error(SPARSERT_EINVAL, "out is NULL, or a device pointer is NULL or not 16-byte aligned");
    }
    // Everything the timing needs lives in `bench`; `Cleanup` releases it on every way out.
    Bench bench;
    bench.s = static_cast<hipStream_t>(stream);
    bench.in = in_dev; bench.out = out_dev; bench.conv = b.conv != 0;
    void *ref_out = nullptr;        // what the first candidate wrote: every other candidate is held against it
    uint32_t *res_dev = nullptr;    // partial and final words of the output comparison
    struct Cleanup {
        Bench &bn; void *&ref; uint32_t *&res;
        ~Cleanup() {
            if (bn.e0) (void)hipEventDestroy(bn.e0);
            if (bn.e1) (void)hipEventDestroy(bn.e1);
            if (bn.scratch) (void)hipFree(bn.scratch);
            if (ref) (void)hipFree(ref);
            if (res) (void)hipFree(res);
        }
    } cleanup{bench, ref_out, res_dev};
    const sparsert::HostPlan &h0 = best->host;
    const size_t out_bytes = (size_t)h0.batch * h0.M * (size_t)(h0.conv ? h0.N : h0.ldc) * h0.out_elem_size();
    bench.scratch_bytes = (size_t)64 << 20;   // twice what the eight 4 MiB L2 caches hold
    if (hipEventCreate(&bench.e0) != hipSuccess || hipEventCreate(&bench.e1) != hipSuccess ||
        hipMalloc(&bench.scratch, bench.scratch_bytes) != hipSuccess || hipMalloc(&ref_out, out_bytes) != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&res_dev), (size_t)(4 * sparsert::compare_blocks(h0) + 4) * sizeof(uint32_t)) != hipSuccess) {
        sparsert_plan_destroy(best);
        return sparsert::set_error(SPARSERT_EHIP, "the tuner could not create its events and scratch buffers");
    }
    for (int i = 0; i < 3; ++i) (void)bench.fill();
    bench.fill_us = bench.loop([&] { return bench.fill(); });
    if (bench.fill_us < 0.0f) {
        sparsert_plan_destroy(best);
        return sparsert::set_error(SPARSERT_EHIP, "timing the cache-displacing fill failed");
    }
    hipStream_t s = bench.s;
    const bool conv = b.conv != 0, f16 = b.dtype == SPARSERT_F16, i8 = b.dtype == SPARSERT_I8;
    const bool rank_cold = !tune_warm;
    const int family = b.kernel;   // AUTO: both executor families; else only that one
    const int64_t nnz = row_ptr[M];

    std::vector<sparsert_options> cands;
    if (!conv) {
        for (int v = 1; v <= (f16 ? 8 : 4); v *= 2) {
            if (N % v || (i8 && v == 2)) continue;
            sparsert_options o = b;
            o.kernel = SPARSERT_KERNEL_ROWS; o.vec = v;
            cands.push_back(o);
            o.split_threshold = 64;
            cands.push_back(o);
        }
    } else {
        for (int thr : {32, 64, 1 << 30}) {
            sparsert_options o = b;
            o.kernel = SPARSERT_KERNEL_ROWS; o.split_threshold = thr;
            cands.push_back(o);
        }
    }
    if (family == SPARSERT_KERNEL_SPEC) cands.clear();
    if (nnz <= (4 << 20) && family != SPARSERT_KERNEL_ROWS) {
        const int64_t images = std::max(1, b.batch);   // every problem of a batch brings its own waves
        const int64_t tiles = (N + 63) / 64 * images;
        // DIRECT and K-split candidates at V columns per lane (V > 1: the halves / int8 packed in one dword)
        auto add_direct = [&](int V) {
            const int64_t vtiles = (N / V + 63) / 64 * images;
            const int max_rows = 192 / V;   // accumulator registers
            // Matrices of some size get a thinner list (a candidate costs 1-2.5 s of assembling per
            // 100 000 nonzeros): blocks of one or two rows - the largest code, and winners only on
            // small problems - and the two-tile twins of the four-tile workgroups are left out.
            const bool sizeable = nnz > (64 << 10);
            for (int r : {1, 2, 4, 8, 16, 24, 48, 96}) {
                if (r > M || r > max_rows || (r == 96 && images == 1)) continue;
                if (sizeable && r < 4 && M >= 1024) continue;
                const int64_t groups = (M + r - 1) / r;
                if (r > 1 && groups * vtiles < 256) continue;   // too few waves to be worth assembling
                if (groups > 8192) continue;
                for (int t : {2, 4}) {
                    if ((V > 1 || sizeable) && t == 2) continue;
                    sparsert_options o = b;
                    o.kernel = SPARSERT_KERNEL_SPEC; o.spec_mode = SPARSERT_SPEC_DIRECT;
                    // (a few more rows where that spares a last round of workgroups on a few compute units)
                    o.spec_rows = sparsert::rows_without_thin_round(M, r, 1, (vtiles / images + t - 1) / t * images, max_rows);
                    o.spec_tiles = t; o.spec_vec = V;
                    cands.push_back(o);
                }
            }
            if (K >= 512) {   // long reduction axis: split it over the waves of a workgroup
                const int rk[][2] = {{1, 8}, {2, 8}, {4, 8}, {8, 8}, {16, 8}, {24, 8}, {32, 8}, {48, 8}, {64, 8}, {96, 8}, {128, 8},
                                     {1, 4}, {2, 4}, {4, 4}, {8, 4}, {16, 4}, {32, 4}, {48, 4}, {64, 4}, {96, 4},
                                     {64, 2}, {96, 2}};
                std::vector<std::pair<int, int>> listed;
                auto add = [&](int r, int ks) {
                    if (std::find(listed.begin(), listed.end(), std::make_pair(r, ks)) != listed.end()) return;
                    listed.push_back({r, ks});
                    sparsert_options o = b;
                    o.kernel = SPARSERT_KERNEL_SPEC; o.spec_mode = SPARSERT_SPEC_DIRECT;
                    o.spec_rows = r; o.spec_ksplit = ks; o.spec_vec = V;
                    cands.push_back(o);
                };
                for (auto &c : rk) {
                    // worth timing with at least two waves for every SIMD of the chip, but not with
                    // more than sixteen (the blocks are then too small to reuse a fetched row)
                    const int64_t waves = (int64_t)((M + c[0] - 1) / c[0]) * vtiles * c[1];
                    if (c[0] > M || c[0] > max_rows || waves < 2048 || waves > 16384) continue;
                    // never a last round of workgroups that only a few compute units take part in
                    add(sparsert::rows_without_thin_round(M, c[0], 1, vtiles, max_rows), c[1]);
                }
                // ... and the row counts that make the launch exactly one, two or four workgroups
                // per compute unit with two or four waves per SIMD: the fewest fetches of B a
                // launch that still fills the chip can have (1024 x 4096 at 95 %, 784 columns:
                // 54 rows x 8 parts = 247 workgroups, 21.3 us; the listed 48 rows = 286: 43.7 us)
                const int whole[][2] = {{8, 1}, {8, 2}, {4, 2}, {4, 4}, {2, 4}};   // parts, workgroups per compute unit
                for (auto &c : whole) {
                    // (eight parts are two waves per SIMD, which leaves each 256 registers: blocks of up to 224 rows;
                    // 1024 x 4096 x 3136 at 95 %: 205 rows, one workgroup per compute unit, 45 us; 103 rows, two: 61 us)
                    const int r = sparsert::rows_for_rounds(M, 1, vtiles, c[1], c[0] == 8 && c[1] == 1 ? 224 / V : max_rows);
                    if (r < 4) continue;
                    const int64_t wgs = (int64_t)((M + r - 1) / r) * vtiles;
                    if (wgs * 4 < (int64_t)256 * c[1] * 3) continue;   // under three quarters of the chip
                    add(r, c[0]);
                }
            }
        };
        {   // what the inspector picks when nothing is set is always in the race
            sparsert_options o = b;
            o.kernel = SPARSERT_KERNEL_SPEC;
            cands.push_back(o);
        }
        add_direct(1);
        if (!conv && f16 && N % 2 == 0) add_direct(2);
        if (!conv && i8 && N % 4 == 0) add_direct(4);
        if (!conv && !f16 && !i8 && K >= 256 && (int64_t)M * tiles >= 1024) {
            for (int r : {12, 24, 48, 96})
                for (int w : {4, 8}) {
                    if (((int64_t)M + r - 1) / r < w) continue;
                    sparsert_options o = b;
                    o.kernel = SPARSERT_KERNEL_SPEC; o.spec_mode = SPARSERT_SPEC_LDS;
                    o.spec_rows = sparsert::rows_without_thin_round(M, r, w, tiles, 128);
                    o.spec_tiles = w;
                    cands.push_back(o);
                }
        }
    }

    // Assembling a candidate costs about 12 s per million nonzeros, so large matrices get a
    // short list of generated kernels: one per family, each at the row count that fills whole
    // rounds of workgroups over the chip's compute units (rows_for_whole_rounds; measured on
    // 4096 x 4096 x 3136 at 95 %: 103 rows per block 127 us, 96 rows 180 us).  The LDS-staged
    // variant leads the list where the reduction axis is long: it is what wins there.
    if (nnz > (256 << 10) && family != SPARSERT_KERNEL_ROWS) {
        const size_t budget = nnz > (1 << 20) ? 3 : 6;
        const int64_t vt = (N + 63) / 64 * std::max(1, b.batch);
        std::vector<sparsert_options> rows_family, spec_family;
        for (const sparsert_options &o : cands)
            if (o.kernel != SPARSERT_KERNEL_SPEC) rows_family.push_back(o);
        auto direct = [&](int ks, int t) {
            sparsert_options o = b;
            o.kernel = SPARSERT_KERNEL_SPEC; o.spec_mode = SPARSERT_SPEC_DIRECT;
            o.spec_ksplit = ks; o.spec_tiles = t;
            o.spec_rows = sparsert::rows_for_whole_rounds(M, 1, ks > 1 ? vt : (vt + t - 1) / t, 32, 128);
            spec_family.push_back(o);
        };
        auto staged = [&](int w) {
            if (conv || K < 256 || ((int64_t)M + 31) / 32 < w) return;
            sparsert_options o = b;
            o.kernel = SPARSERT_KERNEL_SPEC; o.spec_mode = SPARSERT_SPEC_LDS; o.spec_tiles = w;
            o.spec_rows = sparsert::rows_for_whole_rounds(M, w, vt, 32, 128);
            spec_family.push_back(o);
        };
        {   // the inspector's own choice for the generated kernel (no option set) is always in the race
            sparsert_options o = b;
            o.kernel = SPARSERT_KERNEL_SPEC;
            spec_family.push_back(o);
        }
        if (K >= 2048) { staged(8); direct(1, 4); direct(2, 2); staged(4); direct(4, 4); direct(8, 8); }
        else if (K >= 512) { direct(2, 2); direct(1, 4); direct(4, 4); staged(8); direct(8, 8); staged(4); }
        else { direct(1, 4); direct(1, 2); staged(8); staged(4); }
        if (spec_family.size() > budget + 1) spec_family.resize(budget + 1);
        cands = rows_family;
        cands.insert(cands.end(), spec_family.begin(), spec_family.end());
    }

    // One candidate: poison the output, run, hold the result against the first candidate's, time.
    struct Timing { float warm = -1.0f, cold = -1.0f; int agrees = 0; };
    const float tol = i8 ? 0.0f : f16 ? 5e-3f : 1e-3f;   // two correct summation orders differ by far less
    bool have_ref = false;
    auto measure = [&](sparsert_plan *p) {
        Timing t;
        // 0xff bytes: NaN in both floating types, -1 as an integer; an element a plan fails to write shows
        if (hipMemsetAsync(out_dev, 0xff, out_bytes, s) != hipSuccess || bench.run(p) != SPARSERT_OK) return t;
        if (!have_ref) {
            if (hipMemcpyAsync(ref_out, out_dev, out_bytes, hipMemcpyDeviceToDevice, s) != hipSuccess ||
                hipStreamSynchronize(s) != hipSuccess) return t;
            have_ref = true;
            t.agrees = 1;
        } else {
            uint32_t words[4] = {0, 0, 1, 0};
            std::string err;
            uint32_t *final_dev = res_dev + 4 * sparsert::compare_blocks(p->host);
            if (sparsert::launch_compare(p->host, out_dev, ref_out, res_dev, final_dev, s, err) != SPARSERT_OK ||
                hipMemcpyAsync(words, final_dev, sizeof(words), hipMemcpyDeviceToHost, s) != hipSuccess ||
                hipStreamSynchronize(s) != hipSuccess) return t;
            float dmax, rmax;
            std::memcpy(&dmax, &words[0], 4);
            std::memcpy(&rmax, &words[1], 4);
            t.agrees = words[2] == 0 && dmax <= tol * rmax;
            if (!t.agrees) return t;
        }
        t.warm = bench.warm(p);
        t.cold = t.warm > 0.0f ? bench.cold(p) : -1.0f;
        return t;
    };
    auto key = [&](const Timing &t) { return rank_cold ? t.cold : t.warm; };
    // `a` beats `b`: by the ranking figure; cold figures within 1 % of each other are a tie (that is
    // what they scatter by), which the back-to-back figure breaks
    auto beats = [&](const Timing &a, const Timing &b) {
        if (key(a) <= 0.0f) return false;
        if (key(b) <= 0.0f) return true;
        if (rank_cold && a.warm > 0.0f && b.warm > 0.0f && key(a) < 1.01f * key(b) && key(b) < 1.01f * key(a)) return a.warm < b.warm;
        return key(a) < key(b);
    };
    auto log = [&](const sparsert_plan *p, const Timing &tm) {
        if (!report || report->count >= SPARSERT_TUNE_MAX) return;
        sparsert_tune_entry &t = report->entries[report->count++];
        const sparsert::HostPlan &h = p->host;
        t.kernel = h.kernel; t.vec = h.vec; t.split_threshold = h.split_threshold;
        t.spec_mode = h.spec.mode; t.spec_rows = h.spec.rows_per_group; t.spec_tiles = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.tiles_per_wg : 0;
        t.spec_ksplit = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.ksplit : 0;
        t.spec_lanes = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.lanes_per_tile : 0;
        t.spec_swizzle = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.swizzle : 0;
        t.spec_vec = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.vec : 0;
        t.microseconds = tm.warm; t.cold_microseconds = tm.cold; t.agrees = tm.agrees;
        t.spec_prefetch = h.kernel == SPARSERT_KERNEL_SPEC && h.spec.prefetch_lines > 0;
    };
    Timing best_t = measure(best);
    log(best, best_t);
    // The host half of a candidate (analysis, code generation, assembling: seconds for a large
    // matrix) is independent of every other candidate's, so a few host threads build the plans
    // ahead, in list order and at most `window` beyond the one being timed; this thread uploads
    // and times them one after the other.
    struct Built { sparsert_plan *plan = nullptr; bool ready = false; };
    std::vector<Built> built(cands.size());
    std::mutex mu;
    std::condition_variable cv;
    size_t next = 0, consumed = 0;
    bool stop = false;
    const size_t window = 12;
    auto worker = [&]() {
        for (;;) {
            size_t i;
            {
                std::unique_lock<std::mutex> lk(mu);
                cv.wait(lk, [&] { return stop || next >= cands.size() || next < consumed + window; });
                if (stop || next >= cands.size()) return;
                i = next++;
            }
            sparsert_options o = cands[i];
            o.host_only = 1;
            sparsert_plan *p = nullptr;
            if (sparsert_inspect(row_ptr, col_idx, vals, M, K, N, &o, &p) != SPARSERT_OK) p = nullptr;
            {
                std::lock_guard<std::mutex> lk(mu);
                built[i].plan = p;
                built[i].ready = true;
            }
            cv.notify_all();
        }
    };
    struct Pool {   // joins on every way out; plans built but never consumed are released
        std::vector<std::thread> threads;
        std::mutex &mu; std::condition_variable &cv; bool &stop; std::vector<Built> &built;
        ~Pool() {
            { std::lock_guard<std::mutex> lk(mu); stop = true; }
            cv.notify_all();
            for (std::thread &t : threads) if (t.joinable()) t.join();
            for (Built &b : built) if (b.plan) sparsert_plan_destroy(b.plan);
        }
    } pool{{}, mu, cv, stop, built};
    const unsigned hw = std::thread::hardware_concurrency();
    const size_t n_threads = std::min<size_t>(cands.size(), std::max(1u, std::min(8u, hw / 2)));
    for (size_t t = 0; t < n_threads; ++t) pool.threads.emplace_back(worker);
    for (size_t i = 0; i < cands.size(); ++i) {
        sparsert_plan *p = nullptr;
        {
            std::unique_lock<std::mutex> lk(mu);
            cv.wait(lk, [&] { return built[i].ready; });
            p = built[i].plan;
            built[i].plan = nullptr;
            consumed = i + 1;
        }
        cv.notify_all();
        if (!p) continue;
        {
            std::string err;
            if (sparsert::upload_plan(p->host, p->dev, err) != SPARSERT_OK) { sparsert_plan_destroy(p); continue; }
            p->on_device = true;
        }
        const Timing t = measure(p);
        log(p, t);
        if (beats(t, best_t)) {
            sparsert_plan_destroy(best);
            best = p; best_t = t;
        } else {
            sparsert_plan_destroy(p);
        }
    }
    // Last candidate: the winner's configuration with its blocks formed by similarity (row swizzle).
    if (key(best_t) > 0.0f && best->host.kernel == SPARSERT_KERNEL_SPEC && best->host.spec.rows_per_group > 1 &&
        !b.natural_order) {
        const sparsert::SpecPlan &w = best->host.spec;
        sparsert_options o = b;
        o.kernel = SPARSERT_KERNEL_SPEC; o.spec_mode = w.mode; o.spec_rows = w.rows_per_group;
        o.spec_tiles = w.tiles_per_wg; o.spec_ksplit = w.ksplit; o.spec_vec = w.vec; o.spec_swizzle = 1;
        sparsert_plan *p = nullptr;
        if (sparsert_inspect(row_ptr, col_idx, vals, M, K, N, &o, &p) == SPARSERT_OK) {
            const Timing t = measure(p);
            log(p, t);
            if (beats(t, best_t)) {
                sparsert_plan_destroy(best);
                best = p; best_t = t;
            } else {
                sparsert_plan_destroy(p);
            }
        }
    }
    // ... and the winner with its waves prefetching their code: kept if it is worth at least 1.5 %
    // under the condition the ranking uses (it costs time while the code is still in the L2)
    if (key(best_t) > 0.0f && best->host.kernel == SPARSERT_KERNEL_SPEC) {
        const sparsert::SpecPlan &w = best->host.spec;
        sparsert_options o = b;
        o.kernel = SPARSERT_KERNEL_SPEC; o.spec_mode = w.mode; o.spec_rows = w.rows_per_group;
        o.spec_tiles = w.tiles_per_wg; o.spec_ksplit = w.ksplit; o.spec_vec = w.vec; o.spec_swizzle = w.swizzle;
        o.spec_prefetch = 1;
        sparsert_plan *p = nullptr;
        if (sparsert_inspect(row_ptr, col_idx, vals, M, K, N, &o, &p) == SPARSERT_OK) {
            Timing t = measure(p);
            log(p, t);
            // the two are a few percent apart, which is what two timings of one plan minutes apart
            // can differ by: both are timed twice more, alternating, and the best of each counts
            float with = key(t), without = key(best_t);
            for (int i = 0; i < 2 && with > 0.0f; ++i) {
                const float a = rank_cold ? bench.cold(best) : bench.warm(best);
                const float c = rank_cold ? bench.cold(p) : bench.warm(p);
                if (a > 0.0f) without = std::min(without, a);
                if (c > 0.0f) with = std::min(with, c);
            }
            if (with > 0.0f && with < 0.985f * without) {
                sparsert_plan_destroy(best);
                best = p; best_t = t;
            } else {
                sparsert_plan_destroy(p);
            }
        }
    }
    if (report) { report->best_microseconds = best_t.warm; report->best_cold_microseconds = best_t.cold; }
    if (key(best_t) <= 0.0f) {
        sparsert_plan_destroy(best);
        return sparsert::set_error(SPARSERT_EHIP, "no candidate configuration could be launched and timed");
    }
    // leave the winner's result in out_dev (the last candidate timed need not be the winner)
    if (bench.run(best) != SPARSERT_OK || hipStreamSynchronize(s) != hipSuccess) {
        sparsert_plan_destroy(best);
        return sparsert::set_error(SPARSERT_EHIP, "the chosen plan failed to launch");
    }
    *out = best;
    return SPARSERT_OK;
}

extern "C" int sparsert_tune(const int32_t *row_ptr, const int32_t *col_idx, const void *vals,
                             int32_t M, int32_t K, int32_t N, const sparsert_options *base,
                             const void *in_dev, void *out_dev, void *stream,
                             sparsert_plan **out, sparsert_tune_report *report) {
    try {   // no exception may cross the C boundary
        return tune_impl(row_ptr, col_idx, vals, M, K, N, base, in_dev, out_dev, stream, out, report);
    } catch (const std::bad_alloc &) {
        return sparsert::set_error(SPARSERT_ENOMEM, "out of host memory while tuning");
    } catch (const std::exception &ex) {
        return sparsert::set_error(SPARSERT_EINVAL, std::string("internal error while tuning: ") + ex.what());
    }
}
