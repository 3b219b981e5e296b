// Drives the host half of the library (inspector, code generator, serialisation, boundary)
// through a grid of problems and options in one native process, built with
// -fsanitize=address,undefined.  Any out-of-bounds access, use after free, signed overflow or
// misaligned access in that code ends the process with a report; the test expects exit code 0.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/sparsert.h"

namespace {

struct Rng {
    uint64_t s;
    uint32_t next() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(s >> 33); }
    double unit() { return next() / 2147483648.0; }
};

struct Csr { std::vector<int32_t> row_ptr, col; std::vector<uint8_t> vals; };

// `width` bytes per value; the bytes are arbitrary (the host code only moves them), except that
// half values avoid the NaN / infinity exponent so the generator's widening sees ordinary numbers too
Csr make(int M, int K, double density, int width, Rng &r, bool skew) {
    Csr c;
    c.row_ptr.push_back(0);
    for (int m = 0; m < M; ++m) {
        const double d = skew ? density * 4.0 / (1.0 + (m % 7) * (m % 7)) : density;
        for (int k = 0; k < K; ++k)
            if (r.unit() < d) {
                c.col.push_back(k);
                for (int b = 0; b < width; ++b) c.vals.push_back((uint8_t)(r.next() & (width == 2 && b == 1 ? 0x3b : 0xff)));
            }
        c.row_ptr.push_back((int32_t)c.col.size());
    }
    return c;
}

int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) { std::fprintf(stderr, "line %d: %s (%s)\n", __LINE__, #cond, sparsert_last_error()); ++failures; } \
    } while (0)

void exercise(const Csr &c, int M, int K, int N, sparsert_options o, bool may_refuse) {
    o.host_only = 1;
    sparsert_plan *p = nullptr;
    const int rc = sparsert_inspect(c.row_ptr.data(), c.col.data(), c.vals.data(), M, K, N, &o, &p);
    if (rc != SPARSERT_OK) {
        EXPECT(may_refuse && p == nullptr && (rc == SPARSERT_EINVAL || rc == SPARSERT_EUNSUPPORTED));
        return;
    }
    for (int f = SPARSERT_FIELD_INFO; f <= SPARSERT_FIELD_KERNEL_NAME; ++f) {
        size_t need = 0;
        EXPECT(sparsert_plan_export(p, f, nullptr, 0, &need) == SPARSERT_OK);
        std::vector<uint8_t> buf(need + 1);
        EXPECT(sparsert_plan_export(p, f, buf.data(), need, nullptr) == SPARSERT_OK);
        if (need) EXPECT(sparsert_plan_export(p, f, buf.data(), need - 1, nullptr) == SPARSERT_EINVAL);
    }
    size_t need = 0;
    EXPECT(sparsert_plan_save(p, nullptr, 0, &need) == SPARSERT_OK && need > 24);
    std::vector<uint8_t> blob(need), again(need);
    EXPECT(sparsert_plan_save(p, blob.data(), need, nullptr) == SPARSERT_OK);
    sparsert_plan *q = nullptr;
    EXPECT(sparsert_plan_load(blob.data(), need, 1, &q) == SPARSERT_OK && q);
    if (q) {
        size_t need2 = 0;
        EXPECT(sparsert_plan_save(q, again.data(), need, &need2) == SPARSERT_OK && need2 == need);
        EXPECT(std::memcmp(blob.data(), again.data(), need) == 0);
        sparsert_plan_destroy(q);
    }
    // damaged blobs are refused, never dereferenced: a flipped byte, a truncation
    if (need > 64) {
        std::vector<uint8_t> bad(blob);
        bad[need / 2] ^= 0x5a;
        q = nullptr;
        EXPECT(sparsert_plan_load(bad.data(), need, 1, &q) != SPARSERT_OK && !q);
        EXPECT(sparsert_plan_load(blob.data(), need - 9, 1, &q) != SPARSERT_OK && !q);
    }
    // executing a host-only plan is an error, not a crash
    EXPECT(sparsert_spmm(p, blob.data(), again.data(), nullptr) == SPARSERT_EINVAL);
    sparsert_plan_destroy(p);
}

}  // namespace

int main() {
    Rng r{20081184ull};
    const int shapes[][3] = {{1, 1, 1}, {7, 5, 3}, {64, 48, 100}, {70, 150, 196}, {33, 260, 65}};
    int plans = 0;
    for (const auto &s : shapes) {
        const int M = s[0], K = s[1], N = s[2];
        for (int dtype = SPARSERT_F32; dtype <= SPARSERT_I8; ++dtype) {
            const int width = dtype == SPARSERT_F16 ? 2 : dtype == SPARSERT_I8 ? 1 : 4;
            for (double density : {0.08, 1.0}) {
                const Csr c = make(M, K, density, width, r, density == 0.08);
                sparsert_options base;
                std::memset(&base, 0, sizeof(base));
                base.dtype = dtype;
                {   // row-walk plans
                    sparsert_options o = base;
                    o.kernel = SPARSERT_KERNEL_ROWS;
                    exercise(c, M, K, N, o, false); ++plans;
                    o.split_threshold = 3; o.natural_order = (M & 1);
                    exercise(c, M, K, N, o, false); ++plans;
                    o.ldb = N + 8; o.ldc = N + 24; o.batch = 3;
                    exercise(c, M, K, N, o, false); ++plans;
                }
                // generated kernels: defaults, then rows x split x variant x packing
                { sparsert_options o = base; exercise(c, M, K, N, o, false); ++plans; }
                // six of the 24 (rows, split, variant) combinations per case, rotating, so that the
                // whole run meets every combination with every storage type
                const int rows_of[] = {1, 5, 200}, ks_of[] = {1, 8};
                for (int j = 0; j < 6; ++j) {
                    const int combo = (plans * 7 + j * 5) % 24;
                    const int rows = rows_of[combo % 3], ks = ks_of[(combo / 3) % 2], variant = combo / 6;
                    sparsert_options o = base;
                    o.kernel = SPARSERT_KERNEL_SPEC; o.spec_rows = rows; o.spec_ksplit = ks;
                    o.spec_swizzle = variant & 1;
                    if (variant == 1) { o.spec_depth = 2; o.spec_lanes = 32; }
                    if (variant == 2) { o.spec_vec = dtype == SPARSERT_F16 ? 2 : dtype == SPARSERT_I8 ? 4 : 1; o.ldb = N + 12; o.ldc = N + 4; }
                    if (variant == 3) { o.spec_mode = SPARSERT_SPEC_LDS; o.spec_ksplit = 0; o.spec_tiles = ks; o.batch = 2; }
                    exercise(c, M, K, N, o, true); ++plans;
                }
            }
        }
    }
    {   // the empty matrix
        const Csr c = make(9, 12, 0.0, 4, r, false);
        sparsert_options o;
        std::memset(&o, 0, sizeof(o));
        exercise(c, 9, 12, 70, o, false); ++plans;
        o.kernel = SPARSERT_KERNEL_ROWS;
        exercise(c, 9, 12, 70, o, false); ++plans;
    }
    // convolution plans: filter banks [Cout, Cin*9] on H x W images
    const int convs[][4] = {{3, 5, 1, 1}, {4, 6, 2, 3}, {6, 10, 9, 13}, {16, 24, 14, 14}};
    for (const auto &g : convs) {
        const int Cin = g[0], Cout = g[1], H = g[2], W = g[3];
        for (int dtype = SPARSERT_F32; dtype <= SPARSERT_I8; ++dtype) {
            const Csr c = make(Cout, 9 * Cin, 0.3, dtype == SPARSERT_F16 ? 2 : dtype == SPARSERT_I8 ? 1 : 4, r, false);
            sparsert_options o;
            std::memset(&o, 0, sizeof(o));
            o.dtype = dtype; o.conv = 1; o.Cin = Cin; o.H = H; o.W = W;
            for (int kernel : {SPARSERT_KERNEL_ROWS, SPARSERT_KERNEL_AUTO, SPARSERT_KERNEL_SPEC}) {
                o.kernel = kernel;
                for (int batch : {kernel == SPARSERT_KERNEL_AUTO ? 5 : 0}) {
                    o.batch = batch;
                    o.spec_rows = kernel == SPARSERT_KERNEL_SPEC ? 4 : 0;
                    o.spec_ksplit = kernel == SPARSERT_KERNEL_SPEC ? 4 : 0;
                    exercise(c, Cout, 9 * Cin, H * W, o, false); ++plans;
                }
            }
        }
    }
    // malformed input is refused before anything is read past its end
    {
        const int32_t rp_bad[] = {0, 2, 1}, cols[] = {0, 5}, rp_ok[] = {0, 1, 2}, cols_dup[] = {1, 1}, rp2[] = {0, 2, 2};
        const float v[] = {1.0f, 2.0f};
        sparsert_plan *p = nullptr;
        sparsert_options o;
        std::memset(&o, 0, sizeof(o));
        o.host_only = 1;
        EXPECT(sparsert_inspect(rp_bad, cols, v, 2, 8, 4, &o, &p) == SPARSERT_EINVAL && !p);
        EXPECT(sparsert_inspect(rp_ok, cols, v, 2, 4, 4, &o, &p) == SPARSERT_EINVAL && !p);        /* column 5 >= K */
        EXPECT(sparsert_inspect(rp2, cols_dup, v, 2, 4, 4, &o, &p) == SPARSERT_EINVAL && !p);      /* duplicate column */
        EXPECT(sparsert_inspect(nullptr, cols, v, 2, 4, 4, &o, &p) == SPARSERT_EINVAL && !p);
        EXPECT(sparsert_plan_load("SPRT", 4, 1, &p) == SPARSERT_EINVAL && !p);
    }
    std::printf("host sanitize run: %d plans built, exported, saved and reloaded; %d failed expectations\n", plans, failures);
    return failures ? 1 : 0;
}
