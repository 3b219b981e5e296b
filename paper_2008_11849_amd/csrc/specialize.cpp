// Per-matrix specialised executor (Section 3.5 of the paper, re-derived for gfx950).
//
// The paper unrolls the nonzero loop of Algorithm 3 into straight-line code with the
// values of A as instruction constants, so that (i) every accumulator has a fixed
// register, (ii) a row of B is loaded once and reused by every nonzero of that column
// inside the tile, (iii) A costs no data-cache traffic at all.  It emits PTX directly
// instead of going through the high-level compiler (Section 3.7).  The same is done here
// for CDNA4: the inspector emits gfx950 assembly and has the code object manager assemble
// it; going through the HIP compiler took ~50 s for the c3 matrix and serialised every
// load behind its use.
//
// Shape of the generated kernel `sparsert_spec`
//   wave  = one row group g (<= R rows, dealt by the inspector for nonzero balance,
//           Section 3.4) x one column tile (lanes own one column of C each)
//   code  = one straight-line block per group: for each column k that has a nonzero in
//           the group, ascending: fetch b <- B[k, tile columns] (several columns ahead),
//           then  v_fmac_f32 acc[row] += literal(A[row,k]) * b  for every nonzero (row,k);
//           finally one store per row.  No loops, no index loads.
//   DIRECT: workgroup = T waves running the same block on T adjacent tiles; b comes
//           straight from L2/L1 with buffer loads.
//   DIRECT with K split: workgroup = KS waves sharing one block and one tile, each walking
//           a contiguous range of the block's columns with an equal share of its nonzeros
//           (Section 3.4); the partial sums meet in LDS after the walk (Section 3.3).
//   LDS   : workgroup = W waves running W adjacent blocks on the same tile (SpMM; fp32, and half
//           and int8 widened to 32 bits on their way into LDS).  The tile's
//           B rows are staged once per workgroup through LDS in chunks of up to 128 rows
//           (double buffered, one barrier per chunk; each wave fetches a 1/W share) and
//           every wave reads its b values from LDS with compile-time offsets.  Measured
//           on MI355X the vector-memory path delivers ~37 B/clk per CU, the LDS path
//           several times that, and each FMA needs 4 B of b: DIRECT is load bound.
// All global addresses are "descriptor base + row offset literal + lane column offset"
// with the column clamped to the tile, so every access is in bounds by construction.
#include <algorithm>
#include <climits>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <dlfcn.h>
#include <map>
#include <mutex>
#include <stdexcept>
#include <string>

#include "plan.h"

namespace sparsert {

namespace {

// ---------------------------------------------------------------- code object manager
// Loaded at run time so the library itself has no link-time dependency on it.  The entry points
// and the enumerator values below are those of interface version 3 of the code object manager
// (amd_comgr.h); a library that reports another major version is not used.
constexpr size_t kComgrMajor = 3;
typedef struct { uint64_t handle; } comgr_handle;
enum { COMGR_SUCCESS = 0, COMGR_KIND_SOURCE = 1, COMGR_KIND_RELOCATABLE = 7, COMGR_KIND_EXECUTABLE = 8,
       COMGR_KIND_LOG = 5, COMGR_ACTION_LINK_RELOC_TO_EXE = 7, COMGR_ACTION_ASSEMBLE = 8 };

struct Comgr {
    void *lib = nullptr;
    int (*create_data)(int, comgr_handle *) = nullptr;
    int (*release_data)(comgr_handle) = nullptr;
    int (*set_data)(comgr_handle, size_t, const char *) = nullptr;
    int (*set_data_name)(comgr_handle, const char *) = nullptr;
    int (*get_data)(comgr_handle, size_t *, char *) = nullptr;
    int (*create_data_set)(comgr_handle *) = nullptr;
    int (*destroy_data_set)(comgr_handle) = nullptr;
    int (*data_set_add)(comgr_handle, comgr_handle) = nullptr;
    int (*action_data_count)(comgr_handle, int, size_t *) = nullptr;
    int (*action_data_get_data)(comgr_handle, int, size_t, comgr_handle *) = nullptr;
    int (*create_action_info)(comgr_handle *) = nullptr;
    int (*destroy_action_info)(comgr_handle) = nullptr;
    int (*set_isa_name)(comgr_handle, const char *) = nullptr;
    int (*set_logging)(comgr_handle, bool) = nullptr;
    int (*do_action)(int, comgr_handle, comgr_handle, comgr_handle) = nullptr;
    void (*get_version)(size_t *, size_t *) = nullptr;
    size_t major = 0, minor = 0;
    bool ok = false;
};

Comgr &comgr() {
    static Comgr c;
    static std::once_flag once;
    std::call_once(once, [] {
        const char *names[] = {"libamd_comgr.so.3", "libamd_comgr.so", "/opt/rocm/lib/libamd_comgr.so.3",
                               "/opt/rocm/lib/libamd_comgr.so"};
        for (const char *n : names)
            if ((c.lib = dlopen(n, RTLD_NOW | RTLD_LOCAL))) break;
        if (!c.lib) return;
        bool all = true;
        auto sym = [&](const char *n) { void *p = dlsym(c.lib, n); all = all && p; return p; };
#define COMGR_SYM(field, name) c.field = reinterpret_cast<decltype(c.field)>(sym(name))
        COMGR_SYM(create_data, "amd_comgr_create_data");
        COMGR_SYM(release_data, "amd_comgr_release_data");
        COMGR_SYM(set_data, "amd_comgr_set_data");
        COMGR_SYM(set_data_name, "amd_comgr_set_data_name");
        COMGR_SYM(get_data, "amd_comgr_get_data");
        COMGR_SYM(create_data_set, "amd_comgr_create_data_set");
        COMGR_SYM(destroy_data_set, "amd_comgr_destroy_data_set");
        COMGR_SYM(data_set_add, "amd_comgr_data_set_add");
        COMGR_SYM(action_data_count, "amd_comgr_action_data_count");
        COMGR_SYM(action_data_get_data, "amd_comgr_action_data_get_data");
        COMGR_SYM(create_action_info, "amd_comgr_create_action_info");
        COMGR_SYM(destroy_action_info, "amd_comgr_destroy_action_info");
        COMGR_SYM(set_isa_name, "amd_comgr_action_info_set_isa_name");
        COMGR_SYM(set_logging, "amd_comgr_action_info_set_logging");
        COMGR_SYM(do_action, "amd_comgr_do_action");
        COMGR_SYM(get_version, "amd_comgr_get_version");
#undef COMGR_SYM
        if (all) c.get_version(&c.major, &c.minor);
        c.ok = all && c.major == kComgrMajor;
    });
    return c;
}

std::string fetch_log(Comgr &c, comgr_handle set) {
    size_t n = 0;
    std::string out;
    if (c.action_data_count(set, COMGR_KIND_LOG, &n) != COMGR_SUCCESS) return out;
    for (size_t i = 0; i < n; ++i) {
        comgr_handle d;
        if (c.action_data_get_data(set, COMGR_KIND_LOG, i, &d) != COMGR_SUCCESS) continue;
        size_t sz = 0;
        if (c.get_data(d, &sz, nullptr) == COMGR_SUCCESS && sz) {
            std::string s(sz, '\0');
            c.get_data(d, &sz, &s[0]);
            out += s.substr(0, 2000);
        }
        c.release_data(d);
    }
    return out;
}

int assemble(const std::string &text, std::vector<char> &code, std::string &err) {
    Comgr &c = comgr();
    if (!c.ok) {
        err = c.lib && c.major != kComgrMajor
                  ? "code object manager (libamd_comgr) has interface version " + std::to_string(c.major) + "." +
                        std::to_string(c.minor) + ", this library was written against version 3"
                  : std::string("code object manager (libamd_comgr) is not available");
        return SPARSERT_ECOMPILE;
    }
    comgr_handle src{0}, in{0}, rel{0}, exe{0}, info{0}, out{0};
    int rc = SPARSERT_ECOMPILE;
    bool have_src = false, have_in = false, have_rel = false, have_exe = false, have_info = false;
    do {
        if (c.create_data(COMGR_KIND_SOURCE, &src)) { err = "comgr create_data"; break; }
        have_src = true;
        if (c.set_data(src, text.size(), text.data()) || c.set_data_name(src, "sparsert_spec.s")) { err = "comgr set_data"; break; }
        if (c.create_data_set(&in)) { err = "comgr create_data_set"; break; }
        have_in = true;
        if (c.data_set_add(in, src)) { err = "comgr data_set_add"; break; }
        if (c.create_data_set(&rel)) { err = "comgr create_data_set"; break; }
        have_rel = true;
        if (c.create_data_set(&exe)) { err = "comgr create_data_set"; break; }
        have_exe = true;
        if (c.create_action_info(&info)) { err = "comgr create_action_info"; break; }
        have_info = true;
        if (c.set_isa_name(info, "amdgcn-amd-amdhsa--gfx950")) { err = "comgr does not know gfx950"; break; }
        c.set_logging(info, true);
        if (c.do_action(COMGR_ACTION_ASSEMBLE, info, in, rel)) { err = "assembling the generated kernel failed: " + fetch_log(c, rel); break; }
        if (c.do_action(COMGR_ACTION_LINK_RELOC_TO_EXE, info, rel, exe)) { err = "linking the generated kernel failed: " + fetch_log(c, exe); break; }
        size_t n = 0;
        if (c.action_data_count(exe, COMGR_KIND_EXECUTABLE, &n) || n != 1) { err = "comgr produced no executable"; break; }
        if (c.action_data_get_data(exe, COMGR_KIND_EXECUTABLE, 0, &out)) { err = "comgr get executable"; break; }
        size_t sz = 0;
        if (c.get_data(out, &sz, nullptr) == COMGR_SUCCESS && sz) {
            code.resize(sz);
            if (c.get_data(out, &sz, code.data()) == COMGR_SUCCESS) rc = SPARSERT_OK;
        }
        c.release_data(out);
        if (rc != SPARSERT_OK) err = "comgr get executable bytes";
    } while (false);
    if (have_info) c.destroy_action_info(info);
    if (have_exe) c.destroy_data_set(exe);
    if (have_rel) c.destroy_data_set(rel);
    if (have_in) c.destroy_data_set(in);
    if (have_src) c.release_data(src);
    return rc;
}

// ---------------------------------------------------------------- assembly text
struct Emitter {
    std::string s;
    int64_t lines = 0;
    char buf[256];
    void line(const char *fmt, ...) __attribute__((format(printf, 2, 3))) {
        va_list ap;
        va_start(ap, fmt);
        int n = vsnprintf(buf, sizeof(buf), fmt, ap);
        va_end(ap);
        s.append(buf, (size_t)n);
        s.push_back('\n');
        ++lines;
    }
};

// Fixed register plan of the generated kernel.
constexpr int kSgprB = 4, kSgprC = 6;          // kernarg pointers
constexpr int kRsrcB = 8, kRsrcC = 12;         // buffer descriptors (4 SGPRs each)
constexpr int kSgprTile = 16, kSgprBlock = 17, kSgprPc = 18, kSgprTmp = 20, kSgprTmp2 = 21;
constexpr int kSgprOwns = 22;                  // s[22:23] lanes that own a column
constexpr int kSgprOffRing = 24, kOffRing = 8; // s[24:31] row-offset literals in flight
constexpr int kSgprTap0 = 32;                  // conv: s[32:49] = lane masks of the 9 filter taps
constexpr int kSgprFull = 50;                  // conv: s[50:51] = all lanes
constexpr int kSgprImage = 52;                 // batch > 1: workgroup id z = image / matrix of the batch
constexpr int kSgprJump = 53;                  // byte offset of the block's entry in the table
constexpr int kSgprEntry = 54;                 // prologue only, s[54:55]: the block's table entry and the next one's (offsets of their code from the table)
constexpr int kSgprValRing = 54, kValRing = 8; // half / int8 plans: s[54:61] values of A on their way into the multiply-add
constexpr int kSgprTab = 62, kTab = 32;        // DIRECT: s[62:93] = i * (bytes between consecutive operand rows), i < 32
constexpr int kNextFreeSgpr = 94;
constexpr int kVgprOff = 0;                    // byte offset of the lane's column inside a row
constexpr int kVgprLds = 1;                    // LDS byte address of the lane's 16-byte slot
constexpr int kVgprT1 = 2, kVgprT2 = 3, kVgprAcc0 = 4;
constexpr int kVgprOut = kVgprT2;               // byte offset of the lane's column inside a row of C (after the prologue)
constexpr uint32_t kRsrcWord3 = 0x00020000u;   // raw 32-bit buffer, gfx9 family
constexpr int kMaxChunkRows = 128;             // B rows per LDS buffer (32 KiB), two buffers
constexpr int kMaxLdsBytes = 160 * 1024;        // LDS of one gfx950 compute unit, all of it usable by one workgroup
constexpr int kMaxLgkm = 15;                   // lgkmcnt is a 4-bit counter

struct Term { int acc; uint32_t bits; };

struct Gen {
    Emitter e;
    const HostPlan &h;
    SpecPlan &sp;
    int N, K, D;
    int64_t ldb, ldc;    // elements between consecutive rows of B and of C
    bool half = false;   // B, C and the values of A are IEEE half; sums stay fp32
    bool int8 = false;   // B and the values of A are int8, C is int32, sums are exact integers
    int esz = 4;         // bytes of an element of B / X
    int osz = 4;         // bytes of an element of C / Y
    int val_pos = 0;     // half / int8 plans: next slot of the value ring
    int V = 1;           // columns per lane: 2 halves or 4 int8 packed in the dword a lane loads
    int vgpr_unpack0 = 0;  // int8, V = 4: four registers holding the sign-extended bytes of the current operand;
                           // half, V = 2: one register holding the widened high half
    int vgpr_stage0 = 0, vgpr_ring0 = 0, n_vgpr = 0, lds_bytes = 0;
    int ring_size = 0;               // DIRECT: registers of the operand ring (>= D)
    int slot_bytes = 256;            // K split: bytes of one row's partial sums in the exchange area
    int xchg_rows = 0;               // K split: rows exchanged per phase (all of them if they fit the LDS)
    bool stream_stores = false;      // every wave store of C covers whole 128-byte lines
    bool staged = false;             // LDS variant: operands reach the multiply-adds through LDS, already widened to 32 bits
    int chunk_rows = kMaxChunkRows;  // LDS mode: 32 rows per wave of the workgroup, at most 128
    Gen(const HostPlan &hp, SpecPlan &s)
        : h(hp), sp(s), N(hp.N), K(hp.K), D(s.depth), ldb(hp.ldb), ldc(hp.ldc), half(hp.dtype == SPARSERT_F16), int8(hp.dtype == SPARSERT_I8),
          esz(half ? 2 : int8 ? 1 : 4), osz(half ? 2 : 4) {}

    void zero_accs(size_t n) {
        for (size_t i = 0; i < n * (size_t)V; ++i) e.line("\tv_mov_b32_e32 v%d, 0", kVgprAcc0 + (int)i);
    }
    // The value of A is a literal of the multiply-add.  Half storage: the operand just fetched is
    // widened to fp32 in place, once per fetched row of B (exact), and the value - widened to fp32
    // at generation time, exact as well - is the literal, so a nonzero costs one instruction as in
    // fp32 and the sums are the same fp32 multiply-adds.
    int acc_reg(int row, int j = 0) const { return kVgprAcc0 + row * V + j; }
    void fmas(const std::vector<Term> &terms, int vb) {
        if (terms.empty()) return;
        if (int8 && V == 4)   // the four packed operands, sign-extended once per fetched row of B
            for (int j = 0; j < 4; ++j) e.line("\tv_bfe_i32 v%d, v%d, %d, 8", vgpr_unpack0 + j, vb, 8 * j);
        if (half && !staged) {
            if (V == 2)   // the high half of the dword is the next column
                e.line("\tv_cvt_f32_f16_sdwa v%d, v%d dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:WORD_1", vgpr_unpack0, vb);
            e.line("\tv_cvt_f32_f16_e32 v%d, v%d", vb, vb);
        }
        for (const Term &t : terms) {
            if (int8) {
                // exact: both factors fit 24 bits; values in -16..64 are inline constants
                const int32_t a = (int32_t)t.bits;
                char src[16];
                if (a >= -16 && a <= 64) {
                    snprintf(src, sizeof(src), "%d", a);
                } else {
                    const int sv = kSgprValRing + (val_pos++ % kValRing);
                    e.line("\ts_movk_i32 s%d, %d", sv, a);
                    snprintf(src, sizeof(src), "s%d", sv);
                }
                for (int j = 0; j < V; ++j)
                    e.line("\tv_mad_i32_i24 v%d, %s, v%d, v%d", acc_reg(t.acc, j), src, V == 4 ? vgpr_unpack0 + j : vb,
                           acc_reg(t.acc, j));
            } else {
                e.line("\tv_fmac_f32_e32 v%d, 0x%08x, v%d", acc_reg(t.acc), t.bits, vb);
                if (V == 2) e.line("\tv_fmac_f32_e32 v%d, 0x%08x, v%d", acc_reg(t.acc, 1), t.bits, vgpr_unpack0);
            }
        }
    }
    const char *load_op() const {
        return V > 1 ? "buffer_load_dword" : half ? "buffer_load_short_d16" : int8 ? "buffer_load_sbyte" : "buffer_load_dword";
    }
    void load_b_row(int k, int vdst, int ring_pos) {
        const int sreg = kSgprOffRing + (ring_pos % kOffRing);
        e.line("\ts_mov_b32 s%d, 0x%llx", sreg, (unsigned long long)((int64_t)k * ldb * esz));
        e.line("\t%s v%d, v%d, s[%d:%d], s%d offen", load_op(), vdst, kVgprOff, kRsrcB, kRsrcB + 3, sreg);
    }
    // (slot of the permuted CSR, first accumulator register of the row) pairs: one row of C each
    void stores(const std::vector<std::pair<int32_t, int>> &rows) {
        if (rows.empty()) return;
        e.line("\ts_mov_b64 exec, s[%d:%d]", kSgprOwns, kSgprOwns + 1);
        for (size_t i = 0; i < rows.size(); ++i) {
            const int sreg = kSgprOffRing + ((int)i % kOffRing), r = rows[i].second;
            e.line("\ts_mov_b32 s%d, 0x%llx", sreg, (unsigned long long)((int64_t)h.perm[rows[i].first] * ldc * osz));
            const char *op = "buffer_store_dword";
            if (half) {   // one rounding to nearest even, at the store
                for (int j = 0; j < V; ++j) e.line("\tv_cvt_f16_f32_e32 v%d, v%d", r + j, r + j);
                if (V == 2) e.line("\tv_pack_b32_f16 v%d, v%d, v%d", r, r, r + 1);
                else op = "buffer_store_short";
            }
            // C is written once and not read again by this kernel: where a wave's store covers whole
            // 128-byte lines the non-temporal hint keeps C from displacing the code and the rows of B
            // in the L2 (measured: c3 11.5 -> 10.5 us); on partial lines (N = 49, 196, 784) the same
            // hint costs 0.35 us, so it is left off there
            const char *hint = stream_stores ? " nt" : "";
            if (int8 && V == 4)
                e.line("\tbuffer_store_dwordx4 v[%d:%d], v%d, s[%d:%d], s%d offen%s", r, r + 3, kVgprOut, kRsrcC, kRsrcC + 3, sreg, hint);
            else
                e.line("\t%s v%d, v%d, s[%d:%d], s%d offen%s", op, r, kVgprOut, kRsrcC, kRsrcC + 3, sreg, hint);
        }
    }

    // column -> nonzeros of the group, ascending columns
    std::map<int32_t, std::vector<Term>> columns_of(const std::vector<int32_t> &rows) const {
        std::map<int32_t, std::vector<Term>> cols;
        for (size_t i = 0; i < rows.size(); ++i) {
            const int32_t slot = rows[i];
            for (int32_t p = h.p_row_ptr[slot]; p < h.p_row_ptr[slot + 1]; ++p) {
                uint32_t bits;  // the value as stored (the conv stream is reordered, p_vals is not), as fp32
                if (half) {
                    uint16_t hb;
                    std::memcpy(&hb, &h.p_vals[(size_t)p * 2], 2);
                    bits = half_bits_to_float_bits(hb);
                } else if (int8) {
                    bits = (uint32_t)(int32_t)(int8_t)h.p_vals[(size_t)p];   // the integer value itself
                } else {
                    std::memcpy(&bits, &h.p_vals[(size_t)p * 4], 4);
                }
                cols[h.p_col_idx[p]].push_back({(int)i, bits});
            }
        }
        return cols;
    }

    // Convolution (Section 3.6): operand row k = c*9 + tap is the input plane c displaced by the
    // tap; relative to the descriptor base X - (W+1) elements that is c*H*W + r*W + s elements.
    void load_x_row(int k, int vdst, int ring_pos) {
        const int c = k / 9, tap = k % 9, r = tap / 3, t = tap % 3;
        const int sreg = kSgprOffRing + (ring_pos % kOffRing);
        e.line("\ts_mov_b32 s%d, 0x%llx", sreg, (unsigned long long)(((int64_t)c * h.H * h.W + r * h.W + t) * esz));
        e.line("\t%s v%d, v%d, s[%d:%d], s%d offen", load_op(), vdst, kVgprOff, kRsrcB, kRsrcB + 3, sreg);
    }
    int cur_mask = -1;  // conv: tap whose lane mask is in exec; -1 = all lanes
    void want_mask(int tap) {
        if (tap == cur_mask) return;
        if (tap < 0) e.line("\ts_mov_b64 exec, s[%d:%d]", kSgprFull, kSgprFull + 1);
        else e.line("\ts_mov_b64 exec, s[%d:%d]", kSgprTap0 + 2 * tap, kSgprTap0 + 2 * tap + 1);
        cur_mask = tap;
    }

    // DIRECT: b values come straight from global memory, D columns in flight.  For a
    // convolution the columns are walked tap by tap and every load and multiply-add of a tap
    // runs under that tap's lane mask: lanes whose tap falls into the padding neither read
    // nor accumulate, which is the zero contribution of the padding.
    // With `parts` > 1 the waves of a workgroup share the block's rows and tile and split its
    // columns (Section 3.4, thread-group balance: contiguous ranges with equal nonzero counts,
    // the last one takes the remainder); partial accumulators meet in LDS (Section 3.3).
    int block_direct(const std::vector<int32_t> &rows, int part = 0, int parts = 1) {
        auto cols = columns_of(rows);
        std::vector<int32_t> order;
        for (auto &kv : cols) order.push_back(kv.first);
        if (h.conv)
            std::stable_sort(order.begin(), order.end(), [](int32_t a, int32_t b) { return a % 9 < b % 9; });
        if (parts > 1) {
            int64_t total = 0;
            for (int32_t k : order) total += (int64_t)cols[k].size();
            const int64_t share = (total + parts - 1) / parts;
            std::vector<int32_t> mine;
            int64_t seen = 0;
            for (int32_t k : order) {   // a column belongs to the part its first nonzero falls into
                const int p = share ? (int)std::min<int64_t>(parts - 1, seen / share) : 0;
                if (p == part) mine.push_back(k);
                seen += (int64_t)cols[k].size();
            }
            order.swap(mine);
        }
        const int nc = (int)order.size();
        cur_mask = -1;
        // Byte offset of operand row k from the descriptor base (convolution: Section 3.6, operand row
        // k = c*9 + tap is the input plane c displaced by the tap).
        auto offset_of = [&](int32_t k) -> int64_t {
            if (!h.conv) return (int64_t)k * ldb * esz;
            const int c = k / 9, tap = k % 9;
            return ((int64_t)c * h.H * h.W + (tap / 3) * h.W + tap % 3) * esz;
        };
        // Where the rows a block fetches lie close together, their offsets come from a table of
        // multiples of the row pitch kept in scalar registers, and the lane's address register is
        // advanced when a row falls outside the table's reach: no scalar move per fetch.  Blocks
        // whose rows are far apart would advance at every fetch and keep the move instead.
        const int64_t unit = h.conv ? (int64_t)h.H * h.W * esz : ldb * esz;
        bool use_tab = false;
        {
            int64_t base = 0;
            int bumps = 0;
            for (int j = 0; j < nc; ++j) {
                const int64_t d = offset_of(order[j]) - base;
                if (d < 0 || d % unit || d / unit >= kTab) { ++bumps; base += d; }
            }
            use_tab = nc >= 16 && (int64_t)bumps * (h.conv ? 12 : 4) <= nc;
        }
        bool tab_ready[kTab] = {false};   // an entry is written right before its first use, so no fetch waits for the whole table
        int64_t cur_base = 0;             // bytes the address register has been advanced by so far
        auto issue = [&](int j) {
            const int vdst = vgpr_ring0 + (j % D);
            if (!use_tab) {
                if (h.conv) { want_mask(order[j] % 9); load_x_row(order[j], vdst, j); }
                else load_b_row(order[j], vdst, j);
                return;
            }
            int64_t d = offset_of(order[j]) - cur_base;
            if (d < 0 || d % unit || d / unit >= kTab) {
                if (h.conv) want_mask(-1);   // every lane's address moves, whatever tap mask is current
                e.line("\tv_add_u32_e32 v%d, 0x%x, v%d", kVgprOff, (uint32_t)(int32_t)d, kVgprOff);
                cur_base += d;
                d = 0;
            }
            if (h.conv) want_mask(order[j] % 9);
            const int slot = (int)(d / unit);
            if (!tab_ready[slot]) {
                e.line("\ts_mov_b32 s%d, 0x%llx", kSgprTab + slot, (unsigned long long)(slot * unit));
                tab_ready[slot] = true;
            }
            e.line("\t%s v%d, v%d, s[%d:%d], s%d offen", load_op(), vdst, kVgprOff, kRsrcB, kRsrcB + 3, kSgprTab + slot);
        };
        for (int j = 0; j < std::min(D, nc); ++j) issue(j);
        // the accumulators are cleared while the first fetches are on their way
        if (h.conv) want_mask(-1);
        zero_accs(rows.size());
        for (int j = 0; j < nc; ++j) {
            // loads issued so far: columns [0, min(nc, j + D)); those after column j may stay in
            // flight.  (Waiting once per batch of columns was measured slower than once per column.)
            e.line("\ts_waitcnt vmcnt(%d)", std::min(nc, j + D) - 1 - j);
            if (h.conv) want_mask(order[j] % 9);
            fmas(cols[order[j]], vgpr_ring0 + (j % D));
            if (j + D < nc) issue(j + D);
        }
        if (parts > 1) {
            if (h.conv) want_mask(-1);
            // The rows of the block are dealt to the waves in contiguous runs of ceil(rows / parts).
            // Every wave leaves its partial sums of the rows it does not own in LDS, and after
            // one barrier adds the other waves' partials to its own rows in ascending wave order,
            // then stores those rows.  The accumulators of a run are consecutive registers, so
            // they travel four (two, one) at a time: a piece of n registers from one wave is an
            // LDS region [lane][n dwords], written and read with one 16- (8-, 4-) byte access per
            // lane.  Blocks whose partial sums do not fit the LDS at once exchange them in phases
            // of xchg_rows rows, with a second barrier before the area is overwritten.
            const int nr = (int)rows.size();
            const int chunk = (nr + parts - 1) / parts;
            auto own_lo = [&](int q) { return std::min(nr, q * chunk); };
            auto own_hi = [&](int q) { return std::min(nr, (q + 1) * chunk); };
            const int rb = slot_bytes / V;                        // bytes of one register's partials over the lanes of a tile
            const int cq = nr <= xchg_rows ? std::max(1, chunk) : std::max(1, xchg_rows / parts);   // rows per owner and phase
            const int n_phases = (chunk + cq - 1) / cq;
            struct Piece { int reg, len, off; };                  // first register, registers, byte offset of the region
            // address registers: lane * 4n for the three piece sizes, one set per 64 KiB window of
            // the area (ds offsets are 16 bits wide); they and the temporaries borrow the operand ring
            const int n_win = (lds_bytes + 65535) / 65536;
            const int base0 = vgpr_ring0;
            auto addr_reg = [&](int len, int off) {
                const int m = len == 4 ? 2 : len == 2 ? 1 : 0, w = off >> 16;
                return m == 0 && w == 0 ? kVgprLds : base0 + m * n_win + w - 1;
            };
            for (int m = 0; m < 3; ++m)
                for (int w = 0; w < n_win; ++w) {
                    if (m == 0 && w == 0) continue;
                    const int r = addr_reg(1 << m, w << 16);
                    if (m == 0) e.line("\tv_add_u32_e32 v%d, 0x%x, v%d", r, w * 65536, kVgprLds);
                    else if (w == 0) e.line("\tv_lshlrev_b32_e32 v%d, %d, v%d", r, m, kVgprLds);
                    else e.line("\tv_add_u32_e32 v%d, 0x%x, v%d", r, w * 65536, addr_reg(1 << m, 0));
                }
            const int tmp0 = (base0 + 3 * n_win - 1 + 1) / 2 * 2;   // even: 64-bit and wider operands need aligned registers
            const int n_tmp = vgpr_ring0 + ring_size - tmp0;
            if (n_tmp < 4) throw std::runtime_error("operand ring too small for the partial-sum exchange");
            static const char *const kWidth[5] = {"", "b32", "b64", "", "b128"};
            auto vregs = [](int r, int len, char *buf, size_t cap) {
                if (len == 1) snprintf(buf, cap, "v%d", r); else snprintf(buf, cap, "v[%d:%d]", r, r + len - 1);
            };
            std::vector<std::pair<int32_t, int>> mine;
            for (int i = own_lo(part); i < own_hi(part); ++i) mine.push_back({rows[i], acc_reg(i)});
            for (int ph = 0; ph < n_phases; ++ph) {
                // layout of the phase: for every owner q and every other wave s, the pieces of
                // q's rows of this phase as s left them
                std::vector<std::vector<std::vector<Piece>>> lay(parts, std::vector<std::vector<Piece>>(parts));
                int area = 0;
                for (int q = 0; q < parts; ++q) {
                    const int lo = std::min(own_hi(q), own_lo(q) + ph * cq), hi = std::min(own_hi(q), lo + cq);
                    for (int sw = 0; sw < parts; ++sw) {
                        if (sw == q) continue;
                        for (int f = lo * V; f < hi * V;) {
                            const int reg = kVgprAcc0 + f;
                            const int len = (reg & 1) ? 1 : f + 4 <= hi * V ? 4 : f + 2 <= hi * V ? 2 : 1;
                            lay[q][sw].push_back({reg, len, area});
                            area += len * rb;
                            f += len;
                        }
                    }
                }
                if (area > lds_bytes) throw std::runtime_error("partial-sum exchange exceeds its LDS area");
                if (ph > 0) e.line("\ts_barrier");   // every wave has read the previous phase
                char regs[32];
                for (int q = 0; q < parts; ++q)
                    for (const Piece &pc : lay[q][part]) {
                        vregs(pc.reg, pc.len, regs, sizeof(regs));
                        e.line("\tds_write_%s v%d, %s offset:%d", kWidth[pc.len], addr_reg(pc.len, pc.off), regs, pc.off & 65535);
                    }
                e.line("\ts_waitcnt lgkmcnt(0)");
                e.line("\ts_barrier");
                std::vector<Piece> items;   // ascending source wave: the order the partials are added in
                for (int sw = 0; sw < parts; ++sw) items.insert(items.end(), lay[part][sw].begin(), lay[part][sw].end());
                for (size_t b0 = 0; b0 < items.size();) {
                    std::vector<int> at;   // temporary of each piece of the batch
                    int cur = 0;
                    size_t b1 = b0;
                    for (; b1 < items.size() && (int)at.size() < kMaxLgkm; ++b1) {
                        const int len = items[b1].len;
                        const int start = len > 1 ? (cur + 1) / 2 * 2 : cur;
                        if (start + len > n_tmp) break;
                        at.push_back(tmp0 + start);
                        cur = start + len;
                    }
                    for (size_t t = b0; t < b1; ++t) {
                        vregs(at[t - b0], items[t].len, regs, sizeof(regs));
                        e.line("\tds_read_%s %s, v%d offset:%d", kWidth[items[t].len], regs, addr_reg(items[t].len, items[t].off),
                               items[t].off & 65535);
                    }
                    for (size_t t = b0; t < b1; ++t) {
                        e.line("\ts_waitcnt lgkmcnt(%d)", (int)(b1 - 1 - t));
                        for (int j = 0; j < items[t].len; ++j)
                            e.line("\t%s v%d, v%d, v%d", int8 ? "v_add_u32_e32" : "v_add_f32_e32", items[t].reg + j, items[t].reg + j,
                                   at[t - b0] + j);
                    }
                    b0 = b1;
                }
            }
            stores(mine);
            e.line("\ts_endpgm");
            return nc;
        }
        std::vector<std::pair<int32_t, int>> all;
        for (size_t i = 0; i < rows.size(); ++i) all.push_back({rows[i], acc_reg((int)i)});
        stores(all);
        e.line("\ts_endpgm");
        return nc;
    }

    // LDS: wave `w` of W stages quads q == w (mod W) of every chunk; all waves read what
    // they need.  LDS layout per buffer: [quad of 4 consecutive B rows][lane][4 floats].
    int block_lds(const std::vector<int32_t> &rows, int w, int W) {
        auto cols = columns_of(rows);
        const int kChunkRows = chunk_rows;
        const int n_chunks = (K + kChunkRows - 1) / kChunkRows;
        const int quads_per_chunk = kChunkRows / 4;
        const int buf_bytes = kChunkRows * 256;
        int ring_pos = 0;
        zero_accs(rows.size());
        // Staging runs two chunks ahead of the compute: chunk c travels through register set
        // c % 2, so a fetch has two compute phases to arrive before it is copied into LDS.
        const int quads_per_wave = (quads_per_chunk + W - 1) / W;
        std::vector<int> n_loads(n_chunks + 3, 0);
        auto stage_loads = [&](int c) {
            if (c >= n_chunks) return;
            int t = 0, n = 0;
            for (int q = w; q < quads_per_chunk; q += W, ++t)
                for (int j = 0; j < 4; ++j) {
                    const int k = c * kChunkRows + 4 * q + j;
                    if (k < K) { load_b_row(k, vgpr_stage0 + (c & 1) * 4 * quads_per_wave + 4 * t + j, ring_pos++); ++n; }
                }
            n_loads[c] = n;
        };
        auto stage_write = [&](int c) {
            // fetches return in order: chunk c has arrived once only chunk c+1's are outstanding
            e.line("\ts_waitcnt vmcnt(%d)", c + 1 < n_chunks ? n_loads[c + 1] : 0);
            int t = 0;
            for (int q = w; q < quads_per_chunk; q += W, ++t) {
                if (c * kChunkRows + 4 * q >= K) break;
                const int v = vgpr_stage0 + (c & 1) * 4 * quads_per_wave + 4 * t;
                // half storage: widened once here (exact), so the staged tile and everything after
                // it is the fp32 code; int8 arrives sign-extended by the load itself
                if (half)
                    for (int j = 0; j < 4 && c * kChunkRows + 4 * q + j < K; ++j) e.line("\tv_cvt_f32_f16_e32 v%d, v%d", v + j, v + j);
                e.line("\tds_write_b128 v%d, v[%d:%d] offset:%d", kVgprLds, v, v + 3, (c & 1) * buf_bytes + q * 1024);
            }
        };
        stage_loads(0);
        stage_loads(1);
        stage_write(0);
        e.line("\ts_waitcnt lgkmcnt(0)");
        stage_loads(2);
        e.line("\ts_barrier");
        int total_cols = 0;
        for (int c = 0; c < n_chunks; ++c) {
            // quads of this chunk that hold a nonzero column of the group
            struct Quad { int q; std::vector<Term> terms[4]; bool need[4]; };
            std::vector<Quad> quads;
            for (auto it = cols.lower_bound(c * kChunkRows); it != cols.end() && it->first < (c + 1) * kChunkRows; ++it) {
                const int kl = it->first - c * kChunkRows, q = kl / 4, j = kl % 4;
                if (quads.empty() || quads.back().q != q) { quads.push_back(Quad()); quads.back().q = q; for (bool &b : quads.back().need) b = false; }
                quads.back().need[j] = true;
                quads.back().terms[j] = it->second;
                ++total_cols;
            }
            const int nq = (int)quads.size();
            std::vector<int> last_seq(nq, -1);
            int issued = 0;
            auto issue_reads = [&](int i) {
                const Quad &Q = quads[i];
                const int v0 = vgpr_ring0 + 4 * (i % D), off = (c & 1) * buf_bytes + Q.q * 1024;
                const int cnt = Q.need[0] + Q.need[1] + Q.need[2] + Q.need[3];
                if (cnt >= 3) {
                    e.line("\tds_read_b128 v[%d:%d], v%d offset:%d", v0, v0 + 3, kVgprLds, off);
                    ++issued;
                } else {
                    for (int j = 0; j < 4; j += 2) {
                        if (Q.need[j] && Q.need[j + 1]) {
                            e.line("\tds_read_b64 v[%d:%d], v%d offset:%d", v0 + j, v0 + j + 1, kVgprLds, off + 4 * j);
                            ++issued;
                        } else if (Q.need[j] || Q.need[j + 1]) {
                            const int jj = Q.need[j] ? j : j + 1;
                            e.line("\tds_read_b32 v%d, v%d offset:%d", v0 + jj, kVgprLds, off + 4 * jj);
                            ++issued;
                        }
                    }
                }
                last_seq[i] = issued - 1;
            };
            for (int i = 0; i < std::min(D, nq); ++i) issue_reads(i);
            for (int i = 0; i < nq; ++i) {
                // LDS reads return in order: quad i is complete once at most
                // (issued - 1 - last_seq[i]) later reads are outstanding
                e.line("\ts_waitcnt lgkmcnt(%d)", std::min(kMaxLgkm, issued - 1 - last_seq[i]));
                for (int j = 0; j < 4; ++j)
                    if (quads[i].need[j]) fmas(quads[i].terms[j], vgpr_ring0 + 4 * (i % D) + j);
                if (i + D < nq) issue_reads(i + D);
            }
            if (c + 1 < n_chunks) {
                stage_write(c + 1);
                e.line("\ts_waitcnt lgkmcnt(0)");
                stage_loads(c + 3);
                e.line("\ts_barrier");
            }
        }
        std::vector<std::pair<int32_t, int>> all;
        for (size_t i = 0; i < rows.size(); ++i) all.push_back({rows[i], kVgprAcc0 + (int)i});
        stores(all);
        e.line("\ts_endpgm");
        return total_cols;
    }
};

}  // namespace

bool spec_available() { return comgr().ok; }

int rows_for_whole_rounds(int32_t M, int groups_per_wg, int64_t wg_columns, int lo, int hi) {
    constexpr int64_t kComputeUnits = 256;
    lo = std::max(1, std::min<int>(lo, M));
    hi = std::max(lo, std::min<int>(hi, M));
    int best = -1;
    int64_t best_cost = INT64_MAX;
    for (int r = lo; r <= hi; ++r) {
        const int64_t groups = ((int64_t)M + r - 1) / r;
        const int64_t wgs = (groups + groups_per_wg - 1) / groups_per_wg * wg_columns;
        if (wgs < kComputeUnits) continue;   // the model holds while every compute unit has a workgroup
        const int64_t cost = (wgs + kComputeUnits - 1) / kComputeUnits * r;
        if (cost < best_cost || (cost == best_cost && r > best)) { best = r; best_cost = cost; }
    }
    return best > 0 ? best : lo;   // too small a launch for any count in range: the most workgroups
}

static int64_t workgroups_for(int32_t M, int r, int groups_per_wg, int64_t wg_columns) {
    const int64_t groups = ((int64_t)M + r - 1) / r;
    return (groups + groups_per_wg - 1) / groups_per_wg * wg_columns;
}

int rows_for_rounds(int32_t M, int groups_per_wg, int64_t wg_columns, int rounds, int hi) {
    constexpr int64_t kComputeUnits = 256;
    for (int r = 1; r <= std::min<int>(hi, M); ++r)
        if (workgroups_for(M, r, groups_per_wg, wg_columns) <= kComputeUnits * rounds) return r;
    return 0;
}

int rows_without_thin_round(int32_t M, int R, int groups_per_wg, int64_t wg_columns, int hi) {
    constexpr int64_t kComputeUnits = 256;
    const int64_t wgs = workgroups_for(M, R, groups_per_wg, wg_columns);
    const int64_t rounds = (wgs + kComputeUnits - 1) / kComputeUnits;
    // (blocks of a few rows make small workgroups, several of which share a compute unit: no rounds there)
    if (R < 8 || rounds < 2 || rounds > 16 || wgs - kComputeUnits * (rounds - 1) > kComputeUnits / 4) return R;
    const int top = std::min<int>(std::min<int>(hi, M), R + (R * 15 + 99) / 100);
    for (int r = R + 1; r <= top; ++r)
        if (workgroups_for(M, r, groups_per_wg, wg_columns) <= kComputeUnits * (rounds - 1))
            return (rounds - 1) * r < rounds * R ? r : R;
    return R;
}

// What the stages below hand to each other besides the SpecPlan itself.
struct Shape {
    bool lds = false;   // LDS-staged variant
    int max_lanes = kWave, V = 1, nvc = 0, KS = 1, W = 4, wshift = 2;
};

// Stage 1, launch policy: variant, column tiling, columns per lane, rows per block, K split,
// waves per workgroup, fetch depth, number of code blocks.
static int choose_launch_shape(const HostPlan &h, const sparsert_options &opt, SpecPlan &sp, Shape &sh, std::string &err) {
    if (h.conv && opt.spec_mode == SPARSERT_SPEC_LDS) {
        err = "convolution plans use the DIRECT variant of the generated kernel";
        return SPARSERT_EUNSUPPORTED;
    }
    const bool half = h.dtype == SPARSERT_F16, int8 = h.dtype == SPARSERT_I8;
    const int32_t M = h.M, N = h.N;
    sp.mode = opt.spec_mode ? opt.spec_mode : SPARSERT_SPEC_DIRECT;
    // With nothing set, large and very sparse products take the LDS-staged variant with eight waves:
    // every wave fetches a row of B for few multiply-adds there, and staging lets eight blocks share
    // each fetch.  Over the shape sweep it is what the tuner picks from 95 % sparsity on once a
    // compute unit has 512 rows x tiles of C to itself (4096 x 4096 x 4096 at 98 %: 73 us against
    // 156 us for the DIRECT default; 2048 x 2048 x 3136, 392 per compute unit, is better off with
    // DIRECT); below 95 % the multiply-adds dominate and DIRECT is as fast.  M >= 2048 keeps the rule
    // to what was measured: eight waves with blocks of at least 32 rows and several workgroups per tile.
    bool auto_staged = false;
    if (!opt.spec_mode && !opt.spec_rows && !opt.spec_ksplit && !opt.spec_tiles && !opt.spec_lanes && opt.spec_vec <= 1 &&
        h.dtype == SPARSERT_F32 && !h.conv && M >= 2048 && h.K >= 1024 && (int64_t)h.nnz * 18 <= (int64_t)M * h.K &&
        (int64_t)M * ((N + kWave - 1) / kWave) * std::max(1, h.batch) >= 131072) {
        sp.mode = SPARSERT_SPEC_LDS;
        auto_staged = true;
    }
    const bool lds = sp.mode == SPARSERT_SPEC_LDS;
    // Column tiling with one column per lane, balanced tails (same rule as the row-walk plan at V = 1).
    const int max_lanes = opt.spec_lanes ? opt.spec_lanes : kWave;
    if (lds && max_lanes != kWave) { err = "spec_lanes applies to the DIRECT variant"; return SPARSERT_EINVAL; }
    // Columns per lane: 1, or the 2 halves / 4 int8 that share the dword a lane loads (SpMM only).
    const int V = opt.spec_vec ? opt.spec_vec : 1;
    if (!(V == 1 || (V == 2 && half) || (V == 4 && int8))) { err = "spec_vec must be 0/1, 2 for half plans or 4 for int8 plans"; return SPARSERT_EINVAL; }
    if (V > 1 && (h.conv || lds)) { err = "spec_vec > 1 applies to SpMM plans of the DIRECT variant"; return SPARSERT_EINVAL; }
    if (N % V || h.ldb % V || h.ldc % V) { err = "N, ldb and ldc must be multiples of spec_vec"; return SPARSERT_EINVAL; }
    sp.vec = V;
    const int32_t nvc = N / V;   // vector columns
    sp.n_tiles = (nvc + max_lanes - 1) / max_lanes;
    sp.lanes_per_tile = (nvc + sp.n_tiles - 1) / sp.n_tiles;
    sp.tiles_per_wg = opt.spec_tiles ? opt.spec_tiles : auto_staged ? 8 : 4;
    // Rows per block and K split.  Left at 0 they follow what the tuner's winners have in common
    // on this chip: a launch of about two waves per SIMD (2048 waves), with as many rows per
    // block as that allows, because rows per block is what saves fetches of B, and with the
    // reduction axis split over the waves of a workgroup where it is long enough to supply them.
    int R = opt.spec_rows;
    int KS = opt.spec_ksplit;
    if (KS == 0) KS = (!lds && R == 0 && h.K >= 512) ? 8 : 1;
    if (auto_staged) {
        R = rows_for_whole_rounds(M, 8, (int64_t)sp.n_tiles * std::max(1, h.batch), 32, 128);
    } else if (R == 0 && lds) {
        // LDS variant: R1 fills 1024 SIMDs with one wave each, R2 gives a wave about 400 multiply-adds
        const int64_t r1 = (int64_t)M * sp.n_tiles / 1024;
        const int64_t avg = std::max<int64_t>(1, h.nnz / M);
        const int64_t r2 = (400 + avg - 1) / avg;
        R = (int)std::min<int64_t>(96, std::max<int64_t>(4, std::max(r1, r2)));
    } else if (R == 0) {
        const int64_t tiles_all = (int64_t)sp.n_tiles * std::max(1, h.batch);
        const int64_t target = KS > 1 ? 2048 : 1024;
        R = (int)std::max<int64_t>(1, std::min<int64_t>(96 / V, (int64_t)M * tiles_all * KS / target));
        if (opt.spec_ksplit == 0)   // fewer parts where the rows alone already supply the waves
            while (KS > 1 && ((int64_t)M + R - 1) / R * tiles_all * (KS / 2) >= 2048) KS /= 2;
        // 1024 rows in blocks of 52 on 13 column tiles are 260 workgroups, four more than compute
        // units: 34.8 us; in blocks of 54 they are 247: 21.3 us (4096 columns of A at 95 %)
        const int T = opt.spec_tiles ? opt.spec_tiles : 4;
        const int64_t wg_columns = KS > 1 ? tiles_all : (sp.n_tiles + T - 1) / T * std::max(1, h.batch);
        R = rows_without_thin_round(M, R, 1, wg_columns, 128 / V);
    }
    sp.ksplit = KS;
    if (sp.ksplit != 1 && sp.ksplit != 2 && sp.ksplit != 4 && sp.ksplit != 8) { err = "spec_ksplit must be 0,1,2,4,8"; return SPARSERT_EINVAL; }
    if (sp.ksplit > 1 && lds) { err = "spec_ksplit applies to the DIRECT variant"; return SPARSERT_EINVAL; }
    if (sp.ksplit > 1) sp.tiles_per_wg = sp.ksplit;   // the waves of a workgroup are the K parts
    const int W = sp.tiles_per_wg;
    int wshift = 0;
    while ((1 << wshift) < W) ++wshift;
    if (R < 1 || R > 232) { err = "spec_rows must be in 1..232"; return SPARSERT_EINVAL; }
    R = std::min(R, M);
    sp.rows_per_group = R;
    sp.n_groups = (M + R - 1) / R;
    sp.depth = opt.spec_depth ? opt.spec_depth : (lds ? 6 : 16);
    if (lds && sp.depth > 12) sp.depth = 12;
    const int G = sp.n_groups;
    // LDS mode: a workgroup runs W consecutive blocks and every one of them takes part in the
    // staging and the barriers, so the block list is padded with empty blocks.
    sp.n_blocks = lds ? (G + W - 1) / W * W : G * sp.ksplit;
    sh.lds = lds; sh.max_lanes = max_lanes; sh.V = V; sh.nvc = nvc; sh.KS = sp.ksplit; sh.W = W; sh.wshift = wshift;
    return SPARSERT_OK;
}

// Stage 2, block formation: which slots (rows of the permuted CSR) share a code block.
static void form_blocks(const HostPlan &h, const sparsert_options &opt, SpecPlan &sp,
                        std::vector<std::vector<int32_t>> &members) {
    const int32_t M = h.M;
    const int R = sp.rows_per_group, G = sp.n_groups;
    // Block-level balance (Section 3.4, strategy b): slots are in descending-nnz order; deal
    // them to the groups in serpentine order so every group gets nearly the same nonzero count.
    members.assign(sp.n_blocks, {});
    sp.group_of_slot.resize(M);
    sp.swizzle = opt.spec_swizzle && !h.natural_order;
    if (!sp.swizzle) {
        for (int32_t i = 0; i < M; ++i) {
            const int32_t round = i / G, pos = i % G;
            // natural order (ablation): block g is the contiguous row range [g*R, (g+1)*R)
            const int32_t g = h.natural_order ? i / R : ((round & 1) ? G - 1 - pos : pos);
            sp.group_of_slot[i] = g;
            members[g].push_back(i);
        }
    } else {
        // Row swizzle (Section 5, named there as a preprocessing step that would help): rows that share columns go to the
        // same block, so the block fetches fewer rows of B.  The nnz-descending slots are
        // handed out in rounds of G, one row per block and round, which keeps the nonzero
        // counts of the blocks within one row's worth of each other as the serpentine deal
        // does; inside a round each block, in serpentine direction, takes the candidate that
        // shares the most columns with what the block already fetches (ties: lowest slot).
        const int words = (h.K + 63) / 64;
        std::vector<uint64_t> pattern((size_t)M * words, 0), fetched((size_t)G * words, 0);
        for (int32_t i = 0; i < M; ++i)
            for (int32_t p = h.p_row_ptr[i]; p < h.p_row_ptr[i + 1]; ++p)
                pattern[(size_t)i * words + h.p_col_idx[p] / 64] |= 1ull << (h.p_col_idx[p] % 64);
        std::vector<char> taken(M, 0);
        for (int32_t first = 0, round = 0; first < M; first += G, ++round) {
            const int32_t last = std::min<int32_t>(M, first + G);
            for (int32_t step = 0; step < last - first; ++step) {
                const int32_t g = (round & 1) ? G - 1 - step : step;
                int32_t best = -1;
                int64_t best_shared = -1;
                for (int32_t c = first; c < last; ++c) {
                    if (taken[c]) continue;
                    int64_t shared = 0;
                    if (round > 0)
                        for (int w = 0; w < words; ++w)
                            shared += __builtin_popcountll(pattern[(size_t)c * words + w] & fetched[(size_t)g * words + w]);
                    if (shared > best_shared) { best_shared = shared; best = c; }
                    if (round == 0) break;   // seeding: slot first+step goes to block step
                }
                taken[best] = 1;
                sp.group_of_slot[best] = g;
                members[g].push_back(best);
                for (int w = 0; w < words; ++w) fetched[(size_t)g * words + w] |= pattern[(size_t)best * words + w];
            }
        }
    }

}

// Stage 3, register and LDS plan: where accumulators, the operand ring, staging registers and the
// exchange area sit; the descriptor extents; the convolution's pixel-index constant.
struct Extents { int64_t b_bytes = 0, c_bytes = 0; uint32_t magic = 0; };

static int plan_registers(const HostPlan &h, SpecPlan &sp, const Shape &sh, const std::vector<std::vector<int32_t>> &members,
                          Gen &gen, Extents &ex, std::string &err) {
    const bool half = gen.half, int8 = gen.int8, lds = sh.lds;
    const int esz = gen.esz, osz = gen.osz, V = sh.V, KS = sh.KS, W = sh.W, max_lanes = sh.max_lanes;
    const int32_t M = h.M, N = h.N;
    gen.stream_stores = ((int64_t)h.ldc * osz) % 128 == 0 && ((int64_t)sp.lanes_per_tile * V * osz) % 128 == 0;
    // descriptor extents: the last row of a matrix ends after its N columns, whatever the pitch
    ex.b_bytes = h.conv ? ((int64_t)h.Cin * N + 2 * (h.W + 1)) * esz : ((int64_t)(h.K - 1) * h.ldb + N) * esz;
    ex.c_bytes = ((int64_t)(M - 1) * h.ldc + N) * osz;
    // conv: pixel -> (oh, ow) by multiplication with ceil(2^32 / W); verified here for every pixel
    uint32_t &magic = ex.magic;
    if (h.conv && h.W > 1) {
        magic = (uint32_t)(((1ull << 32) + h.W - 1) / h.W);
        for (int64_t p = 0; p < N; ++p)
            if ((int64_t)(((uint64_t)p * magic) >> 32) != p / h.W) {
                err = "image too large for the generated kernel's pixel index arithmetic";
                return SPARSERT_EUNSUPPORTED;
            }
    }
    int max_rows = 0;
    for (auto &m : members) max_rows = std::max<int>(max_rows, (int)m.size());
    const int D = sp.depth;
    if (lds) {
        gen.staged = true;
        gen.chunk_rows = std::min(kMaxChunkRows, 32 * W);
        const int kChunkRows = gen.chunk_rows;
        const int quads_per_wave = (kChunkRows / 4 + W - 1) / W;
        gen.vgpr_stage0 = (kVgprAcc0 + max_rows + 3) / 4 * 4;
        gen.vgpr_ring0 = gen.vgpr_stage0 + 2 * 4 * quads_per_wave;
        gen.n_vgpr = gen.vgpr_ring0 + 4 * D;
        const int n_chunks = (h.K + kChunkRows - 1) / kChunkRows;
        gen.lds_bytes = (n_chunks > 1 ? 2 : 1) * kChunkRows * 256;
    } else {
        gen.V = V;
        gen.vgpr_ring0 = kVgprAcc0 + max_rows * V;
        gen.ring_size = KS > 1 ? std::max(D, 20) : D;   // the K-split exchange borrows the ring: address registers and temporaries
        gen.vgpr_unpack0 = gen.vgpr_ring0 + gen.ring_size;
        gen.n_vgpr = gen.vgpr_unpack0 + (int8 && V == 4 ? 4 : half && V == 2 ? 1 : 0);
        if (KS > 1) {
            gen.slot_bytes = V * ((4 * max_lanes + 15) / 16 * 16);   // a row's partial sums: V registers over the lanes of a tile, 16-byte granules
            gen.xchg_rows = std::min(max_rows, kMaxLdsBytes / ((KS - 1) * gen.slot_bytes));
            gen.lds_bytes = (KS - 1) * gen.xchg_rows * gen.slot_bytes;
            if (gen.lds_bytes == 0) gen.lds_bytes = 256;
        }
    }
    if (gen.n_vgpr > 256) { err = "spec_rows too large for the register file"; return SPARSERT_EINVAL; }
    // A workgroup must fit a compute unit at once: its waves are spread over the four SIMDs, and a
    // SIMD has 512 registers per lane, handed out in granules of eight.  (A dispatch that does not
    // fit is rejected by the hardware queue, which aborts the process.)
    if ((W + 3) / 4 * ((gen.n_vgpr + 7) / 8 * 8) > 512) {
        err = "spec_rows too large for this many waves per workgroup: the workgroup's registers do not fit a compute unit";
        return SPARSERT_EINVAL;
    }
    // The symbol carries the problem shape so that kernel traces tell the plans of a model apart.
    char sym[96];
    snprintf(sym, sizeof(sym), "sparsert_spec_%s%dx%dx%d%s", h.conv ? "conv_" : "", (int)M, (int)h.K, (int)N,
             half ? (V == 2 ? "_f16x2" : "_f16") : int8 ? (V == 4 ? "_i8x4" : "_i8") : "");
    sp.symbol = sym;
    sp.lds_bytes = gen.lds_bytes;

    return SPARSERT_OK;
}

// Stage 4a, emission of everything before the blocks: directives, the prologue that turns the
// workgroup and lane ids into a block, a column and two buffer descriptors, and the jump table.
static void emit_prologue(Gen &gen, Emitter &e, const Shape &sh, const Extents &ex, int prefetch_lines) {
    const HostPlan &h = gen.h;
    SpecPlan &sp = gen.sp;
    const bool lds = sh.lds;
    const int esz = gen.esz, osz = gen.osz, V = sh.V, KS = sh.KS, wshift = sh.wshift, nvc = sh.nvc, n_blocks = sp.n_blocks;
    const int32_t M = h.M, N = h.N;
    const int64_t b_bytes = ex.b_bytes, c_bytes = ex.c_bytes;
    const uint32_t magic = ex.magic;
    e.line("\t.amdgcn_target \"amdgcn-amd-amdhsa--gfx950\"");
    e.line("\t.amdhsa_code_object_version 6");
    e.line("\t.text");
    const char *sym = sp.symbol.c_str();
    e.line("\t.protected\t%s", sym);
    e.line("\t.globl\t%s", sym);
    e.line("\t.p2align\t8");
    e.line("\t.type\t%s,@function", sym);
    e.line("%s:", sym);
    // s[0:1] kernarg, s2 = workgroup id x, s3 = workgroup id y, (s4 = workgroup id z), v0 = thread id
    const bool images = h.batch > 1;
    if (images) e.line("\ts_mov_b32 s%d, s4", kSgprImage);   // s4 is about to receive a kernel argument
    e.line("\ts_load_dwordx4 s[%d:%d], s[0:1], 0x0", kSgprB, kSgprC + 1);
    e.line("\tv_lshrrev_b32_e32 v%d, 6, v0", kVgprT1);
    e.line("\tv_and_b32_e32 v%d, 63, v0", kVgprOff);
    e.line("\ts_nop 1");
    e.line("\tv_readfirstlane_b32 s%d, v%d", kSgprTile, kVgprT1);  // wave index inside the workgroup
    e.line("\ts_nop 4");
    if (!lds && KS > 1) {
        // grid (tiles, groups): the waves of a workgroup run the K parts of one group on one tile
        e.line("\ts_lshl_b32 s%d, s3, %d", kSgprTmp, wshift);
        e.line("\ts_add_u32 s%d, s%d, s%d", kSgprBlock, kSgprTmp, kSgprTile);
        e.line("\ts_mov_b32 s%d, s2", kSgprTile);
        e.line("\tv_lshlrev_b32_e32 v%d, 2, v%d", kVgprLds, kVgprOff);  // lane * 4
    } else if (!lds) {
        // grid (ceil(tiles/W), groups): the waves of a workgroup run one block on adjacent tiles
        e.line("\ts_lshl_b32 s%d, s2, %d", kSgprTmp, wshift);
        e.line("\ts_add_u32 s%d, s%d, s%d", kSgprTile, kSgprTmp, kSgprTile);
        e.line("\ts_mov_b32 s%d, s3", kSgprBlock);
        e.line("\ts_cmp_ge_u32 s%d, %d", kSgprTile, sp.n_tiles);
        e.line("\ts_cbranch_scc1 .Lend");
    } else {
        // grid (tiles, blocks/W): the waves of a workgroup run adjacent blocks on one tile;
        // the block list is padded, so every wave of every workgroup has a block
        e.line("\ts_lshl_b32 s%d, s3, %d", kSgprTmp, wshift);
        e.line("\ts_add_u32 s%d, s%d, s%d", kSgprBlock, kSgprTmp, kSgprTile);
        e.line("\ts_mov_b32 s%d, s2", kSgprTile);
        e.line("\tv_lshlrev_b32_e32 v%d, 4, v%d", kVgprLds, kVgprOff);  // lane * 16
    }
    // offset of this block's code, from a table kept in the text section: fetched now, needed
    // at the end of the prologue, so its latency overlaps the kernel arguments' and the lane set-up
    e.line("\ts_getpc_b64 s[%d:%d]", kSgprPc, kSgprPc + 1);
    e.line(".Lpc:");
    e.line("\ts_add_u32 s%d, s%d, .Ltable-.Lpc", kSgprPc, kSgprPc);
    e.line("\ts_addc_u32 s%d, s%d, 0", kSgprPc + 1, kSgprPc + 1);
    e.line("\ts_lshl_b32 s%d, s%d, 2", kSgprJump, kSgprBlock);
    // this block's entry and the next one's: where the code starts and how long it is
    e.line("\ts_load_dwordx2 s[%d:%d], s[%d:%d], s%d", kSgprEntry, kSgprEntry + 1, kSgprPc, kSgprPc + 1, kSgprJump);
    e.line("\ts_mul_i32 s%d, s%d, %d", kSgprTmp, kSgprTile, sp.lanes_per_tile);  // first column of the tile
    e.line("\tv_add_u32_e32 v%d, s%d, v%d", kVgprT1, kSgprTmp, kVgprOff);        // this lane's column
    e.line("\ts_mov_b32 s%d, %d", kSgprTmp2, nvc);
    e.line("\tv_cmp_gt_u32_e32 vcc, %d, v%d", sp.lanes_per_tile, kVgprOff);     // lane < lanes_per_tile
    e.line("\tv_cmp_gt_u32_e64 s[%d:%d], s%d, v%d", kSgprOwns, kSgprOwns + 1, kSgprTmp2, kVgprT1);  // column < N
    e.line("\ts_nop 4");
    e.line("\ts_and_b64 s[%d:%d], s[%d:%d], vcc", kSgprOwns, kSgprOwns + 1, kSgprOwns, kSgprOwns + 1);
    e.line("\tv_mov_b32_e32 v%d, s%d", kVgprT2, kSgprTmp);
    e.line("\ts_nop 4");
    // lanes without a column redo the tile's first column: loads stay in bounds, nothing is stored
    e.line("\tv_cndmask_b32_e64 v%d, v%d, v%d, s[%d:%d]", kVgprT1, kVgprT2, kVgprT1, kSgprOwns, kSgprOwns + 1);
    auto log2i = [](int x) { int l = 0; while ((1 << l) < x) ++l; return l; };
    e.line("\tv_lshlrev_b32_e32 v%d, %d, v%d", kVgprOut, log2i(V * osz), kVgprT1);   // byte offset of the lane's column(s) in a row of C
    e.line("\tv_lshlrev_b32_e32 v%d, %d, v%d", kVgprOff, log2i(V * esz), kVgprT1);   // ... and in a row of B / X
    // from here on only lanes that own a column are active: idle lanes fetch nothing
    e.line("\ts_mov_b64 exec, s[%d:%d]", kSgprOwns, kSgprOwns + 1);
    if (h.conv) {
        // oh = pixel / W, ow = pixel % W; then one lane mask per filter tap (r, s):
        // 0 <= oh + r - 1 < H and 0 <= ow + s - 1 < W  (Section 3.6: the padding test, made once)
        const int voh = kVgprAcc0, vow = kVgprAcc0 + 1;   // accumulators are not live yet
        const int sa0 = kSgprOffRing, sa2 = kSgprOffRing + 2, sb0 = kSgprOffRing + 4, sb2 = kSgprOffRing + 6;
        if (h.W > 1) {
            e.line("\ts_mov_b32 s%d, 0x%x", kSgprTmp, magic);
            e.line("\tv_mul_hi_u32 v%d, v%d, s%d", voh, kVgprT1, kSgprTmp);
            e.line("\ts_mov_b32 s%d, %d", kSgprTmp, h.W);
            e.line("\tv_mul_lo_u32 v%d, v%d, s%d", vow, voh, kSgprTmp);
            e.line("\tv_sub_u32_e32 v%d, v%d, v%d", vow, kVgprT1, vow);
        } else {  // one pixel per image row
            e.line("\tv_mov_b32_e32 v%d, v%d", voh, kVgprT1);
            e.line("\tv_mov_b32_e32 v%d, 0", vow);
        }
        e.line("\ts_nop 1");
        e.line("\ts_mov_b32 s%d, %d", kSgprTmp, h.H - 2);
        e.line("\ts_mov_b32 s%d, %d", kSgprTmp2, h.W - 2);
        e.line("\tv_cmp_le_i32_e64 s[%d:%d], 1, v%d", sa0, sa0 + 1, voh);             // r = 0 needs oh >= 1
        e.line("\tv_cmp_ge_i32_e64 s[%d:%d], s%d, v%d", sa2, sa2 + 1, kSgprTmp, voh);  // r = 2 needs oh <= H-2
        e.line("\tv_cmp_le_i32_e64 s[%d:%d], 1, v%d", sb0, sb0 + 1, vow);             // s = 0 needs ow >= 1
        e.line("\tv_cmp_ge_i32_e64 s[%d:%d], s%d, v%d", sb2, sb2 + 1, kSgprTmp2, vow); // s = 2 needs ow <= W-2
        e.line("\ts_nop 4");
        e.line("\ts_mov_b64 s[%d:%d], exec", kSgprFull, kSgprFull + 1);
        for (int r = 0; r < 3; ++r)
            for (int t = 0; t < 3; ++t) {
                const int m = kSgprTap0 + 2 * (r * 3 + t);
                e.line("\ts_mov_b64 s[%d:%d], exec", m, m + 1);
                if (r != 1) e.line("\ts_and_b64 s[%d:%d], s[%d:%d], s[%d:%d]", m, m + 1, m, m + 1, r == 0 ? sa0 : sa2, (r == 0 ? sa0 : sa2) + 1);
                if (t != 1) e.line("\ts_and_b64 s[%d:%d], s[%d:%d], s[%d:%d]", m, m + 1, m, m + 1, t == 0 ? sb0 : sb2, (t == 0 ? sb0 : sb2) + 1);
            }
    }
    e.line("\ts_waitcnt lgkmcnt(0)");
    if (h.conv) {
        // operand descriptor starts W+1 elements before X so that every tap displacement is
        // non-negative; lanes that would read before X are always masked off for that tap
        e.line("\ts_sub_u32 s%d, s%d, %d", kSgprB, kSgprB, (h.W + 1) * esz);
        e.line("\ts_subb_u32 s%d, s%d, 0", kSgprB + 1, kSgprB + 1);
    }
    if (images) {
        // problem z of the batch: the operand and the result advance by one image / matrix each
        const int64_t strides[2] = {(h.conv ? (int64_t)h.Cin * N : (int64_t)h.K * h.ldb) * esz, (int64_t)M * h.ldc * osz};
        const int bases[2] = {kSgprB, kSgprC};
        for (int i = 0; i < 2; ++i) {
            e.line("\ts_mov_b32 s%d, 0x%llx", kSgprTmp2, (unsigned long long)strides[i]);
            e.line("\ts_mul_hi_u32 s%d, s%d, s%d", kSgprTmp, kSgprImage, kSgprTmp2);
            e.line("\ts_mul_i32 s%d, s%d, s%d", kSgprTmp2, kSgprImage, kSgprTmp2);
            e.line("\ts_add_u32 s%d, s%d, s%d", bases[i], bases[i], kSgprTmp2);
            e.line("\ts_addc_u32 s%d, s%d, s%d", bases[i] + 1, bases[i] + 1, kSgprTmp);
        }
    }
    e.line("\ts_mov_b32 s%d, s%d", kRsrcB, kSgprB);
    e.line("\ts_and_b32 s%d, s%d, 0xffff", kRsrcB + 1, kSgprB + 1);
    e.line("\ts_mov_b32 s%d, 0x%llx", kRsrcB + 2, (unsigned long long)b_bytes);
    e.line("\ts_mov_b32 s%d, 0x%x", kRsrcB + 3, kRsrcWord3);
    e.line("\ts_mov_b32 s%d, s%d", kRsrcC, kSgprC);
    e.line("\ts_and_b32 s%d, s%d, 0xffff", kRsrcC + 1, kSgprC + 1);
    e.line("\ts_mov_b32 s%d, 0x%llx", kRsrcC + 2, (unsigned long long)c_bytes);
    e.line("\ts_mov_b32 s%d, 0x%x", kRsrcC + 3, kRsrcWord3);
    // jump to the code of this block (the table entry arrived with the kernel arguments)
    e.line("\ts_add_u32 s%d, s%d, s%d", kSgprPc, kSgprPc, kSgprEntry);
    e.line("\ts_addc_u32 s%d, s%d, 0", kSgprPc + 1, kSgprPc + 1);
    if (prefetch_lines > 0) {
        // The block's code is straight-line and read once, so inside a model, where other layers
        // have displaced it from the L2 cache, the wave would take one L2 miss after the other
        // while it runs.  Instead every lane touches `prefetch_lines` 128-byte lines of the block
        // right now, with ordinary loads whose result is never used (lanes past the end of the
        // block are masked off, so nothing outside this block's code is read): the misses overlap
        // each other and the first fetches of B.  The destination register is one no block uses.
        const int stride = 128 * prefetch_lines;
        e.line("\ts_sub_u32 s%d, s%d, s%d", kSgprEntry + 1, kSgprEntry + 1, kSgprEntry);   // bytes of code in this block
        e.line("\ts_mov_b64 exec, -1");
        e.line("\tv_mbcnt_lo_u32_b32 v%d, -1, 0", kVgprAcc0);
        e.line("\tv_mbcnt_hi_u32_b32 v%d, -1, v%d", kVgprAcc0, kVgprAcc0);              // lane id
        e.line("\tv_mul_u32_u24_e32 v%d, 0x%x, v%d", kVgprAcc0, stride, kVgprAcc0);    // first byte this lane touches
        for (int j = 0; j < prefetch_lines; ++j) {
            // lanes whose line starts inside the block stay active (the set only shrinks with j)
            e.line("\tv_cmpx_gt_i32_e32 vcc, s%d, v%d", kSgprEntry + 1, kVgprAcc0);
            e.line("\tglobal_load_dword v%d, v%d, s[%d:%d] offset:%d", kVgprT1, kVgprAcc0, kSgprPc, kSgprPc + 1, 128 * j);
            if (j + 1 < prefetch_lines) e.line("\ts_sub_u32 s%d, s%d, 128", kSgprEntry + 1, kSgprEntry + 1);
        }
        e.line("\ts_mov_b64 exec, s[%d:%d]", kSgprOwns, kSgprOwns + 1);
    }
    e.line("\ts_setpc_b64 s[%d:%d]", kSgprPc, kSgprPc + 1);
    e.line(".Lend:");
    e.line("\ts_endpgm");
    e.line("\t.p2align 2");
    e.line(".Ltable:");
    for (int g = 0; g < n_blocks; ++g) e.line("\t.long .Lg%d-.Ltable", g);
    e.line("\t.long .Lfunc_end-.Ltable");   // end of the last block

}

// Stage 4b, emission of what follows the blocks: the kernel descriptor and the code object metadata.
static void emit_kernel_descriptor(Gen &gen, const Shape &sh) {
    const HostPlan &h = gen.h;
    SpecPlan &sp = gen.sp;
    Emitter &e = gen.e;
    const char *sym = sp.symbol.c_str();
    const bool images = h.batch > 1;
    const int n_vgpr = gen.n_vgpr, W = sh.W;
    e.line(".Lfunc_end:");
    e.line("\t.size\t%s, .Lfunc_end-%s", sym, sym);
    e.line("\t.section\t.rodata,\"a\",@progbits");
    e.line("\t.p2align\t6, 0x0");
    e.line("\t.amdhsa_kernel %s", sym);
    e.line("\t\t.amdhsa_group_segment_fixed_size %d", gen.lds_bytes);
    e.line("\t\t.amdhsa_private_segment_fixed_size 0");
    e.line("\t\t.amdhsa_kernarg_size 16");
    e.line("\t\t.amdhsa_user_sgpr_count 2");
    e.line("\t\t.amdhsa_user_sgpr_dispatch_ptr 0");
    e.line("\t\t.amdhsa_user_sgpr_queue_ptr 0");
    e.line("\t\t.amdhsa_user_sgpr_kernarg_segment_ptr 1");
    e.line("\t\t.amdhsa_user_sgpr_dispatch_id 0");
    e.line("\t\t.amdhsa_user_sgpr_kernarg_preload_length 0");
    e.line("\t\t.amdhsa_user_sgpr_kernarg_preload_offset 0");
    e.line("\t\t.amdhsa_user_sgpr_private_segment_size 0");
    e.line("\t\t.amdhsa_uses_dynamic_stack 0");
    e.line("\t\t.amdhsa_enable_private_segment 0");
    e.line("\t\t.amdhsa_system_sgpr_workgroup_id_x 1");
    e.line("\t\t.amdhsa_system_sgpr_workgroup_id_y 1");
    e.line("\t\t.amdhsa_system_sgpr_workgroup_id_z %d", images ? 1 : 0);
    e.line("\t\t.amdhsa_system_sgpr_workgroup_info 0");
    e.line("\t\t.amdhsa_system_vgpr_workitem_id 0");
    e.line("\t\t.amdhsa_next_free_vgpr %d", n_vgpr);
    e.line("\t\t.amdhsa_next_free_sgpr %d", kNextFreeSgpr);
    e.line("\t\t.amdhsa_accum_offset %d", (n_vgpr + 3) / 4 * 4);
    e.line("\t\t.amdhsa_reserve_vcc 1");
    e.line("\t\t.amdhsa_float_round_mode_32 0");
    e.line("\t\t.amdhsa_float_round_mode_16_64 0");
    e.line("\t\t.amdhsa_float_denorm_mode_32 3");
    e.line("\t\t.amdhsa_float_denorm_mode_16_64 3");
    e.line("\t\t.amdhsa_dx10_clamp 1");
    e.line("\t\t.amdhsa_ieee_mode 1");
    e.line("\t\t.amdhsa_fp16_overflow 0");
    e.line("\t\t.amdhsa_tg_split 0");
    e.line("\t.end_amdhsa_kernel");
    e.line("\t.text");
    e.line("\t.amdgpu_metadata");
    e.line("---");
    e.line("amdhsa.kernels:");
    e.line("  - .agpr_count:     0");
    e.line("    .args:");
    e.line("      - .actual_access:  read_only");
    e.line("        .address_space:  global");
    e.line("        .offset:         0");
    e.line("        .size:           8");
    e.line("        .value_kind:     global_buffer");
    e.line("      - .actual_access:  write_only");
    e.line("        .address_space:  global");
    e.line("        .offset:         8");
    e.line("        .size:           8");
    e.line("        .value_kind:     global_buffer");
    e.line("    .group_segment_fixed_size: %d", gen.lds_bytes);
    e.line("    .kernarg_segment_align: 8");
    e.line("    .kernarg_segment_size: 16");
    e.line("    .max_flat_workgroup_size: %d", W * kWave);
    e.line("    .name:           %s", sym);
    e.line("    .private_segment_fixed_size: 0");
    e.line("    .sgpr_count:     %d", kNextFreeSgpr + 6);
    e.line("    .sgpr_spill_count: 0");
    e.line("    .symbol:         %s.kd", sym);
    e.line("    .uniform_work_group_size: 1");
    e.line("    .uses_dynamic_stack: false");
    e.line("    .vgpr_count:     %d", n_vgpr);
    e.line("    .vgpr_spill_count: 0");
    e.line("    .wavefront_size: 64");
    e.line("amdhsa.target:   amdgcn-amd-amdhsa--gfx950");
    e.line("amdhsa.version:");
    e.line("  - 1");
    e.line("  - 2");
    e.line("...");
    e.line("");
    e.line("\t.end_amdgpu_metadata");

}

int build_spec_plan(HostPlan &h, const sparsert_options &opt, std::string &err) {
    SpecPlan &sp = h.spec;
    Shape sh;
    if (int rc = choose_launch_shape(h, opt, sp, sh, err)) return rc;
    std::vector<std::vector<int32_t>> members;
    form_blocks(h, opt, sp, members);
    Gen gen(h, sp);
    Extents ex;
    if (int rc = plan_registers(h, sp, sh, members, gen, ex, err)) return rc;
    // The blocks are emitted first: the prologue wants to know how long the longest one is.
    Emitter &e = gen.e;
    sp.group_columns.assign(sp.n_blocks, 0);
    int64_t longest = 0;   // instructions of the longest block
    for (int g = 0; g < sp.n_blocks; ++g) {
        const int64_t before = e.lines;
        e.line("\t.p2align 2");
        e.line(".Lg%d:", g);
        sp.group_columns[g] = sh.lds ? gen.block_lds(members[g], g % sh.W, sh.W)
                                     : gen.block_direct(members[g / sh.KS], g % sh.KS, sh.KS);
        longest = std::max(longest, e.lines - before);
    }
    emit_kernel_descriptor(gen, sh);
    // an instruction is at most 8 bytes; 64 lanes touch one 128-byte line each per prefetch
    // instruction, at most 32 of them (their offsets must fit the load's immediate field)
    const int prefetch_lines = !opt.spec_prefetch ? 0 : (int)std::min<int64_t>(32, (longest * 8 + 64 * 128 - 1) / (64 * 128));
    sp.prefetch_lines = prefetch_lines;
    Emitter head;
    emit_prologue(gen, head, sh, ex, prefetch_lines);
    e.s.insert(0, head.s);

    if (const char *dump = getenv("SPARSERT_DUMP_ASM")) {
        if (FILE *f = fopen(dump, "w")) { fwrite(e.s.data(), 1, e.s.size(), f); fclose(f); }
    }
    sp.asm_bytes = (int64_t)e.s.size();
    if (int rc = assemble(e.s, sp.code, err)) return rc;
    return SPARSERT_OK;
}

}  // namespace sparsert
