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
//   grid  = (ceil(n_tiles/4), G);  workgroup = 4 waves = 4 adjacent column tiles
//   wave  = one row group g (<= R rows, chosen by the inspector for nonzero balance,
//           Section 3.4) x one column tile (lanes own one column of C each)
//   code  = per group, for each column k that has a nonzero in the group, ascending:
//             buffer_load  b <- B[k, tile columns]        (issued D columns ahead)
//             v_fmac_f32   acc[row] += literal(A[row,k]) * b     for every nonzero (row,k)
//           then one store per row.  No loops, no index loads, no barriers.
// All addresses are "descriptor base + row offset literal + lane column offset" with the
// column offset clamped to the tile, so every access is in bounds by construction.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <dlfcn.h>
#include <map>
#include <mutex>

#include "plan.h"

namespace sparsert {

namespace {

// ---------------------------------------------------------------- code object manager
// Loaded at run time so the library itself has no link-time dependency on it.
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
#undef COMGR_SYM
        c.ok = all;
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
    if (!c.ok) { err = "code object manager (libamd_comgr) is not available"; return SPARSERT_ECOMPILE; }
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
    char buf[256];
    void line(const char *fmt, ...) __attribute__((format(printf, 2, 3))) {
        va_list ap;
        va_start(ap, fmt);
        int n = vsnprintf(buf, sizeof(buf), fmt, ap);
        va_end(ap);
        s.append(buf, (size_t)n);
        s.push_back('\n');
    }
};

// Fixed register plan of the generated kernel.
constexpr int kSgprB = 4, kSgprC = 6;          // kernarg pointers
constexpr int kRsrcB = 8, kRsrcC = 12;         // buffer descriptors (4 SGPRs each)
constexpr int kSgprTile = 16, kSgprBlock = 17, kSgprPc = 18, kSgprTmp = 20, kSgprTmp2 = 21;
constexpr int kSgprOwns = 22;                  // s[22:23] lanes that own a column
constexpr int kSgprOffRing = 24, kOffRing = 8; // s[24:31] row-offset literals in flight
constexpr int kNextFreeSgpr = 32;
constexpr int kVgprOff = 0, kVgprT1 = 1, kVgprT2 = 2, kVgprAcc0 = 4;
constexpr uint32_t kRsrcWord3 = 0x00020000u;   // raw 32-bit buffer, gfx9 family

}  // namespace

int build_spec_plan(HostPlan &h, const sparsert_options &opt, std::string &err) {
    SpecPlan &sp = h.spec;
    if (h.conv) { err = "the specialised executor does not cover convolution plans yet"; return SPARSERT_EUNSUPPORTED; }
    if (h.dtype != SPARSERT_F32) { err = "the specialised executor is fp32 only"; return SPARSERT_EUNSUPPORTED; }
    const int32_t M = h.M, N = h.N;
    // Column tiling with one column per lane, balanced tails (same rule as the row-walk plan at V = 1).
    sp.n_tiles = (N + kWave - 1) / kWave;
    sp.lanes_per_tile = (N + sp.n_tiles - 1) / sp.n_tiles;
    // Rows per group: enough rows that a loaded B row is reused, few enough that the chip is
    // filled: R1 fills 1024 SIMDs with one wave each, R2 gives a wave about 400 multiply-adds.
    int R = opt.spec_rows;
    if (R == 0) {
        const int64_t r1 = (int64_t)M * sp.n_tiles / 1024;
        const int64_t avg = std::max<int64_t>(1, h.nnz / M);
        const int64_t r2 = (400 + avg - 1) / avg;
        R = (int)std::min<int64_t>(96, std::max<int64_t>(4, std::max(r1, r2)));
    }
    if (R < 1 || R > 200) { err = "spec_rows must be in 1..200"; return SPARSERT_EINVAL; }
    R = std::min(R, M);
    sp.rows_per_group = R;
    sp.n_groups = (M + R - 1) / R;
    sp.depth = opt.spec_depth ? opt.spec_depth : 16;
    sp.tiles_per_wg = opt.spec_tiles ? opt.spec_tiles : 4;
    sp.share_rows = getenv("SPARSERT_SPEC_SHARE") ? atoi(getenv("SPARSERT_SPEC_SHARE")) : 0;
    int tpw_shift = 0;
    while ((1 << tpw_shift) < sp.tiles_per_wg) ++tpw_shift;
    // Block-level balance (Section 3.4, strategy b): slots are in descending-nnz order; deal
    // them to the groups in serpentine order so every group gets nearly the same nonzero count.
    const int G = sp.n_groups;
    sp.group_of_slot.resize(M);
    std::vector<std::vector<int32_t>> members(G);
    for (int32_t i = 0; i < M; ++i) {
        const int32_t round = i / G, pos = i % G;
        const int32_t g = (round & 1) ? G - 1 - pos : pos;
        sp.group_of_slot[i] = g;
        members[g].push_back(i);
    }

    Emitter e;
    const int64_t b_bytes = (int64_t)h.K * N * 4, c_bytes = (int64_t)M * N * 4;
    int max_rows = 0;
    for (auto &m : members) max_rows = std::max<int>(max_rows, (int)m.size());
    const int D = sp.depth;
    const int vgpr_b0 = kVgprAcc0 + max_rows;
    const int n_vgpr = vgpr_b0 + D;
    if (n_vgpr > 256) { err = "spec_rows too large for the register file"; return SPARSERT_EINVAL; }

    e.line("\t.amdgcn_target \"amdgcn-amd-amdhsa--gfx950\"");
    e.line("\t.amdhsa_code_object_version 6");
    e.line("\t.text");
    e.line("\t.protected\tsparsert_spec");
    e.line("\t.globl\tsparsert_spec");
    e.line("\t.p2align\t8");
    e.line("\t.type\tsparsert_spec,@function");
    e.line("sparsert_spec:");
    // s[0:1] kernarg, s2 = workgroup id x (column tile quad), s3 = workgroup id y (row group), v0 = thread id
    e.line("\ts_load_dwordx4 s[%d:%d], s[0:1], 0x0", kSgprB, kSgprC + 1);
    e.line("\tv_lshrrev_b32_e32 v%d, 6, v0", kVgprT1);
    e.line("\tv_and_b32_e32 v%d, 63, v0", kVgprOff);
    e.line("\ts_nop 1");
    e.line("\tv_readfirstlane_b32 s%d, v%d", kSgprTile, kVgprT1);
    e.line("\ts_nop 4");
    if (!sp.share_rows) {
        // the waves of a workgroup run the same code block on adjacent column tiles
        e.line("\ts_lshl_b32 s%d, s2, %d", kSgprTmp, tpw_shift);
        e.line("\ts_add_u32 s%d, s%d, s%d", kSgprTile, kSgprTmp, kSgprTile);  // tile = tiles_per_wg*wg + wave
        e.line("\ts_mov_b32 s%d, s3", kSgprBlock);
    } else {
        // the waves of a workgroup run adjacent code blocks on the same column tile, so the B
        // rows one wave pulls into the L1 are hits for the others
        e.line("\ts_lshl_b32 s%d, s3, %d", kSgprTmp, tpw_shift);
        e.line("\ts_add_u32 s%d, s%d, s%d", kSgprBlock, kSgprTmp, kSgprTile);  // block = waves*wg + wave
        e.line("\ts_mov_b32 s%d, s2", kSgprTile);
        e.line("\ts_cmp_ge_u32 s%d, %d", kSgprBlock, G);
        e.line("\ts_cbranch_scc1 .Lend");
    }
    e.line("\ts_cmp_ge_u32 s%d, %d", kSgprTile, sp.n_tiles);
    e.line("\ts_cbranch_scc1 .Lend");
    e.line("\ts_mul_i32 s%d, s%d, %d", kSgprTmp, kSgprTile, sp.lanes_per_tile);  // first column of the tile
    e.line("\tv_add_u32_e32 v%d, s%d, v%d", kVgprT1, kSgprTmp, kVgprOff);        // this lane's column
    e.line("\ts_mov_b32 s%d, %d", kSgprTmp2, N);
    e.line("\tv_cmp_gt_u32_e32 vcc, %d, v%d", sp.lanes_per_tile, kVgprOff);     // lane < lanes_per_tile
    e.line("\tv_cmp_gt_u32_e64 s[%d:%d], s%d, v%d", kSgprOwns, kSgprOwns + 1, kSgprTmp2, kVgprT1);  // column < N
    e.line("\ts_nop 4");
    e.line("\ts_and_b64 s[%d:%d], s[%d:%d], vcc", kSgprOwns, kSgprOwns + 1, kSgprOwns, kSgprOwns + 1);
    e.line("\tv_mov_b32_e32 v%d, s%d", kVgprT2, kSgprTmp);
    e.line("\ts_nop 4");
    // lanes without a column redo the tile's first column: loads stay in bounds, nothing is stored
    e.line("\tv_cndmask_b32_e64 v%d, v%d, v%d, s[%d:%d]", kVgprT1, kVgprT2, kVgprT1, kSgprOwns, kSgprOwns + 1);
    e.line("\tv_lshlrev_b32_e32 v%d, 2, v%d", kVgprOff, kVgprT1);  // byte offset of the column inside a row
    e.line("\ts_waitcnt lgkmcnt(0)");
    e.line("\ts_mov_b32 s%d, s%d", kRsrcB, kSgprB);
    e.line("\ts_and_b32 s%d, s%d, 0xffff", kRsrcB + 1, kSgprB + 1);
    e.line("\ts_mov_b32 s%d, 0x%llx", kRsrcB + 2, (unsigned long long)b_bytes);
    e.line("\ts_mov_b32 s%d, 0x%x", kRsrcB + 3, kRsrcWord3);
    e.line("\ts_mov_b32 s%d, s%d", kRsrcC, kSgprC);
    e.line("\ts_and_b32 s%d, s%d, 0xffff", kRsrcC + 1, kSgprC + 1);
    e.line("\ts_mov_b32 s%d, 0x%llx", kRsrcC + 2, (unsigned long long)c_bytes);
    e.line("\ts_mov_b32 s%d, 0x%x", kRsrcC + 3, kRsrcWord3);
    // jump to the code of this row group through a table of offsets kept in the text section
    e.line("\ts_getpc_b64 s[%d:%d]", kSgprPc, kSgprPc + 1);
    e.line(".Lpc:");
    e.line("\ts_add_u32 s%d, s%d, .Ltable-.Lpc", kSgprPc, kSgprPc);
    e.line("\ts_addc_u32 s%d, s%d, 0", kSgprPc + 1, kSgprPc + 1);
    e.line("\ts_lshl_b32 s%d, s%d, 2", kSgprTmp, kSgprBlock);
    e.line("\ts_load_dword s%d, s[%d:%d], s%d", kSgprTmp2, kSgprPc, kSgprPc + 1, kSgprTmp);
    e.line("\ts_waitcnt lgkmcnt(0)");
    e.line("\ts_add_u32 s%d, s%d, s%d", kSgprPc, kSgprPc, kSgprTmp2);
    e.line("\ts_addc_u32 s%d, s%d, 0", kSgprPc + 1, kSgprPc + 1);
    e.line("\ts_setpc_b64 s[%d:%d]", kSgprPc, kSgprPc + 1);
    e.line(".Lend:");
    e.line("\ts_endpgm");
    e.line("\t.p2align 2");
    e.line(".Ltable:");
    for (int g = 0; g < G; ++g) e.line("\t.long .Lg%d-.Ltable", g);

    // One straight-line block per row group.
    struct Term { int acc; uint32_t bits; };
    sp.group_columns.assign(G, 0);
    for (int g = 0; g < G; ++g) {
        const std::vector<int32_t> &rows = members[g];
        std::map<int32_t, std::vector<Term>> cols;  // column -> nonzeros of this group
        for (size_t i = 0; i < rows.size(); ++i) {
            const int32_t slot = rows[i];
            for (int32_t p = h.p_row_ptr[slot]; p < h.p_row_ptr[slot + 1]; ++p)
                cols[h.p_col_idx[p]].push_back({(int)i, h.stream[2 * (size_t)p + 1]});
        }
        std::vector<int32_t> order;
        order.reserve(cols.size());
        for (auto &kv : cols) order.push_back(kv.first);
        const int nc = (int)order.size();
        sp.group_columns[g] = nc;
        e.line("\t.p2align 2");
        e.line(".Lg%d:", g);
        for (size_t i = 0; i < rows.size(); ++i) e.line("\tv_mov_b32_e32 v%d, 0", kVgprAcc0 + (int)i);
        const int xp = getenv("SPARSERT_SPEC_XP") ? atoi(getenv("SPARSERT_SPEC_XP")) : 0;  // timing experiments only
        auto issue_load = [&](int j) {
            if ((xp & 2) && j >= D) return;
            const int sreg = kSgprOffRing + (j % kOffRing);
            e.line("\ts_mov_b32 s%d, 0x%llx", sreg, (unsigned long long)((int64_t)order[j] * N * 4));
            e.line("\tbuffer_load_dword v%d, v%d, s[%d:%d], s%d offen", vgpr_b0 + (j % D), kVgprOff,
                   kRsrcB, kRsrcB + 3, sreg);
        };
        for (int j = 0; j < std::min(D, nc); ++j) issue_load(j);
        for (int j = 0; j < nc; ++j) {
            // loads issued so far: columns [0, min(nc, j + D)); those after column j may stay in flight
            if (!(xp & 2)) e.line("\ts_waitcnt vmcnt(%d)", std::min(nc, j + D) - 1 - j);
            else if (j == 0) e.line("\ts_waitcnt vmcnt(0)");
            for (const Term &t : cols[order[j]]) {
                if (xp & 1) e.line("\tv_fmac_f32_e32 v%d, v%d, v%d", kVgprAcc0 + t.acc, vgpr_b0 + (j % D), vgpr_b0 + (j % D));
                else e.line("\tv_fmac_f32_e32 v%d, 0x%08x, v%d", kVgprAcc0 + t.acc, t.bits, vgpr_b0 + (j % D));
            }
            if (j + D < nc) issue_load(j + D);
        }
        e.line("\ts_mov_b64 exec, s[%d:%d]", kSgprOwns, kSgprOwns + 1);
        for (size_t i = 0; i < rows.size(); ++i) {
            const int sreg = kSgprOffRing + ((int)i % kOffRing);
            e.line("\ts_mov_b32 s%d, 0x%llx", sreg, (unsigned long long)((int64_t)h.perm[rows[i]] * N * 4));
            e.line("\tbuffer_store_dword v%d, v%d, s[%d:%d], s%d offen", kVgprAcc0 + (int)i, kVgprOff,
                   kRsrcC, kRsrcC + 3, sreg);
        }
        e.line("\ts_endpgm");
    }
    e.line(".Lfunc_end:");
    e.line("\t.size\tsparsert_spec, .Lfunc_end-sparsert_spec");
    e.line("\t.section\t.rodata,\"a\",@progbits");
    e.line("\t.p2align\t6, 0x0");
    e.line("\t.amdhsa_kernel sparsert_spec");
    e.line("\t\t.amdhsa_group_segment_fixed_size 0");
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
    e.line("\t\t.amdhsa_system_sgpr_workgroup_id_z 0");
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
    e.line("    .group_segment_fixed_size: 0");
    e.line("    .kernarg_segment_align: 8");
    e.line("    .kernarg_segment_size: 16");
    e.line("    .max_flat_workgroup_size: %d", sp.tiles_per_wg * kWave);
    e.line("    .name:           sparsert_spec");
    e.line("    .private_segment_fixed_size: 0");
    e.line("    .sgpr_count:     %d", kNextFreeSgpr + 6);
    e.line("    .sgpr_spill_count: 0");
    e.line("    .symbol:         sparsert_spec.kd");
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

    if (const char *dump = getenv("SPARSERT_DUMP_ASM")) {
        if (FILE *f = fopen(dump, "w")) { fwrite(e.s.data(), 1, e.s.size(), f); fclose(f); }
    }
    sp.asm_bytes = (int64_t)e.s.size();
    if (int rc = assemble(e.s, sp.code, err)) return rc;
    return SPARSERT_OK;
}

}  // namespace sparsert
