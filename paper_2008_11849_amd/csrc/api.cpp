// extern "C" boundary: argument checks, error strings, plan export.
#include <cstring>
#include <exception>
#include <new>
#include <string>

#include "plan.h"

namespace {
thread_local std::string g_err;
int fail(int code, const std::string &msg) { g_err = msg; return code; }
}  // namespace

namespace sparsert {
int set_error(int code, const std::string &msg) { return fail(code, msg); }
}  // namespace sparsert

extern "C" {

int sparsert_inspect(const int32_t *row_ptr, const int32_t *col_idx, const void *vals,
                     int32_t M, int32_t K, int32_t N,
                     const sparsert_options *opt, sparsert_plan **out) {
    if (!out) return fail(SPARSERT_EINVAL, "out is NULL");
    *out = nullptr;
    sparsert_options o;
    if (opt) o = *opt; else std::memset(&o, 0, sizeof(o));
    sparsert_plan *plan = new (std::nothrow) sparsert_plan();
    if (!plan) return fail(SPARSERT_ENOMEM, "out of host memory");
    std::string err;
    int rc;
    try {   // no exception may cross the C boundary
        rc = sparsert::build_host_plan(row_ptr, col_idx, vals, M, K, N, o, plan->host, err);
        if (rc == SPARSERT_OK && plan->host.kernel == SPARSERT_KERNEL_SPEC) {
            rc = sparsert::build_spec_plan(plan->host, o, err);
            if ((rc == SPARSERT_EUNSUPPORTED || rc == SPARSERT_ECOMPILE) && plan->host.kernel_auto) {
                // the inspector's own choice did not work out for this problem (a shape the
                // generator does not cover, an assembler failure): the row-walk kernel always does
                plan->host.spec = sparsert::SpecPlan();
                plan->host.kernel = SPARSERT_KERNEL_ROWS;
                rc = SPARSERT_OK;
                err.clear();
            }
        }
        if (rc == SPARSERT_OK && !o.host_only) {
            rc = sparsert::upload_plan(plan->host, plan->dev, err);
            plan->on_device = (rc == SPARSERT_OK);
        }
    } catch (const std::bad_alloc &) {
        rc = SPARSERT_ENOMEM; err = "out of host memory";
    } catch (const std::exception &ex) {
        rc = SPARSERT_EINVAL; err = std::string("internal error: ") + ex.what();
    }
    if (rc != SPARSERT_OK) {
        sparsert::free_device_plan(plan->dev);
        delete plan;
        return fail(rc, err);
    }
    *out = plan;
    return SPARSERT_OK;
}

static int check_exec(const sparsert_plan *plan, const void *in, void *outp, bool conv) {
    if (!plan) return fail(SPARSERT_EINVAL, "plan is NULL");
    if (!in || !outp) return fail(SPARSERT_EINVAL, "device pointer is NULL");
    if (((uintptr_t)in | (uintptr_t)outp) & 15u) return fail(SPARSERT_EINVAL, "device pointers must be 16-byte aligned");
    if (!plan->on_device) return fail(SPARSERT_EINVAL, "plan was made with host_only and cannot be executed");
    if ((plan->host.conv != 0) != conv)
        return fail(SPARSERT_EINVAL, conv ? "plan is not a convolution plan" : "plan is a convolution plan; use sparsert_conv3x3");
    if (!sparsert::on_plan_device(plan->dev))
        return fail(SPARSERT_EINVAL, "the plan's arrays live on another HIP device than the current one");
    return SPARSERT_OK;
}

int sparsert_spmm(const sparsert_plan *plan, const void *B_dev, void *C_dev, void *stream) {
    if (int rc = check_exec(plan, B_dev, C_dev, false)) return rc;
    std::string err;
    int rc = plan->host.kernel == SPARSERT_KERNEL_SPEC
                 ? sparsert::launch_spec(plan->host, plan->dev, B_dev, C_dev, stream, err)
                 : sparsert::launch_rows(plan->host, plan->dev, B_dev, C_dev, stream, err);
    return rc == SPARSERT_OK ? rc : fail(rc, err);
}

int sparsert_conv3x3(const sparsert_plan *plan, const void *X_dev, void *Y_dev, void *stream) {
    if (int rc = check_exec(plan, X_dev, Y_dev, true)) return rc;
    std::string err;
    int rc = plan->host.kernel == SPARSERT_KERNEL_SPEC
                 ? sparsert::launch_spec(plan->host, plan->dev, X_dev, Y_dev, stream, err)
                 : sparsert::launch_rows(plan->host, plan->dev, X_dev, Y_dev, stream, err);
    return rc == SPARSERT_OK ? rc : fail(rc, err);
}

int sparsert_plan_export(const sparsert_plan *plan, int32_t field, void *buf, size_t cap, size_t *need) {
    if (!plan) return fail(SPARSERT_EINVAL, "plan is NULL");
    const sparsert::HostPlan &h = plan->host;
    int32_t info[SPARSERT_INFO_COUNT] = {0};
    const void *src = nullptr;
    size_t bytes = 0;
    std::string name;
    auto vec32 = [&](const std::vector<int32_t> &v) { src = v.data(); bytes = v.size() * 4; };
    switch (field) {
    case SPARSERT_FIELD_INFO:
        info[SPARSERT_INFO_M] = h.M; info[SPARSERT_INFO_K] = h.K; info[SPARSERT_INFO_N] = h.N;
        info[SPARSERT_INFO_NNZ] = h.nnz; info[SPARSERT_INFO_DTYPE] = h.dtype;
        info[SPARSERT_INFO_CONV] = h.conv; info[SPARSERT_INFO_CIN] = h.Cin;
        info[SPARSERT_INFO_H] = h.H; info[SPARSERT_INFO_W] = h.W;
        info[SPARSERT_INFO_KERNEL] = h.kernel; info[SPARSERT_INFO_VEC] = h.vec;
        info[SPARSERT_INFO_LANES_PER_TILE] = h.lanes_per_tile;
        info[SPARSERT_INFO_N_TILES] = h.n_tiles; info[SPARSERT_INFO_GY] = h.gy;
        info[SPARSERT_INFO_SPLIT_THRESHOLD] = h.split_threshold;
        info[SPARSERT_INFO_N_SPLIT] = h.n_split; info[SPARSERT_INFO_N_WG_ROWS] = h.n_wg_rows;
        info[SPARSERT_INFO_N_BINS] = (int32_t)(h.bins.size() / 4);
        info[SPARSERT_INFO_SPEC_ROWS] = h.spec.rows_per_group;
        info[SPARSERT_INFO_SPEC_GROUPS] = h.spec.n_groups;
        info[SPARSERT_INFO_SPEC_DEPTH] = h.spec.depth;
        info[SPARSERT_INFO_SPEC_CODE_BYTES] = (int32_t)h.spec.code.size();
        info[SPARSERT_INFO_SPEC_TILES] = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.tiles_per_wg : 0;
        info[SPARSERT_INFO_SPEC_MODE] = h.spec.mode;
        info[SPARSERT_INFO_SPEC_LDS_BYTES] = h.spec.lds_bytes;
        info[SPARSERT_INFO_SPEC_KSPLIT] = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.ksplit : 0;
        info[SPARSERT_INFO_NATURAL_ORDER] = h.natural_order;
        info[SPARSERT_INFO_BATCH] = h.batch;
        info[SPARSERT_INFO_SPEC_VEC] = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.vec : 0;
        info[SPARSERT_INFO_LDB] = h.ldb; info[SPARSERT_INFO_LDC] = h.ldc;
        info[SPARSERT_INFO_SPEC_PREFETCH] = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.prefetch_lines : 0;
        info[SPARSERT_INFO_SPEC_LANES] = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.lanes_per_tile : 0;
        info[SPARSERT_INFO_SPEC_SWIZZLE] = h.kernel == SPARSERT_KERNEL_SPEC ? h.spec.swizzle : 0;
        src = info; bytes = sizeof(info);
        break;
    case SPARSERT_FIELD_ROW_NNZ: vec32(h.row_nnz); break;
    case SPARSERT_FIELD_HIST: vec32(h.hist); break;
    case SPARSERT_FIELD_PERM: vec32(h.perm); break;
    case SPARSERT_FIELD_INV_PERM: vec32(h.inv_perm); break;
    case SPARSERT_FIELD_P_ROW_PTR: vec32(h.p_row_ptr); break;
    case SPARSERT_FIELD_P_COL_IDX: vec32(h.p_col_idx); break;
    case SPARSERT_FIELD_P_VALS: src = h.p_vals.data(); bytes = h.p_vals.size(); break;
    case SPARSERT_FIELD_BINS: vec32(h.bins); break;
    case SPARSERT_FIELD_STREAM: src = h.stream.data(); bytes = h.stream.size() * 4; break;
    case SPARSERT_FIELD_CONV_SEG: vec32(h.conv_seg); break;
    case SPARSERT_FIELD_SEGMENTS: vec32(h.segments); break;
    case SPARSERT_FIELD_SPEC_GROUPS: vec32(h.spec.group_of_slot); break;
    case SPARSERT_FIELD_SPEC_COLUMNS: vec32(h.spec.group_columns); break;
    case SPARSERT_FIELD_SPEC_CODE: src = h.spec.code.data(); bytes = h.spec.code.size(); break;
    case SPARSERT_FIELD_KERNEL_NAME:
        if (h.kernel == SPARSERT_KERNEL_SPEC) {
            name = h.spec.symbol;
        } else if (h.dtype == SPARSERT_F16) {
            // the profiler's demangler does not know the half type and shows the symbol as it is
            name = "_ZN8sparsert11rows_kernelIDF16_Li" + std::to_string(h.vec) + "ELb" + (h.conv ? "1" : "0") + "EEEvNS_8RowsArgsE";
        } else {
            name = std::string("void sparsert::rows_kernel<") + (h.dtype == SPARSERT_I8 ? "signed char" : "float") + ", " +
                   std::to_string(h.vec) + ", " + (h.conv ? "true" : "false") + ">(sparsert::RowsArgs)";
        }
        src = name.data(); bytes = name.size();
        break;
    default: return fail(SPARSERT_EINVAL, "unknown plan field");
    }
    if (need) *need = bytes;
    if (!buf) return SPARSERT_OK;
    if (cap < bytes) return fail(SPARSERT_EINVAL, "export buffer too small");
    if (bytes) std::memcpy(buf, src, bytes);
    return SPARSERT_OK;
}

int sparsert_compare_outputs(const sparsert_plan *plan, const void *a_dev, const void *b_dev, void *result_dev, void *stream) {
    if (!plan) return fail(SPARSERT_EINVAL, "plan is NULL");
    if (!a_dev || !b_dev || !result_dev) return fail(SPARSERT_EINVAL, "device pointer is NULL");
    if (((uintptr_t)a_dev | (uintptr_t)b_dev | (uintptr_t)result_dev) & 15u) return fail(SPARSERT_EINVAL, "device pointers must be 16-byte aligned");
    if (!plan->on_device) return fail(SPARSERT_EINVAL, "plan was made with host_only");
    if (!sparsert::on_plan_device(plan->dev)) return fail(SPARSERT_EINVAL, "the plan's arrays live on another HIP device than the current one");
    std::string err;
    int rc = sparsert::compare_with_own_partials(plan->host, a_dev, b_dev, static_cast<uint32_t *>(result_dev), stream, err);
    return rc == SPARSERT_OK ? rc : fail(rc, err);
}

int sparsert_compare_outputs_static(const sparsert_plan *plan, const void *a_dev, const void *b_dev, void *result_dev, void *stream) {
    if (!plan) return fail(SPARSERT_EINVAL, "plan is NULL");
    if (!a_dev || !b_dev || !result_dev) return fail(SPARSERT_EINVAL, "device pointer is NULL");
    if (((uintptr_t)a_dev | (uintptr_t)b_dev | (uintptr_t)result_dev) & 15u) return fail(SPARSERT_EINVAL, "device pointers must be 16-byte aligned");
    if (!plan->on_device) return fail(SPARSERT_EINVAL, "plan was made with host_only");
    if (!sparsert::on_plan_device(plan->dev)) return fail(SPARSERT_EINVAL, "the plan's arrays live on another HIP device than the current one");
    const sparsert::HostPlan &h = plan->host;
    if ((int64_t)h.batch * h.M * h.N > sparsert::static_compare_max_elements())
        return fail(SPARSERT_EUNSUPPORTED, "output has more than 33554432 elements: beyond the static partials array, use sparsert_compare_outputs");
    std::string err;
    uint32_t *partials = nullptr;
    int rc = sparsert::static_compare_scratch(&partials, err);
    if (rc == SPARSERT_OK) rc = sparsert::launch_compare(h, a_dev, b_dev, partials, static_cast<uint32_t *>(result_dev), stream, err);
    return rc == SPARSERT_OK ? rc : fail(rc, err);
}

void sparsert_plan_destroy(sparsert_plan *plan) {
    if (!plan) return;
    sparsert::free_device_plan(plan->dev);
    delete plan;
}

const char *sparsert_last_error(void) { return g_err.c_str(); }

int32_t sparsert_version(void) { return 200; }

}  // extern "C"
