// Internal representation of a plan.  Host arrays mirror exactly what
// sparsert_plan_export hands out; device arrays are what the kernels read.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/sparsert.h"

namespace sparsert {

constexpr int kWave = 64;       // lanes per wavefront on gfx950
constexpr int kGy = 4;          // waves per workgroup (one per SIMD of a CU)
constexpr int kBins = 33;       // bin(0)=0, bin(x)=1+floor(log2 x), x < 2^31
constexpr int kFullTasks = 2048;  // wave tasks wanted before widening per-lane vectors
constexpr int32_t kAutoSpecNnz = 4 << 20;   // SPARSERT_KERNEL_AUTO generates code up to this many nonzeros (about 4 s of assembling per million)

// Per-matrix generated kernel (kernel == SPARSERT_KERNEL_SPEC).
// IEEE binary16 -> binary32, exact for every input (subnormals, inf, NaN payload kept).
inline uint32_t half_bits_to_float_bits(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1fu;
    uint32_t man = h & 0x3ffu;
    if (exp == 0x1fu) return sign | 0x7f800000u | (man << 13);
    if (exp == 0) {
        if (man == 0) return sign;
        int shift = 0;
        while (!(man & 0x400u)) { man <<= 1; ++shift; }
        man &= 0x3ffu;
        exp = 1 - shift;
        return sign | ((exp + 112u) << 23) | (man << 13);
    }
    return sign | ((exp + 112u) << 23) | (man << 13);
}

struct SpecPlan {
    int32_t rows_per_group = 0, n_groups = 0, depth = 0, n_tiles = 0, lanes_per_tile = 0;
    int32_t tiles_per_wg = 4;   // waves per workgroup
    std::string symbol;         // kernel symbol inside the code object
    int32_t swizzle = 0;        // blocks formed by column-pattern similarity
    int32_t vec = 1;            // columns per lane (2 halves or 4 int8 packed in a dword)
    int32_t mode = 0;           // sparsert_spec_mode
    int32_t n_blocks = 0;       // code blocks (n_groups, padded to a multiple of the waves in LDS mode)
    int32_t lds_bytes = 0;
    int32_t ksplit = 1;         // DIRECT: waves of a workgroup that split the K range of one block
    int32_t prefetch_lines = 0; // 128-byte lines of its block's code every lane touches before the block runs
    int64_t asm_bytes = 0;
    std::vector<int32_t> group_of_slot;   // [M]
    std::vector<int32_t> group_columns;   // [n_groups] B rows each group loads per column tile
    std::vector<char> code;               // gfx950 code object
};

struct HostPlan {
    int32_t M = 0, K = 0, N = 0, nnz = 0;
    int32_t dtype = 0, conv = 0, Cin = 0, H = 0, W = 0, kernel = 0;
    int32_t vec = 1, lanes_per_tile = 0, n_tiles = 0, gy = kGy;
    int32_t split_threshold = 0, n_split = 0, n_wg_rows = 0;
    int32_t natural_order = 0;         // rows kept in input order (load-balance ablation)
    int32_t batch = 1;                 // problems per call: images of a convolution, B/C pairs of an SpMM
    int32_t ldb = 0, ldc = 0;          // elements between consecutive rows of B and of C (N unless the caller widens them)
    bool kernel_auto = false;          // the executor family was the inspector's choice, not the caller's

    std::vector<int32_t> row_nnz, hist, perm, inv_perm, p_row_ptr, p_col_idx;
    std::vector<uint8_t> p_vals;       // nnz * elem_size bytes, bit copies
    std::vector<int32_t> bins;         // [nbins][4]
    std::vector<uint32_t> stream;      // [nnz][2]
    std::vector<int32_t> conv_seg;     // [M][10], conv only
    std::vector<int32_t> segments;     // [n_split][gy+1]
    SpecPlan spec;

    int elem_size() const { return dtype == SPARSERT_F16 ? 2 : dtype == SPARSERT_I8 ? 1 : 4; }   // vals, B / X
    int out_elem_size() const { return dtype == SPARSERT_F16 ? 2 : 4; }                            // C / Y
};

struct DevicePlan {
    int device = -1;
    int32_t *p_row_ptr = nullptr;
    int32_t *perm = nullptr;
    uint32_t *stream = nullptr;
    int32_t *conv_seg = nullptr;
    int32_t *segments = nullptr;
    void *spec_module = nullptr;    // hipModule_t
    void *spec_function = nullptr;  // hipFunction_t
};

// Host analysis.  Returns SPARSERT_OK or an error code with `err` filled in.
int build_host_plan(const int32_t *row_ptr, const int32_t *col_idx, const void *vals,
                    int32_t M, int32_t K, int32_t N, const sparsert_options &opt,
                    HostPlan &out, std::string &err);

// Generated-kernel path (specialize.cpp): fills h.spec, including the assembled code object.
int build_spec_plan(HostPlan &h, const sparsert_options &opt, std::string &err);
// Rows per code block, among lo..hi, for which the busiest compute unit has the least work on a
// large launch: workgroups(R) = ceil(ceil(M / R) / groups_per_wg) * wg_columns are dealt to 256
// compute units, a workgroup's work grows with R, so the cost is ceil(workgroups / 256) * R;
// ties go to the larger R (fewer fetches of B).  Only counts that leave no compute unit without a
// workgroup are considered; if there is none, lo is returned.
int rows_for_whole_rounds(int32_t M, int groups_per_wg, int64_t wg_columns, int lo, int hi);
// The smallest number of rows per code block for which the launch is at most `rounds` workgroups
// per compute unit (workgroups counted as above); 0 if more than `hi` rows would be needed.
int rows_for_rounds(int32_t M, int groups_per_wg, int64_t wg_columns, int rounds, int hi);
// A launch a little over a whole number of workgroups per compute unit leaves a few compute units
// with one workgroup more than the rest, and they set the time.  Where the last round is less
// than a quarter full and at most 15 % more rows per block remove it, this returns that row
// count; else R.
int rows_without_thin_round(int32_t M, int R, int groups_per_wg, int64_t wg_columns, int hi);
bool spec_available();   // can generated kernels be assembled in this process (is the code object manager loadable)?

// Records the thread-local error message behind sparsert_last_error (api.cpp); returns `code`.
int set_error(int code, const std::string &msg);

// Device side (kernels.hip).
int upload_plan(const HostPlan &h, DevicePlan &d, std::string &err);
void free_device_plan(DevicePlan &d);
bool on_plan_device(const DevicePlan &d);   // is the plan's device the calling thread's current device?
int launch_rows(const HostPlan &h, const DevicePlan &d, const void *B, void *C,
                void *stream, std::string &err);
int launch_spec(const HostPlan &h, const DevicePlan &d, const void *B, void *C,
                void *stream, std::string &err);
// Comparison of two results of a plan (kernels.hip).  launch_compare: two kernels on `stream`,
// partials_dev must hold 4 words per block of compare_blocks(h), result_dev receives 4 words.
int64_t compare_blocks(const HostPlan &h);
int launch_compare(const HostPlan &h, const void *a, const void *b, uint32_t *partials_dev, uint32_t *result_dev,
                   void *stream, std::string &err);
int compare_with_own_partials(const HostPlan &h, const void *a, const void *b, uint32_t *result_dev, void *stream, std::string &err);
// The library's static partials array: its address on the current device (looked up once per
// device) and the number of output elements it covers.
int static_compare_scratch(uint32_t **out, std::string &err);
int64_t static_compare_max_elements();
// Autotuner helper: overwrites `bytes` of scratch memory so that the L2 caches hold nothing of a plan.
int displace_caches(void *scratch, size_t bytes, void *stream, std::string &err);

}  // namespace sparsert

struct sparsert_plan {
    sparsert::HostPlan host;
    sparsert::DevicePlan dev;
    bool on_device = false;
};
