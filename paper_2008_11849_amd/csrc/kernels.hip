// gfx950 executor kernels: row-walk SpMM and implicit-im2col 3x3 convolution.
//
// Mapping (Section 3.3 keeps N across the threads of a group and broadcasts
// the A operand; the same idea is laid out here for 64-wide wavefronts):
//   - lanes of a wave own V adjacent columns of C each, so B rows and C rows
//     are read and written as contiguous, coalesced segments;
//   - the nonzeros of a row form a wave-uniform stream {operand offset, value}
//     that is fetched with scalar loads and broadcast from SGPRs;
//   - accumulators live in VGPRs and are indexed statically, because a wave
//     owns one row at a time (the paper needs full unrolling for that,
//     Section 3.5; a row-per-wave walk gets it for free);
//   - rows at or above the split threshold are shared by the Gy waves of a
//     workgroup (Section 3.4, thread-group balance) and summed through LDS in a
//     fixed order, so results are reproducible run to run.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <type_traits>

#include "plan.h"

namespace sparsert {

template <typename T, int V> struct VecOf { typedef T type __attribute__((ext_vector_type(V))); };
template <typename T> struct VecOf<T, 1> { typedef T type; };

// Global (address space 1) byte pointer: keeps the loads on the global path with a
// scalar base and a 32-bit per-lane offset.
typedef const char __attribute__((address_space(1))) *gbytes;

// Arithmetic of one storage type at V columns per lane: what an operand fetch yields, how a
// nonzero is accumulated, and how the accumulators are stored.
//   float / half: operands widened to fp32, fp32 multiply-add, the stream word is the fp32 value;
//                 half results are rounded once, to nearest even, at the store.
//   int8:         exact 32-bit integer sums; the stream word is the sign-extended value.  At
//                 V = 4 a lane's four adjacent columns stay packed in one dword and
//                 v_dot4_i32_i8 against the value placed in byte j picks out column j.
template <typename T, int V> struct Ops {
    typedef float acc_t;
    typedef T out_t;
    struct opd_t { float v[V]; };
    typedef typename VecOf<T, V>::type vec_t;
    static __device__ __forceinline__ opd_t load(gbytes p) {
        const vec_t v = *reinterpret_cast<const vec_t __attribute__((address_space(1))) *>(p);
        opd_t o;
        if constexpr (V == 1) {
            o.v[0] = (float)v;
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) o.v[j] = (float)v[j];
        }
        return o;
    }
    static __device__ __forceinline__ void mad(acc_t (&acc)[V], uint32_t word, const opd_t &b) {
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] = __builtin_fmaf(__uint_as_float(word), b.v[j], acc[j]);
    }
    // `stream`: C is not read again, so where a wave's store covers whole 128-byte lines it is
    // written with the non-temporal hint and stays out of the way of B in the L2.
    static __device__ __forceinline__ void store(out_t *dst, const acc_t (&acc)[V], bool stream) {
        vec_t v;
        if constexpr (V == 1) {
            v = (T)acc[0];
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) v[j] = (T)acc[j];  // half: one round-to-nearest-even here
        }
        if (stream) __builtin_nontemporal_store(v, reinterpret_cast<vec_t *>(dst));
        else *reinterpret_cast<vec_t *>(dst) = v;
    }
};

template <int V> struct Ops<int8_t, V> {
    static_assert(V == 1 || V == 4, "int8 plans use one or four columns per lane");
    typedef int32_t acc_t;
    typedef int32_t out_t;
    struct opd_t { int32_t v; };   // V = 1: the operand; V = 4: four packed operands
    static __device__ __forceinline__ opd_t load(gbytes p) {
        opd_t o;
        if constexpr (V == 1) o.v = *reinterpret_cast<const int8_t __attribute__((address_space(1))) *>(p);
        else o.v = *reinterpret_cast<const int32_t __attribute__((address_space(1))) *>(p);
        return o;
    }
    static __device__ __forceinline__ void mad(acc_t (&acc)[V], uint32_t word, const opd_t &b) {
        if constexpr (V == 1) {
            acc[0] += (int32_t)word * b.v;
        } else {
            const uint32_t a8 = word & 0xffu;
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_sdot4(b.v, (int32_t)(a8 << (8 * j)), acc[j], false);
        }
    }
    static __device__ __forceinline__ void store(out_t *dst, const acc_t (&acc)[V], bool stream) {
        if constexpr (V == 1) {
            if (stream) __builtin_nontemporal_store(acc[0], dst);
            else *dst = acc[0];
        } else {
            typedef int32_t i4 __attribute__((ext_vector_type(4)));
            const i4 v = {acc[0], acc[1], acc[2], acc[3]};
            if (stream) __builtin_nontemporal_store(v, reinterpret_cast<i4 *>(dst));
            else *reinterpret_cast<i4 *>(dst) = v;
        }
    }
};

// One operand fetch.  SpMM: the stream word is the byte offset of B's row.  Convolution: the
// top 4 bits name the filter tap (r*3+s), the low 28 bits are the signed byte displacement of
// X[c, oh+r-1, ow+s-1] from X[0, oh, ow]; the caller only walks a tap's nonzeros with the lanes
// whose tap lies inside the image, so no test is needed here.
template <typename T, int V, bool CONV>
__device__ __forceinline__ typename Ops<T, V>::opd_t fetch(gbytes in, uint32_t lane_off, uint32_t word) {
    const int32_t disp = CONV ? (int32_t)(word << 4) >> 4 : (int32_t)word;
    return Ops<T, V>::load(in + disp + lane_off);
}

// acc[:] += sum over stream positions [p0, p1) of value * operand.  p0, p1, the stream and
// `in` are wave-uniform: the {word, value} pairs arrive through scalar loads (the pairs of the
// next chunk are requested before the current chunk's operands are waited for), lane_off is
// the only per-lane part of an address.  The stream is padded by 2*U pairs, so pair loads
// never need a guard.
template <typename T, int V, bool CONV>
__device__ __forceinline__ void walk(const uint2 *__restrict__ stream, int p0, int p1,
                                     gbytes in, uint32_t lane_off, typename Ops<T, V>::acc_t (&acc)[V]) {
    typedef typename Ops<T, V>::opd_t opd_t;
    constexpr int U = 8;
    int p = p0;
    uint2 e[U];
#pragma unroll
    for (int i = 0; i < U; ++i) e[i] = stream[p + i];
    for (; p + U <= p1; p += U) {
        uint2 en[U];
        opd_t b[U];
#pragma unroll
        for (int i = 0; i < U; ++i) en[i] = stream[p + U + i];
#pragma unroll
        for (int i = 0; i < U; ++i) b[i] = fetch<T, V, CONV>(in, lane_off, e[i].x);
#pragma unroll
        for (int i = 0; i < U; ++i) Ops<T, V>::mad(acc, e[i].y, b[i]);
#pragma unroll
        for (int i = 0; i < U; ++i) e[i] = en[i];
    }
    // Tail of fewer than U nonzeros: same shape as a full chunk so the operand loads still go
    // out together.  Loads past the tail are redirected to a row this wave reads anyway; only
    // the multiply-adds are guarded (by a wave-uniform count).
    const int rem = p1 - p;
    if (rem > 0) {
        opd_t b[U - 1];
#pragma unroll
        for (int i = 0; i < U - 1; ++i) b[i] = fetch<T, V, CONV>(in, lane_off, i < rem ? e[i].x : e[0].x);
#pragma unroll
        for (int i = 0; i < U - 1; ++i)
            if (i < rem) Ops<T, V>::mad(acc, e[i].y, b[i]);
    }
}

struct RowsArgs {
    const int32_t *p_row_ptr;
    const int32_t *perm;
    const uint2 *stream;
    const int32_t *segments;
    const int32_t *conv_seg;
    const void *in;   // B [K,N] or X [Cin,H,W]
    void *out;        // C [M,N] or Y [Cout,H,W]
    int32_t M, N, ldc;
    int32_t n_vec_cols, lanes_per_tile, n_tiles;
    int32_t n_split, n_wg_rows;
    int32_t n_tasks, tasks_per_xcd;
    int32_t H, W;
    int32_t stream_stores;   // every wave store of C covers whole 128-byte lines
    int64_t in_image_bytes, out_image_elems;   // distance between the problems of a batch (grid y)
};

template <typename T, int V, bool CONV>
__global__ __launch_bounds__(kGy *kWave) void rows_kernel(const RowsArgs a) {
    // Workgroups are handed to the 8 XCDs round-robin.  Remap so that each XCD works on a
    // contiguous run of tasks; tasks are ordered column-tile major, so the B column slab
    // of a tile is pulled into as few of the per-XCD L2s as possible.
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int task = xcd * a.tasks_per_xcd + idx;
    if (task >= a.n_tasks) return;
    const int tile = task / a.n_wg_rows;
    const int wg_row = task - tile * a.n_wg_rows;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & (kWave - 1);

    // Column ownership.  Lanes past the tile's share redo the tile's first column (their
    // loads stay in bounds, their results are dropped).
    const int vc0 = tile * a.lanes_per_tile;
    const int vc = vc0 + lane;
    const bool owns = lane < a.lanes_per_tile && vc < a.n_vec_cols;
    const int col = (owns ? vc : vc0) * V;

    const gbytes in = (gbytes)a.in + (int64_t)blockIdx.y * a.in_image_bytes;
    const uint32_t lane_off = (uint32_t)col * (uint32_t)sizeof(T);
    unsigned tap_ok = 0x1ff;
    if constexpr (CONV) {
        // Pixel (oh, ow) = col; bit r*3+s of tap_ok says whether (oh+r-1, ow+s-1) is inside.
        const int oh = col / a.W, ow = col - oh * a.W;
        tap_ok = 0;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const int ih = oh + r - 1, iw = ow + s - 1;
                if (ih >= 0 && ih < a.H && iw >= 0 && iw < a.W) tap_ok |= 1u << (r * 3 + s);
            }
    }

    typedef typename Ops<T, V>::acc_t acc_t;
    acc_t acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = 0;

    int slot, p0, p1;
    const bool split = wg_row < a.n_split;
    if (split) {
        slot = wg_row;
        p0 = a.segments[slot * (kGy + 1) + wave];
        p1 = a.segments[slot * (kGy + 1) + wave + 1];
    } else {
        slot = a.n_split + (wg_row - a.n_split) * kGy + wave;
        if (slot >= a.M) return;  // whole wave leaves; no barrier follows on this path
        p0 = a.p_row_ptr[slot];
        p1 = a.p_row_ptr[slot + 1];
    }

    if constexpr (CONV) {
        // The slot's nonzeros are grouped by tap (Section 3.6: the padding test is resolved
        // ahead of time): one lane mask per group instead of a test per multiply-add.
        const int32_t *seg = a.conv_seg + slot * 10;
        for (int t = 0; t < 9; ++t) {
            const int q0 = max(p0, seg[t]), q1 = min(p1, seg[t + 1]);
            if (q0 < q1 && ((tap_ok >> t) & 1u)) walk<T, 1, true>(a.stream, q0, q1, in, lane_off, acc);
        }
    } else {
        walk<T, V, false>(a.stream, p0, p1, in, lane_off, acc);
    }

    if (split) {
        // Section 3.3: partial tiles of the groups are reduced through shared memory at the
        // end.  Summed by wave 0 in wave order: deterministic, no atomics.
        __shared__ acc_t red[kGy][V][kWave];
#pragma unroll
        for (int j = 0; j < V; ++j) red[wave][j][lane] = acc[j];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            acc_t s = red[0][j][lane];
#pragma unroll
            for (int g = 1; g < kGy; ++g) s += red[g][j][lane];
            acc[j] = s;
        }
    }
    if (owns) {
        const int row = a.perm[slot];
        typedef typename Ops<T, V>::out_t out_t;
        out_t *out = static_cast<out_t *>(a.out) + (int64_t)blockIdx.y * a.out_image_elems;
        Ops<T, V>::store(out + (size_t)row * a.ldc + col, acc, a.stream_stores != 0);
    }
}

#define HIP_TRY(call)                                                        \
    do {                                                                     \
        hipError_t e_ = (call);                                              \
        if (e_ != hipSuccess) {                                              \
            err = std::string(#call) + ": " + hipGetErrorString(e_);         \
            return e_ == hipErrorOutOfMemory ? SPARSERT_ENOMEM : SPARSERT_EHIP; \
        }                                                                    \
    } while (0)

template <typename U>
static int to_device(const U *src, size_t count, U **dst, std::string &err) {
    *dst = nullptr;
    const size_t bytes = (count ? count : 1) * sizeof(U);  // never a zero-sized allocation
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(dst), bytes));
    if (count) HIP_TRY(hipMemcpy(*dst, src, count * sizeof(U), hipMemcpyHostToDevice));
    return SPARSERT_OK;
}

bool on_plan_device(const DevicePlan &d) {
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == d.device;
}

int upload_plan(const HostPlan &h, DevicePlan &d, std::string &err) {
    HIP_TRY(hipGetDevice(&d.device));
    if (int rc = to_device(h.p_row_ptr.data(), h.p_row_ptr.size(), &d.p_row_ptr, err)) return rc;
    if (int rc = to_device(h.perm.data(), h.perm.size(), &d.perm, err)) return rc;
    {   // the executor may read up to 16 {word, value} pairs past the last nonzero
        std::vector<uint32_t> padded(h.stream);
        padded.resize(h.stream.size() + 32, 0u);
        if (int rc = to_device(padded.data(), padded.size(), &d.stream, err)) return rc;
    }
    if (int rc = to_device(h.segments.data(), h.segments.size(), &d.segments, err)) return rc;
    if (int rc = to_device(h.conv_seg.data(), h.conv_seg.size(), &d.conv_seg, err)) return rc;
    if (h.kernel == SPARSERT_KERNEL_SPEC) {
        int dev = 0, lds_max = 0;
        HIP_TRY(hipGetDevice(&dev));
        HIP_TRY(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
        if (h.spec.lds_bytes > lds_max) {
            err = "the generated kernel needs more LDS per workgroup than this device has";
            return SPARSERT_EUNSUPPORTED;
        }
        hipModule_t mod = nullptr;
        hipFunction_t fn = nullptr;
        hipError_t e1 = hipModuleLoadData(&mod, h.spec.code.data());
        if (e1 != hipSuccess) { err = std::string("loading the generated kernel: ") + hipGetErrorString(e1); return SPARSERT_ECOMPILE; }
        d.spec_module = mod;
        hipError_t e2 = hipModuleGetFunction(&fn, mod, h.spec.symbol.c_str());
        if (e2 != hipSuccess) { err = std::string("generated kernel symbol: ") + hipGetErrorString(e2); return SPARSERT_ECOMPILE; }
        d.spec_function = fn;
    }
    return SPARSERT_OK;
}

void free_device_plan(DevicePlan &d) {
    if (d.p_row_ptr) (void)hipFree(d.p_row_ptr);
    if (d.perm) (void)hipFree(d.perm);
    if (d.stream) (void)hipFree(d.stream);
    if (d.segments) (void)hipFree(d.segments);
    if (d.conv_seg) (void)hipFree(d.conv_seg);
    if (d.spec_module) (void)hipModuleUnload(static_cast<hipModule_t>(d.spec_module));
    d = DevicePlan();
}

template <typename T, int V, bool CONV>
static int launch_one(const RowsArgs &a, int images, hipStream_t s, std::string &err) {
    const unsigned grid = (unsigned)a.tasks_per_xcd * 8u;
    hipLaunchKernelGGL((rows_kernel<T, V, CONV>), dim3(grid, (unsigned)images), dim3(kGy * kWave), 0, s, a);
    HIP_TRY(hipGetLastError());
    return SPARSERT_OK;
}

int launch_rows(const HostPlan &h, const DevicePlan &d, const void *in, void *out,
                void *stream, std::string &err) {
    // Host-side shape checks: the kernel assumes exactly these relations.
    const int64_t nvc = h.N / h.vec;
    if (h.vec < 1 || h.N % h.vec || h.ldb < h.N || h.ldc < h.N || h.ldb % h.vec || h.ldc % h.vec || h.gy != kGy || h.lanes_per_tile < 1 || h.lanes_per_tile > kWave ||
        (int64_t)h.n_tiles * h.lanes_per_tile < nvc || h.n_split < 0 || h.n_split > h.M ||
        (int64_t)(h.n_tiles - 1) * h.lanes_per_tile >= nvc ||
        h.n_wg_rows != h.n_split + (h.M - h.n_split + kGy - 1) / kGy) {
        err = "plan geometry is inconsistent";
        return SPARSERT_EINVAL;
    }
    const int64_t n_tasks = (int64_t)h.n_wg_rows * h.n_tiles;
    if (n_tasks <= 0 || n_tasks > (1ll << 30)) { err = "too many workgroups"; return SPARSERT_EUNSUPPORTED; }
    RowsArgs a;
    a.p_row_ptr = d.p_row_ptr; a.perm = d.perm;
    a.stream = reinterpret_cast<const uint2 *>(d.stream);
    a.segments = d.segments; a.conv_seg = d.conv_seg;
    a.in = in; a.out = out;
    a.M = h.M; a.N = h.N; a.ldc = h.ldc;
    a.n_vec_cols = (int32_t)nvc; a.lanes_per_tile = h.lanes_per_tile; a.n_tiles = h.n_tiles;
    a.n_split = h.n_split; a.n_wg_rows = h.n_wg_rows;
    a.n_tasks = (int32_t)n_tasks; a.tasks_per_xcd = (int32_t)((n_tasks + 7) / 8);
    a.H = h.H; a.W = h.W;
    a.stream_stores = ((int64_t)h.ldc * h.out_elem_size()) % 128 == 0 &&
                      ((int64_t)h.lanes_per_tile * h.vec * h.out_elem_size()) % 128 == 0;
    a.in_image_bytes = (h.conv ? (int64_t)h.Cin * h.H * h.W : (int64_t)h.K * h.ldb) * h.elem_size();
    a.out_image_elems = (int64_t)h.M * h.ldc;
    const int images = h.batch;
    if (images < 1 || images > 65535) { err = "plan geometry is inconsistent"; return SPARSERT_EINVAL; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool f16 = h.dtype == SPARSERT_F16;
    if (h.dtype == SPARSERT_I8) {
        if (h.conv && h.vec != 1) { err = "conv plans use vec = 1"; return SPARSERT_EINVAL; }
        if (h.conv) return launch_one<int8_t, 1, true>(a, images, s, err);
        if (h.vec == 1) return launch_one<int8_t, 1, false>(a, images, s, err);
        if (h.vec == 4) return launch_one<int8_t, 4, false>(a, images, s, err);
        err = "unsupported vec for this dtype";
        return SPARSERT_EINVAL;
    }
    if (h.conv) {
        if (h.vec != 1) { err = "conv plans use vec = 1"; return SPARSERT_EINVAL; }
        return f16 ? launch_one<_Float16, 1, true>(a, images, s, err) : launch_one<float, 1, true>(a, images, s, err);
    }
    switch (h.vec) {
    case 1: return f16 ? launch_one<_Float16, 1, false>(a, images, s, err) : launch_one<float, 1, false>(a, images, s, err);
    case 2: return f16 ? launch_one<_Float16, 2, false>(a, images, s, err) : launch_one<float, 2, false>(a, images, s, err);
    case 4: return f16 ? launch_one<_Float16, 4, false>(a, images, s, err) : launch_one<float, 4, false>(a, images, s, err);
    case 8:
        if (f16) return launch_one<_Float16, 8, false>(a, images, s, err);
        [[fallthrough]];
    default: err = "unsupported vec for this dtype"; return SPARSERT_EINVAL;
    }
}

// ---------------------------------------------------------------- comparing two results of a plan
// Two passes and no atomics: block b of the first kernel leaves the largest |a - b|, the
// largest |b| (both over the N valid columns of its share of the output rows, as the bits of
// non-negative floats, which order like unsigned integers) and the number of elements that
// differ in kind in slot b of a partials array; one block of the second kernel folds the slots
// into the caller's four result words.  Every slot that is read has been written by the same
// call, so the partials never need clearing.
constexpr int kCmpThreads = 256;
constexpr int64_t kCmpPerBlock = 64 * kCmpThreads;   // output elements per block of the first pass

template <typename T>
__global__ __launch_bounds__(kCmpThreads) void diff_kernel(const T *a, const T *b, int64_t total, int32_t N, int32_t ld,
                                                            uint32_t *partials) {
    float dmax = 0.0f, bmax = 0.0f;
    uint32_t bad = 0;
    const int64_t first = (int64_t)blockIdx.x * kCmpPerBlock, last = min(total, first + kCmpPerBlock);
    for (int64_t i = first + threadIdx.x; i < last; i += kCmpThreads) {
        const int64_t r = i / N, c = i - r * N;
        if constexpr (std::is_integral<T>::value) {
            bad += a[r * ld + c] != b[r * ld + c];
        } else {
            const float x = (float)a[r * ld + c], y = (float)b[r * ld + c];
            const bool fx = __builtin_isfinite(x), fy = __builtin_isfinite(y);
            if (fx && fy) { dmax = fmaxf(dmax, fabsf(x - y)); bmax = fmaxf(bmax, fabsf(y)); }
            else if (fx != fy || (__builtin_isnan(x) != __builtin_isnan(y)) || (!__builtin_isnan(x) && x != y)) ++bad;
        }
    }
    __shared__ uint32_t sd[kCmpThreads], sb[kCmpThreads], sc[kCmpThreads];
    sd[threadIdx.x] = __float_as_uint(dmax); sb[threadIdx.x] = __float_as_uint(bmax); sc[threadIdx.x] = bad;
    __syncthreads();
    for (int w = kCmpThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            sd[threadIdx.x] = max(sd[threadIdx.x], sd[threadIdx.x + w]);
            sb[threadIdx.x] = max(sb[threadIdx.x], sb[threadIdx.x + w]);
            sc[threadIdx.x] += sc[threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        partials[4 * (size_t)blockIdx.x + 0] = sd[0];
        partials[4 * (size_t)blockIdx.x + 1] = sb[0];
        partials[4 * (size_t)blockIdx.x + 2] = sc[0];
        partials[4 * (size_t)blockIdx.x + 3] = 0;
    }
}

__global__ __launch_bounds__(kCmpThreads) void fold_kernel(const uint32_t *partials, int32_t n_blocks, uint32_t *result) {
    uint32_t d = 0, b = 0, c = 0;
    for (int i = threadIdx.x; i < n_blocks; i += kCmpThreads) {
        d = max(d, partials[4 * (size_t)i]); b = max(b, partials[4 * (size_t)i + 1]); c += partials[4 * (size_t)i + 2];
    }
    __shared__ uint32_t sd[kCmpThreads], sb[kCmpThreads], sc[kCmpThreads];
    sd[threadIdx.x] = d; sb[threadIdx.x] = b; sc[threadIdx.x] = c;
    __syncthreads();
    for (int w = kCmpThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            sd[threadIdx.x] = max(sd[threadIdx.x], sd[threadIdx.x + w]);
            sb[threadIdx.x] = max(sb[threadIdx.x], sb[threadIdx.x + w]);
            sc[threadIdx.x] += sc[threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) { result[0] = sd[0]; result[1] = sb[0]; result[2] = sc[0]; result[3] = (uint32_t)n_blocks; }
}

int64_t compare_blocks(const HostPlan &h) {
    const int64_t total = (int64_t)h.batch * h.M * h.N;
    return (total + kCmpPerBlock - 1) / kCmpPerBlock;
}

int launch_compare(const HostPlan &h, const void *a, const void *b, uint32_t *partials_dev, uint32_t *result_dev,
                   void *stream, std::string &err) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t total = (int64_t)h.batch * h.M * h.N, blocks = compare_blocks(h);
    const int32_t ld = h.conv ? h.N : h.ldc;   // the batch's results follow each other at the same pitch
    if (blocks < 1 || blocks > (1ll << 30)) { err = "output too large to compare"; return SPARSERT_EUNSUPPORTED; }
    const dim3 grid((unsigned)blocks), wg(kCmpThreads);
    if (h.dtype == SPARSERT_I8)
        hipLaunchKernelGGL(diff_kernel<int32_t>, grid, wg, 0, s, (const int32_t *)a, (const int32_t *)b, total, h.N, ld, partials_dev);
    else if (h.dtype == SPARSERT_F16)
        hipLaunchKernelGGL(diff_kernel<_Float16>, grid, wg, 0, s, (const _Float16 *)a, (const _Float16 *)b, total, h.N, ld, partials_dev);
    else
        hipLaunchKernelGGL(diff_kernel<float>, grid, wg, 0, s, (const float *)a, (const float *)b, total, h.N, ld, partials_dev);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(fold_kernel, dim3(1), wg, 0, s, partials_dev, (int32_t)blocks, result_dev);
    HIP_TRY(hipGetLastError());
    return SPARSERT_OK;
}

// The variant for callers that cannot allocate keeps its partials in this array: one copy per
// GPU, held until the process ends.  On the host the array's name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returns for the current device.
constexpr int kStaticCmpBlocks = 2048;   // 2048 x 16384 = 33 554 432 output elements
static __device__ __align__(256) uint32_t scratch[4 * kStaticCmpBlocks];

int64_t static_compare_max_elements() { return (int64_t)kStaticCmpBlocks * kCmpPerBlock; }

int static_compare_scratch(uint32_t **out, std::string &err) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static uint32_t *per_device[kMaxDevices] = {nullptr};
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { err = "device ordinal out of range"; return SPARSERT_EUNSUPPORTED; }
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        per_device[dev] = static_cast<uint32_t *>(ptr);
    }
    *out = per_device[dev];
    return SPARSERT_OK;
}

// The partials live in memory allocated for this call and released before it returns, which is
// why this form synchronises the stream.
int compare_with_own_partials(const HostPlan &h, const void *a, const void *b, uint32_t *result_dev, void *stream, std::string &err) {
    uint32_t *partials = nullptr;
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&partials), (size_t)compare_blocks(h) * 4 * sizeof(uint32_t)));
    int rc = launch_compare(h, a, b, partials, result_dev, stream, err);
    const hipError_t e1 = hipStreamSynchronize(static_cast<hipStream_t>(stream));
    (void)hipFree(partials);
    if (rc == SPARSERT_OK && e1 != hipSuccess) { err = std::string("hipStreamSynchronize: ") + hipGetErrorString(e1); rc = SPARSERT_EHIP; }
    return rc;
}

// Writes `bytes` of scratch memory: more than the eight L2 caches hold, so whatever a plan left
// there (its code, its operands) is displaced before the plan's next launch.
__global__ __launch_bounds__(256) void fill_kernel(float4 *p, int64_t n, float v) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = make_float4(v, v, v, v);
}

int displace_caches(void *scratch, size_t bytes, void *stream, std::string &err) {
    hipLaunchKernelGGL(fill_kernel, dim3(2048), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<float4 *>(scratch), (int64_t)(bytes / sizeof(float4)), 1.0f);
    HIP_TRY(hipGetLastError());
    return SPARSERT_OK;
}

int launch_spec(const HostPlan &h, const DevicePlan &d, const void *B, void *C,
                void *stream, std::string &err) {
    const SpecPlan &sp = h.spec;
    if (!d.spec_function || sp.n_groups < 1 || sp.n_tiles < 1) {
        err = "plan has no generated kernel";
        return SPARSERT_EINVAL;
    }
    struct { const void *B; void *C; } args = {B, C};
    size_t size = sizeof(args);
    void *config[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, &args, HIP_LAUNCH_PARAM_BUFFER_SIZE, &size,
                      HIP_LAUNCH_PARAM_END};
    const int tpw = sp.tiles_per_wg;
    if (tpw < 1 || tpw > 16 || (tpw & (tpw - 1))) { err = "plan geometry is inconsistent"; return SPARSERT_EINVAL; }
    const bool lds = sp.mode == SPARSERT_SPEC_LDS;
    if (lds && (sp.n_blocks % tpw || sp.lds_bytes < 1 || sp.lds_bytes > 160 * 1024)) { err = "plan geometry is inconsistent"; return SPARSERT_EINVAL; }
    if (sp.ksplit > 1 && (lds || sp.ksplit != tpw || sp.n_blocks != sp.n_groups * sp.ksplit)) { err = "plan geometry is inconsistent"; return SPARSERT_EINVAL; }
    const unsigned gx = (lds || sp.ksplit > 1) ? (unsigned)sp.n_tiles : (unsigned)((sp.n_tiles + tpw - 1) / tpw);
    const unsigned gy = lds ? (unsigned)(sp.n_blocks / tpw) : (unsigned)sp.n_groups;
    // (that the workgroup's registers fit a compute unit was checked when the plan was generated;
    // a loaded plan carries the symbol's own register count in its code object and is checked by the loader)
    const unsigned gz = (unsigned)h.batch;   // the generated prologue offsets the operand and the result by problem
    if (gz < 1 || gz > 65535) { err = "plan geometry is inconsistent"; return SPARSERT_EINVAL; }
    HIP_TRY(hipModuleLaunchKernel(static_cast<hipFunction_t>(d.spec_function), gx, gy, gz, tpw * kWave, 1, 1,
                                  0, static_cast<hipStream_t>(stream), nullptr, config));
    return SPARSERT_OK;
}

}  // namespace sparsert
