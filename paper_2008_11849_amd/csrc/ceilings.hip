// Measured ceilings for the roofline report of bench.py: three plain kernels whose only job is
// to run one resource of the chip flat out, so that a kernel's time can be held against what
// this GPU delivers, next to the published peaks.  Not on the SpMM path; the benchmark loads
// this library separately.
//   copy  - streams `bytes` from src to dst (16 bytes per lane): the HBM ceiling when the
//           buffers exceed the caches, the L2 / memory-side cache ceiling at a small footprint
//   fma   - independent fp32 multiply-adds on registers: the vector ALU without packed
//           instructions (this build never emits them)
//   loads - every wave pulls 256-byte rows of a cache-resident matrix into registers, one
//           dword per lane, as the generated SpMM kernel fetches rows of B: the rate at which
//           a compute unit can be fed operands through its vector-memory path
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/sparsert_ceilings.h"

namespace {

__global__ __launch_bounds__(256) void copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

constexpr int kAcc = 32;   // independent accumulators per lane: no multiply-add waits for another

__global__ __launch_bounds__(256) void fma_kernel(float *out, int iters, float a, float b) {
    float acc[kAcc];
#pragma unroll
    for (int j = 0; j < kAcc; ++j) acc[j] = (float)(threadIdx.x + j);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < kAcc; ++j) acc[j] = __builtin_fmaf(acc[j], a, b);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < kAcc; ++j) s += acc[j];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Wave w of the launch walks `rows` rows of column tile (w mod tiles): rows are `pitch` floats
// apart, a tile is 64 adjacent floats.  Eight rows are requested before the first is used.
__global__ __launch_bounds__(256) void loads_kernel(const float *__restrict__ m, int rows, int pitch, int tiles,
                                                     int repeats, float *out) {
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
    const float *p = m + (size_t)(wave % tiles) * 64 + lane;
    float s0 = 0.0f, s1 = 0.0f;
    for (int r = 0; r < repeats; ++r) {
        asm volatile("" ::: "memory");   // the rows are fetched again in every repeat
        for (int k = 0; k + 8 <= rows; k += 8) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = p[(size_t)(k + j) * pitch];
#pragma unroll
            for (int j = 0; j < 8; j += 2) { s0 += v[j]; s1 += v[j + 1]; }
        }
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s0 + s1;
}

}  // namespace

extern "C" {

int sparsert_ceiling_copy(const void *src_dev, void *dst_dev, size_t bytes, void *stream) {
    if (!src_dev || !dst_dev || bytes % 16) return -1;
    hipLaunchKernelGGL(copy_kernel, dim3(4096), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const float4 *>(src_dev), static_cast<float4 *>(dst_dev), (int64_t)(bytes / 16));
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int sparsert_ceiling_fma(void *out_dev, int32_t workgroups, int32_t iters, void *stream) {
    if (!out_dev || workgroups < 1 || iters < 1) return -1;
    hipLaunchKernelGGL(fma_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<float *>(out_dev), iters, 1.0000001f, 1e-9f);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int sparsert_ceiling_loads(const void *matrix_dev, int32_t rows, int32_t pitch, int32_t tiles, int32_t workgroups,
                           int32_t repeats, void *out_dev, void *stream) {
    if (!matrix_dev || !out_dev || rows < 8 || rows % 8 || tiles < 1 || pitch < tiles * 64 || workgroups < 1 || repeats < 1) return -1;
    hipLaunchKernelGGL(loads_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const float *>(matrix_dev), rows, pitch, tiles, repeats, static_cast<float *>(out_dev));
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

int32_t sparsert_ceiling_fma_flops_per_thread_iter(void) { return 2 * kAcc; }

}  // extern "C"
