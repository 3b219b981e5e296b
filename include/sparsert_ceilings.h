/*
 * sparsert_ceilings.h - C ABI of the small measurement library behind the roofline report
 * (libsparsert_ceilings.so).  Callers: the benchmark only.  Nothing here is on the SpMM path
 * and the SpMM library does not depend on it.
 *
 * Each call launches one kernel on `stream` (a hipStream_t, NULL = the null stream) and returns
 * at once; the caller times it with events.  Pointers are DEVICE memory, borrowed.
 * Returns 0, -1 for a bad argument, -3 if the launch failed.
 */
#ifndef SPARSERT_CEILINGS_H
#define SPARSERT_CEILINGS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* dst[0..bytes) = src[0..bytes); bytes a multiple of 16, buffers 16-byte aligned, not overlapping. */
int sparsert_ceiling_copy(const void *src_dev, void *dst_dev, size_t bytes, void *stream);

/* `workgroups` x 256 threads each run `iters` x 32 independent fp32 multiply-adds on registers;
 * out_dev receives workgroups*256 floats.  Flops = workgroups*256*iters*sparsert_ceiling_fma_flops_per_thread_iter(). */
int sparsert_ceiling_fma(void *out_dev, int32_t workgroups, int32_t iters, void *stream);
int32_t sparsert_ceiling_fma_flops_per_thread_iter(void);

/* Every wave of `workgroups` x 4 reads `repeats` times `rows` rows (a multiple of 8) of one 64-float
 * column tile of a row-major float matrix (`pitch` floats between rows, `tiles` tiles, wave w takes
 * tile w mod tiles), one dword per lane, eight rows in flight.  Bytes delivered to registers =
 * workgroups*4*repeats*rows*256.  out_dev receives workgroups*256 floats. */
int sparsert_ceiling_loads(const void *matrix_dev, int32_t rows, int32_t pitch, int32_t tiles, int32_t workgroups,
                           int32_t repeats, void *out_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPARSERT_CEILINGS_H */
