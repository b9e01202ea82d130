/* Machine-peak probes: three kernels of known work that measure what this GPU
 * delivers to the simplest possible code - a streaming read, a streaming copy
 * and a loop of nothing but matrix instructions.  bench.py --peaks times them so
 * that a kernel of the library can be priced against the attainable rate next
 * to the data-sheet rate.  They are measurement tools, not part of the method:
 * a library of their own (libzc_peaks.so), nothing in libzipcache.so uses them.
 *
 * All pointers are device memory owned by the caller; work is enqueued on
 * `stream` (a hipStream_t) without synchronisation; the return value is 0 on
 * success, -1 for an invalid argument, -4 when the launch failed.  Nothing is
 * allocated. */
#ifndef ZC_PEAKS_H
#define ZC_PEAKS_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* Reads `bytes` (a multiple of 16, 16-byte aligned) once, 16 bytes a lane, eight
 * requests in flight per lane; `sink` (>= 4 bytes) receives a word only if the
 * data XORs to a pattern random data does not produce. */
int zc_peak_read(const void* src, size_t bytes, uint32_t* sink, void* stream);

/* dst[i] = src[i] over `bytes` (a multiple of 16, both 16-byte aligned, no overlap). */
int zc_peak_copy(void* dst, const void* src, size_t bytes, void* stream);

/* `workgroups` x 256 threads, every wave issues `iters` x 8 independent
 * v_mfma_f32_32x32x16 (bf16 when dtype == 2, fp16 when dtype == 1) on register
 * operands; flops = workgroups * 4 * iters * 8 * 2 * 32 * 32 * 16.  `sink`
 * (>= 4 bytes) receives a word only if an accumulator ends as NaN. */
int zc_peak_mfma(int dtype, int workgroups, int iters, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif
