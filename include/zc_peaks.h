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

/* ---- latency probes: what a launch costs before it does any work -------------------
 * An empty kernel of `workgroups` x 256 threads (every wave ends at once). */
int zc_peak_empty(int workgroups, void* stream);

/* One trip to memory and one store per workgroup: workgroup i reads the 16 bytes at
 * src + ((i * stride_bytes) mod bytes) (lane 0 only), adds `salt` and stores the sum to
 * dst[i].  With stride_bytes >= 4096 and a buffer larger than the last-level cache every
 * read is a miss.  src 16-byte aligned, bytes a multiple of 16, dst holds `workgroups`
 * words.  Two launches, the second reading the first one's dst as its src, make a
 * dependent pair. */
int zc_peak_touch(const void* src, size_t bytes, size_t stride_bytes, int workgroups, uint32_t salt,
                  uint32_t* dst, void* stream);

/* One wave follows `hops` dependent loads through `table` (n 32-bit entries, entry i
 * holding the index of the next entry: the caller builds a permutation with far-apart
 * successors) starting at entry `start`, and stores the index it ends at in *dst: the
 * kernel's duration grows by one memory latency per hop. */
int zc_peak_chase(const uint32_t* table, size_t n, uint32_t start, int hops, uint32_t* dst, void* stream);

#ifdef __cplusplus
}
#endif
#endif
