/* Time stamps inside the decode kernels: a measurement tool, not part of the method.
 *
 * libzipcache_trace.so is libzipcache.so with the bf16 instances of the two kernels of
 * zc_decode_attention (k_decode_mfma, k_decode_reduce) built to record the GPU's 100 MHz
 * real-time counter at their phase boundaries.  It exports everything zipcache.h declares,
 * plus zc_trace_fetch.  bench.py --decode-timeline uses it to show what a decode call's
 * latency is made of; nothing in libzipcache.so records anything.
 *
 * The buffer (device memory of the library, one per GPU):
 *   [ZC_TRACE_WAVES][ZC_TRACE_SLOTS] uint64   one row per wave of k_decode_mfma, row index
 *       ((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 4 + wave; waves past
 *       the end share the last row.  Slots: 0 entry; 1 first batch of kernel arguments in
 *       registers; 2 query operand of the wave's (last) segment built; 3 that segment's first
 *       block in LDS; 4 its half-blocks done; 5 segments folded; 6 at the barrier before the
 *       workgroup's merge; 7 workgroup's result stored; 8 (tail waves) units done.  0 = not
 *       reached.
 *   [ZC_TRACE_HEADS][4] uint64   one row per workgroup (b * Hq + h) of k_decode_reduce:
 *       0 entry; 1 partials landed; 2 end.
 * Every launch overwrites the rows of its waves. */
#ifndef ZC_TRACE_H
#define ZC_TRACE_H
#include <stddef.h>
#ifdef __cplusplus
extern "C" {
#endif

#define ZC_TRACE_SLOTS 16
#define ZC_TRACE_WAVES 8192
#define ZC_TRACE_HEADS 2048

/* Waits for the device to be idle, copies the first `count` uint64 of the buffer to `host`
 * (host memory; count <= ZC_TRACE_WAVES * ZC_TRACE_SLOTS + ZC_TRACE_HEADS * 4) and, with
 * reset != 0, clears the whole buffer.  Synchronises with the host (unlike every call of
 * zipcache.h).  Returns 0, -1 for an invalid argument, -5 when the HIP runtime failed. */
int zc_trace_fetch(unsigned long long* host, size_t count, int reset);

#ifdef __cplusplus
}
#endif
#endif
