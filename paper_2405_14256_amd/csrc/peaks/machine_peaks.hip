// Machine-peak probes (see zc_peaks.h): kernels of known work that do nothing
// clever, for pricing the library's kernels against what the GPU delivers.
#include <hip/hip_runtime.h>
#include "zc_peaks.h"

namespace {

constexpr int kThreads = 256;
constexpr int kInFlight = 8;            // 16-byte requests a lane has outstanding

__global__ __launch_bounds__(kThreads) void k_peak_read(const uint4* __restrict__ src, size_t n16, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  uint4 acc = make_uint4(0u, 0u, 0u, 0u);
  for (; i + (kInFlight - 1) * stride < n16; i += kInFlight * stride) {
    uint4 v[kInFlight];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) v[j] = src[i + j * stride];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) { acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w; }
  }
  for (; i < n16; i += stride) {
    const uint4 v = src[i];
    acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
  }
  if ((acc.x ^ acc.y) == 0x9e3779b9u && (acc.z ^ acc.w) == 0x7f4a7c15u) *sink = acc.x;
}

__global__ __launch_bounds__(kThreads) void k_peak_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  for (; i + (kInFlight - 1) * stride < n16; i += kInFlight * stride) {
    uint4 v[kInFlight];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) v[j] = src[i + j * stride];
#pragma unroll
    for (int j = 0; j < kInFlight; ++j) dst[i + j * stride] = v[j];
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <bool BF16>
__global__ __launch_bounds__(kThreads) void k_peak_mfma(int iters, float* sink) {
  // operands: small numbers that depend on the lane, so nothing folds at compile time
  const float seed = 1.0f / (float)(1 + (threadIdx.x & 7));
  f32x16 acc[8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[a][j] = 0.f;
  if constexpr (BF16) {
    bf16x8 x, y;
#pragma unroll
    for (int j = 0; j < 8; ++j) { x[j] = (__bf16)(seed * (j + 1)); y[j] = (__bf16)(0.001f * (j - 3)); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int a = 0; a < 8; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, acc[a], 0, 0, 0);
    }
  } else {
    f16x8 x, y;
#pragma unroll
    for (int j = 0; j < 8; ++j) { x[j] = (_Float16)(seed * (j + 1)); y[j] = (_Float16)(0.001f * (j - 3)); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int a = 0; a < 8; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x, y, acc[a], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[a][j];
  if (s != s) *sink = s;
}

__global__ __launch_bounds__(kThreads) void k_peak_empty() {}

__global__ __launch_bounds__(kThreads) void k_peak_touch(const uint8_t* __restrict__ src, size_t bytes, size_t stride,
                                                         uint32_t salt, uint32_t* __restrict__ dst) {
  if (threadIdx.x != 0) return;
  const size_t off = ((size_t)blockIdx.x * stride) % bytes & ~(size_t)15;
  const uint4 v = *reinterpret_cast<const uint4*>(src + off);
  dst[blockIdx.x] = v.x + v.y + v.z + v.w + salt;
}

__global__ __launch_bounds__(64) void k_peak_chase(const uint32_t* __restrict__ table, size_t n, uint32_t start, int hops,
                                                   uint32_t* __restrict__ dst) {
  if (threadIdx.x != 0) return;
  uint32_t i = start;
  for (int h = 0; h < hops; ++h) i = __builtin_nontemporal_load(table + (i < n ? i : 0));   // (stays in bounds whatever the table holds)
  *dst = i;
}

int grid_for(size_t n16) {
  // enough workgroups to keep every CU's request queues full, few enough that each
  // still loops: 16 per CU
  hipDeviceProp_t p;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&p, dev) != hipSuccess) return 4096;
  size_t g = (size_t)p.multiProcessorCount * 16;
  const size_t need = (n16 + kThreads - 1) / kThreads;
  if (g > need) g = need;
  return (int)(g ? g : 1);
}

}  // namespace

extern "C" int zc_peak_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
  if (!src || !sink || (bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15)) return -1;
  if (bytes == 0) return 0;
  const size_t n16 = bytes / 16;
  hipLaunchKernelGGL(k_peak_read, dim3(grid_for(n16)), dim3(kThreads), 0, (hipStream_t)stream,
                     static_cast<const uint4*>(src), n16, sink);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

extern "C" int zc_peak_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || (bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15)) return -1;
  const char *d = static_cast<const char*>(dst), *s = static_cast<const char*>(src);
  if (d < s + bytes && s < d + bytes) return -1;
  if (bytes == 0) return 0;
  const size_t n16 = bytes / 16;
  hipLaunchKernelGGL(k_peak_copy, dim3(grid_for(n16)), dim3(kThreads), 0, (hipStream_t)stream,
                     static_cast<uint4*>(dst), static_cast<const uint4*>(src), n16);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

extern "C" int zc_peak_mfma(int dtype, int workgroups, int iters, float* sink, void* stream) {
  if (!sink || workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || (dtype != 1 && dtype != 2)) return -1;
  if (dtype == 2) hipLaunchKernelGGL(k_peak_mfma<true>, dim3(workgroups), dim3(kThreads), 0, (hipStream_t)stream, iters, sink);
  else hipLaunchKernelGGL(k_peak_mfma<false>, dim3(workgroups), dim3(kThreads), 0, (hipStream_t)stream, iters, sink);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

extern "C" int zc_peak_empty(int workgroups, void* stream) {
  if (workgroups <= 0 || workgroups > (1 << 20)) return -1;
  hipLaunchKernelGGL(k_peak_empty, dim3(workgroups), dim3(kThreads), 0, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

extern "C" int zc_peak_touch(const void* src, size_t bytes, size_t stride_bytes, int workgroups, uint32_t salt,
                             uint32_t* dst, void* stream) {
  if (!src || !dst || bytes < 16 || (bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15) || workgroups <= 0 ||
      workgroups > (1 << 20))
    return -1;
  hipLaunchKernelGGL(k_peak_touch, dim3(workgroups), dim3(kThreads), 0, (hipStream_t)stream,
                     static_cast<const uint8_t*>(src), bytes, stride_bytes, salt, dst);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

extern "C" int zc_peak_chase(const uint32_t* table, size_t n, uint32_t start, int hops, uint32_t* dst, void* stream) {
  if (!table || !dst || n == 0 || start >= n || hops < 0 || hops > (1 << 20)) return -1;
  hipLaunchKernelGGL(k_peak_chase, dim3(1), dim3(64), 0, (hipStream_t)stream, table, n, start, hops, dst);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}
