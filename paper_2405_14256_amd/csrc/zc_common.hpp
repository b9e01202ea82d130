// Shared device helpers for the ZipCache gfx950 kernels: element loads,
// wave64 reductions, order-preserving float keys, launch checking.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "zipcache.h"

namespace zc {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

#define ZC_LAUNCH_CHECK()                         \
  do {                                            \
    if (hipGetLastError() != hipSuccess) return ZC_ERR_HIP; \
  } while (0)

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
__host__ __device__ inline int64_t align_up64(int64_t a, int64_t b) { return ceil_div64(a, b) * b; }

inline int elem_bytes(int dtype) { return dtype == ZC_F32 ? 4 : 2; }

// ---- element conversion ---------------------------------------------------
__device__ inline float bf16_bits_to_float(uint32_t u16) { return __uint_as_float(u16 << 16); }
__device__ inline float f16_bits_to_float(uint32_t u16) {
  _Float16 h;
  uint16_t s = (uint16_t)u16;
  __builtin_memcpy(&h, &s, 2);
  return (float)h;
}

template <int DT>
__device__ inline float half_bits_to_float(uint32_t u16) {
  if constexpr (DT == ZC_BF16) return bf16_bits_to_float(u16);
  else return f16_bits_to_float(u16);
}

// Loads 8 consecutive elements starting at element offset `off` (a multiple of
// 8) of a tensor of dtype DT and widens them to float.
template <int DT>
__device__ inline void load8(const void* base, int64_t off, float (&v)[8]) {
  if constexpr (DT == ZC_F32) {
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + off);
    float4 a = p[0], b = p[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
    uint4 r = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(base) + off);
    uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = half_bits_to_float<DT>(w[i] & 0xffffu);
      v[2 * i + 1] = half_bits_to_float<DT>(w[i] >> 16);
    }
  }
}

template <int DT>
__device__ inline float load1(const void* base, int64_t off) {
  if constexpr (DT == ZC_F32) return reinterpret_cast<const float*>(base)[off];
  else return half_bits_to_float<DT>(reinterpret_cast<const uint16_t*>(base)[off]);
}

template <int DT>
__device__ inline void store1(void* base, int64_t off, float x) {
  if constexpr (DT == ZC_F32) {
    reinterpret_cast<float*>(base)[off] = x;
  } else if constexpr (DT == ZC_F16) {
    _Float16 h = (_Float16)x;
    uint16_t s;
    __builtin_memcpy(&s, &h, 2);
    reinterpret_cast<uint16_t*>(base)[off] = s;
  } else {
    // round to nearest even bf16
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
      u = 0x7fc00000u;
    } else {
      u += 0x7fffu + ((u >> 16) & 1u);
    }
    reinterpret_cast<uint16_t*>(base)[off] = (uint16_t)(u >> 16);
  }
}

// ---- order-preserving image of a float in uint32 -----------------------------
__host__ __device__ inline uint32_t float_key(float f) {
  uint32_t u;
#if defined(__HIP_DEVICE_COMPILE__)
  u = __float_as_uint(f);
#else
  memcpy(&u, &f, 4);
#endif
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline float key_float(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
  return __uint_as_float(u);
}

// ---- wave64 reductions ---------------------------------------------------------
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

}  // namespace zc

// Host-side validation shared by the entry points (defined in api.hip).
int zc_validate_tensor(const zc_tensor4* t);
int zc_validate_packed(const zc_packed* p, bool for_append);
