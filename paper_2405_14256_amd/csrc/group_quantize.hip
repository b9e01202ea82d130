// zc_group_quantize: groupwise quantization, the fine-grained baseline the paper compares
// its granularities with (Table 1's first row; Appendix A, Eq. A): every `group`
// consecutive channels of a token row share one (s, z) of Eq. 5.  A comparator, not part of
// the cache format: codes come out unpacked (one byte each) with their parameters and the
// de-quantized values, for error-versus-compression-ratio measurements.
#include "quant_math.hpp"

namespace zc {

struct GQArgs {
  const void* x;
  int64_t sB, sH, sL;
  int B, H, D, W, NV;
  const int32_t* idx;   // [B, n] token list, or null: tokens 0 .. n-1
  int n, bits, group;
  uint8_t* codes;       // [B, n, W] or null
  float* scale;         // [B, n, W / group] or null
  float* zero;
  float* dequant;       // [B, n, W] or null
};

// grid (n, B): one token row per workgroup, a thread per 8 channels, a group = group / 8 lanes
template <int DT>
__global__ __launch_bounds__(256) void k_group_quantize(GQArgs a) {
  const int r = blockIdx.x, b = blockIdx.y;
  const int pos = a.idx ? a.idx[(int64_t)b * a.n + r] : r;
  const int lpg = a.group / 8;                      // lanes per group: 1, 2, 4, 8 or 16
  const float qmax = (float)((1 << a.bits) - 1);
  const int nv_pad = (a.NV + 255) / 256 * 256;
  for (int v = threadIdx.x; v < nv_pad; v += 256) {
    const bool valid = v < a.NV;                    // (a group is valid or not as a whole: W is a multiple of it)
    const int w = (valid ? v : 0) * 8, h = w / a.D, c = w % a.D;
    float x8[8];
    load8<DT>(a.x, (int64_t)b * a.sB + (int64_t)h * a.sH + (int64_t)pos * a.sL + c, x8);
    float lo = x8[0], hi = x8[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) { lo = fminf(lo, x8[i]); hi = fmaxf(hi, x8[i]); }
    for (int o = 1; o < lpg; o <<= 1) { lo = fminf(lo, __shfl_xor(lo, o)); hi = fmaxf(hi, __shfl_xor(hi, o)); }
    float R = hi - lo;
    if (R == 0.f) R = qmax;                         // max == min: s := 1
    const float y = 1.0f / R;
    const float z = -rintf(refined_ratio(lo, qmax, R, y));
    const float s = R / qmax;
    if (!valid) continue;
    const int64_t o8 = ((int64_t)b * a.n + r) * a.W + w;
    float code[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float qv;
      if constexpr (DT == ZC_F32) qv = rintf(refined_ratio(x8[i], qmax, R, y)) + z;
      else qv = rintf(refined_div(x8[i] * qmax, R, y)) + z;       // x * qmax is exact for 16-bit inputs
      code[i] = __builtin_amdgcn_fmed3f(qv, 0.f, qmax);
    }
    if (a.codes) {
      uint32_t lo4 = 0, hi4 = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) { lo4 |= (uint32_t)code[i] << (8 * i); hi4 |= (uint32_t)code[4 + i] << (8 * i); }
      *reinterpret_cast<uint2*>(a.codes + o8) = make_uint2(lo4, hi4);
    }
    if (a.dequant) {
      float4* d = reinterpret_cast<float4*>(a.dequant + o8);
      d[0] = make_float4((code[0] - z) * s, (code[1] - z) * s, (code[2] - z) * s, (code[3] - z) * s);
      d[1] = make_float4((code[4] - z) * s, (code[5] - z) * s, (code[6] - z) * s, (code[7] - z) * s);
    }
    if ((v % lpg) == 0) {
      const int64_t og = ((int64_t)b * a.n + r) * (a.W / a.group) + w / a.group;
      if (a.scale) a.scale[og] = s;
      if (a.zero) a.zero[og] = z;
    }
  }
}

}  // namespace zc

using namespace zc;

extern "C" int zc_group_quantize(const zc_tensor4* x, const int32_t* idx, int64_t n, int32_t bits, int32_t group,
                                 uint8_t* codes_out, float* scale_out, float* zero_out, float* dequant_out, void* stream) {
  int rc = zc_validate_tensor(x);
  if (rc) return rc;
  if (n < 0 || n > 0x7fffffff || (!idx && n > x->L)) return ZC_ERR_INVALID_ARG;
  if (bits != 2 && bits != 4 && bits != 8) return ZC_ERR_UNSUPPORTED;
  if (group != 8 && group != 16 && group != 32 && group != 64 && group != 128) return ZC_ERR_UNSUPPORTED;
  const int64_t W = x->H * x->D;
  if (x->D % group != 0 && group % x->D != 0) return ZC_ERR_UNSUPPORTED;   // groups do not straddle heads unevenly
  if (W % group != 0) return ZC_ERR_INVALID_ARG;
  if (x->B > 65535 || W > (1 << 20)) return ZC_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(codes_out) & 7) || (reinterpret_cast<uintptr_t>(dequant_out) & 15) ||
      (reinterpret_cast<uintptr_t>(scale_out) & 3) || (reinterpret_cast<uintptr_t>(zero_out) & 3))
    return ZC_ERR_INVALID_ARG;
  if (n == 0) return ZC_OK;
  GQArgs a;
  a.x = x->ptr; a.sB = x->sB; a.sH = x->sH; a.sL = x->sL;
  a.B = (int)x->B; a.H = (int)x->H; a.D = (int)x->D; a.W = (int)W; a.NV = (int)(W / 8);
  a.idx = idx; a.n = (int)n; a.bits = bits; a.group = group;
  a.codes = codes_out; a.scale = scale_out; a.zero = zero_out; a.dequant = dequant_out;
  dim3 grid((unsigned)n, (unsigned)x->B);
  hipStream_t st = (hipStream_t)stream;
  if (x->dtype == ZC_F32) hipLaunchKernelGGL(k_group_quantize<ZC_F32>, grid, dim3(256), 0, st, a);
  else if (x->dtype == ZC_F16) hipLaunchKernelGGL(k_group_quantize<ZC_F16>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(k_group_quantize<ZC_BF16>, grid, dim3(256), 0, st, a);
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}
