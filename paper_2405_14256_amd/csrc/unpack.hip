// zc_unpack: the inverse of the bit-packing, and Eq. 5's de-quantization in the
// unified form x_hat = chan_scale * tok_scale * (code - tok_zero - chan_zero).
// A plain gather kernel (one thread per 8 channels of one slot): it exists for
// callers that want canonical codes or values back, not for the hot path.
#include "zc_common.hpp"

namespace zc {

struct UnpackArgs {
  const uint8_t* codes;
  const float* tok_scale;
  const float* tok_zero;
  const float* chan_scale;   // this chunk and subset: [B, W]
  const float* chan_zero;
  int B, H, D, W, bits, layout, tokwise;
  int64_t cap;
  int begin, len;
  uint8_t* codes_out;
  float* dequant_out;
};

__global__ __launch_bounds__(256) void k_unpack(UnpackArgs a) {
  const int r = blockIdx.x, b = blockIdx.y;
  const int slot = a.begin + r;
  const int E = 32 / a.bits, TB = 4 * E;
  float ts = 1.f, tz = 0.f;
  if (a.tokwise) {
    ts = a.tok_scale[(int64_t)b * a.cap + slot];
    tz = a.tok_zero[(int64_t)b * a.cap + slot];
  }
  for (int w = threadIdx.x; w < a.W; w += blockDim.x) {
    const int h = w / a.D, c = w % a.D;
    const int64_t bh = (int64_t)b * a.H + h;
    uint32_t code;
    if (a.layout == ZC_LAYOUT_ROW) {
      const uint8_t* row = a.codes + (bh * a.cap + slot) * (a.D * a.bits / 8);
      const int bit = c * a.bits;
      code = (row[bit >> 3] >> (bit & 7)) & ((1u << a.bits) - 1u);
    } else {
      const int blk = slot / TB, s = slot % TB;
      const int tile = s >> 4, kg = (s & 15) >> 2, rr = s & 3;
      // field e with e % 4 == rr and j(e) == tile; for 2 bits j = (0, 2, 1, 3), its own inverse
      const int q = (a.bits == 2) ? ((tile & 1) * 2 + (tile >> 1)) : tile;
      const int e = 4 * q + rr;
      const uint32_t* words = reinterpret_cast<const uint32_t*>(a.codes);
      const uint32_t word = words[((bh * (a.cap / TB) + blk) * 4 + kg) * a.D + c];
      code = (word >> (a.bits * e)) & ((1u << a.bits) - 1u);
    }
    const int64_t o = ((int64_t)b * a.len + r) * a.W + w;
    if (a.codes_out) a.codes_out[o] = (uint8_t)code;
    if (a.dequant_out) {
      const float cs = a.chan_scale[(int64_t)b * a.W + w], cz = a.chan_zero[(int64_t)b * a.W + w];
      a.dequant_out[o] = cs * ts * ((float)code - tz - cz);
    }
  }
}

}  // namespace zc

using namespace zc;

extern "C" int zc_unpack(const zc_packed* p, int32_t which, int32_t chunk, uint8_t* codes_out, float* dequant_out,
                         void* stream) {
  int rc = zc_validate_packed(p, false);
  if (rc) return rc;
  if (which < 0 || which > 1 || chunk < 0 || chunk >= p->n_chunks) return ZC_ERR_INVALID_ARG;
  const int32_t* row = p->chunk_table_host + 4 * chunk;
  const int begin = row[2 * which], len = row[2 * which + 1];
  if (len == 0 || (!codes_out && !dequant_out)) return ZC_OK;
  if (p->B > 65535) return ZC_ERR_UNSUPPORTED;
  UnpackArgs a;
  a.codes = which ? p->codes_lo : p->codes_hi;
  a.tok_scale = which ? p->tok_scale_lo : p->tok_scale_hi;
  a.tok_zero = which ? p->tok_zero_lo : p->tok_zero_hi;
  const int64_t W = p->H * p->D;
  const int64_t off = ((int64_t)chunk * 2 + which) * p->B * W;
  a.chan_scale = p->chan_scale + off;
  a.chan_zero = p->chan_zero + off;
  a.B = (int)p->B; a.H = (int)p->H; a.D = (int)p->D; a.W = (int)W;
  a.bits = which ? p->bits_lo : p->bits_hi;
  a.layout = p->layout;
  a.tokwise = p->scheme != ZC_SCHEME_CHANNEL;
  a.cap = which ? p->cap_lo : p->cap_hi;
  a.begin = begin; a.len = len;
  a.codes_out = codes_out; a.dequant_out = dequant_out;
  hipLaunchKernelGGL(k_unpack, dim3((unsigned)len, (unsigned)p->B), dim3(256), 0, (hipStream_t)stream, a);
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}
