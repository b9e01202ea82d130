// zc_quantize_pack: mixed-precision quantization and bit-packing of one cache
// tensor (Eq. 5, Eq. 6, Algorithm 1; the four quantizer calls of Algorithm 2).
//
// Channel statistics of a subset must be complete before any of its tokens can
// be quantized, so the work is three launches:
//   1. k_chan_stats     per-channel min / max over a tile of tokens of one
//                       subset (salient or regular), written as partials - no
//                       atomics, so the result does not depend on scheduling.
//   2. k_chan_finalize  reduces the partials and turns them once into the
//                       parameters the quantizer needs (Eq. 5's R = max - min,
//                       1/R and z per channel, or Eq. 6's c and 1/c).
//   3. k_quant_pack     a team of waves owns one "unit" of up to 8 tokens that
//                       share 32-bit words (or their 16-bit halves) in the TGROUP
//                       layout: all rows of the unit's tokens are requested at
//                       once, per-token min / max by DPP wave reduction for the
//                       tokenwise schemes, tie-exact x (2^k-1) / R, round half to
//                       even, + z, clamp, pack along channels (ROW layout) or along
//                       tokens (TGROUP layout).
// Every sweep reads 16 bytes per lane with consecutive lanes on consecutive
// addresses of a (token, head) row; the second sweep of a tensor that fits the
// 256 MB Infinity Cache does not reach HBM.
#include "zc_common.hpp"

namespace zc {

struct QPArgs {
  const void* x;
  int64_t sB, sH, sL;
  int B, H, D, W, NV;          // NV = W / 8 channel vectors per token row
  const int32_t* idx[2];       // [B, n] token lists (salient, regular)
  int n[2];                    // tokens per subset
  int begin[2];                // first arena slot of this chunk
  int bits[2];
  int64_t cap[2];
  uint8_t* codes[2];
  float* tok_scale[2];
  float* tok_zero[2];
  int32_t* pos[2];
  float* chan_scale;           // this chunk: [2, B, W]
  float* chan_zero;
  float* partial;              // workspace [B, tiles_hi + tiles_lo, W, 2] (min, max)
  float4* params;              // workspace [B, 2, W]: CHANNEL {1/R, z, R, -}, CST {1/c, -, -, -}
  int32_t* chunk_row;          // device chunk_table row to fill
  int64_t pos_offset;
  int tiles[2], TT;            // stats sweep tiling
  int units[2];                // quantize sweep: units per subset
  int scheme;
};

constexpr int kStatMaxV = 4;   // channel vectors per thread in the statistics sweep (W <= 8192)

__host__ __device__ inline int stats_tile_tokens(int64_t total_tokens) {
  int64_t tt = ceil_div64(total_tokens, 1024);
  return tt < 16 ? 16 : (tt > 64 ? 64 : (int)tt);
}

template <int DT>
__global__ __launch_bounds__(256) void k_chan_stats(QPArgs a) {
  const int b = blockIdx.y;
  int tile = blockIdx.x;
  const int sub = tile >= a.tiles[0] ? 1 : 0;
  const int gtile = tile;
  if (sub) tile -= a.tiles[0];
  const int t0 = tile * a.TT;
  const int t1 = min(t0 + a.TT, a.n[sub]);
  const int TX = blockDim.x, x = threadIdx.x;
  const int32_t* idx = a.idx[sub] + (int64_t)b * a.n[sub];

  float mn[kStatMaxV][8], mx[kStatMaxV][8];
#pragma unroll
  for (int j = 0; j < kStatMaxV; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) { mn[j][i] = INFINITY; mx[j][i] = -INFINITY; }

  for (int tb = t0; tb < t1; tb += 8) {
    // all rows of the batch are requested before any is reduced
    float vals[8][kStatMaxV][8];
    bool live[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      live[t] = tb + t < t1;
      const int64_t pos = live[t] ? idx[tb + t] : 0;
#pragma unroll
      for (int j = 0; j < kStatMaxV; ++j) {
        const int v = x + j * TX;
        if (live[t] && v < a.NV) {
          const int w = v * 8, h = w / a.D, c = w % a.D;
          load8<DT>(a.x, (int64_t)b * a.sB + (int64_t)h * a.sH + pos * a.sL + c, vals[t][j]);
        }
      }
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
      for (int j = 0; j < kStatMaxV; ++j) {
        const int v = x + j * TX;
        if (live[t] && v < a.NV) {
#pragma unroll
          for (int i = 0; i < 8; ++i) { mn[j][i] = fminf(mn[j][i], vals[t][j][i]); mx[j][i] = fmaxf(mx[j][i], vals[t][j][i]); }
        }
      }
  }
  float* out = a.partial + ((int64_t)b * (a.tiles[0] + a.tiles[1]) + gtile) * a.W * 2;
#pragma unroll
  for (int j = 0; j < kStatMaxV; ++j) {
    const int v = x + j * TX;
    if (v < a.NV) {
      float4* o4 = reinterpret_cast<float4*>(out + (int64_t)v * 16);
      o4[0] = make_float4(mn[j][0], mx[j][0], mn[j][1], mx[j][1]);
      o4[1] = make_float4(mn[j][2], mx[j][2], mn[j][3], mx[j][3]);
      o4[2] = make_float4(mn[j][4], mx[j][4], mn[j][5], mx[j][5]);
      o4[3] = make_float4(mn[j][6], mx[j][6], mn[j][7], mx[j][7]);
    }
  }
}

// N / R from the correctly rounded reciprocal y = 1/R with one residual
// correction.  When the true quotient is representable (in particular an exact
// tie n + 1/2, frequent with 16-bit inputs) the result is that quotient, so the
// round-half-even that follows sees the tie.
__device__ inline float refined_div(float N, float R, float y) {
  const float q0 = N * y;
  const float r = fmaf(-q0, R, N);
  return fmaf(r, y, q0);
}
// x * qmax / R with the rounding error of the product x * qmax carried along, so
// that ties stay exact for 24-bit x too (e.g. the minimum of a token row whose
// maximum is its mirror image: exactly -qmax / 2).
__device__ inline float refined_ratio(float x, float qmax, float R, float y) {
  const float nh = x * qmax;
  const float nl = fmaf(x, qmax, -nh);
  const float q0 = nh * y;
  const float r = fmaf(-q0, R, nh) + nl;
  return fmaf(r, y, q0);
}

// grid (ceil(W / 64), 2 subsets, B), block (64 channels, 4 tile lanes)
__global__ __launch_bounds__(256) void k_chan_finalize(QPArgs a) {
  __shared__ float smn[4][64], smx[4][64];
  const int cx = threadIdx.x, ty = threadIdx.y;
  const int w = blockIdx.x * 64 + cx, sub = blockIdx.y, b = blockIdx.z;
  const int n = a.n[sub];
  const float qmax = (float)((1 << a.bits[sub]) - 1);
  float lo = INFINITY, hi = -INFINITY;
  if (w < a.W && n > 0 && a.scheme != ZC_SCHEME_TOKEN) {
    const int tbeg = sub ? a.tiles[0] : 0, tcnt = a.tiles[sub];
    const float* p = a.partial + ((int64_t)b * (a.tiles[0] + a.tiles[1]) + tbeg) * a.W * 2 + (int64_t)w * 2;
#pragma unroll 4
    for (int t = ty; t < tcnt; t += 4) {
      const float2 v = *reinterpret_cast<const float2*>(p + (int64_t)t * a.W * 2);
      lo = fminf(lo, v.x); hi = fmaxf(hi, v.y);
    }
  }
  smn[ty][cx] = lo; smx[ty][cx] = hi;
  __syncthreads();
  if (ty == 0 && w < a.W) {
    lo = fminf(fminf(smn[0][cx], smn[1][cx]), fminf(smn[2][cx], smn[3][cx]));
    hi = fmaxf(fmaxf(smx[0][cx], smx[1][cx]), fmaxf(smx[2][cx], smx[3][cx]));
    float cs = 1.f, cz = 0.f;
    float4 prm = make_float4(1.f, 0.f, 1.f, 0.f);
    if (n > 0 && a.scheme == ZC_SCHEME_CST) {
      float c = sqrtf(fmaxf(fabsf(lo), fabsf(hi)));       // Eq. 6
      if (c == 0.f) c = 1.f;
      cs = c;
      prm.x = 1.f / c;
    } else if (n > 0 && a.scheme == ZC_SCHEME_CHANNEL) {
      float R = hi - lo;                                     // Eq. 5: s = R / (2^k - 1)
      if (R == 0.f) R = qmax;                                // max == min: s := 1
      cs = R / qmax;
      cz = -rintf(refined_ratio(lo, qmax, R, 1.f / R));
      prm = make_float4(1.f / R, cz, R, 0.f);
    }
    const int64_t o = (int64_t)(sub * a.B + b) * a.W + w;
    a.chan_scale[o] = cs;
    a.chan_zero[o] = cz;
    a.params[(int64_t)(b * 2 + sub) * a.W + w] = prm;
  }
  if (blockIdx.x == 0 && sub == 0 && b == 0 && cx == 0 && ty == 0) {
    a.chunk_row[0] = a.begin[0]; a.chunk_row[1] = a.n[0];
    a.chunk_row[2] = a.begin[1]; a.chunk_row[3] = a.n[1];
  }
}

// ---- wave64 all-reduce through DPP (no LDS traffic) --------------------------------
template <int CTRL, int ROW_MASK>
__device__ inline float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
template <bool IS_MAX>
__device__ inline float wave_allreduce(float v) {
  auto op = [](float x, float y) { return IS_MAX ? fmaxf(x, y) : fminf(x, y); };
  v = op(v, dpp_move<0xB1, 0xF>(v));    // quad_perm [1,0,3,2]
  v = op(v, dpp_move<0x4E, 0xF>(v));    // quad_perm [2,3,0,1]
  v = op(v, dpp_move<0x141, 0xF>(v));   // row_half_mirror
  v = op(v, dpp_move<0x140, 0xF>(v));   // row_mirror: every lane of a 16-lane row has the row result
  v = op(v, dpp_move<0x142, 0xA>(v));   // row_bcast15 into rows 1 and 3
  v = op(v, dpp_move<0x143, 0xC>(v));   // row_bcast31 into rows 2 and 3: lane 63 has the total
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ inline int tile_of_field_group(int bits, int jf) {
  // Slot tile (16 slots) addressed by field group jf of a TGROUP word.
  return (bits == 2) ? ((jf & 1) * 2 + (jf >> 1)) : jf;
}

constexpr int kVPT = 1;  // channel vectors (8 channels each) per thread in the quantize sweep

template <int DT, int BITS, int LAYOUT, bool TOKWISE>
__device__ inline void quant_unit(const QPArgs& a, int sub, int u, int b, float (*red)[8][16]) {
  constexpr int E = 32 / BITS;                       // code fields per 32-bit TGROUP word
  constexpr int TU = E < 8 ? E : 8;                  // tokens per unit: a word, or half of a 2-bit word
  constexpr int UW = E / TU;                         // units that share a word
  constexpr int TBAT = (DT == ZC_F32) ? 4 : TU;      // tokens requested at once
  constexpr int NBAT = TU / TBAT;
  constexpr int TB = 4 * E;                          // slots per TGROUP block
  constexpr float QMAX = (float)((1 << BITS) - 1);
  constexpr int RAW = (DT == ZC_F32) ? 2 : 1;        // 16-byte loads per channel vector

  const int blk = u / (4 * UW), kg = (u / UW) & 3, hf = u % UW;     // unit = (block, k-group, part of the word)
  const int n = a.n[sub];
  const int TX = blockDim.x, x = threadIdx.x;
  const int lane = x & 63, wave = x >> 6, nwaves = TX >> 6;
  const int32_t* idx = a.idx[sub] + (int64_t)b * n;

  // parameters of the channels this thread owns
  float p0[kVPT][8], p1[kVPT][8], p2[kVPT][8];
  bool vvalid[kVPT];
  int64_t xoff[kVPT];
#pragma unroll
  for (int j = 0; j < kVPT; ++j) {
    const int v = x + j * TX;
    vvalid[j] = v < a.NV;
    const int w = (vvalid[j] ? v : 0) * 8, h = w / a.D, c = w % a.D;
    xoff[j] = (int64_t)b * a.sB + (int64_t)h * a.sH + c;
    const float4* pp = a.params + (int64_t)(b * 2 + sub) * a.W + w;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float4 t = pp[i];
      p0[j][i] = t.x; p1[j][i] = t.y; p2[j][i] = t.z;
    }
  }

  uint32_t words[kVPT][8];
#pragma unroll
  for (int j = 0; j < kVPT; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) words[j][i] = 0u;

#pragma unroll
  for (int bt = 0; bt < NBAT; ++bt) {
    // slot (relative to the chunk) and source position of the batch's tokens
    int rel[TBAT];
    uint4 raw[TBAT][kVPT][RAW];
#pragma unroll
    for (int t = 0; t < TBAT; ++t) {
      const int e = hf * TU + bt * TBAT + t;
      rel[t] = blk * TB + 16 * tile_of_field_group(BITS, e >> 2) + 4 * kg + (e & 3);
      const bool tv = rel[t] < n;
      const int64_t pos = tv ? idx[rel[t]] : 0;
#pragma unroll
      for (int j = 0; j < kVPT; ++j)
#pragma unroll
        for (int r = 0; r < RAW; ++r) {
          raw[t][j][r] = make_uint4(0u, 0u, 0u, 0u);
          if (tv && vvalid[j]) {
            const char* src = reinterpret_cast<const char*>(a.x) + (xoff[j] + pos * a.sL) * (DT == ZC_F32 ? 4 : 2) + 16 * r;
            raw[t][j][r] = *reinterpret_cast<const uint4*>(src);
          }
        }
    }
    auto widen = [&](int t, int j, float (&v)[8]) {
      if constexpr (DT == ZC_F32) {
        v[0] = __uint_as_float(raw[t][j][0].x); v[1] = __uint_as_float(raw[t][j][0].y);
        v[2] = __uint_as_float(raw[t][j][0].z); v[3] = __uint_as_float(raw[t][j][0].w);
        v[4] = __uint_as_float(raw[t][j][RAW - 1].x); v[5] = __uint_as_float(raw[t][j][RAW - 1].y);
        v[6] = __uint_as_float(raw[t][j][RAW - 1].z); v[7] = __uint_as_float(raw[t][j][RAW - 1].w);
      } else {
        const uint32_t w4[4] = {raw[t][j][0].x, raw[t][j][0].y, raw[t][j][0].z, raw[t][j][0].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[2 * i] = half_bits_to_float<DT>(w4[i] & 0xffffu);
          v[2 * i + 1] = half_bits_to_float<DT>(w4[i] >> 16);
        }
      }
    };

    float rng[TBAT], inv_r[TBAT], zt[TBAT];
    if constexpr (TOKWISE) {
      float tmin[TBAT], tmax[TBAT];
#pragma unroll
      for (int t = 0; t < TBAT; ++t) {
        float lo = INFINITY, hi = -INFINITY;
#pragma unroll
        for (int j = 0; j < kVPT; ++j) {
          if (vvalid[j]) {
            float v[8];
            widen(t, j, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) { const float y = v[i] * p0[j][i]; lo = fminf(lo, y); hi = fmaxf(hi, y); }
          }
        }
        tmin[t] = wave_allreduce<false>(lo);
        tmax[t] = wave_allreduce<true>(hi);
      }
      if (nwaves > 1) {
        __syncthreads();
        if (lane == 0) {
#pragma unroll
          for (int t = 0; t < TBAT; ++t) { red[0][t][wave] = tmin[t]; red[1][t][wave] = tmax[t]; }
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < TBAT; ++t) {
          float lo = red[0][t][0], hi = red[1][t][0];
          for (int w = 1; w < nwaves; ++w) { lo = fminf(lo, red[0][t][w]); hi = fmaxf(hi, red[1][t][w]); }
          tmin[t] = lo; tmax[t] = hi;
        }
      }
#pragma unroll
      for (int t = 0; t < TBAT; ++t) {
        float R = tmax[t] - tmin[t];
        if (R == 0.f) R = QMAX;                 // max == min: s := 1
        const float y = 1.f / R;
        const float z = -rintf(refined_ratio(tmin[t], QMAX, R, y));
        rng[t] = R; inv_r[t] = y; zt[t] = z;
        if (x == 0 && rel[t] < n) {
          const int64_t o = (int64_t)b * a.cap[sub] + a.begin[sub] + rel[t];
          a.tok_scale[sub][o] = R / QMAX;
          a.tok_zero[sub][o] = z;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < TBAT; ++t) {
      const bool tv = rel[t] < n;
      if (x == 0 && tv && a.pos[sub])
        a.pos[sub][(int64_t)b * a.cap[sub] + a.begin[sub] + rel[t]] = (int32_t)(idx[rel[t]] + a.pos_offset);
#pragma unroll
      for (int j = 0; j < kVPT; ++j) {
        if (!vvalid[j]) continue;
        float v[8];
        widen(t, j, v);
        uint32_t code[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          // Eq. 5: round(x / s) first, then + z, then clip
          float q;
          if constexpr (TOKWISE) q = rintf(refined_ratio(v[i] * p0[j][i], QMAX, rng[t], inv_r[t])) + zt[t];
          else if constexpr (DT == ZC_F32) q = rintf(refined_ratio(v[i], QMAX, p2[j][i], p0[j][i])) + p1[j][i];
          else q = rintf(refined_div(v[i] * QMAX, p2[j][i], p0[j][i])) + p1[j][i];   // x * qmax is exact
          q = __builtin_amdgcn_fmed3f(q, 0.f, QMAX);
          code[i] = tv ? (uint32_t)q : 0u;
        }
        if constexpr (LAYOUT == ZC_LAYOUT_TGROUP) {
          const int e = bt * TBAT + t;             // field inside this unit's part of the word
#pragma unroll
          for (int i = 0; i < 8; ++i) words[j][i] |= code[i] << (BITS * e);
        } else if (tv) {
          const int w = (x + j * TX) * 8, h = w / a.D, c = w % a.D;
          const int64_t slot = a.begin[sub] + rel[t];
          uint8_t* row = a.codes[sub] + (((int64_t)b * a.H + h) * a.cap[sub] + slot) * (a.D * BITS / 8) + c * BITS / 8;
          if constexpr (BITS == 8) {
            uint2 o;
            o.x = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
            o.y = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
            *reinterpret_cast<uint2*>(row) = o;
          } else if constexpr (BITS == 4) {
            uint32_t o = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) o |= code[i] << (4 * i);
            *reinterpret_cast<uint32_t*>(row) = o;
          } else {
            uint32_t o = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) o |= code[i] << (2 * i);
            *reinterpret_cast<uint16_t*>(row) = (uint16_t)o;
          }
        }
      }
    }
  }
  if constexpr (LAYOUT == ZC_LAYOUT_TGROUP) {
#pragma unroll
    for (int j = 0; j < kVPT; ++j) {
      if (!vvalid[j]) continue;
      const int w = (x + j * TX) * 8, h = w / a.D, c = w % a.D;
      const int64_t nblk = a.cap[sub] / TB;
      const int64_t gblk = a.begin[sub] / TB + blk;
      uint32_t* dst = reinterpret_cast<uint32_t*>(a.codes[sub]) +
                      ((((int64_t)b * a.H + h) * nblk + gblk) * 4 + kg) * a.D + c;
      if constexpr (UW == 1) {
        reinterpret_cast<uint4*>(dst)[0] = make_uint4(words[j][0], words[j][1], words[j][2], words[j][3]);
        reinterpret_cast<uint4*>(dst)[1] = make_uint4(words[j][4], words[j][5], words[j][6], words[j][7]);
      } else {
        // this unit fills 16 bits of each word; the other half belongs to a neighbouring workgroup
        uint16_t* d16 = reinterpret_cast<uint16_t*>(dst) + hf;
#pragma unroll
        for (int i = 0; i < 8; ++i) d16[2 * i] = (uint16_t)words[j][i];
      }
    }
  }
}

template <int DT, int LAYOUT, bool TOKWISE>
__global__ __launch_bounds__(1024) void k_quant_pack(QPArgs a) {
  __shared__ float red[2][8][16];    // cross-wave min / max of a batch of tokens (<= 16 waves)
  const int b = blockIdx.y;
  int u = blockIdx.x;
  const int sub = u >= a.units[0] ? 1 : 0;
  if (sub) u -= a.units[0];
  const int bits = a.bits[sub];
  if (bits == 4) quant_unit<DT, 4, LAYOUT, TOKWISE>(a, sub, u, b, red);
  else if (bits == 2) quant_unit<DT, 2, LAYOUT, TOKWISE>(a, sub, u, b, red);
  else quant_unit<DT, 8, LAYOUT, TOKWISE>(a, sub, u, b, red);
}

template <int DT>
static void launch_qp(const QPArgs& a, int layout, bool tokwise, dim3 grid, dim3 block, hipStream_t st) {
  if (layout == ZC_LAYOUT_ROW) {
    if (tokwise) hipLaunchKernelGGL((k_quant_pack<DT, ZC_LAYOUT_ROW, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((k_quant_pack<DT, ZC_LAYOUT_ROW, false>), grid, block, 0, st, a);
  } else {
    if (tokwise) hipLaunchKernelGGL((k_quant_pack<DT, ZC_LAYOUT_TGROUP, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((k_quant_pack<DT, ZC_LAYOUT_TGROUP, false>), grid, block, 0, st, a);
  }
}

static int64_t stats_tiles(int64_t B, int64_t n_tokens, int* TT_out) {
  const int TT = stats_tile_tokens(B * n_tokens);
  if (TT_out) *TT_out = TT;
  return ceil_div64(n_tokens, TT) + 1;     // two subsets: at most one extra ragged tile
}

}  // namespace zc

using namespace zc;

extern "C" size_t zc_quantize_pack_workspace(int64_t B, int64_t H, int64_t L, int64_t D) {
  if (B <= 0 || H <= 0 || D <= 0 || L < 0) return 0;
  const int64_t W = H * D;
  const size_t params = (size_t)align_up64(B * 2 * W * (int64_t)sizeof(float4), 256);
  const size_t partial = (size_t)B * stats_tiles(B, L, nullptr) * W * 2 * sizeof(float);
  return params + partial;
}

extern "C" int zc_quantize_pack(const zc_tensor4* x, const int32_t* salient_idx, int64_t k,
                                const int32_t* regular_idx, int64_t n_reg, int64_t pos_offset,
                                zc_packed* out, void* ws, size_t ws_bytes, void* stream) {
  int rc = zc_validate_tensor(x);
  if (rc) return rc;
  rc = zc_validate_packed(out, true);
  if (rc) return rc;
  if (k < 0 || n_reg < 0 || k > x->L || n_reg > x->L || k + n_reg > x->L) return ZC_ERR_INVALID_ARG;
  if ((k > 0 && !salient_idx) || (n_reg > 0 && !regular_idx)) return ZC_ERR_INVALID_ARG;
  if (x->B != out->B || x->H != out->H || x->D != out->D) return ZC_ERR_INVALID_ARG;
  const int64_t W = x->H * x->D;
  if (W / 8 > kStatMaxV * 256 || W / 8 > kVPT * 1024) return ZC_ERR_UNSUPPORTED;
  if (x->B > 65535) return ZC_ERR_UNSUPPORTED;
  if (out->n_chunks >= out->max_chunks) return ZC_ERR_CAPACITY;
  const int64_t end_hi = align_up64(out->n_hi + k, ZC_SLOT_ALIGN);
  const int64_t end_lo = align_up64(out->n_lo + n_reg, ZC_SLOT_ALIGN);
  if (end_hi > out->cap_hi || end_lo > out->cap_lo) return ZC_ERR_CAPACITY;
  const size_t need = zc_quantize_pack_workspace(x->B, x->H, k + n_reg, x->D);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15)) return ZC_ERR_WORKSPACE;

  hipStream_t st = (hipStream_t)stream;
  QPArgs a;
  a.x = x->ptr; a.sB = x->sB; a.sH = x->sH; a.sL = x->sL;
  a.B = (int)x->B; a.H = (int)x->H; a.D = (int)x->D; a.W = (int)W; a.NV = (int)(W / 8);
  a.idx[0] = salient_idx; a.idx[1] = regular_idx;
  a.n[0] = (int)k; a.n[1] = (int)n_reg;
  a.begin[0] = (int)out->n_hi; a.begin[1] = (int)out->n_lo;
  a.bits[0] = out->bits_hi; a.bits[1] = out->bits_lo;
  a.cap[0] = out->cap_hi; a.cap[1] = out->cap_lo;
  a.codes[0] = out->codes_hi; a.codes[1] = out->codes_lo;
  a.tok_scale[0] = out->tok_scale_hi; a.tok_zero[0] = out->tok_zero_hi;
  a.tok_scale[1] = out->tok_scale_lo; a.tok_zero[1] = out->tok_zero_lo;
  a.pos[0] = out->pos_hi; a.pos[1] = out->pos_lo;
  const int64_t chunk_off = (int64_t)out->n_chunks * 2 * x->B * W;
  a.chan_scale = out->chan_scale + chunk_off;
  a.chan_zero = out->chan_zero + chunk_off;
  a.params = reinterpret_cast<float4*>(ws);
  a.partial = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(ws) + align_up64(x->B * 2 * W * (int64_t)sizeof(float4), 256));
  a.chunk_row = out->chunk_table + 4 * out->n_chunks;
  a.pos_offset = pos_offset;
  a.scheme = out->scheme;
  int TT;
  stats_tiles(x->B, k + n_reg, &TT);
  a.TT = TT;
  a.tiles[0] = (int)ceil_div64(k, TT);
  a.tiles[1] = (int)ceil_div64(n_reg, TT);
  // units of min(32 / bits, 8) tokens; a TGROUP block holds 4 * (32 / bits) slots
  a.units[0] = (int)ceil_div64(k, 4 * (32 / out->bits_hi)) * (out->bits_hi == 2 ? 8 : 4);
  a.units[1] = (int)ceil_div64(n_reg, 4 * (32 / out->bits_lo)) * (out->bits_lo == 2 ? 8 : 4);

  // ---- sweep 1: channel statistics (partials) -----------------------------------
  if (out->scheme != ZC_SCHEME_TOKEN && a.tiles[0] + a.tiles[1] > 0) {
    const int TX = a.NV >= 256 ? 256 : (int)align_up64(a.NV, 64);
    dim3 grid((unsigned)(a.tiles[0] + a.tiles[1]), (unsigned)x->B), block(TX);
    if (x->dtype == ZC_F32) hipLaunchKernelGGL(k_chan_stats<ZC_F32>, grid, block, 0, st, a);
    else if (x->dtype == ZC_F16) hipLaunchKernelGGL(k_chan_stats<ZC_F16>, grid, block, 0, st, a);
    else hipLaunchKernelGGL(k_chan_stats<ZC_BF16>, grid, block, 0, st, a);
    ZC_LAUNCH_CHECK();
  }
  // ---- parameters (also for empty subsets and the tokenwise scheme: defaults) ------
  hipLaunchKernelGGL(k_chan_finalize, dim3((unsigned)ceil_div64(W, 64), 2, (unsigned)x->B), dim3(64, 4), 0, st, a);
  ZC_LAUNCH_CHECK();
  // ---- sweep 2: quantize + pack ---------------------------------------------------
  if (a.units[0] + a.units[1] > 0) {
    const bool tokwise = out->scheme != ZC_SCHEME_CHANNEL;
    const int TXq = (int)align_up64(ceil_div64(a.NV, kVPT), 64);
    dim3 grid((unsigned)(a.units[0] + a.units[1]), (unsigned)x->B), block(TXq);
    if (x->dtype == ZC_F32) launch_qp<ZC_F32>(a, out->layout, tokwise, grid, block, st);
    else if (x->dtype == ZC_F16) launch_qp<ZC_F16>(a, out->layout, tokwise, grid, block, st);
    else launch_qp<ZC_BF16>(a, out->layout, tokwise, grid, block, st);
    ZC_LAUNCH_CHECK();
  }

  int32_t* row = out->chunk_table_host + 4 * out->n_chunks;
  row[0] = (int32_t)out->n_hi; row[1] = (int32_t)k; row[2] = (int32_t)out->n_lo; row[3] = (int32_t)n_reg;
  out->n_hi = end_hi;
  out->n_lo = end_lo;
  out->n_chunks += 1;
  return ZC_OK;
}
