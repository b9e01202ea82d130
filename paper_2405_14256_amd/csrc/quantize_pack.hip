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
//   3. k_quant_pack     a team of waves (one thread per 8 channels) owns one to
//                       four word groups of a TGROUP block - the 32 / bits tokens
//                       whose codes share 32-bit words - and walks them in
//                       batches of 8 tokens, requesting batch i + 1 before it
//                       reduces and quantizes batch i: per-token range by DPP wave
//                       reduction (+ LDS across the team's waves) for the tokenwise
//                       schemes, tie-exact x (2^k-1) / R for the zero points and the
//                       channelwise codes, round half to even, + z, clamp, pack along
//                       channels (ROW layout) or along tokens (TGROUP layout).
// Every sweep reads 16 bytes per lane with consecutive lanes on consecutive
// addresses of a (token, head) row; the second sweep of a tensor that fits the
// 256 MB Infinity Cache does not reach HBM.
#include "quant_math.hpp"

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
  int units[2];                // quantize sweep: word groups per subset (4 per TGROUP block)
  int upw, wgs[2];             // word groups per workgroup (1, 2 or 4: divides a block), workgroups per subset
  int scheme;
};

constexpr int kStatThreads = 256;   // channel vectors (8 channels) per workgroup of the statistics sweep
constexpr int kStatBatch = 8;       // token rows requested at once

__host__ __device__ inline int stats_tile_tokens(int64_t total_tokens) {
  int64_t tt = ceil_div64(total_tokens, 1024);
  return tt < 16 ? 16 : (tt > 64 ? 64 : (int)tt);
}

// grid (tiles, B, ceil(NV / 256)): a workgroup reduces 256 channel vectors over a
// tile of tokens of one subset; a thread owns one vector (8 channels).
struct QPPair { QPArgs t[2]; };   // keys and values of one cache, compressed by the same launches

template <int DT>
__device__ inline void chan_stats_body(const QPArgs& a, int tile, int b, int zchunk) {
  constexpr int RAW = (DT == ZC_F32) ? 2 : 1;        // 16-byte loads per channel vector
  const int sub = tile >= a.tiles[0] ? 1 : 0;
  const int gtile = tile;
  if (sub) tile -= a.tiles[0];
  const int t0 = tile * a.TT;
  const int t1 = min(t0 + a.TT, a.n[sub]);
  const int v = zchunk * kStatThreads + threadIdx.x;
  if (v >= a.NV) return;
  const int32_t* idx = a.idx[sub] + (int64_t)b * a.n[sub];
  const int w = v * 8, h = w / a.D, c = w % a.D;
  const char* base = reinterpret_cast<const char*>(a.x) + ((int64_t)b * a.sB + (int64_t)h * a.sH + c) * (DT == ZC_F32 ? 4 : 2);
  const int64_t row_bytes = a.sL * (DT == ZC_F32 ? 4 : 2);

  float mn[8], mx[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { mn[i] = INFINITY; mx[i] = -INFINITY; }

  for (int tb = t0; tb < t1; tb += kStatBatch) {
    // all rows of the batch are requested before any is reduced; rows past the
    // end repeat the last one (min / max do not care)
    uint4 raw[kStatBatch][RAW];
#pragma unroll
    for (int t = 0; t < kStatBatch; ++t) {
      const int64_t pos = idx[min(tb + t, t1 - 1)];
      const uint4* src = reinterpret_cast<const uint4*>(base + pos * row_bytes);
#pragma unroll
      for (int r = 0; r < RAW; ++r) raw[t][r] = src[r];
    }
#pragma unroll
    for (int t = 0; t < kStatBatch; ++t) {
      float x8[8];
      if constexpr (DT == ZC_F32) {
        x8[0] = __uint_as_float(raw[t][0].x); x8[1] = __uint_as_float(raw[t][0].y);
        x8[2] = __uint_as_float(raw[t][0].z); x8[3] = __uint_as_float(raw[t][0].w);
        x8[4] = __uint_as_float(raw[t][RAW - 1].x); x8[5] = __uint_as_float(raw[t][RAW - 1].y);
        x8[6] = __uint_as_float(raw[t][RAW - 1].z); x8[7] = __uint_as_float(raw[t][RAW - 1].w);
      } else {
        const uint32_t w4[4] = {raw[t][0].x, raw[t][0].y, raw[t][0].z, raw[t][0].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          x8[2 * i] = half_bits_to_float<DT>(w4[i] & 0xffffu);
          x8[2 * i + 1] = half_bits_to_float<DT>(w4[i] >> 16);
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) { mn[i] = fminf(mn[i], x8[i]); mx[i] = fmaxf(mx[i], x8[i]); }
    }
  }
  float* out = a.partial + ((int64_t)b * (a.tiles[0] + a.tiles[1]) + gtile) * a.W * 2;
  float4* o4 = reinterpret_cast<float4*>(out + (int64_t)v * 16);
  o4[0] = make_float4(mn[0], mx[0], mn[1], mx[1]);
  o4[1] = make_float4(mn[2], mx[2], mn[3], mx[3]);
  o4[2] = make_float4(mn[4], mx[4], mn[5], mx[5]);
  o4[3] = make_float4(mn[6], mx[6], mn[7], mx[7]);
}

template <int DT>
__global__ __launch_bounds__(kStatThreads) void k_chan_stats(QPArgs a) {
  chan_stats_body<DT>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}
// both tensors of a cache: grid.x = tiles of the first + tiles of the second
template <int DT>
__global__ __launch_bounds__(kStatThreads) void k_chan_stats_kv(QPPair p) {
  const int nt = p.t[0].tiles[0] + p.t[0].tiles[1];
  const int which = (int)blockIdx.x >= nt ? 1 : 0;
  const QPArgs& a = which ? p.t[1] : p.t[0];
  if (a.scheme == ZC_SCHEME_TOKEN) return;           // plain tokenwise: no channel statistics
  chan_stats_body<DT>(a, blockIdx.x - which * nt, blockIdx.y, blockIdx.z);
}

// grid (ceil(W / 64), 2 subsets, B), block (64 channels, 4 tile lanes)
__device__ inline void chan_finalize_body(const QPArgs& a, int sub, float (*smn)[64], float (*smx)[64]) {
  const int cx = threadIdx.x, ty = threadIdx.y;
  const int w = blockIdx.x * 64 + cx, b = blockIdx.z;
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
__global__ __launch_bounds__(256) void k_chan_finalize(QPArgs a) {
  __shared__ float smn[4][64], smx[4][64];
  chan_finalize_body(a, blockIdx.y, smn, smx);
}
// both tensors of a cache: grid.y = 2 subsets of the first, then of the second
__global__ __launch_bounds__(256) void k_chan_finalize_kv(QPPair p) {
  __shared__ float smn[4][64], smx[4][64];
  const int which = blockIdx.y >> 1;
  chan_finalize_body(which ? p.t[1] : p.t[0], blockIdx.y & 1, smn, smx);
}

// ---- minima of N values over a wave at once -----------------------------------------
// Every lane brings N = 8 or 16 values (value j + N / 2 paired with value j in the first
// step); afterwards lane l holds the minimum over the wave of value number value_of_lane<N>(l).  Each step halves the values a lane still
// carries: two lanes that differ in one bit of the lane number exchange the half the
// other one keeps and reduce the half they keep themselves, so the whole reduction is
// about 2 N instructions instead of 6 per value.  Lane bit 4 and 5 (rows, halves of the
// wave) go through the register-pair swaps, bit 3 and 2 through DPP with a bank mask
// (one instruction per kept half), the last one or two steps (bits 0, 1, and 2 when
// N = 8) reduce the one remaining value over all lanes of a group.  All 64 lanes must
// be active.
__device__ inline float swap_min_rows(float a, float b) {      // rows 0, 2: a over the row pair; rows 1, 3: b
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return fminf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float swap_min_halves(float a, float b) {    // lanes 0-31: a over both halves; lanes 32-63: b
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return fminf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// (the two wait states are what a DPP read of a register needs after the vector
// instruction that wrote it; the compiler does not look inside the block)
__device__ inline float dpp_min_xor8_keep(float a, float b) {  // lanes 0-7 of a row: a; lanes 8-15: b
  asm volatile("s_nop 1\n\t"
               "v_min_f32_dpp %0, %0, %0 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
               "v_min_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0xc" : "+v"(a) : "v"(b));
  return a;
}
__device__ inline float dpp_min_mirror8_keep(float a, float b) {  // lanes 0-3 of every eight: a; lanes 4-7: b
  asm volatile("s_nop 1\n\t"
               "v_min_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0x5\n\t"
               "v_min_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xa" : "+v"(a) : "v"(b));
  return a;
}
__device__ inline float dpp_min_mirror8(float a) {
  asm volatile("s_nop 1\n\tv_min_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf" : "+v"(a));
  return a;
}
__device__ inline float dpp_min_quad(float a) {
  asm volatile("s_nop 1\n\t"
               "v_min_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
               "s_nop 1\n\t"
               "v_min_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "+v"(a));
  return a;
}
template <int N>
__device__ inline int value_of_lane(int lane) {
  const int b2 = (lane >> 2) & 1, b3 = (lane >> 3) & 1, b4 = (lane >> 4) & 1, b5 = (lane >> 5) & 1;
  return N == 16 ? 8 * b4 + 4 * b5 + 2 * b3 + b2 : 4 * b4 + 2 * b5 + b3;
}
// v[j] holds value j in the even rows of the wave and value j + N / 2 in the odd rows,
// already reduced over each row pair (swap_min_rows): the remaining steps.
template <int N>
__device__ inline float wave_min_rest(float (&v)[N / 2]) {
  static_assert(N == 8 || N == 16, "two values (min, -max) for 4 or 8 tokens");
#pragma unroll
  for (int j = 0; j < N / 4; ++j) v[j] = swap_min_halves(v[j], v[j + N / 4]);
#pragma unroll
  for (int j = 0; j < N / 8; ++j) v[j] = dpp_min_xor8_keep(v[j], v[j + N / 8]);
  float r;
  if constexpr (N == 16) r = dpp_min_mirror8_keep(v[0], v[1]);
  else r = dpp_min_mirror8(v[0]);
  return dpp_min_quad(r);
}

__device__ inline int tile_of_field_group(int bits, int jf) {
  // Slot tile (16 slots) addressed by field group jf of a TGROUP word.
  return (bits == 2) ? ((jf & 1) * 2 + (jf >> 1)) : jf;
}

constexpr int kVPT = 1;  // channel vectors (8 channels each) per thread in the quantize sweep

// The quantize sweep of one workgroup: `ng` consecutive word groups of one TGROUP
// block.  A word group is the 32 / bits tokens whose codes share 32-bit words in
// the TGROUP layout (block blk, k-group kg); it is processed in batches of up to
// 8 tokens, a thread owning 8 channels of every token.  The rows of batch i + 1
// are requested before batch i is reduced and quantized.
//   tokenwise schemes: x' = x / c is kept in registers between the range pass and
//   the quantize pass; the per-token range goes through a DPP wave reduction,
//   then (teams of several waves) through LDS; lanes 0..7 then compute the
//   parameters of tokens 0..7 of the batch, once, and broadcast them.
//   codes are assembled in float: sum of code * 2^(bits * position) over a 16-bit
//   group is exact in fp32, so packing costs one FMA per code.
template <int DT, int BITS, int LAYOUT, bool TOKWISE, bool EXACT, bool PIPE>
__device__ inline void quant_units(const QPArgs& a, int sub, int g0, int ng, int b, float (*red)[16][16], int32_t* sidx) {
  constexpr int E = 32 / BITS;                       // tokens of a word group
  constexpr int TBAT = E < 8 ? E : 8;                // tokens per batch
  constexpr int NBAT = E / TBAT;                     // batches per word group
  constexpr int TB = 4 * E;                          // slots per TGROUP block
  constexpr int FPG = 16 / BITS;                     // code fields per 16-bit group
  constexpr float QMAX = (float)((1 << BITS) - 1);
  constexpr int RAW = (DT == ZC_F32) ? 2 : 1;        // 16-byte loads per channel vector
  constexpr int ESZ = (DT == ZC_F32) ? 4 : 2;

  const int n = a.n[sub];
  const int TX = blockDim.x, x = threadIdx.x;
  const int lane = x & 63, wave = x >> 6, nwaves = TX >> 6;
  const int32_t* idx = a.idx[sub] + (int64_t)b * n;
  const int blk = g0 >> 2;                           // every word group of this workgroup lies in this block

  // source positions of the block's slots (-1 past the end of the subset)
  if (x < TB) { const int rel = blk * TB + x; sidx[x] = rel < n ? idx[rel] : -1; }

  // parameters of the channels this thread owns
  // (the channelwise scheme needs no reduction over a token row, so its launches cut
  // the row into chunks of blockDim.x vectors along grid.z)
  const int vec = (int)blockIdx.z * TX + x;
  const bool vvalid = vec < a.NV;
  const int w = (vvalid ? vec : 0) * 8, h = w / a.D, c = w % a.D;
  const char* xbase = reinterpret_cast<const char*>(a.x) + ((int64_t)b * a.sB + (int64_t)h * a.sH + c) * ESZ;
  const int64_t row_bytes = a.sL * ESZ;
  float p0[8], p1[8], p2[8];
  {
    const float4* pp = a.params + (int64_t)(b * 2 + sub) * a.W + w;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float4 t = pp[i];
      p0[i] = t.x; p1[i] = t.y; p2[i] = t.z;
    }
  }
  __syncthreads();

  struct Batch { uint4 raw[TBAT][RAW]; };
  // batch q of the workgroup: word group g0 + q / NBAT, tokens (q % NBAT) * TBAT + t of it
  auto slot_of = [&](int q, int t) {                 // slot inside the block
    const int kg = (g0 + q / NBAT) & 3;
    const int e = (q % NBAT) * TBAT + t;
    return 16 * tile_of_field_group(BITS, e >> 2) + 4 * kg + (e & 3);
  };
  auto issue = [&](int q, Batch& bt) {
#pragma unroll
    for (int t = 0; t < TBAT; ++t) {
      const int pos = sidx[slot_of(q, t)];
#pragma unroll
      for (int r = 0; r < RAW; ++r) {
        bt.raw[t][r] = make_uint4(0u, 0u, 0u, 0u);
        if (pos >= 0 && vvalid) bt.raw[t][r] = *reinterpret_cast<const uint4*>(xbase + (int64_t)pos * row_bytes + 16 * r);
      }
    }
  };
  auto widen = [&](const Batch& bt, int t, float (&v)[8]) {
    if constexpr (DT == ZC_F32) {
      v[0] = __uint_as_float(bt.raw[t][0].x); v[1] = __uint_as_float(bt.raw[t][0].y);
      v[2] = __uint_as_float(bt.raw[t][0].z); v[3] = __uint_as_float(bt.raw[t][0].w);
      v[4] = __uint_as_float(bt.raw[t][RAW - 1].x); v[5] = __uint_as_float(bt.raw[t][RAW - 1].y);
      v[6] = __uint_as_float(bt.raw[t][RAW - 1].z); v[7] = __uint_as_float(bt.raw[t][RAW - 1].w);
    } else {
      const uint32_t w4[4] = {bt.raw[t][0].x, bt.raw[t][0].y, bt.raw[t][0].z, bt.raw[t][0].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[2 * i] = half_bits_to_float<DT>(w4[i] & 0xffffu);
        v[2 * i + 1] = half_bits_to_float<DT>(w4[i] >> 16);
      }
    }
  };

  uint32_t words[8];                                 // TGROUP: the word group's words of this thread's channels

  auto process = [&](int q, const Batch& bt, int parity) {
    const int kg = (g0 + q / NBAT) & 3, bi = q % NBAT;
    bool tv[TBAT];
#pragma unroll
    for (int t = 0; t < TBAT; ++t) tv[t] = blk * TB + slot_of(q, t) < n;
    if (LAYOUT == ZC_LAYOUT_TGROUP && bi == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) words[i] = 0u;
    }
    // bookkeeping of the batch's tokens by lanes 0 .. TBAT-1 of the first wave
    const int my_t = lane < TBAT ? lane : 0;
    const int my_rel = blk * TB + slot_of(q, my_t);
    const bool my_live = x < TBAT && blockIdx.z == 0 && my_rel < n;
    const int64_t my_o = (int64_t)b * a.cap[sub] + a.begin[sub] + my_rel;
    if (my_live && a.pos[sub]) a.pos[sub][my_o] = (int32_t)(sidx[my_rel - blk * TB] + a.pos_offset);

    float xs[TBAT][8];                               // tokenwise: x' = x / c; channelwise: x
    float sinv[TBAT], zt[TBAT];
    float rt[TBAT], yt[TBAT];                        // EXACT (the plain tokenwise scheme) only: range and its reciprocal
#pragma unroll
    for (int t = 0; t < TBAT; ++t) {
      widen(bt, t, xs[t]);
      if constexpr (TOKWISE) {
#pragma unroll
        for (int i = 0; i < 8; ++i) xs[t][i] *= p0[i];
      }
    }
    if constexpr (TOKWISE) {
      // (min, -max) of every token over the wave: values 0 .. TBAT-1 the minima,
      // TBAT .. 2 TBAT-1 the negated maxima
      // (the first step - rows - pairs a token's minimum with its negated maximum, so
      // it is taken as soon as the two exist: TBAT registers live, not 2 TBAT)
      float mm[TBAT];
#pragma unroll
      for (int t = 0; t < TBAT; ++t) {
        float l = xs[t][0], hneg = -xs[t][0];
#pragma unroll
        for (int i = 1; i < 8; ++i) { l = fminf(l, xs[t][i]); hneg = fminf(hneg, -xs[t][i]); }
        if (!vvalid) { l = INFINITY; hneg = INFINITY; }
        mm[t] = swap_min_rows(l, hneg);
      }
      const float wmin = wave_min_rest<2 * TBAT>(mm);
      // through LDS: lane j < 16 ends up with value j (min of token j, or -max of token j - 8)
      // over all waves.  One barrier per batch: the scratch alternates, and the barrier
      // of the next batch separates these reads from the writes of the batch after it.
      float* mine = &red[parity][wave][0];
      if ((lane & 3) == 0) {
        const int vi = value_of_lane<2 * TBAT>(lane);
        mine[vi < TBAT ? vi : 8 + vi - TBAT] = wmin;
      }
      if (nwaves > 1) __syncthreads();
      float r = red[parity][0][lane & 15];
      for (int w2 = 1; w2 < nwaves; ++w2) r = fminf(r, red[parity][w2][lane & 15]);
      const float tmin = r;
      const float tmax = -__shfl(r, (lane & 7) + 8);
      // parameters of token (lane & 7), computed once per lane group
      float R = tmax - tmin;
      if (R == 0.f) R = QMAX;                        // max == min: s := 1
      const float y = __builtin_amdgcn_rcpf(R);
      const float z = -rintf(refined_ratio(tmin, QMAX, R, y));   // tie-exact: a whole row depends on it
      const float si = QMAX * y;
      if (my_live) {
        a.tok_scale[sub][my_o] = R * (1.f / QMAX);
        a.tok_zero[sub][my_o] = z;
      }
#pragma unroll
      for (int t = 0; t < TBAT; ++t) {
        sinv[t] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(si), t));
        zt[t] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(z), t));
        if constexpr (EXACT) {
          rt[t] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(R), t));
          yt[t] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(y), t));
        }
      }
    }

    // Code of a tokenwise element before clipping.  With channel normalization x' = x / c is
    // not on a grid and a plain product decides the rounding; without it (the plain tokenwise
    // scheme, c = 1) 16-bit inputs sit on a grid where x (2^k - 1) / R hits n + 1/2 exactly
    // about once in 10^4 elements, so the quotient is the tie-exact one there.
    auto tok_code = [&](float xv, int t) {
      if constexpr (!EXACT) return rintf(xv * sinv[t]) + zt[t];
      else if constexpr (DT == ZC_F32) return rintf(refined_ratio(xv, QMAX, rt[t], yt[t])) + zt[t];
      else return rintf(refined_div(xv * QMAX, rt[t], yt[t])) + zt[t];      // x * qmax is exact
    };
    if (!vvalid) return;
#pragma unroll
    for (int t = 0; t < TBAT; ++t) {
      // Eq. 5: round(x / s) first, then + z, then clip
      float code[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float qv;
        if constexpr (TOKWISE) qv = tok_code(xs[t][i], t);
        else if constexpr (DT == ZC_F32) qv = rintf(refined_ratio(xs[t][i], QMAX, p2[i], p0[i])) + p1[i];
        else qv = rintf(refined_div(xs[t][i] * QMAX, p2[i], p0[i])) + p1[i];   // x * qmax is exact
        code[i] = __builtin_amdgcn_fmed3f(qv, 0.f, QMAX);
      }
      if constexpr (LAYOUT == ZC_LAYOUT_ROW) {
        if (tv[t]) {
          // the 8 codes of this token, 16 bits at a time
          constexpr int NG = 8 / FPG;                // 16-bit groups of the 8 codes (>= 1: bits >= 2)
          uint32_t half[NG];
#pragma unroll
          for (int g = 0; g < NG; ++g) {
            float acc = 0.f;
#pragma unroll
            for (int f = 0; f < FPG; ++f) acc = fmaf(code[g * FPG + f], (float)(1 << (BITS * f)), acc);
            half[g] = (uint32_t)acc;
          }
          const int64_t slot = a.begin[sub] + blk * TB + slot_of(q, t);
          uint8_t* row = a.codes[sub] + (((int64_t)b * a.H + h) * a.cap[sub] + slot) * (a.D * BITS / 8) + c * BITS / 8;
          if constexpr (BITS == 8) {
            *reinterpret_cast<uint2*>(row) = make_uint2(half[0] | (half[1] << 16), half[2] | (half[3] << 16));
          } else if constexpr (BITS == 4) {
            *reinterpret_cast<uint32_t*>(row) = half[0] | (half[1] << 16);
          } else {
            *reinterpret_cast<uint16_t*>(row) = (uint16_t)half[0];
          }
        }
      }
    }
    if constexpr (LAYOUT == ZC_LAYOUT_TGROUP) {
      // channel i: the batch's tokens, 16 bits (FPG tokens) at a time; dead tokens add nothing
      constexpr int NG = TBAT / FPG > 0 ? TBAT / FPG : 1;
      constexpr int TPG = TBAT < FPG ? TBAT : FPG;   // tokens per 16-bit group
      float mult[TBAT];
#pragma unroll
      for (int t = 0; t < TBAT; ++t) mult[t] = tv[t] ? (float)(1 << (BITS * (t % TPG))) : 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          float acc = 0.f;
#pragma unroll
          for (int f = 0; f < TPG; ++f) {
            const int t = g * TPG + f;
            float qv;
            if constexpr (TOKWISE) qv = tok_code(xs[t][i], t);
            else if constexpr (DT == ZC_F32) qv = rintf(refined_ratio(xs[t][i], QMAX, p2[i], p0[i])) + p1[i];
            else qv = rintf(refined_div(xs[t][i] * QMAX, p2[i], p0[i])) + p1[i];
            acc = fmaf(__builtin_amdgcn_fmed3f(qv, 0.f, QMAX), mult[t], acc);
          }
          words[i] |= (uint32_t)acc << (BITS * (bi * TBAT + g * TPG));
        }
      }
      if (bi == NBAT - 1) {
        const int64_t nblk = a.cap[sub] / TB;
        const int64_t gblk = a.begin[sub] / TB + blk;
        uint32_t* dst = reinterpret_cast<uint32_t*>(a.codes[sub]) + ((((int64_t)b * a.H + h) * nblk + gblk) * 4 + kg) * a.D + c;
        reinterpret_cast<uint4*>(dst)[0] = make_uint4(words[0], words[1], words[2], words[3]);
        reinterpret_cast<uint4*>(dst)[1] = make_uint4(words[4], words[5], words[6], words[7]);
      }
    }
  };

  const int nq = ng * NBAT;
  if constexpr (PIPE) {
    Batch b0, b1;
    issue(0, b0);
    for (int i = 0; i < nq; i += 2) {
      const bool second = i + 1 < nq;
      if (second) issue(i + 1, b1);
      process(i, b0, 0);
      if (second) {
        if (i + 2 < nq) issue(i + 2, b0);
        process(i + 1, b1, 1);
      }
    }
  } else {
    Batch b0;
    for (int i = 0; i < nq; ++i) {
      issue(i, b0);
      process(i, b0, i & 1);
    }
  }
}

// MAXT: most threads of a workgroup (W / 8 rounded up to a wave); it bounds the
// registers of a thread, and with them whether two batches of rows fit.
// EXACT: tokenwise without channel normalization (the plain tokenwise scheme): tie-exact codes.
template <int DT, int LAYOUT, bool TOKWISE, bool EXACT, int MAXT>
__global__ __launch_bounds__(MAXT) void k_quant_pack(QPArgs a) {
  constexpr bool PIPE = (DT != ZC_F32) && MAXT <= 768;
  __shared__ float red[2][16][16];   // [turn][wave][min of token 0..7, -max of token 0..7]
  __shared__ int32_t sidx[64];
  const int b = blockIdx.y;
  int wg = blockIdx.x;
  const int sub = wg >= a.wgs[0] ? 1 : 0;
  if (sub) wg -= a.wgs[0];
  const int g0 = wg * a.upw, ng = a.upw;
  const int bits = a.bits[sub];
  if (bits == 4) quant_units<DT, 4, LAYOUT, TOKWISE, EXACT, PIPE>(a, sub, g0, ng, b, red, sidx);
  else if (bits == 2) quant_units<DT, 2, LAYOUT, TOKWISE, EXACT, PIPE>(a, sub, g0, ng, b, red, sidx);
  else quant_units<DT, 8, LAYOUT, TOKWISE, EXACT, PIPE>(a, sub, g0, ng, b, red, sidx);
}

// Keys (channelwise, ROW layout) and values (channel-separable tokenwise, TGROUP layout) of one
// cache in one launch, for token rows of at most 256 channel vectors (one workgroup width serves
// both): grid.x = workgroups of the keys, then of the values.
template <int DT>
__global__ __launch_bounds__(256) void k_quant_pack_kv(QPPair p) {
  constexpr bool PIPE = (DT != ZC_F32);
  __shared__ float red[2][16][16];
  __shared__ int32_t sidx[64];
  const int b = blockIdx.y;
  const int nk = p.t[0].wgs[0] + p.t[0].wgs[1];
  const int which = (int)blockIdx.x >= nk ? 1 : 0;
  const QPArgs& a = which ? p.t[1] : p.t[0];
  int wg = blockIdx.x - which * nk;
  const int sub = wg >= a.wgs[0] ? 1 : 0;
  if (sub) wg -= a.wgs[0];
  const int g0 = wg * a.upw, ng = a.upw;
  const int bits = a.bits[sub];
  if (which == 0) {
    if (bits == 4) quant_units<DT, 4, ZC_LAYOUT_ROW, false, false, PIPE>(a, sub, g0, ng, b, red, sidx);
    else if (bits == 2) quant_units<DT, 2, ZC_LAYOUT_ROW, false, false, PIPE>(a, sub, g0, ng, b, red, sidx);
    else quant_units<DT, 8, ZC_LAYOUT_ROW, false, false, PIPE>(a, sub, g0, ng, b, red, sidx);
  } else {
    if (bits == 4) quant_units<DT, 4, ZC_LAYOUT_TGROUP, true, false, PIPE>(a, sub, g0, ng, b, red, sidx);
    else if (bits == 2) quant_units<DT, 2, ZC_LAYOUT_TGROUP, true, false, PIPE>(a, sub, g0, ng, b, red, sidx);
    else quant_units<DT, 8, ZC_LAYOUT_TGROUP, true, false, PIPE>(a, sub, g0, ng, b, red, sidx);
  }
}

template <int DT, int LAYOUT, int MAXT>
static void launch_qp_l(const QPArgs& a, bool tokwise, dim3 grid, dim3 block, hipStream_t st) {
  if (!tokwise) hipLaunchKernelGGL((k_quant_pack<DT, LAYOUT, false, false, MAXT>), grid, block, 0, st, a);
  else if (a.scheme == ZC_SCHEME_TOKEN) hipLaunchKernelGGL((k_quant_pack<DT, LAYOUT, true, true, MAXT>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((k_quant_pack<DT, LAYOUT, true, false, MAXT>), grid, block, 0, st, a);
}
template <int DT, int MAXT>
static void launch_qp_t(const QPArgs& a, int layout, bool tokwise, dim3 grid, dim3 block, hipStream_t st) {
  if (layout == ZC_LAYOUT_ROW) launch_qp_l<DT, ZC_LAYOUT_ROW, MAXT>(a, tokwise, grid, block, st);
  else launch_qp_l<DT, ZC_LAYOUT_TGROUP, MAXT>(a, tokwise, grid, block, st);
}
template <int DT>
static void launch_qp(const QPArgs& a, int layout, bool tokwise, dim3 grid, dim3 block, hipStream_t st) {
  if (block.x <= 256) launch_qp_t<DT, 256>(a, layout, tokwise, grid, block, st);
  else if (block.x <= 768) launch_qp_t<DT, 768>(a, layout, tokwise, grid, block, st);
  else launch_qp_t<DT, 1024>(a, layout, tokwise, grid, block, st);
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

// Validation and kernel arguments of one tensor's compression call.
static int qp_prepare(const zc_tensor4* x, const int32_t* salient_idx, int64_t k, const int32_t* regular_idx, int64_t n_reg,
                      int64_t pos_offset, const zc_packed* out, void* ws, size_t ws_bytes, QPArgs& a) {
  int rc = zc_validate_tensor(x);
  if (rc) return rc;
  rc = zc_validate_packed(out, true);
  if (rc) return rc;
  if (k < 0 || n_reg < 0 || k > x->L || n_reg > x->L || k + n_reg > x->L) return ZC_ERR_INVALID_ARG;
  if ((k > 0 && !salient_idx) || (n_reg > 0 && !regular_idx)) return ZC_ERR_INVALID_ARG;
  if (x->B != out->B || x->H != out->H || x->D != out->D) return ZC_ERR_INVALID_ARG;
  const int64_t W = x->H * x->D;
  if (W / 8 > kVPT * 1024) return ZC_ERR_UNSUPPORTED;
  if (x->B > 65535) return ZC_ERR_UNSUPPORTED;
  if (out->n_chunks >= out->max_chunks) return ZC_ERR_CAPACITY;
  const int64_t end_hi = align_up64(out->n_hi + k, ZC_SLOT_ALIGN);
  const int64_t end_lo = align_up64(out->n_lo + n_reg, ZC_SLOT_ALIGN);
  if (end_hi > out->cap_hi || end_lo > out->cap_lo) return ZC_ERR_CAPACITY;
  const size_t need = zc_quantize_pack_workspace(x->B, x->H, k + n_reg, x->D);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15)) return ZC_ERR_WORKSPACE;

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
  // word groups of 32 / bits tokens; a TGROUP block holds 4 of them
  a.units[0] = (int)ceil_div64(k, 4 * (32 / out->bits_hi)) * 4;
  a.units[1] = (int)ceil_div64(n_reg, 4 * (32 / out->bits_lo)) * 4;
  // word groups per workgroup: one while the launch is small (latency), up to a whole
  // block of consecutive slots when there is enough work to fill the chip anyway
  {
    const int64_t total = (int64_t)(a.units[0] + a.units[1]) * x->B;
    int upw = 1;
    while (upw < 4 && total / (2 * upw) >= 1024) upw *= 2;
    a.upw = upw;
    a.wgs[0] = a.units[0] / upw;
    a.wgs[1] = a.units[1] / upw;
  }
  return ZC_OK;
}

// Host bookkeeping of an appended chunk.
static void qp_commit(zc_packed* out, int64_t k, int64_t n_reg) {
  int32_t* row = out->chunk_table_host + 4 * out->n_chunks;
  row[0] = (int32_t)out->n_hi; row[1] = (int32_t)k; row[2] = (int32_t)out->n_lo; row[3] = (int32_t)n_reg;
  out->n_hi = align_up64(out->n_hi + k, ZC_SLOT_ALIGN);
  out->n_lo = align_up64(out->n_lo + n_reg, ZC_SLOT_ALIGN);
  out->n_chunks += 1;
}

static int qp_launch_pack(const QPArgs& a, int dtype, int layout, hipStream_t st) {
  if (a.units[0] + a.units[1] == 0) return ZC_OK;
  const bool tokwise = a.scheme != ZC_SCHEME_CHANNEL;
  int TXq = (int)align_up64(ceil_div64(a.NV, kVPT), 64);
  int zchunks = 1;
  if (!tokwise && TXq > 256) { zchunks = (int)ceil_div64(a.NV, 256); TXq = 256; }
  dim3 grid((unsigned)(a.wgs[0] + a.wgs[1]), (unsigned)a.B, (unsigned)zchunks), block(TXq);
  if (dtype == ZC_F32) launch_qp<ZC_F32>(a, layout, tokwise, grid, block, st);
  else if (dtype == ZC_F16) launch_qp<ZC_F16>(a, layout, tokwise, grid, block, st);
  else launch_qp<ZC_BF16>(a, layout, tokwise, grid, block, st);
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}

extern "C" int zc_quantize_pack(const zc_tensor4* x, const int32_t* salient_idx, int64_t k,
                                const int32_t* regular_idx, int64_t n_reg, int64_t pos_offset,
                                zc_packed* out, void* ws, size_t ws_bytes, void* stream) {
  QPArgs a;
  int rc = qp_prepare(x, salient_idx, k, regular_idx, n_reg, pos_offset, out, ws, ws_bytes, a);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  // ---- sweep 1: channel statistics (partials) -----------------------------------
  if (out->scheme != ZC_SCHEME_TOKEN && a.tiles[0] + a.tiles[1] > 0) {
    const int TX = a.NV >= kStatThreads ? kStatThreads : (int)align_up64(a.NV, 64);
    dim3 grid((unsigned)(a.tiles[0] + a.tiles[1]), (unsigned)x->B, (unsigned)ceil_div64(a.NV, kStatThreads)), block(TX);
    if (x->dtype == ZC_F32) hipLaunchKernelGGL(k_chan_stats<ZC_F32>, grid, block, 0, st, a);
    else if (x->dtype == ZC_F16) hipLaunchKernelGGL(k_chan_stats<ZC_F16>, grid, block, 0, st, a);
    else hipLaunchKernelGGL(k_chan_stats<ZC_BF16>, grid, block, 0, st, a);
    ZC_LAUNCH_CHECK();
  }
  // ---- parameters (also for empty subsets and the tokenwise scheme: defaults) ------
  hipLaunchKernelGGL(k_chan_finalize, dim3((unsigned)ceil_div64(a.W, 64), 2, (unsigned)x->B), dim3(64, 4), 0, st, a);
  ZC_LAUNCH_CHECK();
  // ---- sweep 2: quantize + pack ---------------------------------------------------
  rc = qp_launch_pack(a, x->dtype, out->layout, st);
  if (rc) return rc;
  qp_commit(out, k, n_reg);
  return ZC_OK;
}

extern "C" size_t zc_quantize_pack_kv_workspace(int64_t B, int64_t H, int64_t L, int64_t D) {
  return 2 * (size_t)align_up64((int64_t)zc_quantize_pack_workspace(B, H, L, D), 256);
}

extern "C" int zc_quantize_pack_kv(const zc_tensor4* xk, const zc_tensor4* xv, const int32_t* salient_idx, int64_t k,
                                   const int32_t* regular_idx, int64_t n_reg, int64_t pos_offset,
                                   zc_packed* outK, zc_packed* outV, void* ws, size_t ws_bytes, void* stream) {
  if (!xk || !xv || !outK || !outV || outK == outV) return ZC_ERR_INVALID_ARG;
  if (xk->dtype != xv->dtype || xk->B != xv->B || xk->H != xv->H || xk->D != xv->D || xk->L != xv->L) return ZC_ERR_INVALID_ARG;
  const size_t half = (size_t)align_up64((int64_t)zc_quantize_pack_workspace(xk->B, xk->H, k + n_reg, xk->D), 256);
  if (!ws || ws_bytes < 2 * half || (reinterpret_cast<uintptr_t>(ws) & 15)) return ZC_ERR_WORKSPACE;
  QPPair p;
  int rc = qp_prepare(xk, salient_idx, k, regular_idx, n_reg, pos_offset, outK, ws, half, p.t[0]);
  if (rc) return rc;
  rc = qp_prepare(xv, salient_idx, k, regular_idx, n_reg, pos_offset, outV, reinterpret_cast<uint8_t*>(ws) + half, half, p.t[1]);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  const QPArgs& a = p.t[0];
  const int dt = xk->dtype;
  const int nt = a.tiles[0] + a.tiles[1];
  // ---- sweep 1 of both tensors --------------------------------------------------------
  if (nt > 0 && (outK->scheme != ZC_SCHEME_TOKEN || outV->scheme != ZC_SCHEME_TOKEN)) {
    const int TX = a.NV >= kStatThreads ? kStatThreads : (int)align_up64(a.NV, 64);
    dim3 grid((unsigned)(2 * nt), (unsigned)a.B, (unsigned)ceil_div64(a.NV, kStatThreads)), block(TX);
    if (dt == ZC_F32) hipLaunchKernelGGL(k_chan_stats_kv<ZC_F32>, grid, block, 0, st, p);
    else if (dt == ZC_F16) hipLaunchKernelGGL(k_chan_stats_kv<ZC_F16>, grid, block, 0, st, p);
    else hipLaunchKernelGGL(k_chan_stats_kv<ZC_BF16>, grid, block, 0, st, p);
    ZC_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_chan_finalize_kv, dim3((unsigned)ceil_div64(a.W, 64), 4, (unsigned)a.B), dim3(64, 4), 0, st, p);
  ZC_LAUNCH_CHECK();
  // ---- sweep 2: one launch for both tensors in the paper's configuration (channelwise keys in
  //      ROW layout, channel-separable tokenwise values in TGROUP layout) when a token row fits
  //      one workgroup of 256 threads; else a launch per tensor ------------------------------
  const bool paper_cfg = outK->scheme == ZC_SCHEME_CHANNEL && outK->layout == ZC_LAYOUT_ROW &&
                         outV->scheme == ZC_SCHEME_CST && outV->layout == ZC_LAYOUT_TGROUP;
  const int nwg = a.wgs[0] + a.wgs[1] + p.t[1].wgs[0] + p.t[1].wgs[1];
  if (paper_cfg && a.NV <= 256 && nwg > 0) {
    dim3 grid((unsigned)nwg, (unsigned)a.B), block((unsigned)align_up64(a.NV, 64));
    if (dt == ZC_F32) hipLaunchKernelGGL(k_quant_pack_kv<ZC_F32>, grid, block, 0, st, p);
    else if (dt == ZC_F16) hipLaunchKernelGGL(k_quant_pack_kv<ZC_F16>, grid, block, 0, st, p);
    else hipLaunchKernelGGL(k_quant_pack_kv<ZC_BF16>, grid, block, 0, st, p);
    ZC_LAUNCH_CHECK();
  } else {
    rc = qp_launch_pack(p.t[0], dt, outK->layout, st);
    if (rc) return rc;
    rc = qp_launch_pack(p.t[1], dt, outV->layout, st);
    if (rc) return rc;
  }
  qp_commit(outK, k, n_reg);
  qp_commit(outV, k, n_reg);
  return ZC_OK;
}
