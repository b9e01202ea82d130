// Matrix-core kernel of zc_decode_attention for 2- and 4-bit caches (Eq. 4 over
// the packed cache, Algorithm 3's attention line).
//
// Work unit: one block of the packed cache (32 slots at 4 bits, 64 at 2 bits:
// D*16 bytes of K codes and as many of V codes) or 32 tokens of the
// full-precision tail.  A workgroup takes a contiguous run of units; for every
// segment (chunk x subset, or the tail) in that run its four waves build the
// query operand together, then each wave walks its share of the blocks with its
// own online-softmax state in registers, loading block i+1 while it computes
// block i; there is no barrier inside that loop.  The waves merge through LDS,
// the workgroups of one (batch, KV head) through a partial buffer that the last
// workgroup to arrive reduces (arrival counter, reset to zero by that workgroup).
//
// Both products run on v_mfma_f32_16x16x32_f16 with the codes as one operand:
//   logits  D[token][n]   = sum_c code[token][c] * q'[n][c]      (A = K codes, ROW layout)
//   output  D[n][channel] = sum_t w[n][t] * code[t][channel]     (B = V codes, TGROUP layout)
// The 16 columns n hold the Hq/Hkv query heads of the KV head twice: the fp16
// value of the operand (n even) and its rounding residual times 2^11 (n odd), so
// the fp32 q and softmax weights keep about 21 bits.  A code c enters as the fp16
// number 1 + c / SC (SC = 16 or 4) built by OR-ing its bits into the mantissa of
// 1.0; the "1" terms are removed exactly with the sum of the other operand.  The
// packed layouts are chosen so that the 8 codes a lane feeds to one MFMA are
// contiguous bits of one 32-bit word, and so that the lane that holds a logit is
// the lane that must supply the corresponding softmax weight to the second MFMA.
// De-quantization never happens per element:
//   logit[t] = ts[t] * (dot[t] - tz[t] * sum_c q'[c] - sum_c q'[c] cz[c]),  q' = q cs sm_scale log2(e)
//   o[c]     = cs[c] * (sum_t w[t] code[t][c] - sum_t w[t] tz[t] - cz[c] sum_t w[t]),  w = p ts
#include "decode_args.hpp"

namespace zc {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));

constexpr float kLoScale = 2048.f;          // residual operand is scaled by 2^11
constexpr float kLoInv = 1.f / 2048.f;

__device__ inline f4 mfma16(u4 a, u4 b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
}

// fp16 bit patterns of 1 + c/16 for the eight 4-bit codes of w: register i holds
// code i (low half) and code i + 4 (high half).
__device__ inline u4 unpack4(uint32_t w) {
  const uint32_t M = 0x03C003C0u, E = 0x3C003C00u;
  u4 r;
  r.x = ((w << 6) & M) | E;
  r.y = ((w << 2) & M) | E;
  r.z = ((w >> 2) & M) | E;
  r.w = ((w >> 6) & M) | E;
  return r;
}
// fp16 bit patterns of 1 + c/4 for the sixteen 2-bit codes of w: a.i = codes
// (i, i + 8), b.i = codes (4 + i, 12 + i).
__device__ inline void unpack2(uint32_t w, u4& a, u4& b) {
  const uint32_t M = 0x03000300u, E = 0x3C003C00u;
  a.x = ((w << 8) & M) | E;
  a.y = ((w << 6) & M) | E;
  a.z = ((w << 4) & M) | E;
  a.w = ((w << 2) & M) | E;
  b.x = (w & M) | E;
  b.y = ((w >> 2) & M) | E;
  b.z = ((w >> 4) & M) | E;
  b.w = ((w >> 6) & M) | E;
}

__device__ inline uint32_t pack_h2(_Float16 lo, _Float16 hi) {
  uint16_t a, b;
  __builtin_memcpy(&a, &lo, 2);
  __builtin_memcpy(&b, &hi, 2);
  return (uint32_t)a | ((uint32_t)b << 16);
}

// Splits x into the fp16 nearest to it and the scaled residual; returns the one
// this lane feeds (part 0: value, part 1: residual) and the value both represent.
__device__ inline _Float16 split_part(float x, int part, float& represented) {
  const _Float16 hi = (_Float16)x;
  const float hif = (float)hi;
  const _Float16 lo = (_Float16)((x - hif) * kLoScale);
  represented = hif + (float)lo * kLoInv;
  return part ? lo : hi;
}

__device__ inline float xor1(float x) {   // value of the neighbouring lane (lane ^ 1)
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, true));
}
__device__ inline float grp_max(float x) {  // over the four 16-lane groups
  x = fmaxf(x, __shfl_xor(x, 16));
  return fmaxf(x, __shfl_xor(x, 32));
}
__device__ inline float grp_sum(float x) {
  x += __shfl_xor(x, 16);
  return x + __shfl_xor(x, 32);
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr int kCombineMax = 16;   // most workgroups per (batch, KV head) on this path

template <int DT, int D>
__global__ __launch_bounds__(256) void k_decode_mfma(DecArgs a) {
  constexpr int KS = D / 32;     // k-steps of the logit product
  constexpr int NR = D / 64;     // 16-byte V loads per lane and block
  constexpr int MG = ZC_MAX_GROUP;
  __shared__ float qs[MG][D];             // q * sm_scale * log2(e)
  __shared__ u4 sqB[KS][64];              // query operand of the current segment
  __shared__ float ssum[2][KS][64];
  __shared__ float mO[4][MG][D];
  __shared__ float mM[4][MG], mZ[4][MG];
  __shared__ float ptile[4][MG][kTailUnit];
  __shared__ int s_last;

  const int s = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, grp = lane >> 4;
  const int G = a.G;
  const int g = n >> 1, part = n & 1;
  const bool nvalid = n < 2 * G;
  const int g0 = 2 * grp, g1 = 2 * grp + 1;      // heads of this lane's rows in the output tiles

  for (int i = tid; i < G * D; i += 256) {
    const int gg = i / D, c = i % D;
    qs[gg][c] = load1<DT>(a.q, (int64_t)b * a.q_sB + (int64_t)(hk * G + gg) * a.q_sH + c) * a.scale_log2;
  }
  // (the first barrier of the first segment orders these writes before their readers)

  // running state of this wave
  float m_run = -INFINITY, z_part = 0.f;
  float O[NR][4][2];
  float Ot[MG][NR];
#pragma unroll
  for (int r = 0; r < NR; ++r)
#pragma unroll
    for (int j = 0; j < 4; ++j) { O[r][j][0] = 0.f; O[r][j][1] = 0.f; }
#pragma unroll
  for (int gg = 0; gg < MG; ++gg)
#pragma unroll
    for (int r = 0; r < NR; ++r) Ot[gg][r] = 0.f;

  const int u0 = (int)((int64_t)a.n_units * s / a.S), u1 = (int)((int64_t)a.n_units * (s + 1) / a.S);

  // When the running maximum of a head grows, everything accumulated so far is
  // rescaled; rare after the first blocks, so it sits behind a wave-uniform branch.
  auto rescale_to = [&](float m_new, float& sw, float& a1, float& a2, f4 (*acc)[4]) {
    const bool changed = nvalid && (m_new > m_run);
    if (__any(changed)) {
      const float fac = (m_run > -INFINITY) ? fast_exp2(m_run - m_new) : 0.f;
      z_part *= fac; sw *= fac; a1 *= fac; a2 *= fac;
      const float f0 = __shfl(fac, 2 * g0), f1 = __shfl(fac, 2 * g1);
#pragma unroll
      for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          O[r][j][0] *= f0; O[r][j][1] *= f1;
          if (acc) { acc[r][j].x *= f0; acc[r][j].y *= f0; acc[r][j].z *= f1; acc[r][j].w *= f1; }
        }
#pragma unroll
      for (int gg = 0; gg < MG; ++gg) {
        if (gg < G) {
          const float fg = __shfl(fac, 2 * gg);
#pragma unroll
          for (int r = 0; r < NR; ++r) Ot[gg][r] *= fg;
        }
      }
    }
    m_run = fmaxf(m_run, m_new);
  };

  // The query operand of a segment, built once per workgroup: wave w computes
  // k-step w.  MODE 4 / 2: codes of that width, q' = q cs SC in the channel order
  // the unpacked K words have; MODE 0: the tail, q itself in natural order.
  // Returns the operand registers and sum(q''), sum(q'' cz) over all channels.
  auto build_query_operand = [&](auto mode_c, const float* kcs, const float* kcz, u4 (&qB)[KS], float& sumqq, float& sumqqcz) {
    constexpr int MODE = decltype(mode_c)::value;
    constexpr float SC = MODE == 4 ? 16.f : (MODE == 2 ? 4.f : 1.f);
    __syncthreads();     // qs written; sqB / ssum of the previous segment no longer read
    for (int ks = wave; ks < KS; ks += 4) {
      uint32_t regs[4];
      float sq = 0.f, sqz = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        _Float16 hv[2];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          int c;
          if constexpr (MODE == 4) c = grp * (D / 4) + 8 * ks + i + 4 * half;
          else if constexpr (MODE == 2) c = grp * (D / 4) + 16 * (ks >> 1) + 4 * (ks & 1) + i + 8 * half;
          else c = 32 * ks + 8 * grp + 2 * i + half;
          float qv = nvalid ? qs[g][c] : 0.f;
          if constexpr (MODE != 0) qv *= kcs[c] * SC;
          float rep;
          hv[half] = split_part(qv, part, rep);
          sq += rep;
          if constexpr (MODE != 0) sqz += rep * kcz[c];
        }
        regs[i] = pack_h2(hv[0], hv[1]);
      }
      u4 t; t.x = regs[0]; t.y = regs[1]; t.z = regs[2]; t.w = regs[3];
      sqB[ks][lane] = t;
      ssum[0][ks][lane] = sq;
      ssum[1][ks][lane] = sqz;
    }
    __syncthreads();
    sumqq = 0.f; sumqqcz = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qB[ks] = sqB[ks][lane];
      sumqq += ssum[0][ks][lane];
      sumqqcz += ssum[1][ks][lane];
    }
    sumqq = grp_sum(sumqq);
    sumqqcz = grp_sum(sumqqcz);
  };

  int cursor = 0;
  // ---------------- packed segments --------------------------------------------------
  auto segment = [&](auto bits_c, int ci, int sub, int begin, int len, int lo, int hi) {
    constexpr int BITS = decltype(bits_c)::value;
    constexpr int E = 32 / BITS, TB = 4 * E, NT = TB / 16;
    constexpr float SC = (BITS == 4) ? 16.f : 4.f;
    constexpr int KW = D * BITS / 128;       // 32-bit words of K codes per lane and token
    const int64_t chan_off = ((int64_t)(ci * 2 + sub) * a.B + b) * (a.Hkv * D) + hk * D;
    const int wlo = lo + (hi - lo) * wave / 4, whi = lo + (hi - lo) * (wave + 1) / 4;

    const int64_t bh = (int64_t)b * a.Hkv + hk;
    const int64_t nblk = a.cap[sub] / TB;
    const uint8_t* kbase = a.kc[sub] + bh * a.cap[sub] * (D * BITS / 8) + grp * (KW * 4);
    const int64_t tokbase = (int64_t)b * a.cap[sub];

    struct Buf {
      uint32_t kw[NT][KW];
      uint4 vw[NR];
      float4 kts[NT], ktz[NT], vts[NT], vtz[NT];
    };
    auto load_block = [&](int blk, Buf& bf) {
      const int slot0 = begin + blk * TB;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const uint32_t* kp = reinterpret_cast<const uint32_t*>(kbase + (int64_t)(slot0 + 16 * j + n) * (D * BITS / 8));
        if constexpr (KW == 4) { const uint4 t = *reinterpret_cast<const uint4*>(kp); bf.kw[j][0] = t.x; bf.kw[j][1] = t.y; bf.kw[j][2] = t.z; bf.kw[j][3] = t.w; }
        else if constexpr (KW == 2) { const uint2 t = *reinterpret_cast<const uint2*>(kp); bf.kw[j][0] = t.x; bf.kw[j][1] = t.y; }
        else { bf.kw[j][0] = *kp; }
        const int64_t to = tokbase + slot0 + 16 * j + 4 * grp;
        if (a.k_tok) {
          bf.kts[j] = *reinterpret_cast<const float4*>(a.k_ts[sub] + to);
          bf.ktz[j] = *reinterpret_cast<const float4*>(a.k_tz[sub] + to);
        }
        if (a.v_tok) {
          bf.vts[j] = *reinterpret_cast<const float4*>(a.v_ts[sub] + to);
          bf.vtz[j] = *reinterpret_cast<const float4*>(a.v_tz[sub] + to);
        }
      }
      const uint32_t* vbase = a.vc[sub] + ((bh * nblk + slot0 / TB) * 4 + grp) * D;
#pragma unroll
      for (int r = 0; r < NR; ++r) bf.vw[r] = *reinterpret_cast<const uint4*>(vbase + 4 * (n + 16 * r));
    };

    Buf cur;
    if (wlo < whi) load_block(wlo, cur);      // in flight while the operand is built

    u4 qB[KS];
    float sumqq, sumqqcz;
    build_query_operand(std::integral_constant<int, BITS>{}, a.k_cs + chan_off, a.k_cz + chan_off, qB, sumqq, sumqqcz);
    if (wlo >= whi) return;
    const float Aq = sumqq / SC, Bq = sumqqcz / SC;

    f4 acc[NR][4];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[r][j] = f4{0.f, 0.f, 0.f, 0.f};
    float sw = 0.f, a1 = 0.f, a2 = 0.f;

    for (int blk = wlo; blk < whi; ++blk) {
      Buf nxt = cur;
      if (blk + 1 < whi) load_block(blk + 1, nxt);
      const int ntok = min(TB, len - blk * TB);
      // ---- logits: dot = (value + residual / 2^11 of the head's two columns) - the "1" terms ----
      float lg[NT][4];
      float lmax = -INFINITY;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        f4 sacc = f4{0.f, 0.f, 0.f, 0.f};
        if constexpr (BITS == 4) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) sacc = mfma16(unpack4(cur.kw[j][ks]), qB[ks], sacc);
        } else {
#pragma unroll
          for (int wd = 0; wd < KW; ++wd) {
            u4 ua, ub;
            unpack2(cur.kw[j][wd], ua, ub);
            sacc = mfma16(ua, qB[2 * wd], sacc);
            sacc = mfma16(ub, qB[2 * wd + 1], sacc);
          }
        }
        const float own[4] = {sacc.x, sacc.y, sacc.z, sacc.w};
        float ts[4] = {1.f, 1.f, 1.f, 1.f}, tz[4] = {0.f, 0.f, 0.f, 0.f};
        if (a.k_tok) {
          ts[0] = cur.kts[j].x; ts[1] = cur.kts[j].y; ts[2] = cur.kts[j].z; ts[3] = cur.kts[j].w;
          tz[0] = cur.ktz[j].x; tz[1] = cur.ktz[j].y; tz[2] = cur.ktz[j].z; tz[3] = cur.ktz[j].w;
        }
        const int tb = 16 * j + 4 * grp;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float other = xor1(own[v]);
          const float hi_v = part ? other : own[v], lo_v = part ? own[v] : other;
          const float dot = hi_v + lo_v * kLoInv - sumqq;
          const float x = ts[v] * (dot - tz[v] * Aq - Bq);
          lg[j][v] = (tb + v < ntok) ? x : -INFINITY;
          lmax = fmaxf(lmax, lg[j][v]);
        }
      }
      rescale_to(fmaxf(m_run, grp_max(lmax)), sw, a1, a2, acc);
      // ---- weights w = p ts, and the A operand of the output product ----
      _Float16 wh[NT][4];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        float ts[4] = {1.f, 1.f, 1.f, 1.f}, tz[4] = {0.f, 0.f, 0.f, 0.f};
        if (a.v_tok) {
          ts[0] = cur.vts[j].x; ts[1] = cur.vts[j].y; ts[2] = cur.vts[j].z; ts[3] = cur.vts[j].w;
          tz[0] = cur.vtz[j].x; tz[1] = cur.vtz[j].y; tz[2] = cur.vtz[j].z; tz[3] = cur.vtz[j].w;
        }
        const int tb = 16 * j + 4 * grp;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const bool ok = (tb + v < ntok) && nvalid && (m_run > -INFINITY);
          const float p = ok ? fast_exp2(lg[j][v] - m_run) : 0.f;
          const float w = ok ? p * ts[v] : 0.f;
          z_part += p;
          a1 += ok ? w * tz[v] : 0.f;
          a2 += w;
          float rep;
          wh[j][v] = split_part(w * SC, part, rep);
          sw += rep;
        }
      }
      // ---- output product ----
      if constexpr (BITS == 4) {
        u4 pA;
        pA.x = pack_h2(wh[0][0], wh[1][0]); pA.y = pack_h2(wh[0][1], wh[1][1]);
        pA.z = pack_h2(wh[0][2], wh[1][2]); pA.w = pack_h2(wh[0][3], wh[1][3]);
#pragma unroll
        for (int r = 0; r < NR; ++r) {
          acc[r][0] = mfma16(pA, unpack4(cur.vw[r].x), acc[r][0]);
          acc[r][1] = mfma16(pA, unpack4(cur.vw[r].y), acc[r][1]);
          acc[r][2] = mfma16(pA, unpack4(cur.vw[r].z), acc[r][2]);
          acc[r][3] = mfma16(pA, unpack4(cur.vw[r].w), acc[r][3]);
        }
      } else {
        u4 pA, pB;   // slot tiles (0, 1) and (2, 3)
        pA.x = pack_h2(wh[0][0], wh[1][0]); pA.y = pack_h2(wh[0][1], wh[1][1]);
        pA.z = pack_h2(wh[0][2], wh[1][2]); pA.w = pack_h2(wh[0][3], wh[1][3]);
        pB.x = pack_h2(wh[2][0], wh[3][0]); pB.y = pack_h2(wh[2][1], wh[3][1]);
        pB.z = pack_h2(wh[2][2], wh[3][2]); pB.w = pack_h2(wh[2][3], wh[3][3]);
#pragma unroll
        for (int r = 0; r < NR; ++r) {
          const uint32_t ww[4] = {cur.vw[r].x, cur.vw[r].y, cur.vw[r].z, cur.vw[r].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            u4 ua, ub;
            unpack2(ww[j], ua, ub);
            acc[r][j] = mfma16(pA, ua, acc[r][j]);
            acc[r][j] = mfma16(pB, ub, acc[r][j]);
          }
        }
      }
      cur = nxt;
    }
    // ---- fold the segment into O ----
    // sum_t w code = acc_value + acc_residual / 2^11 - sum_t w'',  w'' = SC w
    sw = grp_sum(sw); a1 = grp_sum(a1); a2 = grp_sum(a2);
    const float sw0 = __shfl(sw, 2 * g0), sw1 = __shfl(sw, 2 * g1);
    const float a10 = __shfl(a1, 2 * g0), a11 = __shfl(a1, 2 * g1);
    const float a20 = __shfl(a2, 2 * g0), a21 = __shfl(a2, 2 * g1);
    const float* vcs = a.v_cs + chan_off;
    const float* vcz = a.v_cz + chan_off;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const float4 cs4 = *reinterpret_cast<const float4*>(vcs + 4 * (n + 16 * r));
      const float4 cz4 = *reinterpret_cast<const float4*>(vcz + 4 * (n + 16 * r));
      const float cs[4] = {cs4.x, cs4.y, cs4.z, cs4.w}, cz[4] = {cz4.x, cz4.y, cz4.z, cz4.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float t0 = acc[r][j].x + acc[r][j].y * kLoInv - sw0;
        const float t1 = acc[r][j].z + acc[r][j].w * kLoInv - sw1;
        O[r][j][0] = fmaf(cs[j], t0 - a10 - cz[j] * a20, O[r][j][0]);
        O[r][j][1] = fmaf(cs[j], t1 - a11 - cz[j] * a21, O[r][j][1]);
      }
    }
  };

  for (int ci = 0; ci < a.n_chunks; ++ci) {
    for (int sub = 0; sub < 2; ++sub) {
      const int begin = a.chunk_table[4 * ci + 2 * sub], len = a.chunk_table[4 * ci + 2 * sub + 1];
      const int bits = a.bits[sub];
      const int TB = 4 * (32 / bits);
      const int nb = ceil_div(len, TB);
      const int seg0 = cursor;
      cursor += nb;
      const int lo = max(u0, seg0) - seg0, hi = min(u1, cursor) - seg0;
      if (lo >= hi) continue;
      if (bits == 4) segment(std::integral_constant<int, 4>{}, ci, sub, begin, len, lo, hi);
      else segment(std::integral_constant<int, 2>{}, ci, sub, begin, len, lo, hi);
    }
  }

  // ---------------- full-precision tail ------------------------------------------------
  {
    const int n_tail = ceil_div(a.tail_len, kTailUnit);
    const int seg0 = cursor;
    const int lo = max(u0, seg0) - seg0, hi = min(u1, seg0 + n_tail) - seg0;
    if (lo < hi) {
      const int wlo = lo + (hi - lo) * wave / 4, whi = lo + (hi - lo) * (wave + 1) / 4;
      u4 qB[KS];
      float dummy0, dummy1;
      build_query_operand(std::integral_constant<int, 0>{}, nullptr, nullptr, qB, dummy0, dummy1);
      const int64_t kb = (int64_t)b * a.tk_sB + (int64_t)hk * a.tk_sH;
      const int64_t vb = (int64_t)b * a.tv_sB + (int64_t)hk * a.tv_sH;
      for (int tu = wlo; tu < whi; ++tu) {
        const int t0 = tu * kTailUnit;
        const int ntok = min(kTailUnit, a.tail_len - t0);
        // values of the unit: every lane owns channels lane + 64 r (issued early)
        float vv[NR][kTailUnit];
#pragma unroll
        for (int t = 0; t < kTailUnit; ++t)
#pragma unroll
          for (int r = 0; r < NR; ++r)
            vv[r][t] = (t < ntok) ? load1<DT>(a.tail_v, vb + (int64_t)(t0 + t) * a.tv_sL + lane + 64 * r) : 0.f;
        float U[2][4];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int tok = 16 * j + n;          // row of the A operand
          f4 s_hi = f4{0.f, 0.f, 0.f, 0.f}, s_lo = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            float kv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (tok < ntok) load8<DT>(a.tail_k, kb + (int64_t)(t0 + tok) * a.tk_sL + 32 * ks + 8 * grp, kv);
            uint32_t rh[4], rl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const _Float16 h0 = (_Float16)kv[2 * i], h1 = (_Float16)kv[2 * i + 1];
              rh[i] = pack_h2(h0, h1);
              if constexpr (DT == ZC_F32)
                rl[i] = pack_h2((_Float16)((kv[2 * i] - (float)h0) * kLoScale), (_Float16)((kv[2 * i + 1] - (float)h1) * kLoScale));
            }
            u4 ah; ah.x = rh[0]; ah.y = rh[1]; ah.z = rh[2]; ah.w = rh[3];
            s_hi = mfma16(ah, qB[ks], s_hi);
            if constexpr (DT == ZC_F32) {
              u4 al; al.x = rl[0]; al.y = rl[1]; al.z = rl[2]; al.w = rl[3];
              s_lo = mfma16(al, qB[ks], s_lo);
            }
          }
          // rows past the end of the tail are zeros; every lane takes part in the MFMAs
          const float own[4] = {s_hi.x + s_lo.x * kLoInv, s_hi.y + s_lo.y * kLoInv, s_hi.z + s_lo.z * kLoInv, s_hi.w + s_lo.w * kLoInv};
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float other = xor1(own[v]);
            U[j][v] = part ? (other + own[v] * kLoInv) : (own[v] + other * kLoInv);
          }
        }
        float lmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            if (16 * j + 4 * grp + v >= ntok) U[j][v] = -INFINITY;
            lmax = fmaxf(lmax, U[j][v]);
          }
        float dsw = 0.f, da1 = 0.f, da2 = 0.f;
        rescale_to(fmaxf(m_run, grp_max(lmax)), dsw, da1, da2, nullptr);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const bool ok = (16 * j + 4 * grp + v < ntok) && nvalid && (m_run > -INFINITY);
            const float p = ok ? fast_exp2(U[j][v] - m_run) : 0.f;
            z_part += p;
            if (nvalid && part == 0) ptile[wave][g][16 * j + 4 * grp + v] = p;
          }
        // weighted sum of the tail values
#pragma unroll
        for (int gg = 0; gg < MG; ++gg) {
          if (gg < G) {
#pragma unroll
            for (int t4 = 0; t4 < kTailUnit; t4 += 4) {
              const float4 p4 = *reinterpret_cast<const float4*>(&ptile[wave][gg][t4]);
#pragma unroll
              for (int r = 0; r < NR; ++r) {
                Ot[gg][r] = fmaf(p4.x, vv[r][t4], Ot[gg][r]);
                Ot[gg][r] = fmaf(p4.y, vv[r][t4 + 1], Ot[gg][r]);
                Ot[gg][r] = fmaf(p4.z, vv[r][t4 + 2], Ot[gg][r]);
                Ot[gg][r] = fmaf(p4.w, vv[r][t4 + 3], Ot[gg][r]);
              }
            }
          }
        }
      }
    }
  }

  // ---------------- merge the four waves --------------------------------------------------
  const float z_tot = grp_sum(z_part);
  if (nvalid && part == 0 && grp == 0) { mM[wave][g] = m_run; mZ[wave][g] = z_tot; }
#pragma unroll
  for (int r = 0; r < NR; ++r)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = 4 * (n + 16 * r) + j;
      if (g0 < G) mO[wave][g0][c] = O[r][j][0];
      if (g1 < G) mO[wave][g1][c] = O[r][j][1];
    }
  __syncthreads();
#pragma unroll
  for (int gg = 0; gg < MG; ++gg) {
    if (gg < G) {
#pragma unroll
      for (int r = 0; r < NR; ++r) mO[wave][gg][lane + 64 * r] += Ot[gg][r];
    }
  }
  __syncthreads();

  const bool direct = a.S == 1;
  for (int i = tid; i < G * D; i += 256) {
    const int gg = i / D, c = i % D;
    float M = fmaxf(fmaxf(mM[0][gg], mM[1][gg]), fmaxf(mM[2][gg], mM[3][gg]));
    float o = 0.f, z = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (mM[w][gg] > -INFINITY) {
        const float f = fast_exp2(mM[w][gg] - M);
        o = fmaf(mO[w][gg][c], f, o);
        z = fmaf(mZ[w][gg], f, z);
      }
    }
    const int64_t hq = (int64_t)b * a.Hq + hk * G + gg;
    if (direct) {
      store1<DT>(a.out, hq * D + c, z > 0.f ? o / z : 0.f);
      if (a.lse_out && c == 0) a.lse_out[hq] = (M + log2f(z)) * kLn2;
    } else {
      a.part_o[(hq * a.S + s) * D + c] = o;
      if (c == 0) { a.part_m[hq * a.S + s] = M; a.part_z[hq * a.S + s] = z; }
    }
  }
  if (direct) return;

  // ---------------- last workgroup of this (batch, KV head) reduces the partials -----------
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const int old = atomicAdd(&a.counters[b * a.Hkv + hk], 1);
    s_last = (old == a.S - 1);
  }
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  for (int i = tid; i < G * D; i += 256) {
    const int gg = i / D, c = i % D;
    const int64_t hq = (int64_t)b * a.Hq + hk * G + gg;
    // all partials are requested before any is used
    float pm[kCombineMax], pz[kCombineMax], po[kCombineMax];
#pragma unroll
    for (int ss = 0; ss < kCombineMax; ++ss) {
      const bool in = ss < a.S;
      pm[ss] = in ? a.part_m[hq * a.S + ss] : -INFINITY;
      pz[ss] = in ? a.part_z[hq * a.S + ss] : 0.f;
      po[ss] = in ? a.part_o[(hq * a.S + ss) * D + c] : 0.f;
    }
    float M = -INFINITY;
#pragma unroll
    for (int ss = 0; ss < kCombineMax; ++ss) M = fmaxf(M, pm[ss]);
    float o = 0.f, z = 0.f;
#pragma unroll
    for (int ss = 0; ss < kCombineMax; ++ss) {
      const float f = (pm[ss] > -INFINITY) ? fast_exp2(pm[ss] - M) : 0.f;
      o = fmaf(po[ss], f, o);
      z = fmaf(pz[ss], f, z);
    }
    store1<DT>(a.out, hq * D + c, z > 0.f ? o / z : 0.f);
    if (a.lse_out && c == 0) a.lse_out[hq] = (M + log2f(z)) * kLn2;
  }
  if (tid == 0) a.counters[b * a.Hkv + hk] = 0;
}


int launch_decode_mfma(const DecArgs& a, int dtype, hipStream_t st) {
  dim3 grid(a.S, a.Hkv, a.B), block(256);
#define ZC_L(DT)                                                                     \
  do {                                                                               \
    if (a.D == 128) hipLaunchKernelGGL((k_decode_mfma<DT, 128>), grid, block, 0, st, a); \
    else hipLaunchKernelGGL((k_decode_mfma<DT, 64>), grid, block, 0, st, a);            \
  } while (0)
  if (dtype == ZC_F32) ZC_L(ZC_F32);
  else if (dtype == ZC_F16) ZC_L(ZC_F16);
  else ZC_L(ZC_BF16);
#undef ZC_L
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}

}  // namespace zc
