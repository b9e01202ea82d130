// zc_decode_attention: single-query attention over the packed mixed-precision
// cache plus the full-precision tail (Eq. 4; the attention line of
// Algorithm 3), de-quantizing on the fly.
//
// Split-K: the packed cache is a sequence of equal-sized blocks (a block is
// 4*32/bits slots, i.e. D*16 bytes of K codes and as many of V codes whatever
// the bit width); every workgroup takes a contiguous share of the blocks of one
// (batch, KV head), keeps an online-softmax state for the Hq/Hkv query heads of
// that KV head, and writes a partial (m, Z, o); a second kernel merges the
// partials.
//
// No value is ever de-quantized element by element.  With
//   x_hat[t,c] = cs[c] * ts[t] * (code[t,c] - tz[t] - cz[c])
// the logit is   ts[t] * ( sum_c q'[c] code[t,c] - tz[t] * sum_c q'[c] - sum_c q'[c] cz[c] ),
// q'[c] = q[c] * cs[c] * sm_scale * log2(e), and the output is
//   o[c] = cs[c] * ( sum_t w[t] code[t,c] - sum_t w[t] tz[t] - cz[c] * sum_t w[t] ),  w[t] = p[t] * ts[t],
// accumulated per chunk and subset (each has its own channel parameters).
#include <atomic>

#include "decode_args.hpp"

namespace zc {

constexpr int kDecThreads = 256;
constexpr int kTailBlock = 16;   // tail tokens per unit of the generic kernel

template <int D>
struct DecShared {
  float qp[ZC_MAX_GROUP][D];
  float sl[ZC_MAX_GROUP][64];
  float aq[ZC_MAX_GROUP], bq[ZC_MAX_GROUP];
  float m_run[ZC_MAX_GROUP], z_run[ZC_MAX_GROUP], a1[ZC_MAX_GROUP], a2[ZC_MAX_GROUP], fac[ZC_MAX_GROUP];
  float red[4][ZC_MAX_GROUP][D];
};

__device__ inline int field_tile(int bits, int jf) { return (bits == 2) ? ((jf & 1) * 2 + (jf >> 1)) : jf; }

// Softmax bookkeeping for one block of up to 64 logits per head held in sh.sl.
// On return sh.sl holds w = p * ts and the running state is updated.
template <int D>
__device__ inline void softmax_block(DecShared<D>& sh, int G, int ntok, const float* ts, const float* tz) {
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < G * 64; i += kDecThreads) {
    const int g = i >> 6, t = i & 63;
    const float v = t < ntok ? sh.sl[g][t] : -INFINITY;
    const float mb = wave_max(v);
    const float m_old = sh.m_run[g];
    const float m_new = fmaxf(m_old, mb);
    float p = 0.f;
    if (m_new > -INFINITY && t < ntok) p = exp2f(v - m_new);
    const float s = (ts && t < ntok) ? ts[t] : 1.f;
    const float z = (tz && t < ntok) ? tz[t] : 0.f;
    const float w = p * s;
    const float sp = wave_sum(p), sw = wave_sum(w), swz = wave_sum(w * z);
    sh.sl[g][t] = w;   // 0 for the slots past the end of the segment
    if (lane == 0) {
      const float f = (m_old > -INFINITY) ? exp2f(m_old - m_new) : 0.f;
      sh.fac[g] = f;
      sh.m_run[g] = m_new;
      sh.z_run[g] = sh.z_run[g] * f + sp;
      sh.a1[g] = sh.a1[g] * f + swz;
      sh.a2[g] = sh.a2[g] * f + sw;
    }
  }
}

template <int DT, int D>
__global__ __launch_bounds__(kDecThreads) void k_decode_partial(DecArgs a) {
  constexpr int NCH = D / 64;            // channels per thread in the V phase
  __shared__ DecShared<D> sh;
  const int s = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int G = a.G;
  const int u0 = (int)((int64_t)a.n_units * s / a.S), u1 = (int)((int64_t)a.n_units * (s + 1) / a.S);

  if (tid < ZC_MAX_GROUP) {
    sh.m_run[tid] = -INFINITY; sh.z_run[tid] = 0.f; sh.a1[tid] = 0.f; sh.a2[tid] = 0.f; sh.fac[tid] = 1.f;
  }
  float O[NCH][ZC_MAX_GROUP];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
    for (int g = 0; g < ZC_MAX_GROUP; ++g) O[ch][g] = 0.f;
  __syncthreads();

  int cursor = 0;
  // ---------------- packed segments ----------------------------------------------------
  for (int ci = 0; ci < a.n_chunks; ++ci) {
    for (int sub = 0; sub < 2; ++sub) {
      const int begin = a.chunk_table[4 * ci + 2 * sub], len = a.chunk_table[4 * ci + 2 * sub + 1];
      const int bits = a.bits[sub];
      const int E = 32 / bits, TB = 4 * E;
      const int nb = ceil_div(len, TB);
      const int seg0 = cursor;
      cursor += nb;
      const int lo = max(u0, seg0) - seg0, hi = min(u1, cursor) - seg0;
      if (lo >= hi) continue;

      const int64_t chan_off = ((int64_t)(ci * 2 + sub) * a.B + b) * (a.Hkv * D) + hk * D;
      const float* kcs = a.k_cs + chan_off;
      const float* kcz = a.k_cz + chan_off;
      const float* vcs = a.v_cs + chan_off;
      const float* vcz = a.v_cz + chan_off;
      // q' and its two channel sums
      for (int i = tid; i < G * D; i += kDecThreads) {
        const int g = i / D, c = i % D;
        const float qv = load1<DT>(a.q, (int64_t)b * a.q_sB + (int64_t)(hk * G + g) * a.q_sH + c);
        sh.qp[g][c] = qv * kcs[c] * a.scale_log2;
      }
      __syncthreads();
      for (int g = wave; g < G; g += kDecThreads / 64) {
        float sa = 0.f, sb = 0.f;
        for (int c = lane; c < D; c += 64) { sa += sh.qp[g][c]; sb += sh.qp[g][c] * kcz[c]; }
        sa = wave_sum(sa); sb = wave_sum(sb);
        if (lane == 0) { sh.aq[g] = sa; sh.bq[g] = sb; }
      }
      if (tid < ZC_MAX_GROUP) { sh.a1[tid] = 0.f; sh.a2[tid] = 0.f; }
      __syncthreads();

      float acc[NCH][ZC_MAX_GROUP];
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
        for (int g = 0; g < ZC_MAX_GROUP; ++g) acc[ch][g] = 0.f;

      const int row_bytes = D * bits / 8, q_bytes = row_bytes / 4;   // K row, and a quarter of it
      const uint32_t cmask = (1u << bits) - 1u;
      for (int blk = lo; blk < hi; ++blk) {
        const int ntok = min(TB, len - blk * TB);
        const int64_t slot0 = (int64_t)begin + blk * TB;
        // ---- phase 1: logits; thread (token, channel quarter) ----
        {
          const int t = tid >> 2, kq = tid & 3;
          float dot[ZC_MAX_GROUP];
#pragma unroll
          for (int g = 0; g < ZC_MAX_GROUP; ++g) dot[g] = 0.f;
          if (t < ntok) {
            const uint8_t* row = a.kc[sub] + (((int64_t)b * a.Hkv + hk) * a.cap[sub] + slot0 + t) * row_bytes + kq * q_bytes;
            const int nwords = q_bytes / 4;
            for (int wi = 0; wi < nwords; ++wi) {
              const uint32_t w = reinterpret_cast<const uint32_t*>(row)[wi];
              for (int e = 0; e < E; ++e) {
                const float code = (float)((w >> (bits * e)) & cmask);
                const int c = kq * (D / 4) + wi * E + e;
#pragma unroll
                for (int g = 0; g < ZC_MAX_GROUP; ++g)
                  if (g < G) dot[g] = fmaf(sh.qp[g][c], code, dot[g]);
              }
            }
          }
#pragma unroll
          for (int g = 0; g < ZC_MAX_GROUP; ++g) {
            if (g < G) {
              dot[g] += __shfl_xor(dot[g], 1);
              dot[g] += __shfl_xor(dot[g], 2);
            }
          }
          if (t < ntok && kq == 0) {
            float ts = 1.f, tz = 0.f;
            if (a.k_tok) {
              ts = a.k_ts[sub][(int64_t)b * a.cap[sub] + slot0 + t];
              tz = a.k_tz[sub][(int64_t)b * a.cap[sub] + slot0 + t];
            }
#pragma unroll
            for (int g = 0; g < ZC_MAX_GROUP; ++g)
              if (g < G) sh.sl[g][t] = ts * (dot[g] - tz * sh.aq[g] - sh.bq[g]);
          }
        }
        __syncthreads();
        // ---- phase 2: softmax bookkeeping ----
        softmax_block<D>(sh, G, ntok,
                         a.v_tok ? a.v_ts[sub] + (int64_t)b * a.cap[sub] + slot0 : nullptr,
                         a.v_tok ? a.v_tz[sub] + (int64_t)b * a.cap[sub] + slot0 : nullptr);
        __syncthreads();
        // ---- phase 3: weighted code sums; thread (kg = wave, channel) ----
        {
          const int kg = wave;
          const int64_t nblk = a.cap[sub] / TB;
          const uint32_t* vb = a.vc[sub] + ((((int64_t)b * a.Hkv + hk) * nblk + (slot0 / TB)) * 4 + kg) * D;
#pragma unroll
          for (int ch = 0; ch < NCH; ++ch) {
            const uint32_t w = vb[lane + 64 * ch];
#pragma unroll
            for (int g = 0; g < ZC_MAX_GROUP; ++g) {
              if (g < G) { const float f = sh.fac[g]; acc[ch][g] *= f; O[ch][g] *= f; }
            }
            for (int jf = 0; jf < E / 4; ++jf) {
              const int tb = 16 * field_tile(bits, jf) + 4 * kg;
              for (int v4 = 0; v4 < 4; ++v4) {
                const float code = (float)((w >> (bits * (4 * jf + v4))) & cmask);
#pragma unroll
                for (int g = 0; g < ZC_MAX_GROUP; ++g)
                  if (g < G) acc[ch][g] = fmaf(sh.sl[g][tb + v4], code, acc[ch][g]);
              }
            }
          }
        }
        __syncthreads();
      }
      // ---- fold the segment into the output accumulators ----
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        const int c = lane + 64 * ch;
        const float cs = vcs[c], cz = vcz[c];
#pragma unroll
        for (int g = 0; g < ZC_MAX_GROUP; ++g) {
          if (g < G) {
            float t = acc[ch][g];
            if (wave == 0) t -= sh.a1[g] + cz * sh.a2[g];
            O[ch][g] = fmaf(cs, t, O[ch][g]);
          }
        }
      }
      __syncthreads();
    }
  }

  // ---------------- full-precision tail ----------------------------------------------
  const int n_tail_units = ceil_div(a.tail_len, kTailBlock);
  {
    const int seg0 = cursor;
    const int lo = max(u0, seg0) - seg0, hi = min(u1, seg0 + n_tail_units) - seg0;
    if (lo < hi) {
      for (int i = tid; i < G * D; i += kDecThreads) {
        const int g = i / D, c = i % D;
        sh.qp[g][c] = load1<DT>(a.q, (int64_t)b * a.q_sB + (int64_t)(hk * G + g) * a.q_sH + c) * a.scale_log2;
      }
      __syncthreads();
      for (int blk = lo; blk < hi; ++blk) {
        const int t0 = blk * kTailBlock;
        const int ntok = min(kTailBlock, a.tail_len - t0);
        {
          const int t = tid >> 2, kq = tid & 3;
          float dot[ZC_MAX_GROUP];
#pragma unroll
          for (int g = 0; g < ZC_MAX_GROUP; ++g) dot[g] = 0.f;
          if (t < ntok) {
            const int64_t off = (int64_t)b * a.tk_sB + (int64_t)hk * a.tk_sH + (int64_t)(t0 + t) * a.tk_sL + kq * (D / 4);
            for (int c8 = 0; c8 < D / 4; c8 += 8) {
              float kv[8];
              load8<DT>(a.tail_k, off + c8, kv);
#pragma unroll
              for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int g = 0; g < ZC_MAX_GROUP; ++g)
                  if (g < G) dot[g] = fmaf(sh.qp[g][kq * (D / 4) + c8 + i], kv[i], dot[g]);
            }
          }
#pragma unroll
          for (int g = 0; g < ZC_MAX_GROUP; ++g) {
            if (g < G) {
              dot[g] += __shfl_xor(dot[g], 1);
              dot[g] += __shfl_xor(dot[g], 2);
            }
          }
          if (t < ntok && kq == 0) {
#pragma unroll
            for (int g = 0; g < ZC_MAX_GROUP; ++g)
              if (g < G) sh.sl[g][t] = dot[g];
          }
        }
        __syncthreads();
        softmax_block<D>(sh, G, ntok, nullptr, nullptr);
        __syncthreads();
        {
          const int kg = wave;
#pragma unroll
          for (int ch = 0; ch < NCH; ++ch) {
            const int c = lane + 64 * ch;
#pragma unroll
            for (int g = 0; g < ZC_MAX_GROUP; ++g)
              if (g < G) O[ch][g] *= sh.fac[g];
            for (int t = kg; t < ntok; t += 4) {
              const float vv = load1<DT>(a.tail_v, (int64_t)b * a.tv_sB + (int64_t)hk * a.tv_sH + (int64_t)(t0 + t) * a.tv_sL + c);
#pragma unroll
              for (int g = 0; g < ZC_MAX_GROUP; ++g)
                if (g < G) O[ch][g] = fmaf(sh.sl[g][t], vv, O[ch][g]);
            }
          }
        }
        __syncthreads();
      }
    }
  }

  // ---------------- write the partial -------------------------------------------------
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
    for (int g = 0; g < ZC_MAX_GROUP; ++g)
      if (g < G) sh.red[wave][g][lane + 64 * ch] = O[ch][g];
  __syncthreads();
  for (int i = tid; i < G * D; i += kDecThreads) {
    const int g = i / D, c = i % D;
    const float o = sh.red[0][g][c] + sh.red[1][g][c] + sh.red[2][g][c] + sh.red[3][g][c];
    const int64_t hq = (int64_t)b * a.Hq + hk * G + g;
    a.part_o[(hq * a.S + s) * D + c] = o;
  }
  if (tid < G) {
    const int64_t hq = (int64_t)b * a.Hq + hk * G + tid;
    a.part_m[hq * a.S + s] = sh.m_run[tid];
    a.part_z[hq * a.S + s] = sh.z_run[tid];
  }
}

template <int DT, int D>
__global__ __launch_bounds__(D) void k_decode_combine(const float* __restrict__ part_m,
                                                      const float* __restrict__ part_z,
                                                      const float* __restrict__ part_o, int S,
                                                      void* __restrict__ out, float* __restrict__ lse_out) {
  const int64_t hq = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;  // b * Hq + h
  const int c = threadIdx.x;
  float m = -INFINITY;
  for (int s = 0; s < S; ++s) m = fmaxf(m, part_m[hq * S + s]);
  float z = 0.f, o = 0.f;
  for (int s = 0; s < S; ++s) {
    const float ms = part_m[hq * S + s];
    if (ms == -INFINITY) continue;
    const float w = exp2f(ms - m);
    z = fmaf(part_z[hq * S + s], w, z);
    o = fmaf(part_o[(hq * S + s) * D + c], w, o);
  }
  store1<DT>(out, hq * D + c, z > 0.f ? o / z : 0.f);
  if (lse_out && c == 0) lse_out[hq] = (m + log2f(z)) * kLn2;
}

template <int DT, int D>
static int launch_decode(const DecArgs& a, void* out, float* lse_out, hipStream_t st) {
  hipLaunchKernelGGL((k_decode_partial<DT, D>), dim3(a.S, a.Hkv, a.B), dim3(kDecThreads), 0, st, a);
  ZC_LAUNCH_CHECK();
  hipLaunchKernelGGL((k_decode_combine<DT, D>), dim3(a.Hq, a.B), dim3(D), 0, st, a.part_m, a.part_z,
                     a.part_o, a.S, out, lse_out);
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}

static int split_cap(int64_t B, int64_t Hq) {
  int64_t s = 2048 / (B * Hq);
  if (s < 1) s = 1;
  if (s > kMaxSplits) s = kMaxSplits;
  return (int)s;
}

}  // namespace zc

using namespace zc;

extern "C" size_t zc_decode_attention_workspace(int64_t B, int64_t Hq, int64_t D) {
  if (B <= 0 || Hq <= 0 || D <= 0) return 0;
  return (size_t)B * Hq * (split_cap(B, Hq) + kTailSplits) * (D + 2) * sizeof(float);
}

// ---- the library's own scratch buffer, for callers that cannot allocate -----------------
// zc_decode_attention_static keeps the partial (m, Z, o) of the split-K workgroups in
// this array instead of a caller's workspace.  Every GPU the library runs on holds its
// own copy at its own address; the name below is only a host-side handle, the address
// on the current device comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[ZC_STATIC_SCRATCH_BYTES];

static int static_scratch_of_current_device(void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> of_device[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ZC_ERR_HIP;
  void* p = of_device[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ZC_ERR_HIP;
    of_device[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return ZC_OK;
}

static int decode_entry(const zc_tensor4* q, const zc_packed* Kp, const zc_packed* Vp,
                        const zc_tensor4* tail_k, const zc_tensor4* tail_v, int64_t tail_len,
                        float sm_scale, void* out, float* lse_out,
                        void* ws, size_t ws_bytes, bool static_ws, void* stream) {
  int rc = zc_validate_tensor(q);
  if (rc) return rc;
  if (q->L != 1) return ZC_ERR_INVALID_ARG;
  rc = zc_validate_packed(Kp, false);
  if (rc) return rc;
  rc = zc_validate_packed(Vp, false);
  if (rc) return rc;
  if (Kp->layout != ZC_LAYOUT_ROW || Vp->layout != ZC_LAYOUT_TGROUP) return ZC_ERR_INVALID_ARG;
  if (Kp->B != q->B || Vp->B != q->B || Kp->H != Vp->H || Kp->D != q->D || Vp->D != q->D) return ZC_ERR_INVALID_ARG;
  if (Kp->bits_hi != Vp->bits_hi || Kp->bits_lo != Vp->bits_lo) return ZC_ERR_INVALID_ARG;
  if (Kp->cap_hi != Vp->cap_hi || Kp->cap_lo != Vp->cap_lo || Kp->n_chunks != Vp->n_chunks) return ZC_ERR_INVALID_ARG;
  if (q->H % Kp->H != 0 || q->H / Kp->H > ZC_MAX_GROUP) return ZC_ERR_UNSUPPORTED;
  if (!out || (reinterpret_cast<uintptr_t>(out) & 15)) return ZC_ERR_INVALID_ARG;
  if (tail_len < 0) return ZC_ERR_INVALID_ARG;
  if (tail_len > 0) {
    rc = zc_validate_tensor(tail_k);
    if (rc) return rc;
    rc = zc_validate_tensor(tail_v);
    if (rc) return rc;
    if (tail_k->dtype != q->dtype || tail_v->dtype != q->dtype) return ZC_ERR_INVALID_ARG;
    if (tail_k->B != q->B || tail_v->B != q->B || tail_k->H != Kp->H || tail_v->H != Kp->H ||
        tail_k->D != q->D || tail_v->D != q->D || tail_k->L < tail_len || tail_v->L < tail_len)
      return ZC_ERR_INVALID_ARG;
    // the matrix-core kernel addresses the tail rows of one (batch, KV head) with 32-bit byte offsets
    const int64_t eb = q->dtype == ZC_F32 ? 4 : 2;
    if (tail_len * tail_k->sL * eb >= 0xFFFFF000ll || tail_len * tail_v->sL * eb >= 0xFFFFF000ll) return ZC_ERR_UNSUPPORTED;
  }
  if (q->B > 65535 || Kp->H > 65535) return ZC_ERR_UNSUPPORTED;
  // the matrix-core kernel addresses one (batch, KV head) part of an arena with 32-bit offsets,
  // and requests "nothing" by pointing every lane at offset 0xFFFFF000, which must lie past the end
  constexpr int64_t kPartLimit = 0xFFFFF000ll;
  if (Kp->cap_hi * (q->D * Kp->bits_hi / 8) >= kPartLimit || Kp->cap_lo * (q->D * Kp->bits_lo / 8) >= kPartLimit ||
      Kp->cap_hi * 4 >= kPartLimit || Kp->cap_lo * 4 >= kPartLimit)
    return ZC_ERR_UNSUPPORTED;
  const size_t need = zc_decode_attention_workspace(q->B, q->H, q->D);
  if (static_ws) {
    if (need > (size_t)ZC_STATIC_SCRATCH_BYTES) return ZC_ERR_STATIC_LIMIT;
    rc = static_scratch_of_current_device(&ws);
    if (rc) return rc;
  } else if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15)) {
    return ZC_ERR_WORKSPACE;
  }

  // the chunk tables must agree; count the work units
  const bool mfma_path = (Kp->bits_hi == 2 || Kp->bits_hi == 4) && (Kp->bits_lo == 2 || Kp->bits_lo == 4);
  int64_t units = 0;
  for (int ci = 0; ci < Kp->n_chunks; ++ci) {
    const int32_t* rk = Kp->chunk_table_host + 4 * ci;
    const int32_t* rv = Vp->chunk_table_host + 4 * ci;
    for (int i = 0; i < 4; ++i)
      if (rk[i] != rv[i]) return ZC_ERR_INVALID_ARG;
    int64_t nh = ceil_div64(rk[1], 4 * (32 / Kp->bits_hi)), nl = ceil_div64(rk[3], 4 * (32 / Kp->bits_lo));
    if (mfma_path) { nh = ceil_div64(rk[1], 32); nl = ceil_div64(rk[3], 32); }   // half-blocks of 32 slots
    units += nh + nl;
    if (mfma_path) units += (nh > 0 ? kSegCost : 0) + (nl > 0 ? kSegCost : 0);   // the MFMA kernel splits a cost line
  }
  if (!mfma_path) units += ceil_div64(tail_len, kTailBlock);   // (the MFMA kernel gives the tail to waves of its own)
  if (units > 0x7fffffff) return ZC_ERR_UNSUPPORTED;

  DecArgs a;
  a.q = q->ptr; a.q_sB = q->sB; a.q_sH = q->sH;
  a.B = (int)q->B; a.Hq = (int)q->H; a.Hkv = (int)Kp->H; a.G = a.Hq / a.Hkv; a.D = (int)q->D;
  a.kc[0] = Kp->codes_hi; a.kc[1] = Kp->codes_lo;
  a.k_ts[0] = Kp->tok_scale_hi; a.k_ts[1] = Kp->tok_scale_lo;
  a.k_tz[0] = Kp->tok_zero_hi; a.k_tz[1] = Kp->tok_zero_lo;
  a.k_cs = Kp->chan_scale; a.k_cz = Kp->chan_zero; a.k_tok = Kp->scheme != ZC_SCHEME_CHANNEL;
  a.vc[0] = reinterpret_cast<const uint32_t*>(Vp->codes_hi);
  a.vc[1] = reinterpret_cast<const uint32_t*>(Vp->codes_lo);
  a.v_ts[0] = Vp->tok_scale_hi; a.v_ts[1] = Vp->tok_scale_lo;
  a.v_tz[0] = Vp->tok_zero_hi; a.v_tz[1] = Vp->tok_zero_lo;
  a.v_cs = Vp->chan_scale; a.v_cz = Vp->chan_zero; a.v_tok = Vp->scheme != ZC_SCHEME_CHANNEL;
  a.cap[0] = Kp->cap_hi; a.cap[1] = Kp->cap_lo;
  a.bits[0] = Kp->bits_hi; a.bits[1] = Kp->bits_lo;
  a.chunk_table = Kp->chunk_table; a.n_chunks = Kp->n_chunks;
  a.chunks_inline = Kp->n_chunks <= kInlineChunks;
  for (int i = 0; i < 4 * kInlineChunks; ++i) a.chunk_rows[i] = (a.chunks_inline && i < 4 * Kp->n_chunks) ? Kp->chunk_table_host[i] : 0;
  a.tail_k = tail_len ? tail_k->ptr : nullptr;
  a.tail_v = tail_len ? tail_v->ptr : nullptr;
  a.tk_sB = tail_len ? tail_k->sB : 0; a.tk_sH = tail_len ? tail_k->sH : 0; a.tk_sL = tail_len ? tail_k->sL : 0;
  a.tv_sB = tail_len ? tail_v->sB : 0; a.tv_sH = tail_len ? tail_v->sH : 0; a.tv_sL = tail_len ? tail_v->sL : 0;
  a.tail_len = (int)tail_len;
  a.scale_log2 = (sm_scale == 0.f ? 1.0f / sqrtf((float)q->D) : sm_scale) * kLog2e;
  a.n_units = (int)units;
  {
    // compute units of the current device (asked once per process and device id)
    static int cu_of_device[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ZC_ERR_HIP;
    int ncu = (dev >= 0 && dev < 64) ? cu_of_device[dev] : 0;
    if (ncu == 0) {
      if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu <= 0) ncu = 256;
      if (dev >= 0 && dev < 64) cu_of_device[dev] = ncu;
    }
    a.n_cu = ncu;
  }
  int S = split_cap(q->B, q->H);
  a.n_pw = 0; a.n_tw = 0; a.tw_full = 0; a.tw_rem = 0; a.tail_alone = 0;
  a.pw_q = a.pw_r = a.tu_q = a.tu_r = 0;
  if (mfma_path) {
    const int64_t heads = q->B * Kp->H;
    const int64_t tail_units = ceil_div64(tail_len, kTailUnit);
    // Packed cache.  About eight cost units per workgroup is the finest useful split;
    // the reduce kernel reads at most 32 partials per head.
    int64_t want = ceil_div64(units, 8);
    if (want > 32) want = 32;
    if (want > S) want = S;
    if (heads * want <= a.n_cu) {
      S = (int)want;                 // one workgroup per CU at most: only latency counts
    } else {
      // The launch runs in rounds of two workgroups per CU; a workgroup costs a fixed
      // part (start-up, operand, merge: about 48 units' worth, measured) plus its units.
      int64_t best = 0, best_cost = 0;
      for (int64_t c = 1; c <= want; ++c) {
        const int64_t cost = ceil_div64(heads * c, 2 * (int64_t)a.n_cu) * (48 + ceil_div64(units, c));
        if (best == 0 || cost < best_cost) { best = c; best_cost = cost; }
      }
      S = (int)best;
    }
    // Tail: waves of its own.  One unit (16 tokens) per wave while the launch stays
    // below one workgroup per CU; else a share of the waves in proportion to its cost
    // (about two half-blocks' worth per unit, plus a start).
    int64_t n_tw = 0;
    bool extra_waves = false;
    if (tail_units > 0) {
      if (units == 0 || heads * (S + ceil_div64(tail_units, 4)) <= a.n_cu) {
        n_tw = tail_units;
        extra_waves = true;
      } else {
        const int64_t tail_cost = 2 * tail_units + kSegCost;
        n_tw = (4 * S * tail_cost + (units + tail_cost) / 2) / (units + tail_cost);
        if (n_tw < 1) n_tw = 1;
        if (n_tw > 4 * S - 1) n_tw = 4 * S - 1;
      }
      if (n_tw > tail_units) n_tw = tail_units;
      if (n_tw > 4 * kTailSplits) n_tw = 4 * kTailSplits;
    }
    if (units == 0) S = 0;
    a.tail_alone = 0;
    int64_t WG = S;
    if (extra_waves) {
      if (units > 0 && heads * (S + n_tw) <= a.n_cu && S + n_tw <= 32 && S + n_tw <= split_cap(q->B, q->H) + kTailSplits) {
        a.tail_alone = 1;            // plenty of idle CUs: a workgroup per tail unit, nothing else in it
        WG = S + n_tw;
      } else {
        WG = ceil_div64(4 * (int64_t)S + n_tw, 4);
      }
    }
    if (WG > 32) WG = 32;
    if (WG < 1) WG = 1;              // empty cache: one workgroup writes the zeros
    if (units == 0) n_tw = 4 * WG;   // every wave is a tail wave (those past the last unit idle)
    a.n_tw = (int)n_tw;
    a.n_pw = a.tail_alone ? (int)(4 * S) : (int)(4 * WG - n_tw);
    a.tw_full = (int)(n_tw / WG);
    a.tw_rem = (int)(n_tw % WG);
    a.pw_q = a.n_pw > 0 ? (int)(units / a.n_pw) : 0;
    a.pw_r = a.n_pw > 0 ? (int)(units % a.n_pw) : 0;
    a.tu_q = a.n_tw > 0 ? (int)(tail_units / a.n_tw) : 0;
    a.tu_r = a.n_tw > 0 ? (int)(tail_units % a.n_tw) : 0;
    S = (int)WG;
  } else if (S > units) {
    S = (int)(units > 0 ? units : 1);
  }
  a.S = S;
  const int64_t nq = q->B * q->H;
  float* wsf = reinterpret_cast<float*>(ws);
  a.part_m = wsf;
  a.part_z = wsf + nq * S;
  a.part_o = wsf + 2 * nq * S;
  a.out = out;
  a.lse_out = lse_out;

  hipStream_t st = (hipStream_t)stream;
  if (mfma_path) return launch_decode_mfma(a, q->dtype, st);
#define ZC_DEC(DT)                                                           \
  (q->D == 128 ? launch_decode<DT, 128>(a, out, lse_out, st) : launch_decode<DT, 64>(a, out, lse_out, st))
  if (q->dtype == ZC_F32) return ZC_DEC(ZC_F32);
  if (q->dtype == ZC_F16) return ZC_DEC(ZC_F16);
  return ZC_DEC(ZC_BF16);
#undef ZC_DEC
}

extern "C" int zc_decode_attention(const zc_tensor4* q, const zc_packed* Kp, const zc_packed* Vp,
                                   const zc_tensor4* tail_k, const zc_tensor4* tail_v, int64_t tail_len,
                                   float sm_scale, void* out, float* lse_out,
                                   void* ws, size_t ws_bytes, void* stream) {
  return decode_entry(q, Kp, Vp, tail_k, tail_v, tail_len, sm_scale, out, lse_out, ws, ws_bytes, false, stream);
}

extern "C" int zc_decode_attention_static(const zc_tensor4* q, const zc_packed* Kp, const zc_packed* Vp,
                                          const zc_tensor4* tail_k, const zc_tensor4* tail_v, int64_t tail_len,
                                          float sm_scale, void* out, float* lse_out, void* stream) {
  return decode_entry(q, Kp, Vp, tail_k, tail_v, tail_len, sm_scale, out, lse_out, nullptr, 0, true, stream);
}
