// The pieces Algorithm 3 needs when its re-compression branch is taken at its word
// (every 100 steps everything but the newest 100 tokens is compressed again, ranked by the
// attention rows of the window's probe steps):
//   zc_decode_probs      the attention row a of one decode step over the whole cache
//                        (Eq. 4's probabilities), in token order, for the probe steps;
//   zc_rows_saliency     Eq. 8 on such explicit rows: column sums over the rows that see a
//                        token, divided by their number, mean over heads;
//   zc_dequantize_cache  the compressed tokens as they now are (Eq. 5's x_hat), scattered
//                        to their token positions in a full-precision tensor - the input
//                        of the next compression.
// None of them is on the per-step hot path (a probe step is one step in ten, a
// re-compression one in a hundred): plain kernels, coalesced, no matrix instructions.
#include "zc_common.hpp"

namespace zc {

struct ProbsArgs {
  const void* q;
  int64_t q_sB, q_sH;
  int B, Hq, Hkv, G, D;
  const uint8_t* kc[2];
  const float* k_ts[2];
  const float* k_tz[2];
  const int32_t* pos[2];
  const float* k_cs;
  const float* k_cz;
  int k_tok;
  int64_t cap[2];
  int bits[2];
  const int32_t* chunk_table;
  int n_chunks;
  int n_seg_tiles;          // 64-slot tiles of all packed segments together
  const void* tail_k;
  int64_t tk_sB, tk_sH, tk_sL;
  int tail_len, tail_pos0;
  float scale_log2;
  const float* lse;         // [B, Hq] natural log
  float* probs;             // [B, Hq, N]
  int N;
};

constexpr int kProbSlots = 64;    // cache slots (or tail tokens) per workgroup

// grid (tiles, Hkv, B), 256 threads: thread (t, kq) = (slot of the tile, quarter of its row)
template <int DT, int D>
__global__ __launch_bounds__(256) void k_decode_probs(ProbsArgs a) {
  __shared__ float qp[ZC_MAX_GROUP][D];
  __shared__ float aq[ZC_MAX_GROUP], bq[ZC_MAX_GROUP];
  const int tile = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int G = a.G;
  const int t = tid >> 2, kq = tid & 3;

  // which segment (chunk, subset) this tile belongs to: walk the chunk table
  int ci = -1, sub = 0, begin = 0, len = 0, first = 0;
  bool is_tail = tile >= a.n_seg_tiles;
  if (!is_tail) {
    int cursor = 0;
    for (int c = 0; c < a.n_chunks && ci < 0; ++c)
      for (int s = 0; s < 2; ++s) {
        const int l = a.chunk_table[4 * c + 2 * s + 1];
        const int nt = ceil_div(l, kProbSlots);
        if (tile < cursor + nt) { ci = c; sub = s; begin = a.chunk_table[4 * c + 2 * s]; len = l; first = (tile - cursor) * kProbSlots; break; }
        cursor += nt;
      }
    if (ci < 0) return;                 // (the host's tile count and the device table disagree: nothing to do)
  } else {
    first = (tile - a.n_seg_tiles) * kProbSlots;
    len = a.tail_len;
  }
  const int ntok = min(kProbSlots, len - first);

  // q' = q * channel scale * sm_scale * log2(e), and its two channel sums
  const int64_t chan_off = is_tail ? 0 : ((int64_t)(ci * 2 + sub) * a.B + b) * (a.Hkv * D) + hk * D;
  for (int i = tid; i < G * D; i += 256) {
    const int g = i / D, c = i % D;
    const float qv = load1<DT>(a.q, (int64_t)b * a.q_sB + (int64_t)(hk * G + g) * a.q_sH + c);
    qp[g][c] = qv * (is_tail ? 1.f : a.k_cs[chan_off + c]) * a.scale_log2;
  }
  __syncthreads();
  for (int g = wave; g < G; g += 4) {
    float sa = 0.f, sb = 0.f;
    for (int c = lane; c < D; c += 64) { sa += qp[g][c]; sb += qp[g][c] * (is_tail ? 0.f : a.k_cz[chan_off + c]); }
    sa = wave_sum(sa); sb = wave_sum(sb);
    if (lane == 0) { aq[g] = sa; bq[g] = sb; }
  }
  __syncthreads();

  float dot[ZC_MAX_GROUP];
#pragma unroll
  for (int g = 0; g < ZC_MAX_GROUP; ++g) dot[g] = 0.f;
  int position = -1;
  float ts = 1.f, tz = 0.f;
  if (t < ntok) {
    if (!is_tail) {
      const int bits = a.bits[sub];
      const int E = 32 / bits;
      const uint32_t cmask = (1u << bits) - 1u;
      const int row_bytes = D * bits / 8, q_bytes = row_bytes / 4;
      const int64_t slot = (int64_t)begin + first + t;
      const uint8_t* row = a.kc[sub] + (((int64_t)b * a.Hkv + hk) * a.cap[sub] + slot) * row_bytes + kq * q_bytes;
      const int nwords = q_bytes / 4;
      for (int wi = 0; wi < nwords; ++wi) {
        const uint32_t wv = reinterpret_cast<const uint32_t*>(row)[wi];
        for (int e = 0; e < E; ++e) {
          const float code = (float)((wv >> (bits * e)) & cmask);
          const int c = kq * (D / 4) + wi * E + e;
#pragma unroll
          for (int g = 0; g < ZC_MAX_GROUP; ++g)
            if (g < G) dot[g] = fmaf(qp[g][c], code, dot[g]);
        }
      }
      position = a.pos[sub][(int64_t)b * a.cap[sub] + slot];
      if (a.k_tok) {
        ts = a.k_ts[sub][(int64_t)b * a.cap[sub] + slot];
        tz = a.k_tz[sub][(int64_t)b * a.cap[sub] + slot];
      }
    } else {
      const int64_t off = (int64_t)b * a.tk_sB + (int64_t)hk * a.tk_sH + (int64_t)(first + t) * a.tk_sL + kq * (D / 4);
      for (int c8 = 0; c8 < D / 4; c8 += 8) {
        float kv[8];
        load8<DT>(a.tail_k, off + c8, kv);
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
          for (int g = 0; g < ZC_MAX_GROUP; ++g)
            if (g < G) dot[g] = fmaf(qp[g][kq * (D / 4) + c8 + i], kv[i], dot[g]);
      }
      position = a.tail_pos0 + first + t;
    }
  }
#pragma unroll
  for (int g = 0; g < ZC_MAX_GROUP; ++g) {
    if (g < G) {
      dot[g] += __shfl_xor(dot[g], 1);
      dot[g] += __shfl_xor(dot[g], 2);
    }
  }
  if (t < ntok && kq == 0 && position >= 0 && position < a.N) {
#pragma unroll
    for (int g = 0; g < ZC_MAX_GROUP; ++g) {
      if (g < G) {
        const int64_t hq = (int64_t)b * a.Hq + hk * G + g;
        const float logit2 = ts * (dot[g] - tz * aq[g] - bq[g]);
        a.probs[hq * a.N + position] = exp2f(logit2 - a.lse[hq] * kLog2e);
      }
    }
  }
}

// scores[b, i] = mean_h ( sum_{j : row_len[j] > i} rows[j, b, h, i] ) / #{j : row_len[j] > i}
__global__ __launch_bounds__(256) void k_rows_saliency(const float* __restrict__ rows, const int32_t* __restrict__ row_len,
                                                       int P, int Hq, int64_t row_stride, int n_out, int normalize,
                                                       float* __restrict__ scores) {
  const int i = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y, B = gridDim.y;
  if (i >= n_out) return;
  float total = 0.f;
  int cnt = 0;
  for (int h = 0; h < Hq; ++h) {
    float col = 0.f;
    for (int j = 0; j < P; ++j)
      if (row_len[j] > i) col += rows[(((int64_t)j * B + b) * Hq + h) * row_stride + i];
    total += col;
  }
  for (int j = 0; j < P; ++j) cnt += row_len[j] > i ? 1 : 0;
  float s = total / (float)Hq;
  if (normalize) s = cnt > 0 ? s / (float)cnt : 0.f;
  scores[(int64_t)b * n_out + i] = s;
}

struct DequantArgs {
  const uint8_t* codes;
  const float* tok_scale;
  const float* tok_zero;
  const int32_t* pos;
  const float* chan_scale;   // this chunk and subset: [B, W]
  const float* chan_zero;
  int B, H, D, W, bits, layout, tokwise;
  int64_t cap;
  int begin, len;
  void* out;
  int64_t o_sB, o_sH, o_sL;
  int out_L;
};

// grid (slots of the subset, B): x_hat of one slot, all channels, to its token position
template <int DT>
__global__ __launch_bounds__(256) void k_dequantize_cache(DequantArgs a) {
  const int r = blockIdx.x, b = blockIdx.y;
  const int slot = a.begin + r;
  const int position = a.pos[(int64_t)b * a.cap + slot];
  if (position < 0 || position >= a.out_L) return;
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
      const int q = (a.bits == 2) ? ((tile & 1) * 2 + (tile >> 1)) : tile;     // field group of the slot's tile
      const int e = 4 * q + rr;
      const uint32_t word = reinterpret_cast<const uint32_t*>(a.codes)[((bh * (a.cap / TB) + blk) * 4 + kg) * a.D + c];
      code = (word >> (a.bits * e)) & ((1u << a.bits) - 1u);
    }
    const float cs = a.chan_scale[(int64_t)b * a.W + w], cz = a.chan_zero[(int64_t)b * a.W + w];
    store1<DT>(a.out, (int64_t)b * a.o_sB + (int64_t)h * a.o_sH + (int64_t)position * a.o_sL + c, cs * ts * ((float)code - tz - cz));
  }
}

}  // namespace zc

using namespace zc;

extern "C" int zc_decode_probs(const zc_tensor4* q, const zc_packed* Kp, const zc_tensor4* tail_k, int64_t tail_len,
                               int64_t tail_pos0, float sm_scale, const float* lse, float* probs_out, int64_t N,
                               void* stream) {
  int rc = zc_validate_tensor(q);
  if (rc) return rc;
  if (q->L != 1) return ZC_ERR_INVALID_ARG;
  rc = zc_validate_packed(Kp, false);
  if (rc) return rc;
  if (Kp->layout != ZC_LAYOUT_ROW || Kp->B != q->B || Kp->D != q->D) return ZC_ERR_INVALID_ARG;
  if (q->H % Kp->H != 0 || q->H / Kp->H > ZC_MAX_GROUP) return ZC_ERR_UNSUPPORTED;
  if (!lse || !probs_out || (reinterpret_cast<uintptr_t>(lse) & 3) || (reinterpret_cast<uintptr_t>(probs_out) & 3)) return ZC_ERR_INVALID_ARG;
  if (tail_len < 0 || tail_pos0 < 0 || N < 1 || N > 0x7fffffff || tail_pos0 + tail_len > N) return ZC_ERR_INVALID_ARG;
  if ((Kp->cap_hi > 0 && !Kp->pos_hi) || (Kp->cap_lo > 0 && !Kp->pos_lo)) return ZC_ERR_INVALID_ARG;   // token order needs the positions
  if (tail_len > 0) {
    rc = zc_validate_tensor(tail_k);
    if (rc) return rc;
    if (tail_k->dtype != q->dtype || tail_k->B != q->B || tail_k->H != Kp->H || tail_k->D != q->D || tail_k->L < tail_len)
      return ZC_ERR_INVALID_ARG;
  }
  if (q->B > 65535 || Kp->H > 65535) return ZC_ERR_UNSUPPORTED;
  int64_t seg_tiles = 0;
  for (int ci = 0; ci < Kp->n_chunks; ++ci)
    for (int s = 0; s < 2; ++s) seg_tiles += ceil_div64(Kp->chunk_table_host[4 * ci + 2 * s + 1], kProbSlots);
  const int64_t tiles = seg_tiles + ceil_div64(tail_len, kProbSlots);
  if (tiles > 0x7fffffff) return ZC_ERR_UNSUPPORTED;
  if (tiles == 0) return ZC_OK;

  ProbsArgs a;
  a.q = q->ptr; a.q_sB = q->sB; a.q_sH = q->sH;
  a.B = (int)q->B; a.Hq = (int)q->H; a.Hkv = (int)Kp->H; a.G = a.Hq / a.Hkv; a.D = (int)q->D;
  a.kc[0] = Kp->codes_hi; a.kc[1] = Kp->codes_lo;
  a.k_ts[0] = Kp->tok_scale_hi; a.k_ts[1] = Kp->tok_scale_lo;
  a.k_tz[0] = Kp->tok_zero_hi; a.k_tz[1] = Kp->tok_zero_lo;
  a.pos[0] = Kp->pos_hi; a.pos[1] = Kp->pos_lo;
  a.k_cs = Kp->chan_scale; a.k_cz = Kp->chan_zero; a.k_tok = Kp->scheme != ZC_SCHEME_CHANNEL;
  a.cap[0] = Kp->cap_hi; a.cap[1] = Kp->cap_lo;
  a.bits[0] = Kp->bits_hi; a.bits[1] = Kp->bits_lo;
  a.chunk_table = Kp->chunk_table; a.n_chunks = Kp->n_chunks;
  a.n_seg_tiles = (int)seg_tiles;
  a.tail_k = tail_len ? tail_k->ptr : nullptr;
  a.tk_sB = tail_len ? tail_k->sB : 0; a.tk_sH = tail_len ? tail_k->sH : 0; a.tk_sL = tail_len ? tail_k->sL : 0;
  a.tail_len = (int)tail_len; a.tail_pos0 = (int)tail_pos0;
  a.scale_log2 = (sm_scale == 0.f ? 1.0f / sqrtf((float)q->D) : sm_scale) * kLog2e;
  a.lse = lse; a.probs = probs_out; a.N = (int)N;
  dim3 grid((unsigned)tiles, (unsigned)a.Hkv, (unsigned)a.B);
  hipStream_t st = (hipStream_t)stream;
#define ZC_PR(DT)                                                                        \
  do {                                                                                   \
    if (q->D == 128) hipLaunchKernelGGL((k_decode_probs<DT, 128>), grid, dim3(256), 0, st, a); \
    else hipLaunchKernelGGL((k_decode_probs<DT, 64>), grid, dim3(256), 0, st, a);          \
  } while (0)
  if (q->dtype == ZC_F32) ZC_PR(ZC_F32);
  else if (q->dtype == ZC_F16) ZC_PR(ZC_F16);
  else ZC_PR(ZC_BF16);
#undef ZC_PR
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}

extern "C" int zc_rows_saliency(const float* rows, const int32_t* row_len, int32_t P, int64_t B, int64_t Hq,
                                int64_t row_stride, int64_t n_out, int32_t normalize, float* scores, void* stream) {
  if (!rows || !row_len || !scores || P < 1 || B < 1 || B > 65535 || Hq < 1 || n_out < 0 || n_out > row_stride ||
      row_stride > 0x7fffffff)
    return ZC_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(rows) & 3) || (reinterpret_cast<uintptr_t>(scores) & 3) || (reinterpret_cast<uintptr_t>(row_len) & 3))
    return ZC_ERR_INVALID_ARG;
  if (n_out == 0) return ZC_OK;
  hipLaunchKernelGGL(k_rows_saliency, dim3((unsigned)ceil_div64(n_out, 256), (unsigned)B), dim3(256), 0, (hipStream_t)stream,
                     rows, row_len, (int)P, (int)Hq, row_stride, (int)n_out, normalize ? 1 : 0, scores);
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}

extern "C" int zc_dequantize_cache(const zc_packed* p, const zc_tensor4* out, void* stream) {
  int rc = zc_validate_packed(p, false);
  if (rc) return rc;
  rc = zc_validate_tensor(out);
  if (rc) return rc;
  if (out->B != p->B || out->H != p->H || out->D != p->D) return ZC_ERR_INVALID_ARG;
  if ((p->cap_hi > 0 && !p->pos_hi) || (p->cap_lo > 0 && !p->pos_lo)) return ZC_ERR_INVALID_ARG;
  if (p->B > 65535 || out->L > 0x7fffffff) return ZC_ERR_UNSUPPORTED;
  const int64_t W = p->H * p->D;
  hipStream_t st = (hipStream_t)stream;
  for (int chunk = 0; chunk < p->n_chunks; ++chunk)
    for (int which = 0; which < 2; ++which) {
      const int32_t* row = p->chunk_table_host + 4 * chunk;
      const int begin = row[2 * which], len = row[2 * which + 1];
      if (len == 0) continue;
      DequantArgs a;
      a.codes = which ? p->codes_lo : p->codes_hi;
      a.tok_scale = which ? p->tok_scale_lo : p->tok_scale_hi;
      a.tok_zero = which ? p->tok_zero_lo : p->tok_zero_hi;
      a.pos = which ? p->pos_lo : p->pos_hi;
      const int64_t off = ((int64_t)chunk * 2 + which) * p->B * W;
      a.chan_scale = p->chan_scale + off;
      a.chan_zero = p->chan_zero + off;
      a.B = (int)p->B; a.H = (int)p->H; a.D = (int)p->D; a.W = (int)W;
      a.bits = which ? p->bits_lo : p->bits_hi;
      a.layout = p->layout;
      a.tokwise = p->scheme != ZC_SCHEME_CHANNEL;
      a.cap = which ? p->cap_lo : p->cap_hi;
      a.begin = begin; a.len = len;
      a.out = out->ptr; a.o_sB = out->sB; a.o_sH = out->sH; a.o_sL = out->sL; a.out_L = (int)out->L;
      dim3 grid((unsigned)len, (unsigned)p->B);
      if (out->dtype == ZC_F32) hipLaunchKernelGGL(k_dequantize_cache<ZC_F32>, grid, dim3(256), 0, st, a);
      else if (out->dtype == ZC_F16) hipLaunchKernelGGL(k_dequantize_cache<ZC_F16>, grid, dim3(256), 0, st, a);
      else hipLaunchKernelGGL(k_dequantize_cache<ZC_BF16>, grid, dim3(256), 0, st, a);
      ZC_LAUNCH_CHECK();
    }
  return ZC_OK;
}
