// zc_prefill_attention: the attention output of every prompt token at once and the
// log-normaliser of every row (Algorithm 2's attention line: Eq. 2 applied to V, with
// the causal mask).  The log-normalisers of the probe rows are what Eq. 9 needs to
// turn a logit into a probability, so zc_probe_saliency given them (lse_ext) runs its
// column sweep only.
//
// One workgroup per 128 query rows of a (batch, query head), a wave per 32 of them;
// 64-key tiles of K and V stream through LDS, long row blocks are launched first.
//   logits  D[key][query]     = sum_c K[key][c] Q[query][c]        (A = K tile, B = Q rows in registers)
//   output  D[channel][query] = sum_key Vt[channel][key] P[query][key]   (A = V tile transposed, B = P)
// Both results put a query in a lane (column r = lane & 31): the running maximum, the
// sum and the rescaling of a row are lane-local (one exchange between the two
// half-waves, which hold different keys of the same query), and the probabilities a
// lane has just computed are, converted in place, exactly the B operand of the
// second product - the order of the keys inside a matrix instruction's k index is
// free as long as both operands use the same one, and the transposed V tile is
// written to LDS in the order the logit accumulators imply.
// K tiles go global -> LDS directly; V tiles pass through registers, where four
// consecutive keys of eight (four) channels are transposed before they are stored.
#include <type_traits>

#include "mfma_tiles.hpp"

namespace zc {

struct PrefillArgs {
  const void *q, *k, *v;
  void* o;
  int64_t q_sB, q_sH, q_sL, k_sB, k_sH, k_sL, v_sB, v_sH, v_sL, o_sB, o_sH, o_sL;
  int B, Hq, Hkv, G, L;
  float scale_log2;
  float* lse;   // [B, Hq, L] natural log, or null
};

constexpr int kPfRows = 128;   // query rows per workgroup
constexpr int kPfKeys = 64;    // keys per tile

// The transposed V tile in LDS: one row per channel, the tile's 64 keys along it.
template <int DT>
struct VtLayout {
  static constexpr int EB = (DT == ZC_F32) ? 4 : 2;
  static constexpr int ROWB = kPfKeys * EB + 16;   // (+16: consecutive channels start four banks apart)
  // Keys a lane feeds to one matrix-instruction chunk: the accumulators v = VPC * s ..
  // VPC * (s + 1) - 1 of a 32-key logit tile, i.e. for 16-bit types the keys
  // 16 s + {4 kh .. 4 kh + 3, 8 + 4 kh .. 8 + 4 kh + 3} of half-wave kh, for fp32 the
  // keys 8 s + 4 kh .. + 3.  A row stores them contiguously per half-wave.
  static constexpr int VPC = (DT == ZC_F32) ? 4 : 8;
  // byte offset inside a row of the four consecutive keys 4 g .. 4 g + 3
  __device__ static int key4_offset(int g) {
    if constexpr (DT == ZC_F32) return g * 16;
    else return (16 * (g >> 2) + 8 * (g & 1) + 4 * ((g >> 1) & 1)) * 2;
  }
  // byte offset of the operand chunk of half-wave kh for chunk pc of the tile
  __device__ static int chunk_offset(int pc, int kh) { return (2 * VPC * pc + VPC * kh) * EB; }
};

template <int DT>
__device__ inline uint32_t pack_pair(float lo, float hi) {
  typedef float f2 __attribute__((ext_vector_type(2)));
  if constexpr (DT == ZC_F16) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{lo, hi}, h2));
  } else {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{lo, hi}, b2));
  }
}

template <int DT, int D>
__global__ __launch_bounds__(256, (DT == ZC_F32) ? 1 : 2) void k_prefill_attention(PrefillArgs a) {
  using T = Tile<DT, D>;
  using VT = VtLayout<DT>;
  constexpr int EB = T::EB;
  constexpr int KTILE_B = kPfKeys * T::ROWB;
  constexpr int VTILE_B = D * VT::ROWB;
  constexpr int NI = kPfKeys / T::RPI / 4;       // K transfers per wave and tile
  constexpr int CT = D / 32;                     // 32-channel tiles of the output
  constexpr int VPC = VT::VPC;
  constexpr int NPC = 16 / VPC;                  // operand chunks per 32-key logit tile
  constexpr int VU = 16 * T::CPR;                // V load units of a tile: 4 keys x one 16-byte chunk
  constexpr int VUPT = (VU + 255) / 256;         // units per thread
  __shared__ __align__(16) uint8_t Ks[2][KTILE_B];
  __shared__ __align__(16) uint8_t Vt[2][VTILE_B];

  // logical order: row block fastest (the longest first), then query head, then batch
  const int nqb = ceil_div(a.L, kPfRows);
  int j = xcd_contiguous(blockIdx.x, gridDim.x);
  const int q0 = (nqb - 1 - j % nqb) * kPfRows; j /= nqb;
  const int hq = j % a.Hq, b = j / a.Hq, hk = hq / a.G;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, kh = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint8_t* qb = reinterpret_cast<const uint8_t*>(a.q) + ((int64_t)b * a.q_sB + (int64_t)hq * a.q_sH) * EB;
  const uint8_t* kb = reinterpret_cast<const uint8_t*>(a.k) + ((int64_t)b * a.k_sB + (int64_t)hk * a.k_sH) * EB;
  const uint8_t* vb = reinterpret_cast<const uint8_t*>(a.v) + ((int64_t)b * a.v_sB + (int64_t)hk * a.v_sH) * EB;
  const uint32_t q_rowb = (uint32_t)(a.q_sL * EB), k_rowb = (uint32_t)(a.k_sL * EB), v_rowb = (uint32_t)(a.v_sL * EB);
  const auto rs_q = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(qb), 0, (uint32_t)(a.L - 1) * q_rowb + T::ROWB, kBufFlags);
  const auto rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(kb), 0, (uint32_t)(a.L - 1) * k_rowb + T::ROWB, kBufFlags);
  const auto rs_v = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(vb), 0, (uint32_t)(a.L - 1) * v_rowb + T::ROWB, kBufFlags);

  const int q_last = min(q0 + kPfRows, a.L) - 1;        // last real row of the block
  const int ntiles = q_last / kPfKeys + 1;               // key tiles it can see
  const int wq0 = q0 + 32 * w;                           // first row of this wave
  const int qpos = wq0 + r;                              // this lane's row

  // ---- K tile: global -> LDS directly, every wave a quarter of the transfers ----------
  const uint32_t ks_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)&Ks[0][0];
  int kvoff[NI];
#pragma unroll
  for (int jj = 0; jj < NI; ++jj) {
    const int row = (w + 4 * jj) * T::RPI + lane / T::CPR;
    kvoff[jj] = (int)(row * k_rowb) + (((lane % T::CPR) ^ T::swz(row)) << 4);
  }
  // (the tile's offset is part of the per-lane offset, which the range check sees: rows
  // past the end of K arrive as zeros)
  auto k_issue = [&](int t, int buf) {
    const int toff = (int)((uint32_t)t * kPfKeys * k_rowb);
#pragma unroll
    for (int jj = 0; jj < NI; ++jj) dma16<0>(ks_lds + buf * KTILE_B + (w + 4 * jj) * 1024, rs_k, kvoff[jj] + toff, 0);
  };
  // ---- V tile: into registers (four consecutive keys of one 16-byte chunk per unit;
  //      consecutive lanes take consecutive key groups, so that the transposed stores of
  //      a wave fill whole rows of the LDS tile) ------------------------------------------
  struct VRegs { u32x4 x[VUPT][4]; };
  auto v_issue = [&](int t, VRegs& vr) {
#pragma unroll
    for (int uu = 0; uu < VUPT; ++uu) {
      const int u = tid + 256 * uu;
      const int g4 = u & 15, cc = u >> 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = t * kPfKeys + 4 * g4 + i;
        const int voff = (u < VU && key < a.L) ? (int)((uint32_t)key * v_rowb) + cc * 16 : kOutOfRange;
        vr.x[uu][i] = __builtin_amdgcn_raw_buffer_load_b128(rs_v, voff, 0, 0);
      }
    }
  };
  auto v_store = [&](int buf, const VRegs& vr) {
#pragma unroll
    for (int uu = 0; uu < VUPT; ++uu) {
      const int u = tid + 256 * uu;
      if (u >= VU) continue;
      const int g4 = u & 15, cc = u >> 4;
      uint8_t* base = &Vt[buf][0] + VT::key4_offset(g4);
      if constexpr (DT == ZC_F32) {
        // chunk cc: channels 4 cc .. 4 cc + 3 of the four keys
        const uint32_t k0[4] = {vr.x[uu][0].x, vr.x[uu][0].y, vr.x[uu][0].z, vr.x[uu][0].w};
        const uint32_t k1[4] = {vr.x[uu][1].x, vr.x[uu][1].y, vr.x[uu][1].z, vr.x[uu][1].w};
        const uint32_t k2[4] = {vr.x[uu][2].x, vr.x[uu][2].y, vr.x[uu][2].z, vr.x[uu][2].w};
        const uint32_t k3[4] = {vr.x[uu][3].x, vr.x[uu][3].y, vr.x[uu][3].z, vr.x[uu][3].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          u32x4 o; o.x = k0[e]; o.y = k1[e]; o.z = k2[e]; o.w = k3[e];
          *reinterpret_cast<u32x4*>(base + (4 * cc + e) * VT::ROWB) = o;
        }
      } else {
        // chunk cc: channels 8 cc .. 8 cc + 7; word jw of a key holds channels 2 jw (low half) and 2 jw + 1
        const uint32_t k0[4] = {vr.x[uu][0].x, vr.x[uu][0].y, vr.x[uu][0].z, vr.x[uu][0].w};
        const uint32_t k1[4] = {vr.x[uu][1].x, vr.x[uu][1].y, vr.x[uu][1].z, vr.x[uu][1].w};
        const uint32_t k2[4] = {vr.x[uu][2].x, vr.x[uu][2].y, vr.x[uu][2].z, vr.x[uu][2].w};
        const uint32_t k3[4] = {vr.x[uu][3].x, vr.x[uu][3].y, vr.x[uu][3].z, vr.x[uu][3].w};
#pragma unroll
        for (int jw = 0; jw < 4; ++jw) {
          const uint2 even = make_uint2((k0[jw] & 0xffffu) | (k1[jw] << 16), (k2[jw] & 0xffffu) | (k3[jw] << 16));
          const uint2 odd = make_uint2((k0[jw] >> 16) | (k1[jw] & 0xffff0000u), (k2[jw] >> 16) | (k3[jw] & 0xffff0000u));
          *reinterpret_cast<uint2*>(base + (8 * cc + 2 * jw) * VT::ROWB) = even;
          *reinterpret_cast<uint2*>(base + (8 * cc + 2 * jw + 1) * VT::ROWB) = odd;
        }
      }
    }
  };

  VRegs vr;
  k_issue(0, 0);
  v_issue(0, vr);
  // this wave's query rows, straight into operand registers (rows past the end: zeros)
  u32x4 qf[T::NKC];
  {
    const int voff = qpos < a.L ? (int)((uint32_t)qpos * q_rowb) + kh * 16 : kOutOfRange;
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc) qf[kc] = __builtin_amdgcn_raw_buffer_load_b128(rs_q, voff + kc * 32, 0, 0);
  }

  v16f oacc[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[ct][i] = 0.f;
  float m = -INFINITY, l = 0.f;       // running maximum (log2 units) and this half-wave's share of the sum

  auto tile = [&](auto masked_c, int t) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int cur = t & 1;
    wait_all_loads();                 // K tile t (this wave's transfers) and V tile t (registers) have landed
    v_store(cur, vr);
    __syncthreads();                  // tile t is complete in LDS; nobody still reads the other buffers
    if (t + 1 < ntiles) { k_issue(t + 1, cur ^ 1); v_issue(t + 1, vr); }
    const int key0 = t * kPfKeys;
    if (key0 > wq0 + 31) return;      // none of this tile's keys is visible to the wave's rows

    // ---- logits of 64 keys x 32 rows ----
    v16f sacc[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) { sacc[0][i] = 0.f; sacc[1][i] = 0.f; }
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc) {
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) {
        const u32x4 af = *reinterpret_cast<const u32x4*>(&Ks[cur][T::slot(32 * jt + r, 2 * kc + kh)]);
        mma_chunk<DT>(sacc[jt], af, qf[kc]);
      }
    }
    // ---- online softmax: a lane owns one row and 32 of the tile's keys ----
    // (the maximum is taken over the raw products - the scale is positive - and the scale
    // enters with the subtraction of the reference: one fused multiply-add per logit)
    float tmax = -INFINITY;
    if constexpr (MASKED) {
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (key0 + 32 * jt + acc_row(v, kh) > qpos) sacc[jt][v] = -INFINITY;
    }
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
      for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, sacc[jt][v]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float m_new = fmaxf(m, tmax * a.scale_log2);
    if (__builtin_amdgcn_ballot_w64(m_new > m)) {
      const float alpha = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - m_new);
      l *= alpha;
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[ct][i] *= alpha;
      m = m_new;
    }
    float s[2][16];
    float psum = 0.f;
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        s[jt][v] = __builtin_amdgcn_exp2f(fmaf(sacc[jt][v], a.scale_log2, -m));   // (m is finite: key 0 is visible to every row)
        psum += s[jt][v];
      }
    l += psum;
    // ---- output += V^T P: the probabilities are the B operand as they stand ----
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
      for (int sp = 0; sp < NPC; ++sp) {
        u32x4 pb;
        if constexpr (DT == ZC_F32) {
          pb.x = __float_as_uint(s[jt][4 * sp]); pb.y = __float_as_uint(s[jt][4 * sp + 1]);
          pb.z = __float_as_uint(s[jt][4 * sp + 2]); pb.w = __float_as_uint(s[jt][4 * sp + 3]);
        } else {
          pb.x = pack_pair<DT>(s[jt][8 * sp], s[jt][8 * sp + 1]); pb.y = pack_pair<DT>(s[jt][8 * sp + 2], s[jt][8 * sp + 3]);
          pb.z = pack_pair<DT>(s[jt][8 * sp + 4], s[jt][8 * sp + 5]); pb.w = pack_pair<DT>(s[jt][8 * sp + 6], s[jt][8 * sp + 7]);
        }
        const int coff = VT::chunk_offset(jt * NPC + sp, kh);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          const u32x4 vf = *reinterpret_cast<const u32x4*>(&Vt[cur][(32 * ct + r) * VT::ROWB + coff]);
          mma_chunk<DT>(oacc[ct], vf, pb);
        }
      }
  };
  // Tiles all of whose keys every row of this wave sees need no mask: they run a copy of the
  // tile code without the position compares (the waves of a workgroup reach their diagonal at
  // different tiles, but every wave passes one barrier per tile either way).
  const int t_full = min(ntiles, (wq0 + 1) / kPfKeys);
  for (int t = 0; t < t_full; ++t) tile(std::false_type{}, t);
  for (int t = t_full; t < ntiles; ++t) tile(std::true_type{}, t);

  // ---- normalise and store: lane = row, accumulator v of tile ct = channel 32 ct + acc_row(v, kh) ----
  const float l_tot = l + __shfl_xor(l, 32);
  if (qpos < a.L) {
    const float inv = 1.f / l_tot;
    uint8_t* orow = reinterpret_cast<uint8_t*>(a.o) + ((int64_t)b * a.o_sB + (int64_t)hq * a.o_sH + (int64_t)qpos * a.o_sL) * EB;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        const int c = 32 * ct + acc_row(4 * v4, kh);        // four consecutive channels
        const float o0 = oacc[ct][4 * v4] * inv, o1 = oacc[ct][4 * v4 + 1] * inv, o2 = oacc[ct][4 * v4 + 2] * inv, o3 = oacc[ct][4 * v4 + 3] * inv;
        if constexpr (DT == ZC_F32) {
          *reinterpret_cast<float4*>(orow + c * 4) = make_float4(o0, o1, o2, o3);
        } else {
          *reinterpret_cast<uint2*>(orow + c * 2) = make_uint2(pack_pair<DT>(o0, o1), pack_pair<DT>(o2, o3));
        }
      }
    if (a.lse && kh == 0) a.lse[((int64_t)b * a.Hq + hq) * a.L + qpos] = (m + log2f(l_tot)) * kLn2;
  }
}

// lse_probe[b, h, p] = lse[b, h, probe_pos[p]]
__global__ void k_gather_lse(const float* __restrict__ lse, const int32_t* __restrict__ probe_pos, float* __restrict__ out,
                             int64_t heads, int L, int P) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= heads * P) return;
  const int64_t h = i / P;
  const int p = (int)(i % P);
  const int pos = probe_pos[p];
  out[i] = (pos >= 0 && pos < L) ? lse[h * L + pos] : 0.f;
}

template <int DT, int D>
static int launch_prefill(const PrefillArgs& a, hipStream_t st) {
  const int64_t grid = (int64_t)ceil_div(a.L, kPfRows) * a.Hq * a.B;
  hipLaunchKernelGGL((k_prefill_attention<DT, D>), dim3((unsigned)grid), dim3(256), 0, st, a);
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}

}  // namespace zc

using namespace zc;

extern "C" int zc_prefill_attention(const zc_tensor4* q, const zc_tensor4* k, const zc_tensor4* v, float sm_scale,
                                    const zc_tensor4* out, float* lse,
                                    const int32_t* probe_pos, int32_t P, float* lse_probe, void* stream) {
  int rc = zc_validate_tensor(q);
  if (rc) return rc;
  rc = zc_validate_tensor(k);
  if (rc) return rc;
  rc = zc_validate_tensor(v);
  if (rc) return rc;
  rc = zc_validate_tensor(out);
  if (rc) return rc;
  if (q->dtype != k->dtype || q->dtype != v->dtype || q->dtype != out->dtype) return ZC_ERR_INVALID_ARG;
  if (q->D != k->D || q->D != v->D || q->D != out->D) return ZC_ERR_INVALID_ARG;
  if (q->B != k->B || q->B != v->B || q->B != out->B || k->H != v->H || q->H != out->H) return ZC_ERR_INVALID_ARG;
  if (q->L < 1 || q->L != k->L || q->L != v->L || q->L != out->L) return ZC_ERR_INVALID_ARG;
  if (q->H % k->H != 0) return ZC_ERR_INVALID_ARG;
  if (lse && (reinterpret_cast<uintptr_t>(lse) & 3)) return ZC_ERR_INVALID_ARG;
  if (P < 0 || (P > 0 && (!probe_pos || !lse_probe || !lse))) return ZC_ERR_INVALID_ARG;
  if (q->B > 65535 || q->H > 65535 || q->L > 0x7fffffff - 256) return ZC_ERR_UNSUPPORTED;
  {
    // one (batch, head) slab of every tensor is addressed with 32-bit byte offsets; a tile may
    // reach up to 63 rows past the end of k and v, and "nothing" is requested at 0xFFFFF000
    const int64_t eb = q->dtype == ZC_F32 ? 4 : 2;
    if (q->L * q->sL * eb >= 0xFFFFF000ll || (k->L + 128) * k->sL * eb >= 0xFFFFF000ll ||
        (v->L + 128) * v->sL * eb >= 0xFFFFF000ll)
      return ZC_ERR_UNSUPPORTED;
  }
  const int64_t grid = ceil_div64(q->L, kPfRows) * q->H * q->B;
  if (grid > 0x7fffffff) return ZC_ERR_UNSUPPORTED;

  PrefillArgs a;
  a.q = q->ptr; a.k = k->ptr; a.v = v->ptr; a.o = out->ptr;
  a.q_sB = q->sB; a.q_sH = q->sH; a.q_sL = q->sL;
  a.k_sB = k->sB; a.k_sH = k->sH; a.k_sL = k->sL;
  a.v_sB = v->sB; a.v_sH = v->sH; a.v_sL = v->sL;
  a.o_sB = out->sB; a.o_sH = out->sH; a.o_sL = out->sL;
  a.B = (int)q->B; a.Hq = (int)q->H; a.Hkv = (int)k->H; a.G = a.Hq / a.Hkv; a.L = (int)q->L;
  a.scale_log2 = (sm_scale == 0.f ? 1.0f / sqrtf((float)q->D) : sm_scale) * kLog2e;
  a.lse = lse;
  hipStream_t st = (hipStream_t)stream;
#define ZC_PF(DT) (q->D == 128 ? launch_prefill<DT, 128>(a, st) : launch_prefill<DT, 64>(a, st))
  if (q->dtype == ZC_F32) rc = ZC_PF(ZC_F32);
  else if (q->dtype == ZC_F16) rc = ZC_PF(ZC_F16);
  else rc = ZC_PF(ZC_BF16);
#undef ZC_PF
  if (rc) return rc;
  if (P > 0) {
    const int64_t heads = q->B * q->H, n = heads * P;
    hipLaunchKernelGGL(k_gather_lse, dim3((unsigned)ceil_div64(n, 256)), dim3(256), 0, st, lse, probe_pos, lse_probe, heads, a.L, (int)P);
    ZC_LAUNCH_CHECK();
  }
  return ZC_OK;
}
