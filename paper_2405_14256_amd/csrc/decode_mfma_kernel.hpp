// Matrix-core kernel of zc_decode_attention for 2- and 4-bit caches (Eq. 4 over
// the packed cache, Algorithm 3's attention line).
//
// The packed cache is a cost line of half-blocks (32 slots: 512 B x D/32 of K
// codes and as many of V codes, equal compute at either bit width) in which
// every segment (chunk x subset) start also counts as kSegCost half-blocks.
// The waves of the S workgroups of a (batch, KV head) are workers of their own:
// the packed waves cut that line into equal contiguous runs, one each; a wave
// builds the query operand of every segment its run touches by itself (there is
// no barrier at a segment start, so the small chunks of a streaming cache spread
// over waves instead of serializing a workgroup), then walks its half-blocks with
// its own online-softmax state in registers while the blocks ahead stream into
// its LDS ring.  The full-precision tail is the role of a few waves spread over
// the workgroups.  The four waves of a workgroup merge through LDS; when several
// workgroups share one (batch, KV head) each writes a partial (m, Z, o) and
// k_decode_reduce reduces them (a kernel boundary is the cheapest device-wide
// release / acquire on this part: in-kernel fences cost more).
//
// Both products run on v_mfma_f32_16x16x32_f16 with the codes as one operand:
//   logits  D[token][n]   = sum_c code[token][c] * q'[n][c]      (A = K codes, ROW layout)
//   output  D[n][channel] = sum_t w[n][t] * code[t][channel]     (B = V codes, TGROUP layout)
// A code enters as an fp16 subnormal: masking a packed word leaves the code's
// bits somewhere in the low ten bits of each 16-bit half, which reads as
// code * 2^pos * 2^-24 (the matrix cores keep subnormal inputs).  The bit
// position pos differs from register to register; the other operand carries
// 2^(P - pos) for the same k index, so every product is code * x * 2^(P - 24) and
// one exact power of two restores the scale.  Unpacking is one AND per operand
// register and one shift per packed word.
// The 16 columns n hold the Hq/Hkv query heads of the KV head twice: the fp16
// value of the operand (n even) and its rounding residual times 2^11 (n odd), so
// the fp32 q keeps about 21 bits; the softmax weights are split the same way for
// fp32 tensors and are single fp16 numbers for 16-bit tensors.  The sum of the
// weights comes from one more MFMA against the constants 2^(pos - P).
// The packed layouts are chosen so that the 8 codes a lane feeds to one MFMA are
// contiguous bits of one 32-bit word, and so that the lane that holds a logit is
// the lane that must supply the corresponding softmax weight to the second MFMA.
// De-quantization never happens per element:
//   logit[t] = ts[t] * (dot[t] - tz[t] * sum_c q'[c] - sum_c q'[c] cz[c]),  q' = q cs sm_scale log2(e)
//   o[c]     = cs[c] * (sum_t w[t] code[t][c] - sum_t w[t] tz[t] - cz[c] sum_t w[t]),  w = p ts
#pragma once

#include "decode_args.hpp"
#include "lds_dma.hpp"

namespace zc {

// ---- time stamps for the latency analysis (bench.py --decode-timeline) ---------------------
// A build with ZC_TRACE (libzipcache_trace.so; include/zc_trace.h) records the 100 MHz
// real-time counter at the phase boundaries marked ZC_MARK below - per wave of k_decode_mfma,
// per workgroup of k_decode_reduce - into a buffer of the library, which zc_trace_fetch copies
// out.  In the library proper the marks are nothing.  A mark inside a segment is overwritten
// by the wave's next segment; waves past the buffer's end share its last row.
#ifdef ZC_TRACE
constexpr int kTraceSlots = 16;              // marks per wave (ZC_TRACE_SLOTS of zc_trace.h)
constexpr int kTraceWaves = 8192;            // rows for waves of k_decode_mfma (ZC_TRACE_WAVES)
constexpr int kTraceHeads = 2048;            // rows of 4 marks for workgroups of k_decode_reduce (ZC_TRACE_HEADS)
static __device__ unsigned long long zc_trace_buf[kTraceWaves * kTraceSlots + kTraceHeads * 4];
#define ZC_TRACE_WAVE_ROW(wave_)                                                                        \
  unsigned long long* zc_tp =                                                                           \
      &zc_trace_buf[(size_t)min((int)(((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 4 + (wave_)), kTraceWaves - 1) * kTraceSlots]; \
  asm volatile("" : "+v"(zc_tp))
#define ZC_TRACE_HEAD_ROW(head_) \
  unsigned long long* zc_tp = &zc_trace_buf[(size_t)kTraceWaves * kTraceSlots + (size_t)min((int)(head_), kTraceHeads - 1) * 4]
#define ZC_MARK(i) do { if ((threadIdx.x & 63) == 0) zc_tp[(i)] = wall_clock64(); } while (0)
#define ZC_MARK_LOADED(i) do { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); ZC_MARK(i); } while (0)
#else
#define ZC_TRACE_WAVE_ROW(wave_) ((void)0)
#define ZC_TRACE_HEAD_ROW(head_) ((void)0)
#define ZC_MARK(i) ((void)0)
#define ZC_MARK_LOADED(i) ((void)0)
#endif

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));

constexpr float kLoScale = 2048.f;          // residual operand is scaled by 2^11
constexpr float kLoInv = 1.f / 2048.f;
constexpr int kCombineMax = 32;             // most workgroups per (batch, KV head) on this path

__device__ inline f4 mfma16(u4 a, u4 b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
}

// Two encodings of a code as an fp16 operand element.
//  * subnormal (16-bit tensors): the masked bits of the packed word, read as
//    code * 2^pos * 2^-24; the other operand carries 2^(P - pos).  The matrix
//    cores align the products of one instruction by their nominal exponents, so a
//    code low in the mantissa loses up to 8 of the 24 accumulator bits; that is far
//    below what 16-bit outputs resolve, but too coarse for fp32 tensors.
//  * normalized (fp32 tensors): 1 + code / SC, the code OR-ed into the top mantissa
//    bits of 1.0 (SC = 16 or 4); the other operand carries SC and the "1" terms are
//    removed with the sum of the other operand.  Exact to the accumulator's 24 bits.
// Register i of unpack4 holds code i (low half) and code i + 4 (high half);
// register i of unpack2 holds codes (i, i + 8) for half 0, (4 + i, 12 + i) for half 1.
template <bool SUBN>
__device__ inline u4 unpack4(uint32_t w) {
  u4 r;
  if constexpr (SUBN) {
    const uint32_t t = w >> 8;
    r.x = w & 0x000F000Fu;
    r.y = w & 0x00F000F0u;
    r.z = t & 0x000F000Fu;
    r.w = t & 0x00F000F0u;
  } else {
    const uint32_t M = 0x03C003C0u, E = 0x3C003C00u;
    r.x = ((w << 6) & M) | E;
    r.y = ((w << 2) & M) | E;
    r.z = ((w >> 2) & M) | E;
    r.w = ((w >> 6) & M) | E;
  }
  return r;
}
template <bool SUBN>
__device__ inline u4 unpack2(uint32_t w, int half) {
  if (half) w >>= 8;
  u4 r;
  if constexpr (SUBN) {
    r.x = w & 0x00030003u;
    r.y = w & 0x000C000Cu;
    r.z = w & 0x00300030u;
    r.w = w & 0x00C000C0u;
  } else {
    const uint32_t M = 0x03000300u, E = 0x3C003C00u;
    r.x = ((w << 8) & M) | E;
    r.y = ((w << 6) & M) | E;
    r.z = ((w << 4) & M) | E;
    r.w = ((w << 2) & M) | E;
  }
  return r;
}
// The factor the other operand carries for operand register i (both halves).
template <int BITS, bool SUBN> __device__ inline float code_comp(int i) {
  if constexpr (!SUBN) return BITS == 4 ? 16.f : 4.f;
  else if constexpr (BITS == 4) return (i & 1) ? 1.f : 16.f;
  else return (float)(64 >> (2 * i));
}
template <int BITS, bool SUBN> __device__ inline int code_comp_log2(int i) {
  if constexpr (!SUBN) return BITS == 4 ? 4 : 2;
  else if constexpr (BITS == 4) return (i & 1) ? 0 : 4;
  else return 6 - 2 * i;
}
// product of a code and x, divided by what the matrix cores accumulate for it
template <int BITS, bool SUBN> constexpr float code_unscale() {
  return SUBN ? (float)(1 << (24 - (BITS == 4 ? 4 : 6))) : 1.f;
}

__device__ inline uint32_t pack_h2(_Float16 lo, _Float16 hi) {
  uint16_t a, b;
  __builtin_memcpy(&a, &lo, 2);
  __builtin_memcpy(&b, &hi, 2);
  return (uint32_t)a | ((uint32_t)b << 16);
}

// Two floats rounded to fp16 in one register (v_cvt_pk_f16_f32).
__device__ inline uint32_t pack_f2(float lo, float hi) {
  typedef float f2 __attribute__((ext_vector_type(2)));
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2{lo, hi}, h2));
}

// Splits x into the fp16 nearest to it and the scaled residual; returns the one
// this lane feeds (part 0: value, part 1: residual).
__device__ inline _Float16 split_part(float x, int part) {
  const _Float16 hi = (_Float16)x;
  const _Float16 lo = (_Float16)((x - (float)hi) * kLoScale);
  return part ? lo : hi;
}
__device__ inline float half_lo_to_float(uint32_t w) {
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  return (float)__builtin_bit_cast(h2, w).x;
}
__device__ inline float half_hi_to_float(uint32_t w) {
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  return (float)__builtin_bit_cast(h2, w).y;
}

__device__ inline float xor1(float x) {   // value of the neighbouring lane (lane ^ 1)
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, true));
}
// Reductions over the four 16-lane rows of a wave with the register-pair swaps of this part
// (vector instructions; a shuffle through the LDS crossbar costs a wave that runs alone on its
// SIMD a round trip each).  v_permlane16_swap exchanges the odd rows of its first operand with
// the even rows of its second, v_permlane32_swap the upper half of the first with the lower
// half of the second.
//   rows16(a, b): rows 0, 2 hold a summed over the row pair, rows 1, 3 hold b;
//   halves32(a, b): lanes 0-31 hold a summed over the two halves, lanes 32-63 hold b.
__device__ inline float rows16(float a, float b) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ inline float halves32(float a, float b) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ inline float grp_max(float x) {  // over the four 16-lane groups, in every lane
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float grp_sum(float x) {  // (row r + row r^1) + (the other pair), as the shuffles gave it
  x = rows16(x, x);
  return halves32(x, x);
}
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Eight consecutive elements of a tensor of dtype DT, as loaded (the conversion
// to float happens where they are used, so that many loads can be in flight).
template <int DT> struct Raw8 { uint4 a; };
template <> struct Raw8<ZC_F32> { uint4 a, b; };
template <int DT>
__device__ inline void raw_to_float(const Raw8<DT>& r, float (&v)[8]) {
  if constexpr (DT == ZC_F32) {
    v[0] = __uint_as_float(r.a.x); v[1] = __uint_as_float(r.a.y); v[2] = __uint_as_float(r.a.z); v[3] = __uint_as_float(r.a.w);
    v[4] = __uint_as_float(r.b.x); v[5] = __uint_as_float(r.b.y); v[6] = __uint_as_float(r.b.z); v[7] = __uint_as_float(r.b.w);
  } else {
    const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = half_bits_to_float<DT>(w[i] & 0xffffu);
      v[2 * i + 1] = half_bits_to_float<DT>(w[i] >> 16);
    }
  }
}

// MINB: workgroups per CU the register budget is sized for.  2 for launches that
// fill the chip; 1 (the whole register file, nothing spilled to scratch) for
// launches of at most one workgroup per CU, where only latency counts.
// STG: the operand's inputs reach LDS by transfers of their own (see the segment): for waves
// with short runs, where a segment's start is a large part of a wave's time.
template <int DT, int D, bool KTOK, bool VTOK, int MINB, bool STG>
__global__ __launch_bounds__(256, MINB) void k_decode_mfma(DecArgs a) {
  constexpr int KS = D / 32;     // k-steps of the logit product
  constexpr int NR = D / 64;     // 16-byte V loads per lane and block
  constexpr int MG = ZC_MAX_GROUP;
  __shared__ __align__(16) float svc[4][256];    // per wave: channel scales [0, D) and zeros [D, 2 D) of V for its current segment (one 1 KB transfer)
  // Per wave a ring of kStages staging buffers for one block of the packed cache
  // each: K codes (D * 16 bytes), V codes (D * 16 bytes), then 256 bytes each of
  // V token scale, V token zero, K token scale, K token zero.  After its last block a
  // wave's ring holds its partial output for the merge (mO).
  constexpr int kStages = 3;
  constexpr int kCodeBytes = D * 16;
  constexpr int kOnesOff = 2 * kCodeBytes + 1024;     // 256 bytes of 1.0f: what the sum-of-p rows read as "token scale"
  constexpr int kStageBytes = kOnesOff + 256;
  constexpr int kRingBytes = kStages * kStageBytes;
  static_assert(kRingBytes >= MG * D * 4, "a wave's ring must hold its partial output");
  __shared__ __align__(16) uint8_t ring[4][kRingBytes];
  auto mO = [&](int w, int gg, int c) -> float& { return reinterpret_cast<float*>(&ring[w][0])[gg * D + c]; };
  __shared__ float mM[4][MG], mZ[4][MG];
  __shared__ float ptile[4][MG][kTailUnit];

  const int s = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int n = lane & 15, grp = lane >> 4;
  const int G = a.G;
  ZC_TRACE_WAVE_ROW(wave);
  ZC_MARK(0);                                   // entry
  const int g = n >> 1, part = n & 1;
  const bool nvalid = n < 2 * G;
  const int g0 = 2 * grp, g1 = 2 * grp + 1;      // heads of this lane's rows in the output tiles
  constexpr bool WSPLIT = (DT == ZC_F32);    // softmax weights as value + residual
  constexpr bool SUBN = (DT != ZC_F32);      // codes enter as fp16 subnormals
  // q' always enters as value + residual (two columns per head).  A single fp16 q'
  // was tried for 16-bit tensors: it saves two instructions per logit but moves the
  // log-sum-exp by up to 3e-3, which the streaming saliency scores inherit.
  constexpr bool QSPLIT = true;

  // running state of this wave; unused columns sit at +inf so that their weights are 0
  float m_run = nvalid ? -INFINITY : INFINITY, z_part = 0.f;
  float Zrun0 = 0.f, Zrun1 = 0.f;            // unsplit weights: sum of p of heads g0, g1 (from the matrix cores)
#pragma unroll
  for (int st = 0; st < kStages; ++st)       // each wave fills (and later reads) its own ring
    reinterpret_cast<float*>(&ring[wave][st * kStageBytes + kOnesOff])[lane] = 1.f;
  float O[NR][4][2];
#pragma unroll
  for (int r = 0; r < NR; ++r)
#pragma unroll
    for (int j = 0; j < 4; ++j) { O[r][j][0] = 0.f; O[r][j][1] = 0.f; }

  // The chunk table that travels in the kernel arguments, one entry per lane: requested first
  // of all (a vector load takes longer than the scalar loads below; whether the table is in
  // the arguments or in memory, these words exist) and used by the chunk loop, which takes its
  // rows from the lanes (a scalar load per row would be a dependent round trip per segment).
  const int rows_v = a.chunk_rows[min(lane, 4 * kInlineChunks - 1)];
  // Likewise the first 64 words of the arguments (everything up to the chunk table), word i in
  // lane i: what a segment starts from - the arrays of its subset, the channel parameters, the
  // query - is read from these lanes, a register read each.  As scalar arguments they cost
  // either registers the kernel does not have (some forty, held from the start) or, fetched
  // where they are used, a round trip per segment; and a choice between the two subsets'
  // arrays is compiled as a choice between the ADDRESSES of the two arguments followed by a
  // load and a wait (per lane, for the channel parameters: three dependent round trips before
  // a segment's first transfer could be issued).
  static_assert(offsetof(DecArgs, chunk_rows) <= 256 && sizeof(DecArgs) >= 256, "the lane table covers the fields before the chunk table");
  // (Only where latency counts, STG: on a compute unit that streams a long cache the answer to
  // a vector load queues behind the other waves' transfers, and a scalar load does not - 16
  // prompts of 4096 tokens with 40 heads took 63.1 us per call this way against 60.9.)
  int args_v = 0;
  if constexpr (STG) args_v = ((const __attribute__((address_space(4))) int*)__builtin_amdgcn_kernarg_segment_ptr())[lane];
  auto arg32 = [&](size_t byte_off) { return __builtin_amdgcn_readlane(args_v, (int)(byte_off / 4)); };
  auto arg64 = [&](size_t byte_off) {
    return (uint64_t)(uint32_t)__builtin_amdgcn_readlane(args_v, (int)(byte_off / 4)) |
           ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(args_v, (int)(byte_off / 4) + 1) << 32);
  };
  // Everything the start of a wave needs from the kernel arguments is requested here, in
  // one batch of scalar loads: left to itself the compiler fetches each field where the
  // control flow first needs it, a dozen dependent round trips before the first load of data.
  {
    int i0 = a.S, i1 = a.n_pw, i2 = a.n_tw, i3 = a.tw_full, i4 = a.tw_rem, i5 = a.tail_alone, i6 = a.pw_q, i7 = a.pw_r,
        i8 = a.tu_q, i9 = a.tu_r, i10 = a.n_chunks, i11 = a.chunks_inline, i12 = a.G, i13 = a.Hq, i14 = a.Hkv, i15 = a.B,
        i16 = a.tail_len;
    float f0 = a.scale_log2;
    int64_t l0 = a.q_sB, l1 = a.q_sH;
    const void *p0 = a.q, *p13 = a.chunk_table;
    asm volatile("" :: "s"(i0), "s"(i1), "s"(i2), "s"(i3), "s"(i4), "s"(i5), "s"(i6), "s"(i7), "s"(i8), "s"(i9), "s"(i10),
                 "s"(i11), "s"(i12), "s"(i13), "s"(i14), "s"(i15), "s"(i16), "s"(f0));
    int64_t t0 = a.tk_sB, t1 = a.tk_sH, t2 = a.tk_sL, t3 = a.tv_sB, t4 = a.tv_sH, t5 = a.tv_sL;
    const void *t6 = a.tail_k, *t7 = a.tail_v;
    asm volatile("" :: "s"(t0), "s"(t1), "s"(t2), "s"(t3), "s"(t4), "s"(t5), "s"(t6), "s"(t7));
    asm volatile("" :: "s"(l0), "s"(l1), "s"(p0), "s"(p13));
  }

  ZC_MARK(1);                                   // the first batch of arguments is in registers
  // What the packed waves need again at their chunk loop: held in scalar registers from here
  // on (as outputs of an empty asm statement they cannot be fetched again where they are used,
  // which the compiler otherwise does - two more dependent round trips before the loop).
  int p_n_chunks = a.n_chunks, p_inline = a.chunks_inline, p_B = a.B, p_Hkv = a.Hkv;
  float p_scale = a.scale_log2;
  asm volatile("" : "+s"(p_n_chunks), "+s"(p_inline), "+s"(p_B), "+s"(p_Hkv), "+s"(p_scale));

  // The waves of the workgroups of one (batch, KV head) are workers of their own:
  // n_tw of them take the full-precision tail, the other n_pw share the cost line of
  // the packed cache (half-blocks + kSegCost per segment start, a contiguous run each).
  // The tail waves are spread over the workgroups -- the last wave of the last
  // workgroups first -- because the tail's loads are many small rows, and one CU
  // has only so many misses in flight.
  // (tail_alone, for launches well below one workgroup per CU where only latency counts:
  // the last n_tw workgroups carry one tail wave each and nothing else)
  // (the split's parameters, pinned like the ones above: the compiler would rather fetch an
  // argument again than keep it in a register, a dependent round trip before the wave knows its run)
  int p_S = a.S, p_n_tw = a.n_tw, p_tw_full = a.tw_full, p_tw_rem = a.tw_rem, p_alone = a.tail_alone, p_pw_q = a.pw_q, p_pw_r = a.pw_r;
  asm volatile("" : "+s"(p_S), "+s"(p_n_tw), "+s"(p_tw_full), "+s"(p_tw_rem), "+s"(p_alone), "+s"(p_pw_q), "+s"(p_pw_r));
  const int my_tails = p_alone ? (s >= p_S - p_n_tw ? 4 : 0) : p_tw_full + (s >= p_S - p_tw_rem ? 1 : 0);
  const bool tail_wave = wave >= 4 - my_tails;
  const int pw = p_alone ? 4 * s + wave
                         : 4 * s - p_tw_full * s - max(0, s - (p_S - p_tw_rem)) + wave;    // index among the packed waves
  // (unit j of the line belongs to packed wave j / q for the first r * (q + 1) units, where the
  // host has divided n_units = q * n_pw + r: the first r waves take one unit more; no division here)
  const int u0 = tail_wave ? 0 : p_pw_q * pw + min(pw, p_pw_r);
  const int u1 = tail_wave ? 0 : p_pw_q * (pw + 1) + min(pw + 1, p_pw_r);

  // The running reference of a head's softmax is only touched when some slot of the
  // half-block exceeds it (a ballot, no data movement otherwise); everything
  // accumulated so far is then rescaled.  Rare after the first half-blocks - but a wave of a
  // short cache has only one or two: its first half-block, which finds nothing accumulated
  // yet, only takes the maximum over, and the factors of the heads of a lane's output rows
  // (columns 4 grp and 4 grp + 2; every row holds the same factors) come from row broadcasts
  // with a row mask instead of two shuffles through the LDS crossbar (head_columns, update_ref).
  // x of this lane's row at columns 4 grp and 4 grp + 2 (the value columns of heads g0 and g1):
  // row broadcasts under a row mask (a value that is the same in every row comes out the same
  // way a shuffle from lanes 2 g0 and 2 g1 would deliver it, without the trip through LDS).
  auto head_columns = [&](float x, float& c0, float& c1) {
    const int xi = __float_as_int(x);
    int i0 = __builtin_amdgcn_update_dpp(0, xi, 0x150, 0x1, 0xF, false);       // row 0 <- its lane 0
    i0 = __builtin_amdgcn_update_dpp(i0, xi, 0x154, 0x2, 0xF, false);          // row 1 <- its lane 4
    i0 = __builtin_amdgcn_update_dpp(i0, xi, 0x158, 0x4, 0xF, false);          // row 2 <- its lane 8
    i0 = __builtin_amdgcn_update_dpp(i0, xi, 0x15C, 0x8, 0xF, false);          // row 3 <- its lane 12
    int i1 = __builtin_amdgcn_update_dpp(0, xi, 0x152, 0x1, 0xF, false);       // lanes 2, 6, 10, 14
    i1 = __builtin_amdgcn_update_dpp(i1, xi, 0x156, 0x2, 0xF, false);
    i1 = __builtin_amdgcn_update_dpp(i1, xi, 0x15A, 0x4, 0xF, false);
    i1 = __builtin_amdgcn_update_dpp(i1, xi, 0x15E, 0x8, 0xF, false);
    c0 = __int_as_float(i0); c1 = __int_as_float(i1);
  };
  // The packed waves keep their logits relative to the running reference m_ref of their column:
  // the reference is folded into the constant that the logit's last multiply-add adds anyway
  // (shift[v] - m_ref), so a weight is exp2 of what that instruction delivers - no subtraction
  // per logit - and "a slot exceeds the reference" is "a relative logit above 0".  The first
  // half-block of a wave takes its maximum over as the reference (nothing is accumulated yet);
  // later ones only raise it, rescaling what is accumulated.  lg: this half-block's relative
  // logits, re-referenced here when the reference moves; rel[v] = base[v] - m_ref.
  float m_ref = nvalid ? 0.f : INFINITY;       // (unused columns: every relative logit -inf, weight 0)
  bool seen = false;                            // (wave-uniform) a half-block has been taken in
  auto update_ref = [&](float lmax, float (&lg)[2][4], float (&rel)[4], const float (&base)[4], float (&a1)[4], f4 (*acc)[4],
                        f4& acc1) {
    if (!seen || __builtin_amdgcn_ballot_w64(lmax > 0.f)) {
      float delta = grp_max(lmax);
      if (seen) {
        delta = fmaxf(delta, 0.f);              // (0 where nothing moved, and in unused columns)
        const float fac = fast_exp2(-delta);
        z_part *= fac;
#pragma unroll
        for (int v = 0; v < 4; ++v) a1[v] *= fac;
        float f0, f1;
        head_columns(fac, f0, f1);
        Zrun0 *= f0; Zrun1 *= f1;
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            O[r][j][0] *= f0; O[r][j][1] *= f1;
            acc[r][j].x *= f0; acc[r][j].y *= f0; acc[r][j].z *= f1; acc[r][j].w *= f1;
          }
        acc1.x *= f0; acc1.y *= f0; acc1.z *= f1; acc1.w *= f1;
      } else {
        delta = nvalid ? delta : 0.f;           // (the first reference may lie below 0)
      }
      m_ref += delta;
#pragma unroll
      for (int v = 0; v < 4; ++v) rel[v] = base[v] - m_ref;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int v = 0; v < 4; ++v) lg[jj][v] -= delta;
      seen = true;
    }
  };

  // The query operand of a segment.  Every wave builds its own (all k-steps): the
  // waves of a workgroup then share nothing until the final merge, so each can
  // work through its own run of segments without a barrier.
  // MODE 4 / 2: codes of that width, q' = q cs sm_scale log2(e) times the factor of
  // its operand register, in the channel order the unpacked K words have; MODE 0:
  // the tail, q itself in natural order.
  // Returns the operand registers and sum(q'), sum(q' cz) over all channels, and the same
  // two sums over the 32 channels of every k-step (what the normalized encoding needs to
  // keep its accumulators centred, see the segment).
  // qsrc + qoff (elements): the query row of this lane's head; kcs, kcz: the K channel
  // parameters of the segment.  In global memory, or in LDS when a packed segment has had
  // the rows and the parameters brought there (see the segment).
  auto build_query_operand = [&](auto mode_c, const void* qsrc, int64_t qoff, const float* kcs, const float* kcz,
                                 u4 (&qB)[KS], float& sumqq, float& sumqqcz, float (&sum_k)[KS], float (&sumcz_k)[KS]) {
    constexpr int MODE = decltype(mode_c)::value;
    // q and the channel parameters of this lane's elements of every k-step
    float q8[KS][8], cs8[KS][8], cz8[KS][8];
#pragma unroll
    for (int ks0 = 0; ks0 < KS; ++ks0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) { cs8[ks0][i] = 1.f; cz8[ks0][i] = 0.f; }
      if constexpr (MODE == 2) {
        // slots (i, half) are channels base + 4 (ks0 & 1) + i + 8 half of a 16-channel word
        const int base = grp * (D / 4) + 16 * (ks0 >> 1) + 4 * (ks0 & 1);
        float qa[8], qb[8];
        load8<DT>(qsrc, qoff + base - 4 * (ks0 & 1), qa);
        load8<DT>(qsrc, qoff + base - 4 * (ks0 & 1) + 8, qb);
        const float4 ca = *reinterpret_cast<const float4*>(kcs + base);
        const float4 cb = *reinterpret_cast<const float4*>(kcs + base + 8);
        const float4 za = *reinterpret_cast<const float4*>(kcz + base);
        const float4 zb = *reinterpret_cast<const float4*>(kcz + base + 8);
        const float csa[4] = {ca.x, ca.y, ca.z, ca.w}, csb[4] = {cb.x, cb.y, cb.z, cb.w};
        const float cza[4] = {za.x, za.y, za.z, za.w}, czb[4] = {zb.x, zb.y, zb.z, zb.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          q8[ks0][2 * i] = qa[4 * (ks0 & 1) + i]; q8[ks0][2 * i + 1] = qb[4 * (ks0 & 1) + i];
          cs8[ks0][2 * i] = csa[i]; cs8[ks0][2 * i + 1] = csb[i];
          cz8[ks0][2 * i] = cza[i]; cz8[ks0][2 * i + 1] = czb[i];
        }
      } else {
        // MODE 4: slots (i, half) are channels base + i + 4 half; MODE 0: base + 2 i + half
        const int base = (MODE == 4) ? grp * (D / 4) + 8 * ks0 : 32 * ks0 + 8 * grp;
        float qa[8];
        load8<DT>(qsrc, qoff + base, qa);
        float ca[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f}, za[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if constexpr (MODE == 4) {
          const float4 c0 = *reinterpret_cast<const float4*>(kcs + base), c1 = *reinterpret_cast<const float4*>(kcs + base + 4);
          const float4 z0 = *reinterpret_cast<const float4*>(kcz + base), z1 = *reinterpret_cast<const float4*>(kcz + base + 4);
          ca[0] = c0.x; ca[1] = c0.y; ca[2] = c0.z; ca[3] = c0.w; ca[4] = c1.x; ca[5] = c1.y; ca[6] = c1.z; ca[7] = c1.w;
          za[0] = z0.x; za[1] = z0.y; za[2] = z0.z; za[3] = z0.w; za[4] = z1.x; za[5] = z1.y; za[6] = z1.z; za[7] = z1.w;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const int e = (MODE == 4) ? i + 4 * half : 2 * i + half;
            q8[ks0][2 * i + half] = qa[e]; cs8[ks0][2 * i + half] = ca[e]; cz8[ks0][2 * i + half] = za[e];
          }
      }
    }
    // Value and residual columns: the residual of the query operand is NOT scaled, so its
    // column comes out of the matrix cores in the unit of the value column and the two are
    // simply added.  A residual below 2^-14 is an fp16 subnormal (absolute step 2^-24),
    // which bounds the error of a logit by 2^-25 per channel and code unit.
    // Unused columns get q' = 0.  For 16-bit tensors the sums take q' itself rather than
    // the value the two fp16 columns represent (they differ by 2^-22 relative: nothing
    // next to the rounding of a 16-bit output); fp32 tensors take the represented value.
    const float lane_scale = nvalid ? p_scale : 0.f;
    float sq = 0.f, sqz = 0.f;
#pragma unroll
    for (int ks0 = 0; ks0 < KS; ++ks0) {
      const float sq_before = sq, sqz_before = sqz;
      uint32_t regs[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float comp = (MODE == 0) ? 1.f : code_comp<MODE == 0 ? 4 : MODE, SUBN>(i);
        const float qn0 = q8[ks0][2 * i] * lane_scale * cs8[ks0][2 * i], qn1 = q8[ks0][2 * i + 1] * lane_scale * cs8[ks0][2 * i + 1];
        const float qv0 = qn0 * comp, qv1 = qn1 * comp;
        if constexpr (QSPLIT) {
          const uint32_t hi2 = pack_f2(qv0, qv1);                       // both values rounded to fp16
          const float h0 = half_lo_to_float(hi2), h1 = half_hi_to_float(hi2);
          const uint32_t lo2 = pack_f2(qv0 - h0, qv1 - h1);             // the residuals (exact differences), rounded
          regs[i] = part ? lo2 : hi2;
          if constexpr (SUBN) {
            sq += qn0 + qn1;
            sqz = fmaf(qn0, cz8[ks0][2 * i], fmaf(qn1, cz8[ks0][2 * i + 1], sqz));
          } else {
            const float inv_comp = 1.f / comp;      // a power of two
            const float r0 = (h0 + half_lo_to_float(lo2)) * inv_comp, r1 = (h1 + half_hi_to_float(lo2)) * inv_comp;
            sq += r0 + r1;
            sqz = fmaf(r0, cz8[ks0][2 * i], fmaf(r1, cz8[ks0][2 * i + 1], sqz));
          }
        } else {
          regs[i] = pack_f2(qv0, qv1);
          sq += qn0 + qn1;
          sqz = fmaf(qn0, cz8[ks0][2 * i], fmaf(qn1, cz8[ks0][2 * i + 1], sqz));
        }
      }
      qB[ks0].x = regs[0]; qB[ks0].y = regs[1]; qB[ks0].z = regs[2]; qB[ks0].w = regs[3];
      if constexpr (!SUBN && MODE != 0) {
        sum_k[ks0] = grp_sum(sq - sq_before);
        sumcz_k[ks0] = grp_sum(sqz - sqz_before);
      } else {
        sum_k[ks0] = 0.f; sumcz_k[ks0] = 0.f;
      }
    }
    sumqq = grp_sum(sq);
    sumqqcz = grp_sum(sqz);
  };

  // Combines the (m, Z, o) the four waves left in LDS and writes the workgroup's
  // result: the output itself when it is the only workgroup of its KV head.
  // (Everything is read from LDS before anything is computed, and a wave without tokens -
  // m = -inf; its sums are zeros - takes part with weight 0 instead of being branched
  // around: this is the end of the call's critical path, and with a branch per wave the
  // reads went out one dependent round trip after the other.)
  auto write_result = [&]() {
    const bool direct = a.S == 1;
    constexpr int NIT = MG * D / 256;               // most elements per thread
    static_assert(256 % D == 0, "a thread's elements share their channel");
    const int c = tid % D, g_first = tid / D;       // (tid is below 256: shifts and masks)
    const int64_t hq0 = (int64_t)b * a.Hq + hk * G; // first head of this KV head's group
    float pm[NIT][4], pz[NIT][4], po[NIT][4];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      if (256 * it >= G * D) break;                 // (wave-uniform)
      const int gg = min(g_first + it * (256 / D), G - 1);       // (element tid + 256 it: head gg, channel c)
#pragma unroll
      for (int w = 0; w < 4; ++w) { pm[it][w] = mM[w][gg]; pz[it][w] = mZ[w][gg]; po[it][w] = mO(w, gg, c); }
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int gg = g_first + it * (256 / D);
      if (gg >= G) break;
      const float M = fmaxf(fmaxf(pm[it][0], pm[it][1]), fmaxf(pm[it][2], pm[it][3]));
      float o = 0.f, z = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float f = (pm[it][w] > -INFINITY) ? fast_exp2(pm[it][w] - M) : 0.f;
        o = fmaf(po[it][w], f, o);
        z = fmaf(pz[it][w], f, z);
      }
      // (the uniform part of every index in scalar registers, the thread's own part in 32 bits)
      if (direct) {
        store1<DT>(a.out, hq0 * D + (gg * D + c), z > 0.f ? o / z : 0.f);
        if (a.lse_out && c == 0) a.lse_out[hq0 + gg] = (M + log2f(z)) * kLn2;
      } else {
        const int64_t row0 = hq0 * a.S + s;
        a.part_o[row0 * D + ((gg * a.S) * D + c)] = o;
        if (c == 0) { a.part_m[row0 + gg * a.S] = M; a.part_z[row0 + gg * a.S] = z; }
      }
    }
  };

  // ---------------- full-precision tail: waves of its own ---------------------------------
  // Units of kTailUnit tokens (one 16-row MFMA tile).  All K and V rows of a unit are
  // requested before the query operand is built, so the unit costs one trip to
  // memory.  Logits on the matrix cores (K rows as the A operand); the weighted
  // sum of V on the vector ALUs, lane = (token mod TPI, 8 channels).
  if (tail_wave) {
    constexpr int LPT = D / 8, TPI = 64 / LPT, NI = kTailUnit / TPI, NJ = kTailUnit / 16;
    const int tw = (3 - wave) * a.S + (a.S - 1 - s);     // index among the tail waves
    const bool working = tw < a.n_tw;              // (tail_alone: only the last wave of a tail workgroup works)
    // the tail's units over its waves, as above: units = tu_q * n_tw + tu_r
    const int wlo = working ? a.tu_q * tw + min(tw, a.tu_r) : 0, whi = working ? a.tu_q * (tw + 1) + min(tw + 1, a.tu_r) : 0;
    // Buffer resources over this (batch, KV head)'s rows of the tail: rows past its end are
    // asked for at an offset beyond the buffer and arrive as zeros (no branch per load).
    constexpr int EB = (DT == ZC_F32) ? 4 : 2;
    constexpr int kTailFlags = 0x00020000;
    constexpr int kTailOOR = (int)0xFFFFF000u;
    const uint8_t* tkp = reinterpret_cast<const uint8_t*>(a.tail_k) + ((int64_t)b * a.tk_sB + (int64_t)hk * a.tk_sH) * EB;
    const uint8_t* tvp = reinterpret_cast<const uint8_t*>(a.tail_v) + ((int64_t)b * a.tv_sB + (int64_t)hk * a.tv_sH) * EB;
    const uint32_t tk_rowb = (uint32_t)a.tk_sL * EB, tv_rowb = (uint32_t)a.tv_sL * EB;
    const auto rs_tk = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(tkp), 0, (uint32_t)(a.tail_len - 1) * tk_rowb + D * EB, kTailFlags);
    const auto rs_tv = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(tvp), 0, (uint32_t)(a.tail_len - 1) * tv_rowb + D * EB, kTailFlags);
    const int vtok = lane / LPT, vch = 8 * (lane % LPT);
    auto load8 = [&](__amdgpu_buffer_rsrc_t rs, int voff) {
      Raw8<DT> r;
      const u4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, 0, 0);
      r.a = uint4{x.x, x.y, x.z, x.w};
      if constexpr (DT == ZC_F32) {
        const u4 y = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 16, 0, 0);
        r.b = uint4{y.x, y.y, y.z, y.w};
      }
      return r;
    };
    struct TBuf {
      Raw8<DT> k[NJ][KS];
      Raw8<DT> v[NI];
    };
    auto load_unit = [&](int tu, TBuf& bf) {
      const int t0 = tu * kTailUnit;
      const int ntok = min(kTailUnit, a.tail_len - t0);
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int row = 16 * j + n;
        const int voff = row < ntok ? (int)((uint32_t)(t0 + row) * tk_rowb) + 8 * grp * EB : kTailOOR;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bf.k[j][ks] = load8(rs_tk, voff + 32 * ks * EB);
      }
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int row = i * TPI + vtok;
        bf.v[i] = load8(rs_tv, row < ntok ? (int)((uint32_t)(t0 + row) * tv_rowb) + vch * EB : kTailOOR);
      }
    };
    // 16-bit tensors: two units are in flight, so a wave with at most two units pays one
    // trip to memory (fp32 rows take twice the registers: one unit at a time)
    constexpr bool kTwoUnits = (DT != ZC_F32);
    TBuf bf0, bf1;
    if (wlo < whi) load_unit(wlo, bf0);
    if (kTwoUnits && wlo + 1 < whi) load_unit(wlo + 1, bf1);
    u4 qB[KS];
    float dummy0, dummy1;
    float dummy_k[KS], dummy_kz[KS];
    build_query_operand(std::integral_constant<int, 0>{}, a.q, (int64_t)b * a.q_sB + (int64_t)(hk * G + (nvalid ? g : 0)) * a.q_sH,
                        nullptr, nullptr, qB, dummy0, dummy1, dummy_k, dummy_kz);
    float Ot[MG][8];
#pragma unroll
    for (int gg = 0; gg < MG; ++gg)
#pragma unroll
      for (int i = 0; i < 8; ++i) Ot[gg][i] = 0.f;

    auto tail_unit = [&](int tu, const TBuf& bf) {
      const int ntok = min(kTailUnit, a.tail_len - tu * kTailUnit);
      float U[NJ][4];
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        // rows past the end of the tail are zeros; every lane takes part in the MFMAs
        f4 s_hi = f4{0.f, 0.f, 0.f, 0.f}, s_lo = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          if constexpr (DT == ZC_F16) {
            u4 ah; ah.x = bf.k[j][ks].a.x; ah.y = bf.k[j][ks].a.y; ah.z = bf.k[j][ks].a.z; ah.w = bf.k[j][ks].a.w;
            s_hi = mfma16(ah, qB[ks], s_hi);
          } else {
            float kv[8];
            raw_to_float<DT>(bf.k[j][ks], kv);
            uint32_t rh[4], rl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              if constexpr (DT == ZC_F32) {
                const _Float16 h0 = (_Float16)kv[2 * i], h1 = (_Float16)kv[2 * i + 1];
                rh[i] = pack_h2(h0, h1);
                rl[i] = pack_h2((_Float16)((kv[2 * i] - (float)h0) * kLoScale), (_Float16)((kv[2 * i + 1] - (float)h1) * kLoScale));
              } else {
                rh[i] = pack_f2(kv[2 * i], kv[2 * i + 1]);
              }
            }
            u4 ah; ah.x = rh[0]; ah.y = rh[1]; ah.z = rh[2]; ah.w = rh[3];
            s_hi = mfma16(ah, qB[ks], s_hi);
            if constexpr (DT == ZC_F32) {
              u4 al; al.x = rl[0]; al.y = rl[1]; al.z = rl[2]; al.w = rl[3];
              s_lo = mfma16(al, qB[ks], s_lo);
            }
          }
        }
        const float own[4] = {s_hi.x + s_lo.x * kLoInv, s_hi.y + s_lo.y * kLoInv, s_hi.z + s_lo.z * kLoInv, s_hi.w + s_lo.w * kLoInv};
#pragma unroll
        for (int v = 0; v < 4; ++v) U[j][v] = QSPLIT ? own[v] + xor1(own[v]) : own[v];
      }
      float lmax = -INFINITY;
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          if (16 * j + 4 * grp + v >= ntok) U[j][v] = -INFINITY;
          lmax = fmaxf(lmax, U[j][v]);
        }
      // a unit holds at least one token, so the new maximum is finite
      const float m_new = fmaxf(m_run, grp_max(lmax));
      if (__any(nvalid && m_new > m_run)) {
        const float fac = (m_run > -INFINITY) ? fast_exp2(m_run - m_new) : 0.f;
        z_part *= fac;
#pragma unroll
        for (int gg = 0; gg < MG; ++gg) {
          if (gg < G) {
            const float fg = __shfl(fac, 2 * gg);
#pragma unroll
            for (int i = 0; i < 8; ++i) Ot[gg][i] *= fg;
          }
        }
      }
      m_run = m_new;
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float p = nvalid ? fast_exp2(U[j][v] - m_run) : 0.f;     // 0 past the end of the tail
          z_part += p;
          if (nvalid && part == 0) ptile[wave][g][16 * j + 4 * grp + v] = p;
        }
      // weighted sum of the unit's V rows (ptile is written and read by this wave only)
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        float vv[8];
        raw_to_float<DT>(bf.v[i], vv);
#pragma unroll
        for (int gg = 0; gg < MG; ++gg) {
          if (gg < G) {
            const float p = ptile[wave][gg][i * TPI + vtok];
#pragma unroll
            for (int e = 0; e < 8; ++e) Ot[gg][e] = fmaf(p, vv[e], Ot[gg][e]);
          }
        }
      }
    };
    if constexpr (kTwoUnits) {
      for (int tu = wlo; tu < whi; tu += 2) {
        tail_unit(tu, bf0);
        if (tu + 2 < whi) load_unit(tu + 2, bf0);
        if (tu + 1 < whi) {
          tail_unit(tu + 1, bf1);
          if (tu + 3 < whi) load_unit(tu + 3, bf1);
        }
      }
    } else {
      for (int tu = wlo; tu < whi; ++tu) {
        if (tu > wlo) load_unit(tu, bf0);
        tail_unit(tu, bf0);
      }
    }
    // merge: sum the token sub-rows, then the four waves through LDS.  Four values at a
    // time are summed over the four rows with three swaps and three additions, after which
    // row r holds the sum of value r - and writes it.
    const float z_tot = grp_sum(z_part);
    if (nvalid && part == 0 && grp == 0) { mM[wave][g] = m_run; mZ[wave][g] = z_tot; }
#pragma unroll
    for (int gg = 0; gg < MG; ++gg) {
      if (gg < G) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            x[e] = Ot[gg][4 * h + e];
            if constexpr (LPT == 8) x[e] += __shfl_xor(x[e], 8);      // (D = 64: two tokens per row)
          }
          const float sum = halves32(rows16(x[0], x[1]), rows16(x[2], x[3]));
          if ((lane & 15) < LPT) mO(wave, gg, vch + 4 * h + grp) = sum;
        }
      }
    }
  }

  if (tail_wave) ZC_MARK(8);                    // a tail wave has finished its units
  int cursor = 0;
  // ---------------- packed segments --------------------------------------------------
  auto segment = [&](auto bits_c, int ci, int sub, int begin, int len, int lo, int hi) {
    constexpr int BITS = decltype(bits_c)::value;
    constexpr int TB = 4 * (32 / BITS), NH = TB / 32;   // slots and half-blocks per block
    constexpr int KW = D * BITS / 128;                  // 32-bit words of K codes per lane and token
    constexpr int ROWB = D * BITS / 8;                  // bytes of one K row
    constexpr float UNSCALE = code_unscale<BITS, SUBN>();
    constexpr float SC = (BITS == 4) ? 16.f : 4.f;     // normalized encoding: 1 + code / SC
    const int64_t chan_off = ((int64_t)(ci * 2 + sub) * p_B + b) * (p_Hkv * D) + hk * D;
    // lo, hi: this wave's range of the segment in half-blocks (not empty)
    const int hlo = lo, hhi = hi;

    // Buffer resources over this (batch, KV head)'s part of each array: the
    // per-lane offset is fixed, the half-block adds a scalar offset, reads past
    // the end return zeros.  (The host checks that each part is below 4 GiB.)
    const int64_t bh = (int64_t)b * p_Hkv + hk;
    // (selects between the two subsets' kernel arguments, which are in registers already:
    // an index would be another scalar load and another wait)
    int64_t cap, p_qsB, p_qsH;
    const uint8_t* kc;
    const uint32_t* vc;
    const float *k_ts = nullptr, *k_tz = nullptr, *v_ts = nullptr, *v_tz = nullptr, *p_kcs, *p_kcz, *p_vcs, *p_vcz;
    const void* p_q;
    if constexpr (STG) {
      const size_t so = 8 * (size_t)sub;                // (a lane index in a scalar register)
      cap = (int64_t)arg64(offsetof(DecArgs, cap) + so);
      kc = reinterpret_cast<const uint8_t*>(arg64(offsetof(DecArgs, kc) + so));
      vc = reinterpret_cast<const uint32_t*>(arg64(offsetof(DecArgs, vc) + so));
      if constexpr (KTOK) {
        k_ts = reinterpret_cast<const float*>(arg64(offsetof(DecArgs, k_ts) + so));
        k_tz = reinterpret_cast<const float*>(arg64(offsetof(DecArgs, k_tz) + so));
      }
      if constexpr (VTOK) {
        v_ts = reinterpret_cast<const float*>(arg64(offsetof(DecArgs, v_ts) + so));
        v_tz = reinterpret_cast<const float*>(arg64(offsetof(DecArgs, v_tz) + so));
      }
      p_kcs = reinterpret_cast<const float*>(arg64(offsetof(DecArgs, k_cs)));
      p_kcz = reinterpret_cast<const float*>(arg64(offsetof(DecArgs, k_cz)));
      p_vcs = reinterpret_cast<const float*>(arg64(offsetof(DecArgs, v_cs)));
      p_vcz = reinterpret_cast<const float*>(arg64(offsetof(DecArgs, v_cz)));
      p_q = reinterpret_cast<const void*>(arg64(offsetof(DecArgs, q)));
      p_qsB = (int64_t)arg64(offsetof(DecArgs, q_sB)); p_qsH = (int64_t)arg64(offsetof(DecArgs, q_sH));
    } else {
      cap = sub ? a.cap[1] : a.cap[0];
      kc = sub ? a.kc[1] : a.kc[0];
      vc = sub ? a.vc[1] : a.vc[0];
      k_ts = sub ? a.k_ts[1] : a.k_ts[0]; k_tz = sub ? a.k_tz[1] : a.k_tz[0];
      v_ts = sub ? a.v_ts[1] : a.v_ts[0]; v_tz = sub ? a.v_tz[1] : a.v_tz[0];
      p_kcs = a.k_cs; p_kcz = a.k_cz; p_vcs = a.v_cs; p_vcz = a.v_cz;
      p_q = a.q; p_qsB = a.q_sB; p_qsH = a.q_sH;
    }
    const uint32_t code_bytes = (uint32_t)(cap * ROWB);
    const uint32_t tok_bytes = (uint32_t)(cap * 4);
    constexpr int kRsrcFlags = 0x00020000;              // raw 32-bit data, no swizzle
    const auto rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(kc + bh * (int64_t)code_bytes), 0, code_bytes, kRsrcFlags);
    const auto rs_v = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(reinterpret_cast<const uint8_t*>(vc) + bh * (int64_t)code_bytes), 0, code_bytes, kRsrcFlags);
    const int64_t tokbase = (int64_t)b * cap;
    const auto rs_kts = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(KTOK ? k_ts + tokbase : nullptr), 0, KTOK ? tok_bytes : 0, kRsrcFlags);
    const auto rs_ktz = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(KTOK ? k_tz + tokbase : nullptr), 0, KTOK ? tok_bytes : 0, kRsrcFlags);
    const auto rs_vts = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(VTOK ? v_ts + tokbase : nullptr), 0, VTOK ? tok_bytes : 0, kRsrcFlags);
    const auto rs_vtz = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(VTOK ? v_tz + tokbase : nullptr), 0, VTOK ? tok_bytes : 0, kRsrcFlags);
    // Staging: block bi of the segment is D * 16 contiguous bytes of K codes and as
    // many of V codes; each goes to LDS with KCH 1 KB transfers.  (Token parameters:
    // 64 floats per array, of which a 4-bit block uses - and requests - the first 32.)
    constexpr int KCH = D / 64;                           // 1 KB transfers per code array and block
    constexpr int L_STAGE = 2 * KCH + (VTOK ? 2 : 0) + (KTOK ? 2 : 0);   // transfers per block
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)&ring[wave][0];
    const uint8_t* ring_gen = &ring[wave][0];
    const int bl_lo = hlo / NH, bl_hi = hlo < hhi ? (hhi - 1) / NH + 1 : hlo / NH;    // this wave's blocks
    // (live == false: the same number of transfers, all out of range -- they move
    // zeros and touch no memory -- so that the wait counts below are constants)
    // (A token-parameter transfer is 64 floats, a 4-bit block 32 slots: lanes past the block
    // ask out of range too.  The block's offset travels in the scalar offset, which the
    // range check does not see, so for the last block of an arena that is full to its
    // capacity those lanes would otherwise read past the end of the array.)
    const int tok_lane = (4 * lane) | ((TB < 64 && lane >= TB) ? (int)0xFFFFF000u : 0);
    auto issue = [&](uint32_t dst, int bi, bool live) {
      const int ko = (int)((uint32_t)(begin + bi * TB) * (uint32_t)ROWB);          // = block index * D * 16
      const int to = (int)((uint32_t)(begin + bi * TB) * 4u);
      const int oob = live ? 0 : (int)0xFFFFF000u;     // per-lane offsets beyond any buffer the host admits
      const int v16 = (16 * lane) | oob, v4 = tok_lane | oob;
      dma16<0>(dst, rs_k, v16, ko);
      if constexpr (KCH == 2) dma16<1024>(dst, rs_k, v16, ko);
      dma16<0>(dst + kCodeBytes, rs_v, v16, ko);
      if constexpr (KCH == 2) dma16<1024>(dst + kCodeBytes, rs_v, v16, ko);
      if constexpr (VTOK) {
        dma4(dst + 2 * kCodeBytes, rs_vts, v4, to);
        dma4(dst + 2 * kCodeBytes + 256, rs_vtz, v4, to);
      }
      if constexpr (KTOK) {
        dma4(dst + 2 * kCodeBytes + 512, rs_kts, v4, to);
        dma4(dst + 2 * kCodeBytes + 768, rs_ktz, v4, to);
      }
    };
    // Launches whose waves have short runs (STG; always when only latency counts): what the
    // query operand is built from goes to LDS by three or four transfers of its own (with a
    // load per lane and k-step - some thirty of them, each with its address arithmetic - a wave
    // needed 0.8 us just to issue them): the K channel scales and zeros (1 KB: lanes pick their
    // 16-byte piece of either array) and the query rows of the KV head's G heads go to the
    // ring's last stage, which is free until the block loop's first request; the V channel
    // scales and zeros go to svc, where they wait until the segment is folded.  Launches that
    // fill the chip keep the loads per lane: there the transfers cost throughput (16 prompts
    // of 4096 tokens with 40 heads: 61 -> 62.5 us per call with them, 79 -> 84 us with cold caches).
    constexpr bool STAGED = STG;
    constexpr int ESZ = (DT == ZC_F32) ? 4 : 2;
    constexpr int PA = D / 4;                           // 16-byte pieces of a parameter row
    constexpr int PR = D * ESZ / 16, RP = 64 / PR;      // 16-byte pieces of a query row; rows per transfer
    constexpr int NQ = (MG + RP - 1) / RP;
    static_assert(1024 + NQ * 1024 <= kStageBytes, "the parameters fit a stage of the ring");
    const uint32_t par_lds = ring_lds + (kStages - 1) * kStageBytes;
    const uint8_t* par = ring_gen + (kStages - 1) * kStageBytes;
    if constexpr (STAGED) {
      const int piece = lane % PA;
      const bool zeros = (lane / PA) & 1;
      gdma16(par_lds, (zeros ? p_kcz : p_kcs) + chan_off + 4 * piece);
      gdma16((uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)&svc[wave][0],
             (zeros ? p_vcz : p_vcs) + chan_off + 4 * piece);
      const uint8_t* qrows = reinterpret_cast<const uint8_t*>(p_q) + ((int64_t)b * p_qsB + (int64_t)hk * G * p_qsH) * ESZ + 16 * (lane % PR);
#pragma unroll
      for (int t = 0; t < NQ; ++t)
        if (t * RP < G)                                 // (wave-uniform; rows past the last head repeat it)
          gdma16(par_lds + 1024 + t * 1024, qrows + (int64_t)min(t * RP + lane / PR, G - 1) * p_qsH * ESZ);
    }
    // the first blocks are in flight while the operand is built
#pragma unroll
    for (int i = 0; i < kStages - 1; ++i) issue(ring_lds + i * kStageBytes, bl_lo + i, bl_lo + i < bl_hi);

    u4 qB[KS];
    float Aq, sumqcz, Aq_k[KS], sumqcz_k[KS];
    if constexpr (STAGED) {
      wait_vmem<(kStages - 1) * L_STAGE>();             // the parameters have landed (the blocks need not have)
      build_query_operand(std::integral_constant<int, BITS>{}, par + 1024, (int64_t)(nvalid ? g : 0) * D,
                          reinterpret_cast<const float*>(par), reinterpret_cast<const float*>(par) + D, qB, Aq, sumqcz, Aq_k, sumqcz_k);
    } else {
      // the V channel parameters wait in this wave's part of LDS until the segment is folded
      if (lane < D / 2) {
        const bool zero_half = lane >= D / 4;
        const int c4 = 4 * (zero_half ? lane - D / 4 : lane);
        const float4 t = *reinterpret_cast<const float4*>((zero_half ? p_vcz : p_vcs) + chan_off + c4);
        *reinterpret_cast<float4*>(&svc[wave][(zero_half ? D : 0) + c4]) = t;
      }
      build_query_operand(std::integral_constant<int, BITS>{}, p_q, (int64_t)b * p_qsB + (int64_t)(hk * G + (nvalid ? g : 0)) * p_qsH,
                          p_kcs + chan_off, p_kcz + chan_off, qB, Aq, sumqcz, Aq_k, sumqcz_k);
    }
    ZC_MARK(2);                                 // the segment's query operand is built
    // Subnormal codes: the logit is ts (dot - tz sum(q') - sum(q' cz)), the two sums taken off
    // after the matrix instructions.  Normalized codes (fp32 tensors) add SC sum(q') to the
    // accumulator on top; there everything that is taken off is taken off k-step by k-step,
    // between the matrix instructions, so that the accumulator never holds more than one
    // k-step's worth of what cancels: with fp64 as the yardstick a quarter of the rounding
    // error when sum(q') is large (queries with a common component, a large token scale).
    //   corr_c[ks] + tz corr_s[ks], in accumulator units; value column only (the residual
    //   column is added to it afterwards)
    const float kconst = SUBN ? -sumqcz : 0.f;
    float corr_c[KS], corr_s[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      corr_c[ks] = (SUBN || part) ? 0.f : -(SC * Aq_k[ks] + sumqcz_k[ks]) * (1.f / UNSCALE);
      corr_s[ks] = (SUBN || part) ? 0.f : -Aq_k[ks] * (1.f / UNSCALE);
    }
    // factor of operand register v of the weights.  When the weights are not split,
    // the second row of a head carries p instead of w = p ts: its product with the
    // constants below is the sum of p (the softmax denominator), at no VALU cost
    float wcomp[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) wcomp[v] = code_comp<BITS, SUBN>(v);
    // Unsplit weights: that factor (a power of two) is folded into the logit, so exp2
    // delivers p times the factor; the running maximum is then the maximum of the
    // shifted logits, which is as good a reference point as the true one.
    // base[v]: what the last multiply-add of a logit adds (tokenwise keys: the factor's power;
    // else that plus the segment's constant); rel[v] = base[v] - m_ref is what it adds here.
    float base[4], rel[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float lshift = WSPLIT ? 0.f : (float)code_comp_log2<BITS, SUBN>(v);
      base[v] = KTOK ? lshift : kconst + lshift;
      rel[v] = base[v] - m_ref;
    }
    // B operand that sums the weights: 1 / factor of each operand register
    // (normalized codes: plain ones, the sum then carries SC and is also the "1" term of the output product)
    u4 ones;
    if constexpr (!SUBN) ones = u4{0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
    else if constexpr (BITS == 4) ones = u4{0x2C002C00u, 0x3C003C00u, 0x2C002C00u, 0x3C003C00u};   // 1/16, 1, 1/16, 1
    else ones = u4{0x24002400u, 0x2C002C00u, 0x34003400u, 0x3C003C00u};                            // 1/64, 1/16, 1/4, 1

    f4 acc[NR][4];
    f4 acc1 = f4{0.f, 0.f, 0.f, 0.f};     // sum of the weights
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[r][j] = f4{0.f, 0.f, 0.f, 0.f};
    float a1[4] = {0.f, 0.f, 0.f, 0.f};   // sum of w tz, one per operand register of the weights

    // this lane's addresses in the current stage (they move with the ring, once per
    // block); the half-block adds constants
    const uint8_t* kbase = ring_gen + n * ROWB + grp * (KW * 4);
    const uint8_t* vbase = ring_gen + kCodeBytes + grp * (D * 4) + 16 * n;
    const uint8_t* tbase = ring_gen + 2 * kCodeBytes + 16 * grp;
    const uint8_t* tsbase = (!WSPLIT && part) ? ring_gen + kOnesOff : tbase;
    auto half_block = [&](auto h_c, int hb) {
      constexpr int SB = 0;
      constexpr int h = decltype(h_c)::value;
      // operands of this half-block from the staging buffer
      struct { uint32_t kw[2][KW]; u4 vw[NR]; u4 kts[2], ktz[2], vts[2], vtz[2]; } bf;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const uint8_t* kp = kbase + SB + 16 * (2 * h + jj) * ROWB;
        if constexpr (KW == 4) { const u4 t = *reinterpret_cast<const u4*>(kp); bf.kw[jj][0] = t.x; bf.kw[jj][1] = t.y; bf.kw[jj][2] = t.z; bf.kw[jj][3] = t.w; }
        else if constexpr (KW == 2) { const uint2 t = *reinterpret_cast<const uint2*>(kp); bf.kw[jj][0] = t.x; bf.kw[jj][1] = t.y; }
        else { bf.kw[jj][0] = *reinterpret_cast<const uint32_t*>(kp); }
        const uint8_t* tp = tbase + SB + 64 * (2 * h + jj);
        if constexpr (VTOK) {
          bf.vts[jj] = *reinterpret_cast<const u4*>(tsbase + SB + 64 * (2 * h + jj));
          bf.vtz[jj] = *reinterpret_cast<const u4*>(tp + 256);
        }
        if constexpr (KTOK) { bf.kts[jj] = *reinterpret_cast<const u4*>(tp + 512); bf.ktz[jj] = *reinterpret_cast<const u4*>(tp + 768); }
      }
#pragma unroll
      for (int r = 0; r < NR; ++r) bf.vw[r] = *reinterpret_cast<const u4*>(vbase + SB + 256 * r);
      const int ntok = len - 32 * hb;                  // slots of this half-block inside the segment, >= 1
      const bool masked = ntok < 32;                   // only the last half-block of a segment
      float lg[2][4], vts[2][4], vtz[2][4];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const float kts[4] = {__uint_as_float(bf.kts[jj].x), __uint_as_float(bf.kts[jj].y), __uint_as_float(bf.kts[jj].z), __uint_as_float(bf.kts[jj].w)};
        const float ktz[4] = {__uint_as_float(bf.ktz[jj].x), __uint_as_float(bf.ktz[jj].y), __uint_as_float(bf.ktz[jj].z), __uint_as_float(bf.ktz[jj].w)};
        f4 sacc = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          if constexpr (BITS == 4) sacc = mfma16(unpack4<SUBN>(bf.kw[jj][ks]), qB[ks], sacc);
          else sacc = mfma16(unpack2<SUBN>(bf.kw[jj][ks >> 1], ks & 1), qB[ks], sacc);
          if constexpr (!SUBN) {
            if constexpr (KTOK) {
              sacc.x += fmaf(ktz[0], corr_s[ks], corr_c[ks]); sacc.y += fmaf(ktz[1], corr_s[ks], corr_c[ks]);
              sacc.z += fmaf(ktz[2], corr_s[ks], corr_c[ks]); sacc.w += fmaf(ktz[3], corr_s[ks], corr_c[ks]);
            } else {
              sacc.x += corr_c[ks]; sacc.y += corr_c[ks]; sacc.z += corr_c[ks]; sacc.w += corr_c[ks];
            }
          }
        }
        const float own[4] = {sacc.x, sacc.y, sacc.z, sacc.w};
        vts[jj][0] = __uint_as_float(bf.vts[jj].x); vts[jj][1] = __uint_as_float(bf.vts[jj].y);
        vts[jj][2] = __uint_as_float(bf.vts[jj].z); vts[jj][3] = __uint_as_float(bf.vts[jj].w);
        vtz[jj][0] = __uint_as_float(bf.vtz[jj].x); vtz[jj][1] = __uint_as_float(bf.vtz[jj].y);
        vtz[jj][2] = __uint_as_float(bf.vtz[jj].z); vtz[jj][3] = __uint_as_float(bf.vtz[jj].w);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float x;
          const float dot = QSPLIT ? own[v] + xor1(own[v]) : own[v];     // value + residual column
          if constexpr (KTOK && !SUBN) x = fmaf(kts[v], dot * UNSCALE, rel[v]);        // already centred
          else if constexpr (KTOK) x = fmaf(kts[v], fmaf(-ktz[v], Aq, fmaf(dot, UNSCALE, kconst)), rel[v]);
          else x = fmaf(dot, UNSCALE, rel[v]);
          lg[jj][v] = x;
        }
      }
      if (masked) {
        // slots past the end of the segment: no weight, and their per-token
        // parameters were never written
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const bool live = 16 * jj + 4 * grp + v < ntok;
            lg[jj][v] = live ? lg[jj][v] : -INFINITY;
            vts[jj][v] = live ? vts[jj][v] : 0.f;
            vtz[jj][v] = live ? vtz[jj][v] : 0.f;
          }
      }
      const float lmax = fmaxf(fmaxf(fmaxf(fmaxf(lg[0][0], lg[0][1]), lg[0][2]), fmaxf(fmaxf(lg[0][3], lg[1][0]), lg[1][1])),
                               fmaxf(lg[1][2], lg[1][3]));       // three v_max3 and one v_max
      update_ref(lmax, lg, rel, base, a1, acc, acc1);
      // weights w = p ts and the A operand of the output product
      float w2[2][4];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float p = fast_exp2(lg[jj][v]);              // 0 for masked slots and unused columns
          float w = p;
          if constexpr (VTOK) {
            w = p * vts[jj][v];
            a1[v] = fmaf(w, vtz[jj][v], a1[v]);
          }
          if constexpr (WSPLIT) { z_part += p; w2[jj][v] = w * wcomp[v]; }
          else w2[jj][v] = w;
        }
      u4 pA;
      if constexpr (WSPLIT) {
        pA.x = pack_h2(split_part(w2[0][0], part), split_part(w2[1][0], part));
        pA.y = pack_h2(split_part(w2[0][1], part), split_part(w2[1][1], part));
        pA.z = pack_h2(split_part(w2[0][2], part), split_part(w2[1][2], part));
        pA.w = pack_h2(split_part(w2[0][3], part), split_part(w2[1][3], part));
      } else {
        pA.x = pack_f2(w2[0][0], w2[1][0]); pA.y = pack_f2(w2[0][1], w2[1][1]);
        pA.z = pack_f2(w2[0][2], w2[1][2]); pA.w = pack_f2(w2[0][3], w2[1][3]);
      }
      acc1 = mfma16(pA, ones, acc1);
#pragma unroll
      for (int r = 0; r < NR; ++r) {
        const uint32_t ww[4] = {bf.vw[r].x, bf.vw[r].y, bf.vw[r].z, bf.vw[r].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if constexpr (BITS == 4) acc[r][j] = mfma16(pA, unpack4<SUBN>(ww[j]), acc[r][j]);
          else acc[r][j] = mfma16(pA, unpack2<SUBN>(ww[j], h), acc[r][j]);
        }
      }
    };

    // Blocks in turn through the ring: the block kStages - 1 ahead is requested (out of
    // range past the wave's last block), then the wave waits for all but the two blocks'
    // loads issued after the current one's.
    int st = 0, st_ahead = kStages - 1;
    uint32_t dst_ahead = ring_lds + (kStages - 1) * kStageBytes;
    for (int bi = bl_lo; bi < bl_hi; ++bi) {
      dma_reuse_fence();                         // the reads of the buffer about to be refilled are complete
      issue(dst_ahead, bi + kStages - 1, bi + kStages - 1 < bl_hi);
      wait_vmem<(kStages - 1) * L_STAGE>();
      if (bi == bl_lo) ZC_MARK(3);              // the segment's first block has landed
      if constexpr (NH == 1) {
        half_block(std::integral_constant<int, 0>{}, bi);
      } else {
        const unsigned span = (unsigned)(hhi - hlo);
        if ((unsigned)(bi * NH - hlo) < span) half_block(std::integral_constant<int, 0>{}, bi * NH);
        if ((unsigned)(bi * NH + 1 - hlo) < span) half_block(std::integral_constant<int, 1>{}, bi * NH + 1);
      }
      const int step = (st == kStages - 1) ? -(kStages - 1) * kStageBytes : kStageBytes;
      kbase += step; vbase += step; tbase += step; tsbase += step;
      st = (st == kStages - 1) ? 0 : st + 1;
      dst_ahead = (st_ahead == kStages - 1) ? ring_lds : dst_ahead + kStageBytes;
      st_ahead = (st_ahead == kStages - 1) ? 0 : st_ahead + 1;
    }
    ZC_MARK(4);                                 // the segment's half-blocks are done
    wait_vmem<0>();                              // the out-of-range requests have landed too
    dma_reuse_fence();                           // the ring is reused (next segment, merge)
    // ---- fold the segment into O ----
    //   subnormal codes:   sum_t w code = acc 2^(24 - P),  sum_t w = acc1
    //   normalized codes:  sum_t w code = acc - acc1,         sum_t w = acc1 / SC
    //   (value + residual / 2^11 when the weights are split)
    const float r0 = WSPLIT ? acc1.x + acc1.y * kLoInv : acc1.x;
    const float r1 = WSPLIT ? acc1.z + acc1.w * kLoInv : acc1.z;
    const float sw0 = SUBN ? r0 : r0 * (1.f / SC), sw1 = SUBN ? r1 : r1 * (1.f / SC);
    const float bias0 = SUBN ? 0.f : r0, bias1 = SUBN ? 0.f : r1;
    if constexpr (!WSPLIT) { Zrun0 += acc1.y; Zrun1 += acc1.w; }
    float a10 = 0.f, a11 = 0.f;
    if constexpr (VTOK) {
      float a1s = 0.f;
#pragma unroll
      for (int v = 0; v < 4; ++v) a1s = fmaf(a1[v], WSPLIT ? 1.f : 1.f / wcomp[v], a1s);
      a1s = grp_sum(a1s);                          // (the same in every row)
      head_columns(a1s, a10, a11);
    }
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const float4 vcs4 = *reinterpret_cast<const float4*>(&svc[wave][4 * (n + 16 * r)]);
      const float4 vcz4 = *reinterpret_cast<const float4*>(&svc[wave][D + 4 * (n + 16 * r)]);
      const float cs[4] = {vcs4.x, vcs4.y, vcs4.z, vcs4.w}, cz[4] = {vcz4.x, vcz4.y, vcz4.z, vcz4.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float t0 = ((WSPLIT ? acc[r][j].x + acc[r][j].y * kLoInv : acc[r][j].x) - bias0) * UNSCALE;
        const float t1 = ((WSPLIT ? acc[r][j].z + acc[r][j].w * kLoInv : acc[r][j].z) - bias1) * UNSCALE;
        O[r][j][0] = fmaf(cs[j], t0 - a10 - cz[j] * sw0, O[r][j][0]);
        O[r][j][1] = fmaf(cs[j], t1 - a11 - cz[j] * sw1, O[r][j][1]);
      }
    }
  };

  if (!tail_wave) {
    for (int ci = 0; ci < p_n_chunks && cursor < u1; ++ci) {
      for (int sub = 0; sub < 2; ++sub) {
        if (cursor >= u1) break;                   // the wave's run ends before this segment: nothing left to do
        // The row of the chunk table: from the lanes of rows_v when the table travels in the
        // kernel arguments, else from memory.
        int begin, len;
        if (p_inline) {
          begin = __builtin_amdgcn_readlane(rows_v, 4 * ci + 2 * sub);
          len = __builtin_amdgcn_readlane(rows_v, 4 * ci + 2 * sub + 1);
        } else {
          begin = __builtin_amdgcn_readfirstlane(a.chunk_table[4 * ci + 2 * sub]);
          len = __builtin_amdgcn_readfirstlane(a.chunk_table[4 * ci + 2 * sub + 1]);
          asm volatile("" : "+s"(begin), "+s"(len));
        }
        int bits;
        if constexpr (STG) bits = arg32(offsetof(DecArgs, bits) + 4 * (size_t)sub);
        else bits = sub ? a.bits[1] : a.bits[0];
        const int TB = 4 * (32 / bits);
        const int nb = ceil_div(len, 32);          // half-blocks of 32 slots (equal compute at either width)
        if (nb == 0) continue;
        const int seg0 = cursor + kSegCost;        // the segment's half-blocks sit after its start-up slots
        cursor = seg0 + nb;
        const int lo = max(u0 - seg0, 0), hi = min(u1 - seg0, nb);
        if (lo >= hi) continue;
        if (bits == 4) segment(std::integral_constant<int, 4>{}, ci, sub, begin, len, lo, hi);
        else segment(std::integral_constant<int, 2>{}, ci, sub, begin, len, lo, hi);
      }
    }

    ZC_MARK(5);                                 // the segments are folded
    // ---------------- this wave's partial, for the merge of the four waves ---------------
    const float m_out = seen ? m_ref : -INFINITY;    // (a wave without a half-block: empty)
    if constexpr (WSPLIT) {
      const float z_tot = grp_sum(z_part);
      if (nvalid && part == 0 && grp == 0) { mM[wave][g] = m_out; mZ[wave][g] = z_tot; }
    } else {
      if (nvalid && part == 0 && grp == 0) mM[wave][g] = m_out;
      if (n == 0) { mZ[wave][g0] = Zrun0; mZ[wave][g1] = Zrun1; }      // (rows below G are read)
    }
    // (four consecutive channels a store, and no condition on the head: the ring has rows for
    // ZC_MAX_GROUP heads, the merge reads those below G - 32 single stores, each with a branch
    // around it, were 0.4 us at the end of every wave's path)
    static_assert(2 * 3 + 1 < MG, "rows g0, g1 of every lane exist in the ring");
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const int c = 4 * (n + 16 * r);
      *reinterpret_cast<float4*>(&mO(wave, g0, c)) = make_float4(O[r][0][0], O[r][1][0], O[r][2][0], O[r][3][0]);
      *reinterpret_cast<float4*>(&mO(wave, g1, c)) = make_float4(O[r][0][1], O[r][1][1], O[r][2][1], O[r][3][1]);
    }
  }
  ZC_MARK(6);                                   // at the barrier before the merge
  __syncthreads();
  write_result();
  ZC_MARK(7);                                   // the workgroup's result is stored
}

// Reduces the partial (m, Z, o) of the workgroups of one query head.  The call's latency is
// this kernel's too, so nothing here branches: lane ss of every wave fetches (m, Z) of split
// ss with one load each (lanes past the last split repeat the last one and count as empty),
// the NMAX possible output partials of this thread's channel are requested back to back (splits
// past the last one are out of range of the buffer: zeros, with weight 0), and the weights 2^(m - M) come from one
// exponential over the lanes, handed round as scalars.  (With a branch per split - which
// loads exist depends on S - the loads took 1.6 us to issue and land, against 0.8 us here.)
// NMAX: the most splits this instance handles (8, 16, 24 or kCombineMax: the smallest that holds S -
// an output partial that does not exist still costs its load and its two instructions).
template <int DT, int D, int NMAX>
__global__ __launch_bounds__(D) void k_decode_reduce(const float* __restrict__ part_m, const float* __restrict__ part_z,
                                                      const float* __restrict__ part_o, int S,
                                                      void* __restrict__ out, float* __restrict__ lse_out) {
  static_assert(NMAX <= kCombineMax && kCombineMax <= 64, "one lane per split");
  const int64_t hq = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;  // b * Hq + h
  const int c = threadIdx.x, lane = c & 63;
  const int last = S - 1;
  ZC_TRACE_HEAD_ROW(hq);
  if (c == 0) ZC_MARK(0);                       // entry
  const int64_t row = hq * S;
  float pmv = part_m[row + min(lane, last)], pzv = part_z[row + min(lane, last)];
  // (through a buffer descriptor over this head's S rows: a row past the last is out of range
  // and arrives as zero - its weight is zero too - and the row's offset is a constant of the
  // instruction; with plain loads each address took six instructions, 0.3 us of them in
  // front of the first load)
  const auto rs_o = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(part_o + row * D), 0, (uint32_t)S * D * 4u, 0x00020000);
  float po[NMAX];
#pragma unroll
  for (int ss = 0; ss < NMAX; ++ss) po[ss] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs_o, 4 * c + ss * (D * 4), 0, 0));
  if (lane > last) { pmv = -INFINITY; pzv = 0.f; }
  if (c == 0) ZC_MARK_LOADED(1);                // the partials have landed (the trace build waits for them here)
  // maximum over the lanes: inside the rows of 16, then row to row into lane 63 (vector
  // instructions with lane permutation; no round trips through the LDS crossbar)
  float M = pmv;
  M = fmaxf(M, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(M), __float_as_int(M), 0x111, 0xF, 0xF, false)));   // row_shr:1
  M = fmaxf(M, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(M), __float_as_int(M), 0x112, 0xF, 0xF, false)));   // row_shr:2
  M = fmaxf(M, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(M), __float_as_int(M), 0x114, 0xF, 0xF, false)));   // row_shr:4
  M = fmaxf(M, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(M), __float_as_int(M), 0x118, 0xF, 0xF, false)));   // row_shr:8
  M = fmaxf(M, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(M), __float_as_int(M), 0x142, 0xA, 0xF, false)));   // row_bcast:15
  M = fmaxf(M, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(M), __float_as_int(M), 0x143, 0xC, 0xF, false)));   // row_bcast:31
  M = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(M), 63));
  const float fv = (pmv > -INFINITY) ? fast_exp2(pmv - M) : 0.f;
  // the denominator: one product per lane, summed the way the maximum was taken
  float z = pzv * fv;
  z += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(z), 0x111, 0xF, 0xF, false));    // row_shr:1 (0 shifted in)
  z += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(z), 0x112, 0xF, 0xF, false));    // row_shr:2
  z += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(z), 0x114, 0xF, 0xF, false));    // row_shr:4
  z += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(z), 0x118, 0xF, 0xF, false));    // row_shr:8
  z += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(z), 0x142, 0xA, 0xF, false));    // row_bcast:15
  z += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(z), 0x143, 0xC, 0xF, false));    // row_bcast:31
  z = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(z), 63));
  float o = 0.f;
#pragma unroll
  for (int ss = 0; ss < NMAX; ++ss) o = fmaf(po[ss], __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fv), ss)), o);
  store1<DT>(out, hq * D + c, z > 0.f ? o / z : 0.f);
  if (lse_out && c == 0) lse_out[hq] = (M + log2f(z)) * kLn2;
  if (c == 0) ZC_MARK(2);                       // end
}

template <int DT>
static int launch_decode_mfma_dt(const DecArgs& a, hipStream_t st) {
  dim3 grid(a.S, a.Hkv, a.B), block(256);
  const bool small = (int64_t)a.S * a.Hkv * a.B <= a.n_cu;
  const bool staged = small || a.pw_q < kStagedRun;          // cost units per packed wave
#define ZC_L(KT, VT)                                                                                          \
  do {                                                                                                        \
    if (a.D == 128) {                                                                                         \
      if (small) hipLaunchKernelGGL((k_decode_mfma<DT, 128, KT, VT, 1, true>), grid, block, 0, st, a);        \
      else if (staged) hipLaunchKernelGGL((k_decode_mfma<DT, 128, KT, VT, 2, true>), grid, block, 0, st, a);  \
      else hipLaunchKernelGGL((k_decode_mfma<DT, 128, KT, VT, 2, false>), grid, block, 0, st, a);             \
    } else {                                                                                                  \
      if (small) hipLaunchKernelGGL((k_decode_mfma<DT, 64, KT, VT, 1, true>), grid, block, 0, st, a);         \
      else if (staged) hipLaunchKernelGGL((k_decode_mfma<DT, 64, KT, VT, 2, true>), grid, block, 0, st, a);   \
      else hipLaunchKernelGGL((k_decode_mfma<DT, 64, KT, VT, 2, false>), grid, block, 0, st, a);              \
    }                                                                                                         \
  } while (0)
  if (a.k_tok && a.v_tok) ZC_L(true, true);
  else if (a.k_tok) ZC_L(true, false);
  else if (a.v_tok) ZC_L(false, true);
  else ZC_L(false, false);
#undef ZC_L
  ZC_LAUNCH_CHECK();
  if (a.S > 1) {
#define ZC_R(DD, NM) hipLaunchKernelGGL((k_decode_reduce<DT, DD, NM>), dim3(a.Hq, a.B), dim3(DD), 0, st, a.part_m, a.part_z, a.part_o, a.S, a.out, a.lse_out)
    if (a.D == 128) { if (a.S <= 8) ZC_R(128, 8); else if (a.S <= 16) ZC_R(128, 16); else if (a.S <= 24) ZC_R(128, 24); else ZC_R(128, kCombineMax); }
    else { if (a.S <= 8) ZC_R(64, 8); else if (a.S <= 16) ZC_R(64, 16); else if (a.S <= 24) ZC_R(64, 24); else ZC_R(64, kCombineMax); }
#undef ZC_R
    ZC_LAUNCH_CHECK();
  }
  return ZC_OK;
}

}  // namespace zc
