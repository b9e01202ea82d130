// zc_select_salient: exact top-k split of the token scores (Algorithm 2,
// "Split(., p~, r%)").  One workgroup per batch row: an MSB-first radix select
// on the order-preserving uint32 image of the scores finds the k-th largest
// key and how many tokens equal to it are taken (lowest indices first); one
// ordered compaction pass then writes both index lists in ascending order.
// Rows of up to 34816 tokens are read from memory once and kept in LDS
// (k_select_cached); longer rows are re-read from memory by every pass
// (k_select_stream).
#include <type_traits>

#include "zc_common.hpp"

namespace zc {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

constexpr int kSelMaxCached = 34816;     // keys of one row that fit the LDS of a CU next to the small arrays
// The digit histogram is kept in kSelRep copies, a lane adding to copy (lane mod kSelRep); the
// copies are 257 words apart, so they sit in different LDS banks.  Scores of one prompt share
// their exponent bits: with a single histogram all 64 lanes of a wave add to the same few
// words and the adds serialize (a pass over 32 k keys took 13 us that way).
constexpr int kSelRep = 16;
constexpr int kSelRepStride = 257;

// Which bin of a digit histogram holds the `need`-th largest key: threads 0..255 own a bin
// each (hist[tid] filled by its owner), suffix sums from the largest digit down; the owner of
// the one bin with (keys above) < need <= (keys above) + (keys in it) publishes the digit,
// what is still to take inside it and how many keys it holds.  Called by all threads; two barriers inside.
__device__ inline void pick_bin(const int* hist, int* wave_tot, int need, int tid, int* s_bin, int* s_need, int* s_cnt) {
  const int lane_ = tid & 63, wv = tid >> 6;
  int suf = 0;
  if (tid < 256) {
    suf = hist[tid];                               // becomes the sum of bins >= tid inside the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_down(suf, o);
      if (lane_ + o < 64) suf += t;
    }
    if (lane_ == 0) wave_tot[wv] = suf;
  }
  __syncthreads();
  if (tid < 256) {
    for (int w2 = wv + 1; w2 < 4; ++w2) suf += wave_tot[w2];
    const int above = suf - hist[tid];             // keys in bins > tid
    if (above < need && suf >= need) {             // exactly one bin satisfies this
      *s_bin = tid;
      *s_need = need - above;
      *s_cnt = hist[tid];
    }
  }
  __syncthreads();
}

// Inclusive sum over the 64 lanes of a wave (row shifts inside the rows of 16 lanes, then
// lane 15 of a row to the next row, lane 31 to the upper half).
__device__ inline int wave_inclusive_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);    // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);    // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);    // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);    // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
  return v;
}

constexpr int kSelCand = 1024;                 // candidates one wave finishes the search on
constexpr int kSelBufFlags = 0x00020000;       // buffer descriptor: raw 32-bit data, no swizzle
constexpr int kSelDropped = (int)0xFFFFF000u;  // a store offset past the end of every output: the store is dropped

// The row's keys live in LDS, four to a 16-byte word (the row padded to a multiple of 256 with
// key 0, which lies below the key of every number: -inf maps to 0x007fffff).
//   1. load: scores -> keys -> LDS, and the smallest and largest key of the row.  Their common
//      leading bits are decided already: the radix passes start at the first bit in which two
//      keys of the row differ (scores of one prompt share sign and most exponent bits - a pass
//      over those bits would put every key into one or two bins).
//   2. radix passes of eight bits by the whole workgroup, until the chosen bin holds at most
//      kSelCand keys (normally after the first) or no bit is left.
//   3. one sweep in which every wave counts, in its run of consecutive tokens, the keys above
//      the chosen bin and collects those inside it (the candidates).
//   4. wave 0 alone finishes the radix select on the candidates - no barriers - and adds, per
//      run, how many candidates lie above the k-th key and how many equal it.
//   5. ordered compaction: a lane owns four consecutive tokens, a wave its run; the index lists
//      are written through buffer descriptors, a store that does not apply (the other list's,
//      a pad's) being pointed past the end of its buffer, where it is dropped.
// VEC: the row starts on a 16-byte boundary (16-byte loads of the scores).
template <bool VEC>
__global__ __launch_bounds__(kSelThreads) void k_select_cached(
    const float* __restrict__ scores, int L, int k, int32_t* __restrict__ salient,
    int32_t* __restrict__ regular, uint8_t* __restrict__ mask) {
  extern __shared__ uint4 skeys4[];       // the row's keys
  __shared__ __align__(16) int hist[256];
  __shared__ __align__(16) int hrep[kSelRep * kSelRepStride];   // histogram copies; then the candidates
  __shared__ int s_bin, s_need, s_cnt, s_ncand;
  __shared__ uint32_t s_thr;
  __shared__ int s_wave_gt[kSelWaves], s_wave_eq[kSelWaves];
  __shared__ uint32_t s_wave_min[kSelWaves], s_wave_max[kSelWaves];
  static_assert(kSelCand * 2 <= kSelRep * kSelRepStride && kSelWaves * 256 <= kSelRep * kSelRepStride,
                "the candidates and the compaction stages reuse the histogram copies");

  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const float* sc = scores + (int64_t)b * L;
  const int n4 = ((L + 255) & ~255) >> 2;            // 16-byte words of keys, pads included

  // ---- 1. load ----------------------------------------------------------------
  for (int i = tid; i < kSelRep * kSelRepStride; i += kSelThreads) hrep[i] = 0;
  if (tid == 0) s_ncand = 0;
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for (int c = tid; c < n4; c += kSelThreads) {
    const int i = 4 * c;
    uint32_t kk[4] = {0u, 0u, 0u, 0u};
    if (i + 3 < L) {
      float f[4];
      if constexpr (VEC) {
        const float4 t = reinterpret_cast<const float4*>(sc)[c];
        f[0] = t.x; f[1] = t.y; f[2] = t.z; f[3] = t.w;
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) f[u] = sc[i + u];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        kk[u] = float_key(f[u]);
        kmin = min(kmin, kk[u]); kmax = max(kmax, kk[u]);
      }
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i + u < L) {
          kk[u] = float_key(sc[i + u]);
          kmin = min(kmin, kk[u]); kmax = max(kmax, kk[u]);
        }
    }
    skeys4[c] = make_uint4(kk[0], kk[1], kk[2], kk[3]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
  }
  if (lane == 0) { s_wave_min[wave] = kmin; s_wave_max[wave] = kmax; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) { kmin = min(kmin, s_wave_min[w]); kmax = max(kmax, s_wave_max[w]); }
  // (values every lane holds alike are moved to scalar registers, here and below: what is
  // computed from them then costs no vector instruction)
  kmin = __builtin_amdgcn_readfirstlane(kmin);
  kmax = __builtin_amdgcn_readfirstlane(kmax);

  // ---- 2. radix passes by the whole workgroup ----------------------------------------
  const uint32_t diff = kmin ^ kmax;
  int lo = diff ? 32 - __clz(diff) : 0;              // the low `lo` bits are undecided
  uint32_t prefix = lo >= 32 ? 0u : ((kmax >> lo) << lo);
  int need = k;          // how many still to take among keys matching the prefix
  if (k > 0 && k < L) {
    bool first = true;
    while (lo > 0) {
      const int top = lo;
      lo = top > 8 ? top - 8 : 0;
      const uint32_t hi_mask = top >= 32 ? 0u : (0xffffffffu << top);
      const uint32_t dmask = (1u << (top - lo)) - 1u;
      if (!first) {
        for (int i = tid; i < kSelRep * kSelRepStride; i += kSelThreads) hrep[i] = 0;
        __syncthreads();
      }
      first = false;
      int* mine = &hrep[(tid & (kSelRep - 1)) * kSelRepStride];
      for (int c = tid; c < n4; c += kSelThreads) {
        const uint4 kk = skeys4[c];
        // (a pad matches only an all-zero prefix and then falls into bin 0, below every key)
        if ((kk.x & hi_mask) == prefix) atomicAdd(&mine[(kk.x >> lo) & dmask], 1);
        if ((kk.y & hi_mask) == prefix) atomicAdd(&mine[(kk.y >> lo) & dmask], 1);
        if ((kk.z & hi_mask) == prefix) atomicAdd(&mine[(kk.z >> lo) & dmask], 1);
        if ((kk.w & hi_mask) == prefix) atomicAdd(&mine[(kk.w >> lo) & dmask], 1);
      }
      __syncthreads();
      if (tid < 256) {
        int h = 0;
#pragma unroll
        for (int r = 0; r < kSelRep; ++r) h += hrep[r * kSelRepStride + tid];
        hist[tid] = h;                               // (read back by this thread only)
      }
      pick_bin(hist, s_wave_gt, need, tid, &s_bin, &s_need, &s_cnt);
      prefix |= (uint32_t)__builtin_amdgcn_readfirstlane(s_bin) << lo;
      need = __builtin_amdgcn_readfirstlane(s_need);
      const int in_bin = __builtin_amdgcn_readfirstlane(s_cnt);       // (pads included when the bin is the lowest of all)
      __syncthreads();
      if (in_bin <= kSelCand) break;
    }
  }
  // Tokens with key > thr_gt are salient; of those equal to thr_eq, the first `need` by index.
  // k == 0 takes none, k == L takes all (every key of a number lies above 0).
  uint32_t thr_gt = prefix, thr_eq = prefix;
  if (k >= L) { thr_gt = 0u; thr_eq = 0xffffffffu; need = 0; lo = 0; }
  if (k <= 0) { thr_gt = 0xffffffffu; thr_eq = 0xffffffffu; need = 0; lo = 0; }

  // ---- 3. per run: keys above the chosen bin, keys inside it ----------------------------
  const int seg = (((L + kSelWaves - 1) / kSelWaves) + 255) & ~255;   // tokens per wave, whole pieces
  const int i0 = min(wave * seg, L), i1 = min(i0 + seg, L);
  const bool collect = lo > 0;                      // bits left: the keys inside the bin are candidates
  uint2* cand = reinterpret_cast<uint2*>(hrep);     // (key, run)
  {
    const uint32_t pg = thr_gt >> lo, pe = thr_eq >> lo;
    int cnt = 0;                                    // low half: keys above, high half: keys equal (no bits left)
    auto piece = [&](auto whole_c, int base) {
      constexpr bool WHOLE = decltype(whole_c)::value;              // no pad in this piece
      const uint4 kk = skeys4[(base >> 2) + lane];
      const int i = base + 4 * lane;
      const uint32_t k4[4] = {kk.x, kk.y, kk.z, kk.w};
      bool in[4];
      int nin = 0;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t t = k4[u] >> lo;
        cnt += t > pg ? 1 : 0;                       // (a pad is never above: its key is 0)
        in[u] = WHOLE ? t == pe : (t == pe && i + u < i1);
        nin += in[u] ? 1 : 0;
      }
      if (!collect) cnt += nin << 16;
      else if (__ballot(nin != 0)) {                 // wave-uniform; rare: a bin holds a small part of the row
        const int incl = wave_inclusive_sum(nin);
        int at = 0;
        if (lane == 63) at = atomicAdd(&s_ncand, incl);
        at = __builtin_amdgcn_readlane(at, 63) + incl - nin;
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (in[u]) cand[at++] = make_uint2(k4[u], (uint32_t)wave);
      }
    };
    for (int base = i0; base < i1; base += 256) {
      if (base + 256 <= i1) piece(std::true_type{}, base);
      else piece(std::false_type{}, base);
    }
    // (a wave's run has at most 34816 / 16 rounded up to 256 = 2304 tokens: the halves cannot carry)
    cnt = __builtin_amdgcn_readlane(wave_inclusive_sum(cnt), 63);
    if (lane == 0) { s_wave_gt[wave] = cnt & 0xffff; s_wave_eq[wave] = cnt >> 16; }
  }
  __syncthreads();

  // ---- 4. wave 0 finishes the search on the candidates --------------------------------------
  if (collect) {
    if (wave == 0) {
      const int n = __builtin_amdgcn_readfirstlane(s_ncand);          // <= kSelCand: the chosen bin's count bounds it
      const int nq = (n + 63) >> 6;
      // the candidates in registers, 16 a lane at most; an unused place holds a key that differs
      // from the prefix in the decided bits and so never matches below
      uint32_t ck[kSelCand / 64];
#pragma unroll
      for (int q = 0; q < kSelCand / 64; ++q) {
        ck[q] = ~prefix;
        if (q < nq && q * 64 + lane < n) ck[q] = cand[q * 64 + lane].x;
      }
      int top = lo, nd = need;
      uint32_t pre = prefix;
      while (top > 0) {
        const int lo2 = top > 8 ? top - 8 : 0;
        const uint32_t dm = (1u << (top - lo2)) - 1u;
        reinterpret_cast<int4*>(hist)[lane] = make_int4(0, 0, 0, 0);
#pragma unroll
        for (int q = 0; q < kSelCand / 64; ++q)
          if (q < nq && (ck[q] >> top) == (pre >> top)) atomicAdd(&hist[(ck[q] >> lo2) & dm], 1);
        // (LDS serves a wave's requests in order; the compiler must not move the read up)
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const int4 h = reinterpret_cast<const int4*>(hist)[lane];      // bins 4 lane .. 4 lane + 3
        const int incl = wave_inclusive_sum(h.x + h.y + h.z + h.w);
        const int a3 = __builtin_amdgcn_readlane(incl, 63) - incl;    // candidates in bins above this lane's
        const int a2 = a3 + h.w, a1 = a2 + h.z, a0 = a1 + h.y;
        int d = -1, rest = 0;
        if (a3 < nd && nd <= a3 + h.w) { d = 3; rest = nd - a3; }
        else if (a2 < nd && nd <= a2 + h.z) { d = 2; rest = nd - a2; }
        else if (a1 < nd && nd <= a1 + h.y) { d = 1; rest = nd - a1; }
        else if (a0 < nd && nd <= a0 + h.x) { d = 0; rest = nd - a0; }
        const int owner = __builtin_ctzll(__ballot(d >= 0));          // exactly one lane owns the bin
        const int bin = __builtin_amdgcn_readlane(4 * lane + d, owner);
        nd = __builtin_amdgcn_readlane(rest, owner);
        pre |= (uint32_t)bin << lo2;
        top = lo2;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      }
      for (int j = lane; j < n; j += 64) {
        const uint2 c = cand[j];
        if (c.x > pre) atomicAdd(&s_wave_gt[c.y], 1);
        else if (c.x == pre) atomicAdd(&s_wave_eq[c.y], 1);
      }
      if (lane == 0) { s_thr = pre; s_need = nd; }
    }
    __syncthreads();
    thr_gt = thr_eq = __builtin_amdgcn_readfirstlane(s_thr);
    need = __builtin_amdgcn_readfirstlane(s_need);
  }

  // ---- 5. ordered compaction -------------------------------------------------------
  int run_gt = 0, run_eq = 0;
  for (int w = 0; w < wave; ++w) { run_gt += s_wave_gt[w]; run_eq += s_wave_eq[w]; }
  run_gt = __builtin_amdgcn_readfirstlane(run_gt);
  run_eq = __builtin_amdgcn_readfirstlane(run_eq);
  const auto rs_sal = __builtin_amdgcn_make_buffer_rsrc(salient + (int64_t)b * k, 0, (uint32_t)k * 4u, kSelBufFlags);
  const auto rs_reg = __builtin_amdgcn_make_buffer_rsrc(regular + (int64_t)b * (L - k), 0, (uint32_t)(L - k) * 4u, kSelBufFlags);
  uint8_t* mk = mask ? mask + (int64_t)b * L : nullptr;
  const bool mk_words = (reinterpret_cast<uintptr_t>(mk) & 3) == 0;
  // A lane classifies four consecutive tokens, but consecutive lanes must write consecutive
  // list entries (a store instruction costs what the number of memory lines it touches costs):
  // the tokens of a piece go to a 256-word stage of the wave in list order - the salient ones,
  // then the others - and leave it 64 consecutive words at a time.
  int32_t* stage = hrep + wave * 256;               // (the candidates are no longer needed)
  for (int base = i0; base < i1; base += 256) {
    const uint4 kk = skeys4[(base >> 2) + lane];
    const int i = base + 4 * lane;
    const uint32_t k4[4] = {kk.x, kk.y, kk.z, kk.w};
    bool gt[4], eq[4];                               // (a pad is neither: thr_eq is the key of a number, or ~0)
    int mine = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      gt[u] = k4[u] > thr_gt;
      eq[u] = k4[u] == thr_eq;
      mine += (gt[u] ? 1 : 0) + (eq[u] ? 0x10000 : 0);
    }
    const int incl = wave_inclusive_sum(mine);
    const int total = __builtin_amdgcn_readlane(incl, 63);
    const int sal0 = run_gt + min(run_eq, need);                      // salient tokens before this piece
    const int nsal = run_gt + (total & 0xffff) + min(run_eq + (total >> 16), need) - sal0;   // ... inside it
    int eq_before = run_eq + ((incl - mine) >> 16);
    int p = run_gt + ((incl - mine) & 0xffff) + min(eq_before, need) - sal0;   // salient before this token, inside the piece
    uint32_t mbytes = 0u;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      // (no token of the piece equals the k-th key, nearly always: then salient means above it)
      const bool is_sal = gt[u] || (eq[u] && eq_before < need);
      stage[is_sal ? p : nsal + (4 * lane + u - p)] = i + u;
      mbytes |= (is_sal ? 1u : 0u) << (8 * u);
      p += is_sal ? 1 : 0;
      eq_before += eq[u] ? 1 : 0;
    }
    if (mk) {
      if (mk_words && base + 256 <= L) *reinterpret_cast<uint32_t*>(mk + i) = mbytes;
      else {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (i + u < L) mk[i + u] = (uint8_t)((mbytes >> (8 * u)) & 1u);
      }
    }
    // (LDS serves a wave's requests in order; the compiler must keep the order too)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // An entry past the end of its list is dropped by the buffer's range check: a pad (token
    // >= L, "regular", only at the end of the row) lands at an index >= L - k.
    const int reg0 = base - sal0 - nsal;              // list index of the piece's first regular token, minus nsal
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = 64 * u + lane;
      const uint32_t tok = (uint32_t)stage[j];
      if (64 * u < nsal)                             // wave-uniform: some of these 64 are salient
        __builtin_amdgcn_raw_buffer_store_b32(tok, rs_sal, j < nsal ? 4 * (sal0 + j) : kSelDropped, 0, 0);
      if (64 * u + 64 > nsal)                        // ... some are not
        __builtin_amdgcn_raw_buffer_store_b32(tok, rs_reg, j < nsal ? kSelDropped : 4 * (reg0 + j), 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    run_gt += total & 0xffff;
    run_eq += total >> 16;
  }
}

// Rows too long for LDS: every pass reads the scores from memory.  (Keeping a thread's keys
// in registers instead, with every loop unrolled, was slower at every size - 17 us against
// 10 us for a row of 4096: the straight-line code is fetched cold at every launch.)
__global__ __launch_bounds__(kSelThreads) void k_select_stream(
    const float* __restrict__ scores, int L, int k, int32_t* __restrict__ salient,
    int32_t* __restrict__ regular, uint8_t* __restrict__ mask) {
  __shared__ int hist[256];
  __shared__ int hrep[kSelRep * kSelRepStride];
  __shared__ int s_bin, s_need, s_cnt;
  __shared__ int s_wave_gt[kSelWaves], s_wave_eq[kSelWaves];

  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const float* sc = scores + (int64_t)b * L;
  int32_t* sal = salient + (int64_t)b * k;
  int32_t* reg = regular + (int64_t)b * (L - k);
  uint8_t* mk = mask ? mask + (int64_t)b * L : nullptr;
  const int seg = ((L + kSelWaves - 1) / kSelWaves + 63) & ~63;      // keys per wave, a multiple of 64
  const int i0 = min(wave * seg, L), i1 = min(i0 + seg, L);
  auto key_at = [&](int i) -> uint32_t { return float_key(sc[i]); };

  // ---- radix select of the k-th largest key ---------------------------------
  uint32_t prefix = 0;   // key bits decided so far (high bits)
  int need = k;          // how many still to take among keys matching the prefix
  if (k > 0 && k < L) {
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
      for (int i = tid; i < kSelRep * kSelRepStride; i += kSelThreads) hrep[i] = 0;
      __syncthreads();
      int* mine = &hrep[(tid & (kSelRep - 1)) * kSelRepStride];
      for (int i = tid; i < L; i += 4 * kSelThreads) {      // four keys requested before the first add
        uint32_t k4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) k4[u] = i + u * kSelThreads < L ? key_at(i + u * kSelThreads) : 0u;
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (i + u * kSelThreads < L && (k4[u] & hi_mask) == prefix) atomicAdd(&mine[(k4[u] >> shift) & 0xff], 1);
      }
      __syncthreads();
      if (tid < 256) {
        int h = 0;
#pragma unroll
        for (int r = 0; r < kSelRep; ++r) h += hrep[r * kSelRepStride + tid];
        hist[tid] = h;                               // (read back by this thread only)
      }
      pick_bin(hist, s_wave_gt, need, tid, &s_bin, &s_need, &s_cnt);
      prefix |= (uint32_t)s_bin << shift;
      need = s_need;
      __syncthreads();
    }
  }
  // Tokens with key > prefix are salient; of those equal to it, the first
  // `need` by index.  k == 0 takes none, k == L takes all.
  const bool take_all = (k >= L);
  const bool take_none = (k <= 0);

  // Ordered compaction without a barrier per step: every wave first counts the salient
  // candidates of its run (> and == the k-th key), the waves exchange the counts once, then
  // every wave writes its run in order from its own base offsets.
  auto classify = [&](int i, uint32_t key, bool& gt, bool& eq) {
    gt = false; eq = false;
    if (i < i1) {
      if (take_all) gt = true;
      else if (!take_none) { gt = key > prefix; eq = key == prefix; }
    }
  };
  int cnt_gt = 0, cnt_eq = 0;
  for (int base = i0; base < i1; base += 64) {
    bool gt, eq;
    const int i = base + lane;
    classify(i, (i < i1 && !take_all && !take_none) ? key_at(i) : 0u, gt, eq);
    cnt_gt += __popcll(__ballot(gt));
    cnt_eq += __popcll(__ballot(eq));
  }
  if (lane == 0) { s_wave_gt[wave] = cnt_gt; s_wave_eq[wave] = cnt_eq; }
  __syncthreads();
  int run_gt = 0, run_eq = 0;
  for (int w = 0; w < wave; ++w) { run_gt += s_wave_gt[w]; run_eq += s_wave_eq[w]; }
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  auto emit = [&](int i, uint32_t key) {
    bool gt, eq;
    classify(i, key, gt, eq);
    const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
    const int gt_before = run_gt + __popcll(bgt & below);
    const int eq_before = run_eq + __popcll(beq & below);
    if (i < i1) {
      const bool is_sal = gt || (eq && eq_before < need);
      const int sal_before = gt_before + min(eq_before, need);
      if (is_sal) sal[sal_before] = i;
      else reg[i - sal_before] = i;
      if (mk) mk[i] = is_sal ? 1 : 0;
    }
    run_gt += __popcll(bgt);
    run_eq += __popcll(beq);
  };
  for (int base = i0; base < i1; base += 64) {
    const int i = base + lane;
    emit(i, (i < i1 && !take_all && !take_none) ? key_at(i) : 0u);
  }
}

}  // namespace zc

extern "C" size_t zc_select_salient_workspace(int64_t, int64_t) { return 0; }

extern "C" int zc_select_salient(const float* scores, int64_t B, int64_t L, int64_t k,
                                 int32_t* salient_idx, int32_t* regular_idx, uint8_t* mask,
                                 void* ws, size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  if (B < 0 || L < 0 || k < 0 || k > L || L > 0x7fffffff || B > 65535 * 32) return ZC_ERR_INVALID_ARG;
  if (B == 0 || L == 0) return ZC_OK;
  if (!scores || (k > 0 && !salient_idx) || (k < L && !regular_idx)) return ZC_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(scores) & 3) || (reinterpret_cast<uintptr_t>(salient_idx) & 3) ||
      (reinterpret_cast<uintptr_t>(regular_idx) & 3))
    return ZC_ERR_INVALID_ARG;
  if (L <= zc::kSelMaxCached) {
    const size_t lds = (size_t)((L + 255) & ~(int64_t)255) * sizeof(uint32_t);
    // rows start on 16-byte boundaries when the array does and L is a multiple of four (or B is 1)
    const bool vec = (reinterpret_cast<uintptr_t>(scores) & 15) == 0 && (B == 1 || (L & 3) == 0);
    const void* fn = vec ? reinterpret_cast<const void*>(&zc::k_select_cached<true>)
                         : reinterpret_cast<const void*>(&zc::k_select_cached<false>);
    if (lds > 32 * 1024) {
      // a launch above the default dynamic-LDS limit needs the attribute raised (idempotent)
      if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(zc::kSelMaxCached * sizeof(uint32_t))) != hipSuccess)
        return ZC_ERR_HIP;
    }
    if (vec)
      hipLaunchKernelGGL(zc::k_select_cached<true>, dim3((unsigned)B), dim3(zc::kSelThreads), lds,
                         (hipStream_t)stream, scores, (int)L, (int)k, salient_idx, regular_idx, mask);
    else
      hipLaunchKernelGGL(zc::k_select_cached<false>, dim3((unsigned)B), dim3(zc::kSelThreads), lds,
                         (hipStream_t)stream, scores, (int)L, (int)k, salient_idx, regular_idx, mask);
  } else {
    hipLaunchKernelGGL(zc::k_select_stream, dim3((unsigned)B), dim3(zc::kSelThreads), 0,
                       (hipStream_t)stream, scores, (int)L, (int)k, salient_idx, regular_idx, mask);
  }
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}
