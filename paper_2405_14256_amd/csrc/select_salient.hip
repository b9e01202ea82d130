// zc_select_salient: exact top-k split of the token scores (Algorithm 2,
// "Split(., p~, r%)").  One workgroup per batch row: an MSB-first radix select
// on the order-preserving uint32 image of the scores finds the k-th largest
// key and how many tokens equal to it are taken (lowest indices first); one
// ordered compaction pass then writes both index lists in ascending order.
// The keys of a row are read from memory once and kept in LDS (rows of up to 34816
// tokens; longer rows are re-read from memory by every pass).
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

// CACHED: the row's keys are in LDS (at most kSelMaxCached of them).  (Keeping a thread's keys
// in registers instead, with every loop unrolled, was slower at every size - 17 us against
// 10 us for a row of 4096: the straight-line code is fetched cold at every launch.)
template <bool CACHED>
__global__ __launch_bounds__(kSelThreads) void k_select_salient(
    const float* __restrict__ scores, int L, int k, int32_t* __restrict__ salient,
    int32_t* __restrict__ regular, uint8_t* __restrict__ mask) {
  extern __shared__ uint32_t skeys[];     // CACHED: the row's keys
  __shared__ int hist[256];
  __shared__ int hrep[kSelRep * kSelRepStride];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
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
  if constexpr (CACHED) {
    for (int i = tid; i < L; i += kSelThreads) skeys[i] = float_key(sc[i]);
    __syncthreads();
  }
  auto key_at = [&](int i) -> uint32_t {
    if constexpr (CACHED) return skeys[i];
    else return float_key(sc[i]);
  };

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
        hist[tid] = h;                               // (read back below by this thread only)
      }
      // suffix sums over the bins (largest digit first): thread d owns bin d
      if (tid < 256) {
        const int lane_ = tid & 63, wv = tid >> 6;
        int suf = hist[tid];                         // becomes sum of bins >= tid inside the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int t = __shfl_down(suf, o);
          if (lane_ + o < 64) suf += t;
        }
        if (lane_ == 0) s_wave_gt[wv] = suf;         // wave totals (array reused as scratch)
      }
      __syncthreads();
      if (tid < 256) {
        const int lane_ = tid & 63, wv = tid >> 6;
        int suf = hist[tid];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int t = __shfl_down(suf, o);
          if (lane_ + o < 64) suf += t;
        }
        for (int w2 = wv + 1; w2 < 4; ++w2) suf += s_wave_gt[w2];
        const int above = suf - hist[tid];           // elements in bins > tid
        if (above < need && suf >= need) {           // exactly one bin satisfies this
          s_prefix = prefix | ((uint32_t)tid << shift);
          s_need = need - above;
        }
      }
      __syncthreads();
      prefix = s_prefix;
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
    const size_t lds = (size_t)L * sizeof(uint32_t);
    if (lds > 32 * 1024) {
      // a launch above the default dynamic-LDS limit needs the attribute raised (idempotent)
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(&zc::k_select_salient<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)(zc::kSelMaxCached * sizeof(uint32_t))) != hipSuccess)
        return ZC_ERR_HIP;
    }
    hipLaunchKernelGGL(zc::k_select_salient<true>, dim3((unsigned)B), dim3(zc::kSelThreads), lds,
                       (hipStream_t)stream, scores, (int)L, (int)k, salient_idx, regular_idx, mask);
  } else {
    hipLaunchKernelGGL(zc::k_select_salient<false>, dim3((unsigned)B), dim3(zc::kSelThreads), 0,
                       (hipStream_t)stream, scores, (int)L, (int)k, salient_idx, regular_idx, mask);
  }
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}
