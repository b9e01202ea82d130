// zc_select_salient: exact top-k split of the token scores (Algorithm 2,
// "Split(., p~, r%)").  One workgroup per batch row: an MSB-first radix select
// on the order-preserving uint32 image of the scores finds the k-th largest
// key and how many tokens equal to it are taken (lowest indices first); one
// ordered compaction pass then writes both index lists in ascending order.
#include "zc_common.hpp"

namespace zc {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

__global__ __launch_bounds__(kSelThreads) void k_select_salient(
    const float* __restrict__ scores, int L, int k, int32_t* __restrict__ salient,
    int32_t* __restrict__ regular, uint8_t* __restrict__ mask) {
  __shared__ int hist[256];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
  __shared__ int s_wave_gt[kSelWaves], s_wave_eq[kSelWaves];
  __shared__ int s_base_gt, s_base_eq;

  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const float* sc = scores + (int64_t)b * L;
  int32_t* sal = salient + (int64_t)b * k;
  int32_t* reg = regular + (int64_t)b * (L - k);
  uint8_t* mk = mask ? mask + (int64_t)b * L : nullptr;

  // ---- radix select of the k-th largest key ---------------------------------
  uint32_t prefix = 0;   // key bits decided so far (high bits)
  int need = k;          // how many still to take among keys matching the prefix
  if (k > 0 && k < L) {
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      for (int i = tid; i < L; i += kSelThreads) {
        uint32_t key = float_key(sc[i]);
        if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xff], 1);
      }
      __syncthreads();
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

  if (tid == 0) { s_base_gt = 0; s_base_eq = 0; }
  __syncthreads();

  const int lane = tid & 63, wave = tid >> 6;
  for (int base = 0; base < L; base += kSelThreads) {
    const int i = base + tid;
    bool gt = false, eq = false;
    if (i < L) {
      if (take_all) gt = true;
      else if (!take_none) {
        uint32_t key = float_key(sc[i]);
        gt = key > prefix;
        eq = key == prefix;
      }
    }
    const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    int pre_gt = __popcll(bgt & below), pre_eq = __popcll(beq & below);
    if (lane == 0) { s_wave_gt[wave] = __popcll(bgt); s_wave_eq[wave] = __popcll(beq); }
    __syncthreads();
    int tot_gt = 0, tot_eq = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      int g = s_wave_gt[w], e = s_wave_eq[w];
      if (w < wave) { pre_gt += g; pre_eq += e; }
      tot_gt += g; tot_eq += e;
    }
    const int gt_before = s_base_gt + pre_gt;
    const int eq_before = s_base_eq + pre_eq;
    if (i < L) {
      const bool is_sal = gt || (eq && eq_before < need);
      const int sal_before = gt_before + min(eq_before, need);
      if (is_sal) sal[sal_before] = i;
      else reg[i - sal_before] = i;
      if (mk) mk[i] = is_sal ? 1 : 0;
    }
    __syncthreads();
    if (tid == 0) { s_base_gt += tot_gt; s_base_eq += tot_eq; }
    __syncthreads();
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
  hipLaunchKernelGGL(zc::k_select_salient, dim3((unsigned)B), dim3(zc::kSelThreads), 0,
                     (hipStream_t)stream, scores, (int)L, (int)k, salient_idx, regular_idx, mask);
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}
