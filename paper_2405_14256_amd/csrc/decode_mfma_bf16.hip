// Instantiates the matrix-core decode kernel for bf16 queries (one translation
// unit per dtype so that the variants compile in parallel).
#include "decode_mfma_kernel.hpp"

namespace zc {
int launch_decode_mfma_bf16(const DecArgs& a, hipStream_t st) { return launch_decode_mfma_dt<ZC_BF16>(a, st); }
}  // namespace zc

#ifdef ZC_TRACE
#include "zc_trace.h"
static_assert(ZC_TRACE_SLOTS == zc::kTraceSlots && ZC_TRACE_WAVES == zc::kTraceWaves && ZC_TRACE_HEADS == zc::kTraceHeads,
              "zc_trace.h describes the buffer of this file");
// Copies the time stamps of the bf16 kernels out (and clears them when asked to).
extern "C" int zc_trace_fetch(unsigned long long* host, size_t count, int reset) {
  constexpr size_t kTotal = (size_t)zc::kTraceWaves * zc::kTraceSlots + (size_t)zc::kTraceHeads * 4;
  if (count > kTotal || (count > 0 && !host)) return ZC_ERR_INVALID_ARG;
  if (hipDeviceSynchronize() != hipSuccess) return ZC_ERR_HIP;
  if (count > 0 && hipMemcpyFromSymbol(host, HIP_SYMBOL(zc::zc_trace_buf), count * sizeof(unsigned long long)) != hipSuccess) return ZC_ERR_HIP;
  if (reset) {
    void* dev = nullptr;
    if (hipGetSymbolAddress(&dev, HIP_SYMBOL(zc::zc_trace_buf)) != hipSuccess) return ZC_ERR_HIP;
    if (hipMemset(dev, 0, kTotal * sizeof(unsigned long long)) != hipSuccess) return ZC_ERR_HIP;
  }
  return ZC_OK;
}
#endif
