// Dispatch of the matrix-core decode kernel by query dtype.
#include "decode_args.hpp"

namespace zc {
int launch_decode_mfma_f32(const DecArgs& a, hipStream_t st);
int launch_decode_mfma_f16(const DecArgs& a, hipStream_t st);
int launch_decode_mfma_bf16(const DecArgs& a, hipStream_t st);

int launch_decode_mfma(const DecArgs& a, int dtype, hipStream_t st) {
  if (dtype == ZC_F32) return launch_decode_mfma_f32(a, st);
  if (dtype == ZC_F16) return launch_decode_mfma_f16(a, st);
  return launch_decode_mfma_bf16(a, st);
}
}  // namespace zc
