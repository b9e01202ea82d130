// Instantiates the matrix-core decode kernel for f16 queries (one translation
// unit per dtype so that the variants compile in parallel).
#include "decode_mfma_kernel.hpp"

namespace zc {
int launch_decode_mfma_f16(const DecArgs& a, hipStream_t st) { return launch_decode_mfma_dt<ZC_F16>(a, st); }
}  // namespace zc
