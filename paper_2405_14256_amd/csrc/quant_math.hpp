// The quotient x / s of Eq. 5 in fp32 such that exact ties survive: shared by the
// quantizers (zc_quantize_pack, zc_group_quantize).
#pragma once

#include "zc_common.hpp"

namespace zc {

// N / R from the correctly rounded reciprocal y = 1/R with one residual
// correction.  When the true quotient is representable (in particular an exact
// tie n + 1/2, frequent with 16-bit inputs) the result is that quotient, so the
// round-half-even that follows sees the tie.
__device__ inline float refined_div(float N, float R, float y) {
  const float q0 = N * y;
  const float r = fmaf(-q0, R, N);
  return fmaf(r, y, q0);
}
// x * qmax / R with the rounding error of the product x * qmax carried along, so
// that ties stay exact for 24-bit x too (e.g. the minimum of a token row whose
// maximum is its mirror image: exactly -qmax / 2).
__device__ inline float refined_ratio(float x, float qmax, float R, float y) {
  const float nh = x * qmax;
  const float nl = fmaf(x, qmax, -nh);
  const float q0 = nh * y;
  const float r = fmaf(-q0, R, nh) + nl;
  return fmaf(r, y, q0);
}

}  // namespace zc
