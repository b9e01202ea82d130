// Pieces shared by the matrix-core kernels that tile dense products for wave64
// (probe saliency, prefill attention): the 32x32 MFMA on one 16-byte operand chunk
// per lane, the LDS tile layout that global -> LDS transfers fill, the workgroup ->
// XCD mapping, the accumulator layout of a 32x32 result.
#pragma once

#include "lds_dma.hpp"

namespace zc {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// One 16-byte operand chunk per lane: a single 32x32x16 MFMA for 16-bit types,
// four 32x32x2 MFMAs for fp32 (element m of both half-waves forms one k pair).
template <int DT>
__device__ inline void mma_chunk(v16f& acc, u32x4 a, u32x4 b) {
  if constexpr (DT == ZC_BF16) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  } else if constexpr (DT == ZC_F16) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
  } else {
    // (the elements are extracted one by one on purpose: a loop over a[i] inside
    // a bit-cast collapsed to element 0 with this compiler)
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
}

template <int DT, int D>
struct Tile {
  static constexpr int EB = (DT == ZC_F32) ? 4 : 2;
  static constexpr int ROWB = D * EB;          // bytes of one row
  static constexpr int CPR = ROWB / 16;        // 16-byte chunks per row (8, 16 or 32)
  static constexpr int NKC = ROWB / 32;        // operand chunks per lane and row
  static constexpr int RPI = 64 / CPR;         // rows one 64-lane transfer covers
  // Rows sit in LDS unpadded (a transfer writes 64 consecutive chunks); chunk c of
  // a row goes to chunk slot c ^ swz(row), which spreads the 16 rows that one
  // quarter-wave reads at the same c over all 64 banks.
  static constexpr int SW = CPR < 16 ? CPR : 16;
  static constexpr int RP256 = ROWB >= 256 ? 1 : 256 / ROWB;
  __device__ static int swz(int row) { return (row / RP256) % SW; }
  __device__ static int slot(int row, int c) { return row * ROWB + ((c ^ swz(row)) << 4); }
};

// Workgroups are handed to the 8 XCDs round-robin by their linear index, and
// every XCD has its own L2.  This maps the hardware index to a logical index such
// that each XCD gets one contiguous range of logical indices: workgroups that
// read the same K head (or the same probe rows) then share an L2.
__device__ inline int xcd_contiguous(int id, int n) {
  const int xcd = id & 7, slot = id >> 3;
  return xcd * (n >> 3) + min(xcd, n & 7) + slot;
}

// Row index inside a 32x32 MFMA result held by accumulator register v of a lane
// in half-wave kh.
__device__ inline int acc_row(int v, int kh) { return 8 * (v >> 2) + 4 * kh + (v & 3); }

constexpr int kBufFlags = 0x00020000;          // raw 32-bit data, no swizzle
constexpr int kOutOfRange = (int)0xFFFFF000u;  // a per-lane offset past the end of every admitted buffer

// The tile transfers (inline assembly) are invisible to the compiler, ordinary loads - the
// stationary operand before the loop, table look-ups inside it - are tracked by it.  If it
// believes one of "its" loads may still be in flight somewhere in the tile loop it waits for
// it with a count that also covers the transfers of the next tile, issued just before: the
// prefetch is waited for at once.  A wait it understands (all vector-memory loads of the
// wave done), where the loop waits for its transfers anyway, leaves it nothing to wait for.
__device__ inline void wait_all_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0) only

}  // namespace zc
