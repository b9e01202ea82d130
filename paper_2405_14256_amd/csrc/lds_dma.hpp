// Global -> LDS transfers that do not pass through registers (buffer_load ... lds).
#pragma once

#include "zc_common.hpp"

namespace zc {

// ---- global -> LDS without passing through registers -----------------------------------
// One instruction moves 64 x 16 (or 64 x 4) bytes: lane l's bytes go to
// lds_addr + OFF + l * 16 (or * 4); OFF is added to the memory address too.  Lanes
// whose address is outside the buffer write zeros.  The compiler does not know
// about these transfers: the reader waits with wait_vmem<N>() for all but the N
// newest loads of the wave, and must have its own reads of a staging buffer
// complete (dma_reuse_fence) before loads into the same buffer are issued.
template <int OFF>
__device__ inline void dma16(uint32_t lds_addr, __amdgpu_buffer_rsrc_t rs, int voff, int soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen offset:%4 lds"
               :: "s"(lds_addr), "v"(voff), "s"(rs), "s"(soff), "n"(OFF) : "memory");
}
__device__ inline void dma4(uint32_t lds_addr, __amdgpu_buffer_rsrc_t rs, int voff, int soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rs), "s"(soff) : "memory");
}
// The same with an address of its own per lane (no buffer descriptor, no range check).
__device__ inline void gdma16(uint32_t lds_addr, const void* lane_src) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(lds_addr), "v"(lane_src) : "memory");
}
template <int N>
__device__ inline void wait_vmem() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
__device__ inline void dma_reuse_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

}  // namespace zc
