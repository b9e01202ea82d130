// Kernel argument block shared by the decode-attention kernels.
#pragma once

#include "zc_common.hpp"

namespace zc {

constexpr int kTailUnit = 16;    // tail tokens per work unit of the MFMA decode kernel (a multiple of 16)
constexpr int kMaxSplits = 128;
constexpr int kTailSplits = 8;    // 4 * kTailSplits: most waves per (batch, KV head) that share the tail
constexpr int kStagedRun = 16;   // packed waves with fewer cost units than this get the staged operand inputs
constexpr int kSegCost = 3;        // cost, in blocks, charged for starting a segment (query operand)
constexpr int kInlineChunks = 12;  // chunk-table rows that travel in the kernel arguments

struct DecArgs {
  const void* q;
  int64_t q_sB, q_sH;
  int B, Hq, Hkv, G, D;
  const uint8_t* kc[2];
  const float* k_ts[2];
  const float* k_tz[2];
  const float* k_cs;
  const float* k_cz;
  int k_tok;
  const uint32_t* vc[2];
  const float* v_ts[2];
  const float* v_tz[2];
  const float* v_cs;
  const float* v_cz;
  int v_tok;
  int64_t cap[2];
  int bits[2];
  const int32_t* chunk_table;
  int n_chunks;
  int chunks_inline;                       // 1: chunk_rows holds the whole table
  int32_t chunk_rows[4 * kInlineChunks];   // host copy of the chunk table, passed by value
  const void* tail_k;
  const void* tail_v;
  int64_t tk_sB, tk_sH, tk_sL, tv_sB, tv_sH, tv_sL;
  int tail_len;
  float scale_log2;
  int S, n_units;  // workgroups per (batch, KV head); length of the packed cache's cost line
  int n_pw, n_tw;  // waves per (batch, KV head) that share the packed cache / the tail; n_pw + n_tw = 4 S
  int tw_full, tw_rem;   // n_tw = tw_full * S + tw_rem: tail waves per workgroup, and workgroups with one more
  int tail_alone;        // 1: instead, the last n_tw workgroups hold one tail wave each and no packed wave
  int pw_q, pw_r;        // n_units = pw_q * n_pw + pw_r: cost units per packed wave, and waves with one more
  int tu_q, tu_r;        // tail units = tu_q * n_tw + tu_r, likewise
  int n_cu;        // compute units of the device
  float* part_m;   // [B, Hq, S]
  float* part_z;   // [B, Hq, S]
  float* part_o;   // [B, Hq, S, D]
  void* out;       // [B, Hq, D], q's dtype
  float* lse_out;  // [B, Hq] or null
};

// Defined in decode_mfma.hip: the matrix-core kernel for 2- and 4-bit caches.
int launch_decode_mfma(const DecArgs& a, int dtype, hipStream_t st);

}  // namespace zc
