// zc_probe_saliency: normalized attention score of every key token from a
// probe subset of query rows (Eq. 9 substituted into Eq. 8).
//
// The probe rows of A = Softmax(Q_probe K^T / sqrt(d)) are never stored.  Two
// matrix-core sweeps recompute the logits instead:
//   k_probe_lse     one workgroup per 128 probe rows and column range (the columns a
//                   row block can see are cut into up to 8 ranges: to fill the chip
//                   when the launch is small, and to even out row blocks that see
//                   very different numbers of columns): the probe rows sit in
//                   registers as matrix operands, 64-column K tiles stream through
//                   LDS (global -> LDS transfers, the next tile's in flight), logits
//                   come out of the MFMA as D[column][row] so that every lane owns
//                   one probe row and keeps its running (reference, sum) in two
//                   registers; writes the pair per row and column range
//                   (k_probe_lse_merge joins the ranges).
//   k_probe_colsum  one workgroup per 128 key columns: K fragments stay in
//                   registers, 64-row probe tiles stream through LDS with their
//                   positions and log-sum-exps, logits come out as D[row][column] so
//                   that every lane owns one column and sums exp(logit - lse) over
//                   the rows in registers; divides by the number of probes that can
//                   see the column.
//   k_probe_mean    mean over query heads.
// Causality: rows are sorted by position, so a column tile starts at the first
// probe that can see it and a row tile stops at its last row's position.
// Inputs in fp16 / bf16 use the 32x32x16 MFMA, fp32 inputs the 32x32x2 fp32 MFMA
// (no rounding of the operands); accumulation and softmax are fp32.
#include "mfma_tiles.hpp"

namespace zc {

constexpr int kMaxProbeSplit = 8;

struct ProbeArgs {
  const void* q;
  const void* k;
  int64_t q_sB, q_sH, q_sL, k_sB, k_sH, k_sL;
  int B, Hq, Hkv, G, Lk, Lq, P;
  const int32_t* probe_rows;
  const int32_t* probe_pos;
  float scale_log2;
  const float* lse_in;   // natural log, [B, Hq, P]; null: use lse2
  float* lse2;           // [B, Hq, P] log-sum-exp in log2 units: sweep 1's result
  float2* lse_part;      // [B, Hq, P, nsplit] (running maximum in log2 units, sum) when nsplit > 1
  int nsplit;            // column ranges a row block's sweep 1 is split into
  float* per_head;       // [B, Hq, Lk]
  int normalize;         // 1: divide a column's sum by the number of probes that see it (Eq. 8); 0: Eq. 7
};

constexpr int kLseRows = 128;                  // probe rows per workgroup of sweep 1
constexpr int kLseCols = 64;                   // columns per K tile of sweep 1

template <int DT, int D>
__global__ __launch_bounds__(256, 2) void k_probe_lse(ProbeArgs a) {
  using T = Tile<DT, D>;
  constexpr int TILE_B = kLseCols * T::ROWB;
  constexpr int NI = kLseCols / T::RPI / 4;     // transfers per wave and K tile
  __shared__ __align__(16) uint8_t Ks[2][TILE_B];
  __shared__ int spos[kLseRows];
  __shared__ float sm[2][kLseRows], sz[2][kLseRows];

  // logical order: probe-row block fastest, then column range, then query head, then batch
  const int nrb = ceil_div(a.P, kLseRows);
  int j = xcd_contiguous(blockIdx.x, gridDim.x);
  const int rb0 = (j % nrb) * kLseRows; j /= nrb;
  const int split = j % a.nsplit; j /= a.nsplit;
  const int hq = j % a.Hq, b = j / a.Hq, hk = hq / a.G;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, kh = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rh = w >> 1, ch = w & 1;            // this wave: rows rh * 64 .. + 63, columns ch * 32 .. + 31 of a tile
  const uint8_t* qb = reinterpret_cast<const uint8_t*>(a.q) + ((int64_t)b * a.q_sB + (int64_t)hq * a.q_sH) * T::EB;
  const uint8_t* kb = reinterpret_cast<const uint8_t*>(a.k) + ((int64_t)b * a.k_sB + (int64_t)hk * a.k_sH) * T::EB;
  const uint32_t k_rowb = (uint32_t)(a.k_sL * T::EB), q_rowb = (uint32_t)(a.q_sL * T::EB);
  const auto rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(kb), 0, (uint32_t)(a.Lk - 1) * k_rowb + T::ROWB, kBufFlags);
  const auto rs_q = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(qb), 0, (uint32_t)(a.Lq - 1) * q_rowb + T::ROWB, kBufFlags);

  // the block's last row decides how many column tiles it sees
  const int nvalid = min(kLseRows, a.P - rb0);
  const int pmax = min(a.probe_pos[rb0 + nvalid - 1], a.Lk - 1);
  const int ntiles = pmax / kLseCols + 1;
  // this workgroup's share of the column tiles
  const int per = ceil_div(ntiles, a.nsplit);
  const int t_begin = split * per, t_end = min(t_begin + per, ntiles);

  // A K tile goes global -> LDS directly, every wave a quarter of its transfers;
  // the per-lane part of the addresses is fixed, the tile adds a scalar.
  const uint32_t ks_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)&Ks[0][0];
  int kvoff[NI];
#pragma unroll
  for (int jj = 0; jj < NI; ++jj) {
    const int row = (w + 4 * jj) * T::RPI + lane / T::CPR;
    kvoff[jj] = (int)(row * k_rowb) + (((lane % T::CPR) ^ T::swz(row)) << 4);
  }
  // (the tile's offset goes into the per-lane offset, which is what the range check
  // sees: rows past the end of K then arrive as zeros)
  auto issue = [&](int t, int buf) {
    const int toff = (int)((uint32_t)t * kLseCols * k_rowb);
#pragma unroll
    for (int jj = 0; jj < NI; ++jj) dma16<0>(ks_lds + buf * TILE_B + (w + 4 * jj) * 1024, rs_k, kvoff[jj] + toff, 0);
  };
  if (t_begin < t_end) issue(t_begin, 0);

  // the probe rows of this wave, straight into operand registers
  u32x4 qf[2][T::NKC];
  int myp[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int p = rb0 + rh * 64 + rb * 32 + r;
    int voff = kOutOfRange;
    myp[rb] = -1;
    if (p < a.P) {
      myp[rb] = a.probe_pos[p];
      voff = (int)((uint32_t)(a.probe_rows ? a.probe_rows[p] : myp[rb]) * q_rowb) + kh * 16;
    }
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc) qf[rb][kc] = __builtin_amdgcn_raw_buffer_load_b128(rs_q, voff + kc * 32, 0, 0);
  }
  if (tid < kLseRows) spos[tid] = (rb0 + tid < a.P) ? a.probe_pos[rb0 + tid] : -1;
  __syncthreads();
  // rows are sorted by position: a block's first row bounds what is fully visible,
  // its last real row what is visible at all
  int pos_last = -1;
  if (rb0 + rh * 64 < a.P) pos_last = spos[min(rh * 64 + 63, nvalid - 1)];
  // the same per 32-row block: its first row's position (-1: no row) and its last real row's
  int pfirst[2], plast[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int base = rh * 64 + rb * 32;
    pfirst[rb] = spos[base];
    plast[rb] = rb0 + base < a.P ? spos[min(base + 31, nvalid - 1)] : -1;
  }
  float m[2] = {-INFINITY, -INFINITY}, z[2] = {0.f, 0.f};
  const int krow = ch * 32 + r;                  // this lane's column inside a tile

  for (int t = t_begin; t < t_end; ++t) {
    const int cur = (t - t_begin) & 1;
    wait_all_loads();    // this wave's transfers of tile t have landed ...
    __syncthreads();     // ... and everyone's; nobody still reads the other buffer
    if (t + 1 < t_end) issue(t + 1, cur ^ 1);
    if (t * kLseCols > pos_last) continue;       // nothing of this tile is visible to the wave's rows
    v16f acc[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[0][i] = 0.f; acc[1][i] = 0.f; }
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc) {
      const u32x4 af = *reinterpret_cast<const u32x4*>(&Ks[cur][T::slot(krow, 2 * kc + kh)]);
      mma_chunk<DT>(acc[0], af, qf[0][kc]);
      mma_chunk<DT>(acc[1], af, qf[1][kc]);
    }
    const int colb = t * kLseCols + ch * 32;     // this wave's 32 columns of the tile
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      if (colb > plast[rb]) continue;            // none of them visible to this block's rows
      if (colb + 31 <= pfirst[rb]) {
        // Every logit of the tile counts.  The reference point m of a row only has to keep
        // exp2 in range, not to be the maximum: it is taken from the row's first tile
        // and moved only when a tile's sum shows that some logit lies 2^60 above it
        // (the log-sum-exp m + log2(z) does not depend on the choice).
        bool redo = __builtin_amdgcn_ballot_w64(m[rb] == -INFINITY) != 0;
        if (!redo) {
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(fmaf(acc[rb][v], a.scale_log2, -m[rb]));
          redo = __builtin_amdgcn_ballot_w64(!(sum < 0x1p60f)) != 0;
          if (!redo) z[rb] += sum;
        }
        if (redo) {
          float tmax = fmaxf(acc[rb][0], acc[rb][1]);
#pragma unroll
          for (int v = 2; v < 16; v += 2) tmax = fmaxf(fmaxf(tmax, acc[rb][v]), acc[rb][v + 1]);
          const float m_new = fmaxf(m[rb], tmax * a.scale_log2);
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(fmaf(acc[rb][v], a.scale_log2, -m_new));
          z[rb] = z[rb] * __builtin_amdgcn_exp2f(m[rb] - m_new) + sum;
          m[rb] = m_new;
        }
      } else {
        float sv[16];
        float tmax = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int col = colb + acc_row(v, kh);
          const float sc = (col <= myp[rb]) ? acc[rb][v] * a.scale_log2 : -INFINITY;
          sv[v] = sc;
          tmax = fmaxf(tmax, sc);
        }
        const float m_new = fmaxf(m[rb], tmax);
        if (m_new > -INFINITY) {
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(sv[v] - m_new);
          z[rb] = z[rb] * __builtin_amdgcn_exp2f(m[rb] - m_new) + sum;
          m[rb] = m_new;
        }
      }
    }
  }
  // merge the two half-waves, then the two column halves
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const float mo = __shfl_xor(m[rb], 32), zo = __shfl_xor(z[rb], 32);
    const float M = fmaxf(m[rb], mo);
    float Z = 0.f;
    if (M > -INFINITY) Z = z[rb] * exp2f(m[rb] - M) + zo * exp2f(mo - M);
    if (kh == 0) { sm[ch][rh * 64 + rb * 32 + r] = M; sz[ch][rh * 64 + rb * 32 + r] = Z; }
  }
  __syncthreads();
  if (tid < kLseRows && rb0 + tid < a.P) {
    const float M = fmaxf(sm[0][tid], sm[1][tid]);
    float Z = 0.f;
    if (M > -INFINITY) Z = sz[0][tid] * exp2f(sm[0][tid] - M) + sz[1][tid] * exp2f(sm[1][tid] - M);
    const int64_t row = ((int64_t)b * a.Hq + hq) * a.P + rb0 + tid;
    if (a.nsplit == 1) a.lse2[row] = M + log2f(Z);
    else a.lse_part[row * a.nsplit + split] = make_float2(M, Z);
  }
}

// Merges the (maximum, sum) pairs of a probe row's column ranges.
__global__ void k_probe_lse_merge(const float2* __restrict__ part, float* __restrict__ lse2, int64_t rows, int nsplit) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows) return;
  float2 v[kMaxProbeSplit];
#pragma unroll
  for (int sp = 0; sp < kMaxProbeSplit; ++sp) v[sp] = sp < nsplit ? part[i * nsplit + sp] : make_float2(-INFINITY, 0.f);
  float M = -INFINITY;
#pragma unroll
  for (int sp = 0; sp < kMaxProbeSplit; ++sp) M = fmaxf(M, v[sp].x);
  float Z = 0.f;
#pragma unroll
  for (int sp = 0; sp < kMaxProbeSplit; ++sp)
    if (v[sp].x > -INFINITY) Z += v[sp].y * exp2f(v[sp].x - M);
  lse2[i] = M + log2f(Z);
}

__device__ inline int lower_bound_pos(const int32_t* pos, int n, int key) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (pos[mid] < key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

constexpr int kPosTable = 4096;     // probe positions kept in LDS (larger sets are read from memory)

template <int DT, int D>
__global__ __launch_bounds__(256, (DT == ZC_F32 && D == 128) ? 1 : 2) void k_probe_colsum(ProbeArgs a) {
  using T = Tile<DT, D>;
  constexpr int QT = 64;                        // probe rows per tile
  constexpr int TILE_B = QT * T::ROWB;
  constexpr int NI = QT / T::RPI / 4;           // transfers per wave and tile
  __shared__ __align__(16) uint8_t Qs[2][TILE_B];
  __shared__ int32_t lpos[kPosTable];
  __shared__ __align__(16) int spos[2][QT];
  __shared__ __align__(16) float slse[2][QT];
  __shared__ float scol[2][128];

  // logical order: column tile fastest, then query head, then batch
  const int nct = ceil_div(a.Lk, 128);
  int j = xcd_contiguous(blockIdx.x, gridDim.x);
  const int col0 = (j % nct) * 128; j /= nct;
  const int hq = j % a.Hq, b = j / a.Hq, hk = hq / a.G;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, kh = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rbw = w >> 1, cbp = w & 1;
  const uint8_t* qb = reinterpret_cast<const uint8_t*>(a.q) + ((int64_t)b * a.q_sB + (int64_t)hq * a.q_sH) * T::EB;
  const uint8_t* kb = reinterpret_cast<const uint8_t*>(a.k) + ((int64_t)b * a.k_sB + (int64_t)hk * a.k_sH) * T::EB;
  const int64_t lrow = ((int64_t)b * a.Hq + hq) * a.P;
  const uint32_t k_rowb = (uint32_t)(a.k_sL * T::EB), q_rowb = (uint32_t)(a.q_sL * T::EB);
  const auto rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(kb), 0, (uint32_t)(a.Lk - 1) * k_rowb + T::ROWB, kBufFlags);
  const auto rs_q = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(qb), 0, (uint32_t)(a.Lq - 1) * q_rowb + T::ROWB, kBufFlags);
  const auto rs_pos = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(a.probe_pos), 0, (uint32_t)a.P * 4u, kBufFlags);
  const float* lse_src = (a.lse_in ? a.lse_in : a.lse2) + lrow;
  const auto rs_lse = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(lse_src), 0, (uint32_t)a.P * 4u, kBufFlags);

  // this wave's K columns, straight into operand registers (columns past the end: zeros)
  u32x4 kf[2][T::NKC];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const int col = col0 + (cbp * 2 + cb) * 32 + r;
    const int voff = col < a.Lk ? (int)((uint32_t)col * k_rowb) + kh * 16 : kOutOfRange;
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc) kf[cb][kc] = __builtin_amdgcn_raw_buffer_load_b128(rs_k, voff + kc * 32, 0, 0);
  }
  // the probe positions go to LDS, so that the binary searches and the row addresses
  // of this workgroup do not go to memory
  const bool pos_in_lds = a.P <= kPosTable;
  if (pos_in_lds) {
    for (int i = tid; i < a.P; i += 256) lpos[i] = a.probe_pos[i];
    __syncthreads();
  }
  const bool rows_in_lds = pos_in_lds && !a.probe_rows;              // the rows of q are the positions themselves
  const auto lds_tab = (__attribute__((address_space(3))) const int32_t*)lpos;
  const auto g_rows = (__attribute__((address_space(1))) const int32_t*)a.probe_rows;
  const auto g_pos = (__attribute__((address_space(1))) const int32_t*)a.probe_pos;
  const int pstart = pos_in_lds ? lower_bound_pos(lpos, a.P, col0) : lower_bound_pos(a.probe_pos, a.P, col0);
  float colsum[2] = {0.f, 0.f};

  // A tile of 64 probe rows goes global -> LDS directly, every wave a quarter of its
  // transfers; wave 0 also brings the rows' positions and log-sum-exps.
  const uint32_t qs_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)&Qs[0][0];
  const uint32_t spos_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int*)&spos[0][0];
  const uint32_t slse_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)&slse[0][0];
  auto issue = [&](int pr, int buf) {
    // the rows of q this lane fetches: from the LDS table, or from memory (uniform branches
    // over pointers of known address space: never a read through a generic pointer); the
    // reads from memory are waited for here, where their values are needed anyway, so that
    // the compiler carries no load of its own into the rest of the loop (see wait_all_loads)
    uint32_t qrow[NI];
    if (rows_in_lds) {
#pragma unroll
      for (int jj = 0; jj < NI; ++jj) qrow[jj] = (uint32_t)lds_tab[min(pr + (w + 4 * jj) * T::RPI + lane / T::CPR, a.P - 1)];
    } else {
#pragma unroll
      for (int jj = 0; jj < NI; ++jj) {
        const int pc = min(pr + (w + 4 * jj) * T::RPI + lane / T::CPR, a.P - 1);
        qrow[jj] = a.probe_rows ? (uint32_t)g_rows[pc] : (uint32_t)g_pos[pc];
      }
      wait_all_loads();
    }
#pragma unroll
    for (int jj = 0; jj < NI; ++jj) {
      const int row = (w + 4 * jj) * T::RPI + lane / T::CPR;
      const int p = pr + row;
      const int voff = p < a.P ? (int)(qrow[jj] * q_rowb) + (((lane % T::CPR) ^ T::swz(row)) << 4) : kOutOfRange;
      dma16<0>(qs_lds + buf * TILE_B + (w + 4 * jj) * 1024, rs_q, voff, 0);
    }
    if (w == 0) {
      dma4(spos_lds + buf * (QT * 4), rs_pos, (pr + lane) * 4, 0);
      dma4(slse_lds + buf * (QT * 4), rs_lse, (pr + lane) * 4, 0);
    }
  };
  if (pstart < a.P) issue(pstart, 0);
  const int qrow_l = rbw * 32 + r;               // this lane's row inside a tile

  for (int pr = pstart; pr < a.P; pr += QT) {
    const int cur = ((pr - pstart) / QT) & 1;
    wait_all_loads();    // this wave's transfers of the tile have landed ...
    __syncthreads();     // ... and everyone's; nobody still reads the other buffer
    if (pr + QT < a.P) issue(pr + QT, cur ^ 1);
    float rl[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) rl[v] = slse[cur][rbw * 32 + acc_row(v, kh)];
    if (a.lse_in) {
#pragma unroll
      for (int v = 0; v < 16; ++v) rl[v] *= kLog2e;       // an external log-sum-exp is in natural units
    }
    v16f acc[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[0][i] = 0.f; acc[1][i] = 0.f; }
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc) {
      const u32x4 af = *reinterpret_cast<const u32x4*>(&Qs[cur][T::slot(qrow_l, 2 * kc + kh)]);
      mma_chunk<DT>(acc[0], af, kf[0][kc]);
      mma_chunk<DT>(acc[1], af, kf[1][kc]);
    }
    // a tile of 64 real rows whose first position is past this workgroup's last
    // column needs no mask
    const bool tile_full = pr + QT <= a.P && col0 + 127 <= spos[cur][0];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      const int col = col0 + (cbp * 2 + cb) * 32 + r;
      if (tile_full) {
#pragma unroll
        for (int v = 0; v < 16; ++v) colsum[cb] += __builtin_amdgcn_exp2f(fmaf(acc[cb][v], a.scale_log2, -rl[v]));
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float e = __builtin_amdgcn_exp2f(fmaf(acc[cb][v], a.scale_log2, -rl[v]));
          const int row = rbw * 32 + acc_row(v, kh);
          const bool seen = col <= spos[cur][row] && pr + row < a.P;    // (rows past the last probe arrive as zeros)
          colsum[cb] += seen ? e : 0.f;
        }
      }
    }
  }
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    colsum[cb] += __shfl_xor(colsum[cb], 32);
    if (kh == 0) scol[rbw][(cbp * 2 + cb) * 32 + r] = colsum[cb];
  }
  __syncthreads();
  if (tid < 128 && col0 + tid < a.Lk) {
    const int col = col0 + tid;
    const float total = scol[0][tid] + scol[1][tid];
    const int cnt = a.P - (pos_in_lds ? lower_bound_pos(lpos, a.P, col) : lower_bound_pos(a.probe_pos, a.P, col));
    a.per_head[((int64_t)b * a.Hq + hq) * a.Lk + col] = !a.normalize ? total : (cnt > 0 ? total / (float)cnt : 0.f);
  }
}

// Mean over the query heads: block (64 columns, 4 head groups); every group
// sums its heads in order, the four partial sums are then added in order.
__global__ __launch_bounds__(256) void k_probe_mean(const float* __restrict__ per_head, float* __restrict__ scores, int Hq, int Lk) {
  __shared__ float part[4][64];
  const int b = blockIdx.y;
  const int cx = threadIdx.x, gy = threadIdx.y;
  const int i = blockIdx.x * 64 + cx;
  const int per = (Hq + 3) / 4;
  float s = 0.f;
  if (i < Lk) {
    const int h1 = min(Hq, (gy + 1) * per);
    for (int h = gy * per; h < h1; ++h) s += per_head[((int64_t)b * Hq + h) * Lk + i];
  }
  part[gy][cx] = s;
  __syncthreads();
  if (gy == 0 && i < Lk) scores[(int64_t)b * Lk + i] = (((part[0][cx] + part[1][cx]) + part[2][cx]) + part[3][cx]) / (float)Hq;
}

template <int DT, int D>
static int launch_probe(const ProbeArgs& a, bool need_lse, float* scores, hipStream_t st) {
  if (need_lse) {
    hipLaunchKernelGGL((k_probe_lse<DT, D>), dim3((unsigned)((int64_t)ceil_div(a.P, kLseRows) * a.Hq * a.B * a.nsplit)), dim3(256), 0, st, a);
    ZC_LAUNCH_CHECK();
    if (a.nsplit > 1) {
      const int64_t rows = (int64_t)a.B * a.Hq * a.P;
      hipLaunchKernelGGL(k_probe_lse_merge, dim3((unsigned)ceil_div64(rows, 256)), dim3(256), 0, st, a.lse_part, a.lse2, rows, a.nsplit);
      ZC_LAUNCH_CHECK();
    }
  }
  hipLaunchKernelGGL((k_probe_colsum<DT, D>), dim3((unsigned)((int64_t)ceil_div(a.Lk, 128) * a.Hq * a.B)), dim3(256), 0, st, a);
  ZC_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_probe_mean, dim3(ceil_div(a.Lk, 64), a.B), dim3(64, 4), 0, st, a.per_head, scores, a.Hq, a.Lk);
  ZC_LAUNCH_CHECK();
  return ZC_OK;
}

}  // namespace zc

using namespace zc;

// Column ranges per row block of sweep 1.  Enough workgroups to fill the chip once (three fit
// a CU); and, however many there are, up to four ranges of at least 16 tiles each: a row block
// near the end of a long prompt sees ten times the columns of one near the start, and whole
// row blocks as units leave the chip half empty while the long ones finish.
static int probe_splits(int64_t B, int64_t Hq, int64_t P, int64_t Lk) {
  const int64_t wgs = B * Hq * ceil_div64(P, kLseRows);
  const int64_t fill = 768 / wgs;
  int64_t even = ceil_div64(Lk, kLseCols) / 16;
  if (even > 4) even = 4;
  const int64_t ns = fill > even ? fill : even;
  return (int)(ns < 1 ? 1 : (ns > kMaxProbeSplit ? kMaxProbeSplit : ns));
}
static size_t lse_bytes(int64_t B, int64_t Hq, int64_t P) { return (size_t)align_up64(B * Hq * P * (kMaxProbeSplit * (int64_t)sizeof(float2) + 4), 256); }

extern "C" size_t zc_probe_saliency_workspace(int64_t B, int64_t Hq, int64_t Lk, int64_t P) {
  if (B <= 0 || Hq <= 0 || Lk <= 0 || P <= 0) return 0;
  return lse_bytes(B, Hq, P) + (size_t)B * Hq * Lk * 4;
}

static int probe_scores(const zc_tensor4* q, const zc_tensor4* k,
                        const int32_t* probe_rows, const int32_t* probe_pos, int32_t P,
                        float sm_scale, const float* lse_ext,
                        float* scores, float* scores_per_head,
                        void* ws, size_t ws_bytes, void* stream, bool normalize) {
  int rc = zc_validate_tensor(q);
  if (rc) return rc;
  rc = zc_validate_tensor(k);
  if (rc) return rc;
  if (q->dtype != k->dtype || q->D != k->D || q->B != k->B) return ZC_ERR_INVALID_ARG;
  if (q->H % k->H != 0) return ZC_ERR_INVALID_ARG;
  if (P < 1 || !probe_pos || !scores || k->L < 1 || q->L < 1) return ZC_ERR_INVALID_ARG;
  if (q->B > 65535 || q->H > 65535 || k->L > 0x7fffffff - 256) return ZC_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(probe_pos) & 3) || (reinterpret_cast<uintptr_t>(scores) & 3)) return ZC_ERR_INVALID_ARG;
  {
    // the kernels address one (batch, head) slab of q and of k with 32-bit byte offsets,
    // and request "nothing" at offset 0xFFFFF000, which must lie past the end of a slab
    const int64_t eb = q->dtype == ZC_F32 ? 4 : 2;
    // (a K tile may start up to 63 rows before the end of k and reach as far past it: those
    // offsets must not wrap either)
    if (q->L * q->sL * eb >= 0xFFFFF000ll || (k->L + 128) * k->sL * eb >= 0xFFFFF000ll || (int64_t)P * 4 >= 0xFFFFF000ll) return ZC_ERR_UNSUPPORTED;
  }
  const size_t need = zc_probe_saliency_workspace(q->B, q->H, k->L, P);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15)) return ZC_ERR_WORKSPACE;

  ProbeArgs a;
  a.q = q->ptr; a.k = k->ptr;
  a.q_sB = q->sB; a.q_sH = q->sH; a.q_sL = q->sL;
  a.k_sB = k->sB; a.k_sH = k->sH; a.k_sL = k->sL;
  a.B = (int)q->B; a.Hq = (int)q->H; a.Hkv = (int)k->H; a.G = a.Hq / a.Hkv; a.Lk = (int)k->L; a.Lq = (int)q->L; a.P = P;
  a.probe_rows = probe_rows; a.probe_pos = probe_pos;
  a.scale_log2 = (sm_scale == 0.f ? 1.0f / sqrtf((float)q->D) : sm_scale) * kLog2e;
  float* ws_ph = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(ws) + lse_bytes(q->B, q->H, P));
  a.lse_in = lse_ext;
  a.lse_part = reinterpret_cast<float2*>(ws);
  a.lse2 = reinterpret_cast<float*>(a.lse_part + (int64_t)q->B * q->H * P * kMaxProbeSplit);
  a.nsplit = probe_splits(q->B, q->H, P, k->L);
  if ((int64_t)ceil_div64(P, kLseRows) * q->H * q->B * a.nsplit > 0x7fffffff || (int64_t)ceil_div64(k->L, 128) * q->H * q->B > 0x7fffffff)
    return ZC_ERR_UNSUPPORTED;
  a.per_head = scores_per_head ? scores_per_head : ws_ph;
  a.normalize = normalize ? 1 : 0;

  hipStream_t st = (hipStream_t)stream;
  const bool need_lse = lse_ext == nullptr;
#define ZC_PROBE(DT) (q->D == 128 ? launch_probe<DT, 128>(a, need_lse, scores, st) : launch_probe<DT, 64>(a, need_lse, scores, st))
  if (q->dtype == ZC_F32) return ZC_PROBE(ZC_F32);
  if (q->dtype == ZC_F16) return ZC_PROBE(ZC_F16);
  return ZC_PROBE(ZC_BF16);
#undef ZC_PROBE
}

extern "C" int zc_probe_saliency(const zc_tensor4* q, const zc_tensor4* k,
                                 const int32_t* probe_rows, const int32_t* probe_pos, int32_t P,
                                 float sm_scale, const float* lse_ext,
                                 float* scores, float* scores_per_head,
                                 void* ws, size_t ws_bytes, void* stream) {
  return probe_scores(q, k, probe_rows, probe_pos, P, sm_scale, lse_ext, scores, scores_per_head, ws, ws_bytes, stream, true);
}

extern "C" int zc_probe_accumulated(const zc_tensor4* q, const zc_tensor4* k,
                                    const int32_t* probe_rows, const int32_t* probe_pos, int32_t P,
                                    float sm_scale, const float* lse_ext,
                                    float* scores, float* scores_per_head,
                                    void* ws, size_t ws_bytes, void* stream) {
  return probe_scores(q, k, probe_rows, probe_pos, P, sm_scale, lse_ext, scores, scores_per_head, ws, ws_bytes, stream, false);
}
