// zc_probe_saliency: normalized attention score of every key token from a
// probe subset of query rows (Eq. 9 substituted into Eq. 8).
//
// The probe rows of A = Softmax(Q_probe K^T / sqrt(d)) are never stored.  Two
// matrix-core sweeps recompute the logits instead:
//   k_probe_lse     one workgroup per 64 probe rows and column range (the columns a
//                   row block can see are split over up to 8 workgroups when the
//                   launch would not fill the chip): streams 128-column K tiles
//                   through LDS (the next tile's loads in flight), logits come
//                   out of the MFMA as D[column][row] so that every lane owns one
//                   probe row and keeps its running (max, sum) in two registers;
//                   writes the (max, sum) pair per row and column range.
//   k_probe_colsum  one workgroup per 128 key columns: K fragments stay in
//                   registers, 64-row probe tiles stream through LDS (merging the
//                   (max, sum) pairs of a row into its log-sum-exp on the way), logits
//                   come out as D[row][column] so that every lane owns one
//                   column and sums exp(logit - lse) over the rows in registers;
//                   divides by the number of probes that can see the column.
//   k_probe_mean    mean over query heads.
// Causality: rows are sorted by position, so a column tile starts at the first
// probe that can see it and a row tile stops at its last row's position.
// Inputs in fp16 / bf16 use the 32x32x16 MFMA, fp32 inputs the 32x32x2 fp32 MFMA
// (no rounding of the operands); accumulation and softmax are fp32.
#include "zc_common.hpp"

namespace zc {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int kMaxProbeSplit = 8;

struct ProbeArgs {
  const void* q;
  const void* k;
  int64_t q_sB, q_sH, q_sL, k_sB, k_sH, k_sL;
  int B, Hq, Hkv, G, Lk, P;
  const int32_t* probe_rows;
  const int32_t* probe_pos;
  float scale_log2;
  const float* lse_in;   // natural log, [B, Hq, P]; null: use lse2
  float* lse2;           // [B, Hq, P] log-sum-exp in log2 units: sweep 1's result
  float2* lse_part;      // [B, Hq, P, nsplit] (running maximum in log2 units, sum) when nsplit > 1
  int nsplit;            // column ranges a row block's sweep 1 is split into
  float* per_head;       // [B, Hq, Lk]
};

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
  static constexpr int CPR = ROWB / 16;        // 16-byte chunks per row
  static constexpr int STRIDE = ROWB + 16;     // padded LDS row stride
  static constexpr int NKC = ROWB / 32;        // operand chunks per lane and row
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

template <int DT, int D>
__global__ __launch_bounds__(256) void k_probe_lse(ProbeArgs a) {
  using T = Tile<DT, D>;
  // the probe rows go through the same LDS space as the K tiles: they are in
  // registers before the first tile arrives (four workgroups fit a CU this way)
  __shared__ __align__(16) uint8_t Ks[128 * T::STRIDE];
  uint8_t* Qs = Ks;
  __shared__ int spos[64];
  __shared__ float sm[4][64], sz[4][64];

  // logical order: probe-row block fastest, then column range, then query head, then batch
  const int nrb = ceil_div(a.P, 64);
  int j = xcd_contiguous(blockIdx.x, gridDim.x);
  const int rb0 = (j % nrb) * 64; j /= nrb;
  const int split = j % a.nsplit; j /= a.nsplit;
  const int hq = j % a.Hq, b = j / a.Hq, hk = hq / a.G;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, kh = lane >> 5;
  const uint8_t* qb = reinterpret_cast<const uint8_t*>(a.q) + ((int64_t)b * a.q_sB + (int64_t)hq * a.q_sH) * T::EB;
  const uint8_t* kb = reinterpret_cast<const uint8_t*>(a.k) + ((int64_t)b * a.k_sB + (int64_t)hk * a.k_sH) * T::EB;

  // the block's last row decides how many column tiles it sees; read it first so
  // that the first K tile is requested together with the probe rows
  const int nvalid = min(64, a.P - rb0);
  const int pmax = min(a.probe_pos[rb0 + nvalid - 1], a.Lk - 1);
  const int ntiles = pmax / 128 + 1;
  // this workgroup's share of the column tiles
  const int per = ceil_div(ntiles, a.nsplit);
  const int t_begin = split * per, t_end = min(t_begin + per, ntiles);

  // a K tile travels global -> registers -> LDS; the next tile's loads are in
  // flight while the current one is multiplied
  constexpr int KCH = 128 * T::CPR / 256;      // 16-byte chunks per thread and tile
  u32x4 kreg[KCH];
  auto fetch = [&](int t) {
#pragma unroll
    for (int j = 0; j < KCH; ++j) {
      const int i = tid + j * 256;
      const int row = i / T::CPR, cc = i % T::CPR;
      const int col = t * 128 + row;
      kreg[j] = u32x4{0, 0, 0, 0};
      if (col < a.Lk) kreg[j] = *reinterpret_cast<const u32x4*>(kb + (int64_t)col * a.k_sL * T::EB + cc * 16);
    }
  };
  if (t_begin < t_end) fetch(t_begin);

  for (int i = tid; i < 64 * T::CPR; i += 256) {
    const int row = i / T::CPR, cc = i % T::CPR;
    const int p = rb0 + row;
    u32x4 v = {0, 0, 0, 0};
    if (p < a.P) {
      const int64_t qrow = a.probe_rows ? a.probe_rows[p] : a.probe_pos[p];
      v = *reinterpret_cast<const u32x4*>(qb + qrow * a.q_sL * T::EB + cc * 16);
    }
    *reinterpret_cast<u32x4*>(Qs + row * T::STRIDE + cc * 16) = v;
  }
  if (tid < 64) spos[tid] = (rb0 + tid < a.P) ? a.probe_pos[rb0 + tid] : -1;
  __syncthreads();

  u32x4 qf[2][T::NKC];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc)
      qf[rb][kc] = *reinterpret_cast<const u32x4*>(Qs + (rb * 32 + r) * T::STRIDE + kc * 32 + kh * 16);
  const int myp[2] = {spos[r], spos[32 + r]};
  float m[2] = {-INFINITY, -INFINITY}, z[2] = {0.f, 0.f};

  for (int t = t_begin; t < t_end; ++t) {
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KCH; ++j) {
      const int i = tid + j * 256;
      *reinterpret_cast<u32x4*>(Ks + (i / T::CPR) * T::STRIDE + (i % T::CPR) * 16) = kreg[j];
    }
    __syncthreads();
    if (t + 1 < t_end) fetch(t + 1);
    v16f acc[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[0][i] = 0.f; acc[1][i] = 0.f; }
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc) {
      const u32x4 af = *reinterpret_cast<const u32x4*>(Ks + (w * 32 + r) * T::STRIDE + kc * 32 + kh * 16);
      mma_chunk<DT>(acc[0], af, qf[0][kc]);
      mma_chunk<DT>(acc[1], af, qf[1][kc]);
    }
    const int colb = t * 128 + w * 32;
    // rows are sorted by position: when the tile's last column is visible to the
    // block's first row, nothing in the tile is masked
    const bool tile_full = t * 128 + 127 <= spos[0];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      if (tile_full) {
        float tmax = acc[rb][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, acc[rb][v]);
        const float m_new = fmaxf(m[rb], tmax * a.scale_log2);
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(fmaf(acc[rb][v], a.scale_log2, -m_new));
        z[rb] = z[rb] * __builtin_amdgcn_exp2f(m[rb] - m_new) + sum;
        m[rb] = m_new;
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
  // merge the two half-waves, then the four waves
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const float mo = __shfl_xor(m[rb], 32), zo = __shfl_xor(z[rb], 32);
    const float M = fmaxf(m[rb], mo);
    float Z = 0.f;
    if (M > -INFINITY) Z = z[rb] * exp2f(m[rb] - M) + zo * exp2f(mo - M);
    if (kh == 0) { sm[w][rb * 32 + r] = M; sz[w][rb * 32 + r] = Z; }
  }
  __syncthreads();
  if (tid < 64 && rb0 + tid < a.P) {
    float M = fmaxf(fmaxf(sm[0][tid], sm[1][tid]), fmaxf(sm[2][tid], sm[3][tid]));
    float Z = 0.f;
    if (M > -INFINITY) {
#pragma unroll
      for (int i = 0; i < 4; ++i) Z += sz[i][tid] * exp2f(sm[i][tid] - M);
    }
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

template <int DT, int D>
__global__ __launch_bounds__(256) void k_probe_colsum(ProbeArgs a) {
  using T = Tile<DT, D>;
  // one LDS space: first the K tile (until its fragments are in registers), then
  // the probe positions followed by the current tile of probe rows
  __shared__ __align__(16) uint8_t Ks[128 * T::STRIDE];
  __shared__ int spos[64];
  __shared__ float slse[64];
  __shared__ float scol[2][128];

  // logical order: column tile fastest, then query head, then batch
  const int nct = ceil_div(a.Lk, 128);
  int j = xcd_contiguous(blockIdx.x, gridDim.x);
  const int col0 = (j % nct) * 128; j /= nct;
  const int hq = j % a.Hq, b = j / a.Hq, hk = hq / a.G;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, kh = lane >> 5;
  const int rbw = w >> 1, cbp = w & 1;
  const uint8_t* qb = reinterpret_cast<const uint8_t*>(a.q) + ((int64_t)b * a.q_sB + (int64_t)hq * a.q_sH) * T::EB;
  const uint8_t* kb = reinterpret_cast<const uint8_t*>(a.k) + ((int64_t)b * a.k_sB + (int64_t)hk * a.k_sH) * T::EB;
  const int64_t lrow = ((int64_t)b * a.Hq + hq) * a.P;

  for (int i = tid; i < 128 * T::CPR; i += 256) {
    const int row = i / T::CPR, cc = i % T::CPR;
    const int col = col0 + row;
    u32x4 v = {0, 0, 0, 0};
    if (col < a.Lk) v = *reinterpret_cast<const u32x4*>(kb + (int64_t)col * a.k_sL * T::EB + cc * 16);
    *reinterpret_cast<u32x4*>(Ks + row * T::STRIDE + cc * 16) = v;
  }
  __syncthreads();
  u32x4 kf[2][T::NKC];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc)
      kf[cb][kc] = *reinterpret_cast<const u32x4*>(Ks + ((cbp * 2 + cb) * 32 + r) * T::STRIDE + kc * 32 + kh * 16);

  // the K tile is in registers now: its LDS space takes the probe positions, so
  // that the two binary searches of this workgroup do not go to memory
  __syncthreads();
  constexpr int kPosCap = (128 - 64) * T::STRIDE / 4;     // what the tile of probe rows leaves free
  const int32_t* ppos = a.probe_pos;
  uint8_t* Qs = Ks + 64 * T::STRIDE;
  if (a.P <= kPosCap) {
    int32_t* lp = reinterpret_cast<int32_t*>(Ks);
    for (int i = tid; i < a.P; i += 256) lp[i] = a.probe_pos[i];
    __syncthreads();
    ppos = lp;
  }
  const int pstart = lower_bound_pos(ppos, a.P, col0);
  float colsum[2] = {0.f, 0.f};

  // a tile of 64 probe rows travels global -> registers -> LDS, the next one in
  // flight while the current one is multiplied; threads 0..63 also carry the
  // row's position and its log-sum-exp (log2 units)
  constexpr int QCH = 64 * T::CPR / 256;
  u32x4 qreg[QCH];
  int pos_reg = -1;
  float lse_reg = 0.f;
  auto fetch = [&](int pr) {
#pragma unroll
    for (int j = 0; j < QCH; ++j) {
      const int i = tid + j * 256;
      const int row = i / T::CPR, cc = i % T::CPR;
      const int p = pr + row;
      qreg[j] = u32x4{0, 0, 0, 0};
      if (p < a.P) {
        // (the positions are in LDS by now: no second trip to memory for the row address)
        const int64_t qrow = a.probe_rows ? a.probe_rows[p] : ppos[p];
        qreg[j] = *reinterpret_cast<const u32x4*>(qb + qrow * a.q_sL * T::EB + cc * 16);
      }
    }
    if (tid < 64) {
      const int p = pr + tid;
      pos_reg = p < a.P ? ppos[p] : -1;
      lse_reg = 0.f;
      if (p < a.P) {
        lse_reg = a.lse_in ? a.lse_in[lrow + p] * kLog2e : a.lse2[lrow + p];
      }
    }
  };
  if (pstart < a.P) fetch(pstart);

  for (int pr = pstart; pr < a.P; pr += 64) {
    __syncthreads();
#pragma unroll
    for (int j = 0; j < QCH; ++j) {
      const int i = tid + j * 256;
      *reinterpret_cast<u32x4*>(Qs + (i / T::CPR) * T::STRIDE + (i % T::CPR) * 16) = qreg[j];
    }
    if (tid < 64) { spos[tid] = pos_reg; slse[tid] = lse_reg; }
    __syncthreads();
    if (pr + 64 < a.P) fetch(pr + 64);
    int rp[16];
    float rl[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      rp[v] = spos[rbw * 32 + acc_row(v, kh)];
      rl[v] = slse[rbw * 32 + acc_row(v, kh)];
    }
    v16f acc[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[0][i] = 0.f; acc[1][i] = 0.f; }
#pragma unroll
    for (int kc = 0; kc < T::NKC; ++kc) {
      const u32x4 af = *reinterpret_cast<const u32x4*>(Qs + (rbw * 32 + r) * T::STRIDE + kc * 32 + kh * 16);
      mma_chunk<DT>(acc[0], af, kf[0][kc]);
      mma_chunk<DT>(acc[1], af, kf[1][kc]);
    }
    // a tile of 64 real rows whose first position is past this workgroup's last
    // column needs no mask
    const bool tile_full = pr + 64 <= a.P && col0 + 127 <= spos[0];
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
          colsum[cb] += (col <= rp[v]) ? e : 0.f;
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
    const int cnt = a.P - lower_bound_pos(ppos, a.P, col);
    a.per_head[((int64_t)b * a.Hq + hq) * a.Lk + col] = cnt > 0 ? total / (float)cnt : 0.f;
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
    hipLaunchKernelGGL((k_probe_lse<DT, D>), dim3((unsigned)((int64_t)ceil_div(a.P, 64) * a.Hq * a.B * a.nsplit)), dim3(256), 0, st, a);
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

// column ranges per row block of sweep 1: enough workgroups to fill the chip
static int probe_splits(int64_t B, int64_t Hq, int64_t P) {
  const int64_t wgs = B * Hq * ceil_div64(P, 64);
  int64_t ns = 1024 / wgs;      // four workgroups fit a CU
  return (int)(ns < 1 ? 1 : (ns > kMaxProbeSplit ? kMaxProbeSplit : ns));
}
static size_t lse_bytes(int64_t B, int64_t Hq, int64_t P) { return (size_t)align_up64(B * Hq * P * (kMaxProbeSplit * (int64_t)sizeof(float2) + 4), 256); }

extern "C" size_t zc_probe_saliency_workspace(int64_t B, int64_t Hq, int64_t Lk, int64_t P) {
  if (B <= 0 || Hq <= 0 || Lk <= 0 || P <= 0) return 0;
  return lse_bytes(B, Hq, P) + (size_t)B * Hq * Lk * 4;
}

extern "C" int zc_probe_saliency(const zc_tensor4* q, const zc_tensor4* k,
                                 const int32_t* probe_rows, const int32_t* probe_pos, int32_t P,
                                 float sm_scale, const float* lse_ext,
                                 float* scores, float* scores_per_head,
                                 void* ws, size_t ws_bytes, void* stream) {
  int rc = zc_validate_tensor(q);
  if (rc) return rc;
  rc = zc_validate_tensor(k);
  if (rc) return rc;
  if (q->dtype != k->dtype || q->D != k->D || q->B != k->B) return ZC_ERR_INVALID_ARG;
  if (q->H % k->H != 0) return ZC_ERR_INVALID_ARG;
  if (P < 1 || !probe_pos || !scores || k->L < 1 || q->L < 1) return ZC_ERR_INVALID_ARG;
  if (q->B > 65535 || q->H > 65535 || k->L > 0x7fffffff - 256) return ZC_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(probe_pos) & 3) || (reinterpret_cast<uintptr_t>(scores) & 3)) return ZC_ERR_INVALID_ARG;
  const size_t need = zc_probe_saliency_workspace(q->B, q->H, k->L, P);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15)) return ZC_ERR_WORKSPACE;

  ProbeArgs a;
  a.q = q->ptr; a.k = k->ptr;
  a.q_sB = q->sB; a.q_sH = q->sH; a.q_sL = q->sL;
  a.k_sB = k->sB; a.k_sH = k->sH; a.k_sL = k->sL;
  a.B = (int)q->B; a.Hq = (int)q->H; a.Hkv = (int)k->H; a.G = a.Hq / a.Hkv; a.Lk = (int)k->L; a.P = P;
  a.probe_rows = probe_rows; a.probe_pos = probe_pos;
  a.scale_log2 = (sm_scale == 0.f ? 1.0f / sqrtf((float)q->D) : sm_scale) * kLog2e;
  float* ws_ph = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(ws) + lse_bytes(q->B, q->H, P));
  a.lse_in = lse_ext;
  a.lse_part = reinterpret_cast<float2*>(ws);
  a.lse2 = reinterpret_cast<float*>(a.lse_part + (int64_t)q->B * q->H * P * kMaxProbeSplit);
  a.nsplit = probe_splits(q->B, q->H, P);
  if ((int64_t)ceil_div64(P, 64) * q->H * q->B * a.nsplit > 0x7fffffff || (int64_t)ceil_div64(k->L, 128) * q->H * q->B > 0x7fffffff)
    return ZC_ERR_UNSUPPORTED;
  a.per_head = scores_per_head ? scores_per_head : ws_ph;

  hipStream_t st = (hipStream_t)stream;
  const bool need_lse = lse_ext == nullptr;
#define ZC_PROBE(DT) (q->D == 128 ? launch_probe<DT, 128>(a, need_lse, scores, st) : launch_probe<DT, 64>(a, need_lse, scores, st))
  if (q->dtype == ZC_F32) return ZC_PROBE(ZC_F32);
  if (q->dtype == ZC_F16) return ZC_PROBE(ZC_F16);
  return ZC_PROBE(ZC_BF16);
#undef ZC_PROBE
}
