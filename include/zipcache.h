/*
 * zipcache.h - C ABI of the MI355X (gfx950) implementation of ZipCache's
 * data-parallel hot path (arXiv 2405.14256).
 *
 * Four operations, in the order Algorithm 2 (prefill) and Algorithm 3 (decode)
 * use them (and, beside them, the prefill attention of Algorithm 2 itself,
 * zc_prefill_attention, whose row normalisers feed the first):
 *
 *   zc_probe_saliency    Eq. 9 + Eq. 8: normalized attention score of every
 *                        key token from a probe subset of query rows.
 *   zc_select_salient    Algorithm 2 "Split": the k most salient tokens.
 *   zc_quantize_pack     Eq. 5, Eq. 6, Algorithm 1: channelwise or
 *                        channel-separable tokenwise quantization of the
 *                        salient subset at bits_hi and of the rest at bits_lo,
 *                        bit-packed into the cache arenas as a new chunk.
 *   zc_decode_attention  Eq. 4 over the packed cache (de-quantized on the
 *                        fly) plus a full-precision tail of recent tokens.
 *
 * General rules
 *   - Every pointer marked "device" is GPU memory owned by the caller; every
 *     other pointer is host memory.  The library allocates nothing, keeps no
 *     pointer after a call returns and has no global mutable state (apart from
 *     a cached copy of the device's compute-unit count and, for
 *     zc_decode_attention_static, its per-device scratch buffer).
 *   - All work is enqueued on the given HIP stream (`stream` is a hipStream_t
 *     passed as void*; NULL is the default stream).  Calls never synchronise
 *     with the host and never read results back.
 *   - Every function returns a zc_status.  Arguments are validated on the host
 *     before anything is launched; a failed validation launches nothing and
 *     leaves outputs untouched.  A launch failure returns ZC_ERR_HIP.
 *   - Device pointers must be 16-byte aligned; tensors must have unit stride
 *     along the last (channel) axis and all other strides multiples of 8
 *     elements.
 *   - Supported: head dimension D in {64, 128}; dtypes f32, f16, bf16;
 *     code widths in {2, 4, 8}; Hq a multiple of Hkv with Hq/Hkv <= 8.
 *   - HIP graph capture.  Every call may be captured (nothing synchronises or
 *     allocates).  The state of a zc_packed on the host - slots in use, number of
 *     chunks, the mirror of the chunk table - is read when a call is *issued* and
 *     travels in the kernel arguments: a captured zc_decode_attention replays over the
 *     chunks the cache had at capture time, a captured zc_quantize_pack appends at the
 *     slots it was captured for.  A graph therefore has to be captured in the order its
 *     calls will run and replayed as a whole sequence from the same starting state
 *     (after the host fields have been reset to what they were when capture began);
 *     the library cannot check this.
 *   - Value ranges (not checked: the data lives on the device).  All inputs must be
 *     finite - no NaN, no infinity (the quantizer takes minima and maxima without
 *     regard to NaN).  zc_decode_attention feeds the matrix cores fp16 operands:
 *     every |q[c] * chan_scale[c] * sm_scale| of the keys' channel scales must stay
 *     below 700 and every token scale of the values below 1000 (an fp16 overflow
 *     there turns the output into NaN); activations of the models the paper
 *     compresses are orders of magnitude inside these bounds.
 *   - Size limits (beyond them a call returns ZC_ERR_UNSUPPORTED and launches
 *     nothing): B <= 65535 and heads <= 65535; a token row of a cache tensor at
 *     most 8192 channels (W = H*D) in zc_quantize_pack; the kernels address one
 *     (batch, head) slab with 32-bit byte offsets, so the span of such a slab -
 *     L * sL elements of q, (L + 128) * sL of k in the probe calls, tail_len * sL
 *     of the tail, cap * D * bits / 8 bytes of a code arena in the decode call -
 *     must stay below 4 GiB - 4 KiB.
 */
#ifndef ZIPCACHE_H
#define ZIPCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ZC_OK = 0,
  ZC_ERR_INVALID_ARG = -1, /* null / misaligned pointer, bad size or stride  */
  ZC_ERR_UNSUPPORTED = -2, /* dtype, head dim, bit width, scheme, size limit  */
  ZC_ERR_WORKSPACE = -3,   /* workspace smaller than the *_workspace() size  */
  ZC_ERR_CAPACITY = -4,    /* arena or chunk table of a zc_packed is full    */
  ZC_ERR_HIP = -5,         /* the HIP runtime refused a launch               */
  ZC_ERR_STATIC_LIMIT = -6 /* needs more scratch than ZC_STATIC_SCRATCH_BYTES */
} zc_status;

typedef enum { ZC_F32 = 0, ZC_F16 = 1, ZC_BF16 = 2 } zc_dtype;

/* Quantization granularity of one cache tensor.
 *   CHANNEL: one (s, z) of Eq. 5 per channel over the tokens of the subset
 *            (the paper's choice for keys, Section 4.1).
 *   CST:     Algorithm 1 - c_i = sqrt(max|X_i|) per channel (Eq. 6), then one
 *            (s, z) per token over the W = H*D normalized values of its row
 *            (the paper's choice for values).
 *   TOKEN:   CST with c = 1 (plain tokenwise quantization, Table 1 row 3).
 * In every scheme
 *   x_hat[t, w] = chan_scale[w] * tok_scale[t] * (code[t, w] - tok_zero[t] - chan_zero[w])
 * with tok_scale = 1, tok_zero = 0 for CHANNEL and chan_zero = 0 otherwise. */
typedef enum { ZC_SCHEME_CHANNEL = 0, ZC_SCHEME_CST = 1, ZC_SCHEME_TOKEN = 2 } zc_scheme;

/* Bit layout of the codes of one (batch, head) inside an arena.
 *   ROW    (keys): slot-major rows of D codes; code of channel c sits at bit
 *          offset c*bits of its row, little-endian (for 4 bits: channel 2j in
 *          the low nibble of byte j).
 *   TGROUP (values): 32-bit words indexed [block][kg][c], kg in 0..3, c the
 *          channel, each word holding E = 32/bits codes of one channel for E
 *          different slots; a block covers 4*E consecutive slots.  Field e
 *          (bits e*bits .. (e+1)*bits-1) of word [blk][kg][c] belongs to slot
 *             blk*4*E + 16*j(e) + 4*kg + e%4,
 *          j(e) = e/4 for bits in {4, 8};  for bits == 2, j(e) = 0,2,1,3 for
 *          e/4 = 0,1,2,3.
 *          (Keys are contracted over channels and values over tokens, so each
 *          tensor packs along the axis its matrix-core operand runs over.)
 * Both layouts take B*H*cap*D*bits/8 bytes per arena. */
typedef enum { ZC_LAYOUT_ROW = 0, ZC_LAYOUT_TGROUP = 1 } zc_layout;

#define ZC_SLOT_ALIGN 64 /* every chunk starts at a multiple of this many slots */
#define ZC_MAX_GROUP 8   /* largest supported Hq / Hkv                          */

/* A strided 4-D view [B, H, L, D] of device memory; strides in elements,
 * the D axis is contiguous. */
typedef struct zc_tensor4 {
  void* ptr; /* device */
  int32_t dtype; /* zc_dtype */
  int32_t reserved;
  int64_t B, H, L, D;
  int64_t sB, sH, sL;
} zc_tensor4;

/* One tensor (K or V) of the compressed cache.  The struct lives on the host;
 * all arrays are caller-allocated.  Salient tokens go to the "hi" arena at
 * bits_hi, the others to the "lo" arena at bits_lo.  Each zc_quantize_pack
 * call appends one chunk: chunk_table row i = {begin_hi, len_hi, begin_lo,
 * len_lo} in slots.  A chunk has its own channel parameters (one set per
 * subset); slot r of the hi part of chunk i is slot begin_hi + r of the hi
 * arena for the codes, the token parameters and the positions alike.  The K
 * and V structs of one cache must be filled by the same sequence of calls so
 * that their chunk tables agree. */
typedef struct zc_packed {
  int32_t layout;  /* zc_layout */
  int32_t scheme;  /* zc_scheme */
  int32_t bits_hi, bits_lo;
  int64_t B, H, D;          /* W = H*D channels per token row */
  int64_t cap_hi, cap_lo;   /* slots per arena, multiples of ZC_SLOT_ALIGN */
  int64_t n_hi, n_lo;       /* slots in use (aligned end of the last chunk) */
  uint8_t* codes_hi;        /* device, B*H*cap_hi*D*bits_hi/8 bytes */
  uint8_t* codes_lo;        /* device */
  float* tok_scale_hi;      /* device [B, cap_hi]; unused for CHANNEL (may be NULL) */
  float* tok_zero_hi;
  float* tok_scale_lo;      /* device [B, cap_lo] */
  float* tok_zero_lo;
  int32_t* pos_hi;          /* device [B, cap_hi] original token positions, or NULL */
  int32_t* pos_lo;          /* device [B, cap_lo], or NULL */
  float* chan_scale;        /* device [max_chunks, 2 (hi, lo), B, W] */
  float* chan_zero;         /* device [max_chunks, 2, B, W] */
  int32_t* chunk_table;     /* device [max_chunks, 4] */
  int32_t* chunk_table_host; /* host   [max_chunks, 4], kept equal to the above */
  int32_t n_chunks, max_chunks;
} zc_packed;

/* ---- Eq. 9 + Eq. 8 ------------------------------------------------------
 * q [B, Hq, Lq, D], k [B, Hkv, Lk, D], same dtype.  Probe p uses query row
 * probe_rows[p] of q (probe_pos[p] when probe_rows is NULL) and attends key
 * columns i <= probe_pos[p]; probe_pos must be ascending (device int32 [P],
 * values in [0, Lk)).  Logits are q.k * sm_scale (sm_scale == 0 means
 * 1/sqrt(D)); query head h reads KV head h / (Hq/Hkv).
 * With lse_ext == NULL each probe row is soft-maxed over its visible columns.
 * With lse_ext (device float [B, Hq, P], natural log) the probabilities are
 * exp(logit - lse_ext): decode-time probes whose softmax also covered tokens
 * outside k.
 * Output scores (device float [B, Lk]): mean over query heads of
 *   sum_{p : probe_pos[p] >= i} A[p, i] / #{p : probe_pos[p] >= i}
 * (0 where no probe sees column i).  scores_per_head (device float
 * [B, Hq, Lk]) receives the per-head values when not NULL.
 * The result is deterministic: no floating-point atomics are used. */
size_t zc_probe_saliency_workspace(int64_t B, int64_t Hq, int64_t Lk, int64_t P);
int zc_probe_saliency(const zc_tensor4* q, const zc_tensor4* k,
                      const int32_t* probe_rows, const int32_t* probe_pos, int32_t P,
                      float sm_scale, const float* lse_ext,
                      float* scores, float* scores_per_head,
                      void* ws, size_t ws_bytes, void* stream);

/* ---- Eq. 7 (the accumulated attention score the paper argues against) ------
 * Same arguments, workspace and error behaviour as zc_probe_saliency; the
 * column sums are NOT divided by the number of probes that see the column:
 *   scores[b, i] = mean over query heads of sum_{p : probe_pos[p] >= i} A[p, i].
 * With all rows as probes this is Eq. 7 itself (earlier tokens accumulate more
 * terms: the bias of Section 4.2); serves as the comparison metric. */
int zc_probe_accumulated(const zc_tensor4* q, const zc_tensor4* k,
                         const int32_t* probe_rows, const int32_t* probe_pos, int32_t P,
                         float sm_scale, const float* lse_ext,
                         float* scores, float* scores_per_head,
                         void* ws, size_t ws_bytes, void* stream);

/* ---- Algorithm 2, the attention line (Eq. 2 applied to V; Appendix B, prefill) -------
 * The attention output of all prompt tokens at once, with the causal mask:
 *   out[b, h, p, :] = sum_{i <= p} softmax_i(q[b,h,p] . k[b,h/G,i] * sm_scale) v[b,h/G,i, :]
 * q, out [B, Hq, L, D]; k, v [B, Hkv, L, D]; all four of one dtype (out may have strides of
 * its own); sm_scale == 0 means 1/sqrt(D).  lse (device float [B, Hq, L], optional)
 * receives the natural-log normaliser of every row.  With P > 0 the normalisers of the
 * rows probe_pos[0..P) (device int32, values in [0, L)) are also gathered into lse_probe
 * (device float [B, Hq, P]; needs lse): exactly the lse_ext argument with which
 * zc_probe_saliency scores the same probe rows in one sweep instead of two.
 * fp32 tensors are multiplied on the fp32 matrix pipes, never rounded to 16 bits; the
 * probabilities of 16-bit tensors enter the second product rounded to the tensors' type.
 * Needs no workspace; enqueued on `stream`.
 * Errors: ZC_ERR_INVALID_ARG for mismatching shapes or types, ZC_ERR_UNSUPPORTED for a
 * (batch, head) slab of 4 GiB or more. */
int zc_prefill_attention(const zc_tensor4* q, const zc_tensor4* k, const zc_tensor4* v, float sm_scale,
                         const zc_tensor4* out, float* lse,
                         const int32_t* probe_pos, int32_t P, float* lse_probe, void* stream);

/* ---- Algorithm 2, Split(., p~, r%) ------------------------------------------
 * scores: device float [B, L] (must not contain NaN).  For every batch row
 * the k largest scores are salient; among equal scores the lower index wins.
 * salient_idx (device int32 [B, k]) and regular_idx (device int32 [B, L-k])
 * are both ascending; mask (device uint8 [B, L], optional) is 1 for salient.
 * 0 <= k <= L.  Exact and deterministic. */
size_t zc_select_salient_workspace(int64_t B, int64_t L);
int zc_select_salient(const float* scores, int64_t B, int64_t L, int64_t k,
                      int32_t* salient_idx, int32_t* regular_idx, uint8_t* mask,
                      void* ws, size_t ws_bytes, void* stream);

/* ---- Eq. 5, Eq. 6, Algorithm 1; the four quantizer calls of Algorithm 2 -----
 * x [B, H, L, D] is one cache tensor.  Tokens salient_idx[b, 0..k) are
 * quantized at out->bits_hi, tokens regular_idx[b, 0..n_reg) at out->bits_lo,
 * each subset with its own channel statistics, by out->scheme, rounding half
 * to even; s := 1 when max == min, c := 1 when the channel is all zero.  An
 * empty subset gets chan_scale = 1, chan_zero = 0.  The codes are appended as
 * chunk out->n_chunks in out->layout; positions idx + pos_offset are stored
 * when pos arrays are present.  On success the host fields n_hi, n_lo,
 * n_chunks and chunk_table_host are updated (the device copy is written by
 * the enqueued work).  Index lists must hold distinct values in [0, L). */
size_t zc_quantize_pack_workspace(int64_t B, int64_t H, int64_t L /* tokens per call, k + n_reg */, int64_t D);
int zc_quantize_pack(const zc_tensor4* x, const int32_t* salient_idx, int64_t k,
                     const int32_t* regular_idx, int64_t n_reg, int64_t pos_offset,
                     zc_packed* out, void* ws, size_t ws_bytes, void* stream);

/* ---- the four quantizer calls of Algorithm 2 at once ------------------------------------
 * Keys and values of one cache compressed by the same launches: exactly what two
 * zc_quantize_pack calls (xk into outK, then xv into outV, same index lists and offset)
 * leave behind, bit for bit, in half the launches (three, when outK is CHANNEL / ROW, outV is
 * CST / TGROUP and a token row has at most 2048 channels; four or five otherwise).  xk and xv
 * must agree in shape and dtype; outK and outV are two different descriptors.  Workspace:
 * zc_quantize_pack_kv_workspace(B, H, k + n_reg, D).  Errors as for zc_quantize_pack; when
 * one is returned neither descriptor has been changed. */
size_t zc_quantize_pack_kv_workspace(int64_t B, int64_t H, int64_t L, int64_t D);
int zc_quantize_pack_kv(const zc_tensor4* xk, const zc_tensor4* xv, const int32_t* salient_idx, int64_t k,
                        const int32_t* regular_idx, int64_t n_reg, int64_t pos_offset,
                        zc_packed* outK, zc_packed* outV, void* ws, size_t ws_bytes, void* stream);

/* ---- Eq. 4 over the packed cache (Algorithm 3, attention line) -------------------
 * q [B, Hq, 1, D]; Kp (ROW layout) and Vp (TGROUP layout) hold the same
 * chunks; tail_k / tail_v [B, Hkv, >=tail_len, D] are the full-precision
 * recent tokens (same dtype as q; may be NULL when tail_len == 0).
 * out (device, q's dtype, [B, Hq, D]) = softmax(q.K^T * sm_scale) V over all
 * packed tokens and the first tail_len tail tokens; lse_out (device float
 * [B, Hq], optional) receives the natural-log normaliser of each row.
 * Deterministic for fixed shapes.  Calls that share a workspace must not run
 * concurrently. */
size_t zc_decode_attention_workspace(int64_t B, int64_t Hq, int64_t D);
int zc_decode_attention(const zc_tensor4* q, const zc_packed* Kp, const zc_packed* Vp,
                        const zc_tensor4* tail_k, const zc_tensor4* tail_v, int64_t tail_len,
                        float sm_scale, void* out, float* lse_out,
                        void* ws, size_t ws_bytes, void* stream);

/* ---- groupwise quantization: the baseline granularity of Table 1 / Appendix A (Eq. A) -----
 * Every `group` (8, 16, 32, 64 or 128; the paper's n = 32) consecutive channels of a token
 * row w = h*D + c share one (s, z) of Eq. 5 (s := 1 when the group is constant; round half to
 * even).  x [B, H, L, D]; the n token rows idx[b, 0..n) (device int32, or NULL for rows 0..n-1)
 * are quantized at `bits` (2, 4 or 8).  A comparator, not a cache format: outputs are
 * token-major and unpacked, each optional - codes_out device uint8 [B, n, W], scale_out /
 * zero_out device float [B, n, W / group], dequant_out device float [B, n, W] =
 * (code - z) * s.  Needs no workspace. */
int zc_group_quantize(const zc_tensor4* x, const int32_t* idx, int64_t n, int32_t bits, int32_t group,
                      uint8_t* codes_out, float* scale_out, float* zero_out, float* dequant_out, void* stream);

/* ---- Algorithm 3 with its re-compression branch taken at its word ----------------------
 * ("Extract K[:-100] and V[:-100] and adaptively compress them with A_probe": every 100
 * steps everything but the newest 100 tokens is compressed again as a whole, ranked by the
 * explicit attention rows of the window's probe steps.)  Three building blocks; together
 * with zc_select_salient and zc_quantize_pack into a fresh zc_packed they make that branch.
 *
 * zc_decode_probs: the attention row a of one decode step (Eq. 4's probabilities; the
 * "Compute attention scores a of current token" line), in token order:
 *   probs_out[b, h, pos] = exp(q[b,h] . k_hat[b, h/G, pos] * sm_scale - lse[b, h])
 * over every token of Kp (at its stored position: Kp needs its pos arrays) and the first
 * tail_len rows of tail_k (token tail_pos0 + t).  lse (device float [B, Hq]) is the
 * normaliser zc_decode_attention returned for the same step; probs_out is device float
 * [B, Hq, N], N >= tail_pos0 + tail_len, and entries of positions the cache does not hold
 * are left untouched.  Arguments as for zc_decode_attention otherwise.
 *
 * zc_rows_saliency: Eq. 8 on explicit rows.  rows is device float [P, B, Hq, row_stride]
 * (row j valid for tokens i < row_len[j]; row_len device int32 [P]):
 *   scores[b, i] = mean over heads of sum_{j : row_len[j] > i} rows[j, b, h, i] / #{j : row_len[j] > i}
 * for i < n_out (scores: device float [B, n_out]; 0 where no row sees the token; without the
 * division when normalize == 0: Eq. 7).  Deterministic (fixed summation order).
 *
 * zc_dequantize_cache: out[b, h, pos, :] = x_hat of every token of p (all chunks), rounded to
 * out's dtype, at its stored position (p needs its pos arrays; positions >= out->L are
 * skipped).  out [B, H, L', D] is typically the caller's full-precision token buffer, whose
 * rows pos >= (tokens in p) already hold the tokens not compressed yet. */
int zc_decode_probs(const zc_tensor4* q, const zc_packed* Kp, const zc_tensor4* tail_k, int64_t tail_len,
                    int64_t tail_pos0, float sm_scale, const float* lse, float* probs_out, int64_t N, void* stream);
int zc_rows_saliency(const float* rows, const int32_t* row_len, int32_t P, int64_t B, int64_t Hq,
                     int64_t row_stride, int64_t n_out, int32_t normalize, float* scores, void* stream);
int zc_dequantize_cache(const zc_packed* p, const zc_tensor4* out, void* stream);

/* ---- zc_decode_attention for callers that cannot allocate ----------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid
 * hipMalloc: the same operation, arguments, kernels and results as zc_decode_attention,
 * without a workspace argument.  The partial results of the split-K workgroups go to a
 * buffer of ZC_STATIC_SCRATCH_BYTES that lives in the library's own device image (one
 * copy per GPU, held until the process ends); the call allocates and frees nothing.
 * Limit: zc_decode_attention_workspace(B, Hq, D) must not exceed ZC_STATIC_SCRATCH_BYTES
 * (B*Hq <= 1790 query heads at D = 128 is always within it), else the call returns
 * ZC_ERR_STATIC_LIMIT and launches nothing.  All calls on one GPU share that buffer: two
 * calls that may overlap on the same GPU (different streams) race; calls on one stream,
 * or ordered by events, are safe.  Nothing in the buffer has to start at zero: every
 * partial a call reads was written by that call. */
#define ZC_STATIC_SCRATCH_BYTES (8u << 20)
int zc_decode_attention_static(const zc_tensor4* q, const zc_packed* Kp, const zc_packed* Vp,
                               const zc_tensor4* tail_k, const zc_tensor4* tail_v, int64_t tail_len,
                               float sm_scale, void* out, float* lse_out, void* stream);

/* ---- helpers ------------------------------------------------------------------ */
/* Bytes of one code arena of `cap` slots. */
size_t zc_arena_bytes(int64_t B, int64_t H, int64_t D, int64_t cap, int32_t bits);
/* Smallest legal capacity that holds `n_chunks` chunks totalling n tokens. */
int64_t zc_arena_slots(int64_t n_tokens, int64_t n_chunks);
/* ---- inverse of the packing (Eq. 5's de-quantization; the bit layouts above) ----
 * Unpacks subset `which` (0: hi / salient, 1: lo / regular) of chunk `chunk` of
 * a packed tensor into canonical token-major arrays: element [b, r, w] belongs
 * to slot r of that chunk's subset (ascending original position) and channel
 * w = h*D + c.  codes_out (device uint8 [B, len, W], one byte per code) and
 * dequant_out (device float [B, len, W], x_hat of the formula at zc_scheme) may
 * each be NULL.  len is the subset's length in the chunk table (host mirror).
 * Nothing is allocated; the work is enqueued on `stream`.
 * Errors: ZC_ERR_INVALID_ARG for a bad descriptor, chunk or subset index. */
int zc_unpack(const zc_packed* p, int32_t which, int32_t chunk, uint8_t* codes_out, float* dequant_out,
              void* stream);

const char* zc_status_string(int status);
int zc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ZIPCACHE_H */
