"""CPU oracle for the ZipCache hot path (arXiv 2405.14256).

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, float64 numpy
implementation of what the GPU library computes.  It exists so that the HIP
kernels can be checked element by element; it is never used by the product
path, and it shares no code with it.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it.

Every function follows the paper's definition or algorithm step by step, in
the paper's order, with no blocking, fusion or reordering.  Conventions used
throughout (tokens and channels are 0-indexed):

  * Q is [B, Hq, L, d]; K and V are [B, Hkv, L, d]; query head h reads KV head
    h // (Hq // Hkv).
  * A "token row" of K or V is the W = Hkv*d values of one token across all KV
    heads (the l x hd matrix of Algorithm 1), channel index w = head*d + c.
  * Rounding is round-half-to-even (numpy.rint).
  * The de-quantizer is (code - z) * s: Eq. 5 as printed omits the "- z", but
    its stated error behaviour only holds with it.
  * A degenerate group with max == min takes s := 1; a channel whose maximum
    magnitude is 0 takes c := 1.

Parity pins live in tests/test_oracle_*.py; both readings of Algorithm 3's
re-compression branch (StreamingCache: chunk-local; LiteralStreamingCache: the
text taken at its word) are pinned only by self-consistency ("parity unpinned"
by the paper, whose text is ambiguous there).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Attention (Eq. 2, Eq. 4, Eq. 9)
# --------------------------------------------------------------------------

def _scale(d: int, sm_scale: Optional[float]) -> float:
    return 1.0 / np.sqrt(float(d)) if not sm_scale else float(sm_scale)


def causal_attention(q: np.ndarray, k: np.ndarray, sm_scale: Optional[float] = None) -> np.ndarray:
    """Eq. 2, one head: A = Softmax(q k^T / sqrt(d)), lower triangular.

    q, k: [L, d].  Returns A [L, L] with A[p, i] = 0 for i > p (Section 4.2
    states the matrix is lower triangular).
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    L, d = q.shape
    S = (q @ k.T) * _scale(d, sm_scale)
    row = np.arange(L)[:, None]
    col = np.arange(L)[None, :]
    S = np.where(col <= row, S, -np.inf)
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    return E / E.sum(axis=1, keepdims=True)


def probe_attention(q_rows: np.ndarray, pos: np.ndarray, k: np.ndarray,
                    sm_scale: Optional[float] = None,
                    lse: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 9, one head: the rows of A that belong to the probe tokens.

    q_rows: [P, d] probe queries; pos: [P] causal position of each probe (it
    attends key columns i <= pos); k: [Lk, d].  Returns (A_probe [P, Lk],
    lse [P]).  When `lse` is given it is used as the log-normaliser of each row
    instead of the one computed over the visible columns (decode-time probes,
    whose softmax also ran over tokens that are not columns of `k`).
    """
    q_rows = np.asarray(q_rows, F64)
    k = np.asarray(k, F64)
    pos = np.asarray(pos, np.int64)
    P, d = q_rows.shape
    Lk = k.shape[0]
    S = (q_rows @ k.T) * _scale(d, sm_scale)
    visible = np.arange(Lk)[None, :] <= pos[:, None]
    S = np.where(visible, S, -np.inf)
    if lse is None:
        m = S.max(axis=1)
        lse = m + np.log(np.exp(S - m[:, None]).sum(axis=1))
    lse = np.asarray(lse, F64)
    A = np.exp(S - lse[:, None])
    return A, lse


def prefill_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray,
                      sm_scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 2's attention line: the prefill output of every token at once,
    O = Softmax(Q K^T / sqrt(d)) V with the causal mask (Eq. 2 applied to V), and
    the log-normaliser of every row (the natural log of its softmax denominator,
    what a row needs to be re-normalised later: the probe rows of Eq. 9).

    Q: [B, Hq, L, d]; K, V: [B, Hkv, L, d]; query head h reads KV head h // (Hq // Hkv).
    Returns (O [B, Hq, L, d], lse [B, Hq, L])."""
    Q = np.asarray(Q, F64)
    K = np.asarray(K, F64)
    V = np.asarray(V, F64)
    B, Hq, L, d = Q.shape
    G = Hq // K.shape[1]
    O = np.zeros((B, Hq, L, d), F64)
    lse = np.zeros((B, Hq, L), F64)
    row = np.arange(L)[:, None]
    col = np.arange(L)[None, :]
    for b in range(B):
        for h in range(Hq):
            A = causal_attention(Q[b, h], K[b, h // G], sm_scale)
            O[b, h] = A @ V[b, h // G]
            S = np.where(col <= row, (Q[b, h] @ K[b, h // G].T) * _scale(d, sm_scale), -np.inf)
            m = S.max(axis=1)
            lse[b, h] = m + np.log(np.exp(S - m[:, None]).sum(axis=1))
    return O, lse


def unmasked_count(pos: np.ndarray, Lk: int) -> np.ndarray:
    """nnz(A[:, i]) of Eq. 8 read structurally: the number of probe rows whose
    causal window contains column i."""
    pos = np.asarray(pos, np.int64)
    return (pos[:, None] >= np.arange(Lk)[None, :]).sum(axis=0)


def saliency_scores(Q: np.ndarray, K: np.ndarray, probe_pos: Sequence[int],
                    probe_rows: Optional[Sequence[int]] = None,
                    sm_scale: Optional[float] = None,
                    lse_ext: Optional[np.ndarray] = None,
                    normalized: bool = True) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 8 with the probe rows of Eq. 9 substituted (Eq. 7 when
    normalized=False).

    Q: [B, Hq, Lq, d]; K: [B, Hkv, Lk, d]; probe_pos: [P] causal positions;
    probe_rows: [P] rows of Q holding the probe queries (default: probe_pos);
    lse_ext: optional [B, Hq, P] external log-normalisers.
    Returns (scores [B, Lk], per_head [B, Hq, Lk]); the per-token score is the
    mean over query heads of the per-head column-sum / unmasked-count.
    Columns no probe can see get score 0.
    """
    Q = np.asarray(Q, F64)
    K = np.asarray(K, F64)
    B, Hq, _, d = Q.shape
    _, Hkv, Lk, _ = K.shape
    G = Hq // Hkv
    pos = np.asarray(probe_pos, np.int64)
    rows = pos if probe_rows is None else np.asarray(probe_rows, np.int64)
    cnt = unmasked_count(pos, Lk)
    per_head = np.zeros((B, Hq, Lk), F64)
    for b in range(B):
        for h in range(Hq):
            ext = None if lse_ext is None else np.asarray(lse_ext, F64)[b, h]
            A, _ = probe_attention(Q[b, h, rows], pos, K[b, h // G], sm_scale, ext)
            col = A.sum(axis=0)
            if normalized:
                col = np.where(cnt > 0, col / np.maximum(cnt, 1), 0.0)
            per_head[b, h] = col
    return per_head.mean(axis=1), per_head


# --------------------------------------------------------------------------
# Salient-token split (Algorithm 2, "Split")
# --------------------------------------------------------------------------

def select_salient(score: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """The k tokens with the largest score; equal scores go to the lower index.
    Returns (salient, regular), both ascending."""
    score = np.asarray(score)
    L = score.shape[0]
    order = np.lexsort((np.arange(L), -score.astype(F64)))  # score desc, index asc
    chosen = np.zeros(L, bool)
    chosen[order[:k]] = True
    idx = np.arange(L)
    return idx[chosen], idx[~chosen]


# --------------------------------------------------------------------------
# Uniform quantizer (Eq. 5) and the three granularities built on it
# --------------------------------------------------------------------------

def _ratio(x, xmin, xmax, bits: int):
    """x / s of Eq. 5 with s = (max - min) / (2^k - 1), evaluated as
    x * (2^k - 1) / (max - min) (the same real number).  A group with
    max == min uses s = 1."""
    x = np.asarray(x, F64)
    rng = np.asarray(xmax, F64) - np.asarray(xmin, F64)
    flat = rng == 0.0
    return np.where(flat, x, x * float(2 ** bits - 1) / np.where(flat, 1.0, rng))


def _round_ratio(x, xmin, xmax, bits: int):
    """round(x / s) of Eq. 5, half-to-even, decided in exact arithmetic.

    fp16 / bf16 data sit on a coarse grid, so x / s lands exactly halfway
    between two integers far more often than chance (for instance the minimum
    of a token row whose maximum is its mirror image gives exactly -(2^k-1)/2).
    Floating-point evaluation would decide those ties by its own rounding
    noise; here every value within 1e-9 of a tie is re-evaluated as the exact
    rational x (2^k - 1) / (max - min) of the given float64 numbers.
    Returns (rounded, value before rounding)."""
    from fractions import Fraction
    pre = _ratio(x, xmin, xmax, bits)
    out = np.array(np.rint(pre), dtype=F64)
    frac = np.abs(pre - np.floor(pre) - 0.5)
    near = np.argwhere(frac < 1e-9 * np.maximum(1.0, np.abs(pre)))
    if len(near):
        xb, lob, hib = np.broadcast_arrays(np.asarray(x, F64), np.asarray(xmin, F64), np.asarray(xmax, F64))
        qmax = 2 ** bits - 1
        for ix in map(tuple, near):
            lo, hi = Fraction(float(lob[ix])), Fraction(float(hib[ix]))
            if hi == lo:
                continue
            out[ix] = float(round(Fraction(float(xb[ix])) * qmax / (hi - lo)))   # half-to-even
    return out, pre


def quant_params(xmin, xmax, bits: int):
    """s = (max - min) / (2^k - 1), z = -round(min / s); s := 1 if max == min."""
    xmin = np.asarray(xmin, F64)
    xmax = np.asarray(xmax, F64)
    s = (xmax - xmin) / float(2 ** bits - 1)
    s = np.where(s == 0.0, 1.0, s)
    z = -_round_ratio(xmin, xmin, xmax, bits)[0]
    return s, z + 0.0


def quantize(x, xmin, xmax, bits: int):
    """clip(round(x / s) + z, 0, 2^k - 1) for a group with the given extrema.
    Returns (codes, x / s before rounding)."""
    _, z = quant_params(xmin, xmax, bits)
    r, pre = _round_ratio(x, xmin, xmax, bits)
    return np.clip(r + z, 0.0, float(2 ** bits - 1)), pre


def dequantize(code, s, z):
    return (np.asarray(code, F64) - z) * s


@dataclass
class QuantSubset:
    """One token subset of one tensor after quantization.

    x_hat[b, t, w] = chan_scale[b, w] * tok_scale[b, t]
                     * (codes[b, t, w] - tok_zero[b, t] - chan_zero[b, w])
    (channelwise: tok_scale = 1, tok_zero = 0; channel-separable tokenwise:
    chan_scale = c, chan_zero = 0).
    """
    scheme: str
    bits: int
    idx: np.ndarray          # [B, n] token positions, ascending
    codes: np.ndarray        # [B, n, W] integers stored as float64
    chan_scale: np.ndarray   # [B, W]
    chan_zero: np.ndarray    # [B, W]
    tok_scale: np.ndarray    # [B, n]
    tok_zero: np.ndarray     # [B, n]
    pre_round: Optional[np.ndarray] = None  # x/s before rounding (diagnostics)
    grp_scale: Optional[np.ndarray] = None  # groupwise only: [B, n, W / group]
    grp_zero: Optional[np.ndarray] = None

    def dequant(self) -> np.ndarray:
        if self.scheme == "group":
            g = self.codes.shape[2] // self.grp_scale.shape[2]
            return (self.codes - np.repeat(self.grp_zero, g, axis=2)) * np.repeat(self.grp_scale, g, axis=2)
        return (self.chan_scale[:, None, :] * self.tok_scale[:, :, None]
                * (self.codes - self.tok_zero[:, :, None] - self.chan_zero[:, None, :]))


def quantize_rows(X: np.ndarray, bits: int, scheme: str, idx: Optional[np.ndarray] = None,
                  group: int = 32) -> QuantSubset:
    """Quantize token rows X [B, n, W] of one subset.

    scheme "group": groupwise quantization, the fine-grained baseline of Table 1 and
      Appendix A (Eq. A): every `group` consecutive channels of a token row share one
      (s, z) of Eq. 5 - 2 l h d / n parameters per tensor.
    scheme "channel": one (s, z) per channel over the subset's tokens (the
      paper's key-cache scheme, Section 4.1).
    scheme "cst": Algorithm 1 - c_i = sqrt(max |X_i|), X_i /= c_i, tokenwise
      Eq. 5 over each row of W values, rescale by c_i on de-quantization.
    scheme "token": plain tokenwise quantization (Algorithm 1 with c = 1).
    """
    X = np.asarray(X, F64)
    B, n, W = X.shape
    if idx is None:
        idx = np.tile(np.arange(n), (B, 1))
    ones_t = np.ones((B, n), F64)
    zeros_t = np.zeros((B, n), F64)
    ones_c = np.ones((B, W), F64)
    zeros_c = np.zeros((B, W), F64)
    if n == 0:
        return QuantSubset(scheme, bits, idx, np.zeros((B, 0, W)), ones_c, zeros_c, ones_t, zeros_t,
                           np.zeros((B, 0, W)))
    if scheme == "group":
        assert W % group == 0
        Xg = X.reshape(B, n, W // group, group)
        lo, hi = Xg.min(axis=3), Xg.max(axis=3)                          # [B, n, W / group]
        s, z = quant_params(lo, hi, bits)
        codes, pre = quantize(Xg, lo[..., None], hi[..., None], bits)
        return QuantSubset(scheme, bits, idx, codes.reshape(B, n, W), ones_c, zeros_c, ones_t, zeros_t,
                           pre.reshape(B, n, W), s, z)
    if scheme == "channel":
        lo, hi = X.min(axis=1), X.max(axis=1)                            # [B, W]
        s, z = quant_params(lo, hi, bits)
        codes, pre = quantize(X, lo[:, None, :], hi[:, None, :], bits)
        return QuantSubset(scheme, bits, idx, codes, s, z, ones_t, zeros_t, pre)
    if scheme == "cst":
        c = np.sqrt(np.abs(X).max(axis=1))                               # [B, W]
        c = np.where(c == 0.0, 1.0, c)
    elif scheme == "token":
        c = ones_c
    else:
        raise ValueError(scheme)
    Xn = X / c[:, None, :]
    lo, hi = Xn.min(axis=2), Xn.max(axis=2)                              # [B, n]
    s, z = quant_params(lo, hi, bits)
    codes, pre = quantize(Xn, lo[:, :, None], hi[:, :, None], bits)
    return QuantSubset(scheme, bits, idx, codes, c, zeros_c, s, z, pre)


def token_rows(X: np.ndarray) -> np.ndarray:
    """[B, H, L, d] -> [B, L, H*d] (the l x hd matrix of Algorithm 1)."""
    X = np.asarray(X, F64)
    B, H, L, d = X.shape
    return X.transpose(0, 2, 1, 3).reshape(B, L, H * d)


def head_rows(Xr: np.ndarray, H: int) -> np.ndarray:
    """Inverse of token_rows: [B, n, H*d] -> [B, H, n, d]."""
    B, n, W = Xr.shape
    return Xr.reshape(B, n, H, W // H).transpose(0, 2, 1, 3)


@dataclass
class QuantChunk:
    """Salient ("hi") and regular ("lo") subsets of one tensor for one
    compression call (Algorithm 2, the four quantizer calls)."""
    hi: QuantSubset
    lo: QuantSubset


def compress_tensor(X: np.ndarray, salient: np.ndarray, regular: np.ndarray,
                    bits_hi: int, bits_lo: int, scheme: str, pos_offset: int = 0) -> QuantChunk:
    """Split X [B, H, L, d] by the per-batch index lists and quantize each
    subset on its own (its own channel parameters), salient at bits_hi and
    regular at bits_lo."""
    R = token_rows(X)
    B = R.shape[0]
    salient = np.asarray(salient, np.int64).reshape(B, -1)
    regular = np.asarray(regular, np.int64).reshape(B, -1)
    hi_rows = np.stack([R[b, salient[b]] for b in range(B)])
    lo_rows = np.stack([R[b, regular[b]] for b in range(B)])
    return QuantChunk(quantize_rows(hi_rows, bits_hi, scheme, salient + pos_offset),
                      quantize_rows(lo_rows, bits_lo, scheme, regular + pos_offset))


def compress_prefill(K: np.ndarray, V: np.ndarray, scores: np.ndarray, k: int,
                     bits_hi: int = 4, bits_lo: int = 2,
                     k_scheme: str = "channel", v_scheme: str = "cst"):
    """Algorithm 2, compression part: per batch element pick the k salient
    tokens from `scores` [B, L], then quantize K and V subsets."""
    B = scores.shape[0]
    sal, reg = zip(*(select_salient(scores[b], k) for b in range(B)))
    sal = np.stack(sal)
    reg = np.stack(reg)
    return (compress_tensor(K, sal, reg, bits_hi, bits_lo, k_scheme),
            compress_tensor(V, sal, reg, bits_hi, bits_lo, v_scheme), sal, reg)


# --------------------------------------------------------------------------
# Decode attention over the de-quantized cache (Eq. 4, Algorithm 3)
# --------------------------------------------------------------------------

def decode_attention(q: np.ndarray, Kc: np.ndarray, Vc: np.ndarray,
                     sm_scale: Optional[float] = None):
    """Eq. 4 for every (batch, query head): q [B, Hq, d]; Kc, Vc [B, Hkv, N, d]
    already de-quantized / concatenated.  Returns (out [B, Hq, d],
    lse [B, Hq] natural log, probs [B, Hq, N])."""
    q = np.asarray(q, F64)
    Kc = np.asarray(Kc, F64)
    Vc = np.asarray(Vc, F64)
    B, Hq, d = q.shape
    Hkv = Kc.shape[1]
    G = Hq // Hkv
    N = Kc.shape[2]
    out = np.zeros((B, Hq, d), F64)
    lse = np.zeros((B, Hq), F64)
    probs = np.zeros((B, Hq, N), F64)
    sc = _scale(d, sm_scale)
    for b in range(B):
        for h in range(Hq):
            s = (Kc[b, h // G] @ q[b, h]) * sc
            m = s.max()
            e = np.exp(s - m)
            Z = e.sum()
            a = e / Z
            probs[b, h] = a
            lse[b, h] = m + np.log(Z)
            out[b, h] = a @ Vc[b, h // G]
    return out, lse, probs


def cache_matrices(chunks_K: List[QuantChunk], chunks_V: List[QuantChunk], Hkv: int,
                   tail_k: Optional[np.ndarray] = None, tail_v: Optional[np.ndarray] = None):
    """De-quantize every chunk (salient subset, then regular subset, chunk by
    chunk) and append the full-precision tail [B, Hkv, T, d]."""
    ks, vs = [], []
    for ck, cv in zip(chunks_K, chunks_V):
        for sk, sv in ((ck.hi, cv.hi), (ck.lo, cv.lo)):
            ks.append(head_rows(sk.dequant(), Hkv))
            vs.append(head_rows(sv.dequant(), Hkv))
    if tail_k is not None and tail_k.shape[2] > 0:
        ks.append(np.asarray(tail_k, F64))
        vs.append(np.asarray(tail_v, F64))
    return np.concatenate(ks, axis=2), np.concatenate(vs, axis=2)


@dataclass
class StreamingCache:
    """Algorithm 3 under the chunk-local reading: new tokens are appended in
    full precision; once `interval` of them have accumulated they are scored
    with that window's probe rows, split and quantized as a new chunk; older
    chunks are never re-quantized."""
    Hkv: int
    bits_hi: int = 4
    bits_lo: int = 2
    k_scheme: str = "channel"
    v_scheme: str = "cst"
    interval: int = 100
    chunks_K: List[QuantChunk] = field(default_factory=list)
    chunks_V: List[QuantChunk] = field(default_factory=list)
    tail_k: List[np.ndarray] = field(default_factory=list)   # each [B, Hkv, d]
    tail_v: List[np.ndarray] = field(default_factory=list)
    probe_q: List[np.ndarray] = field(default_factory=list)  # [B, Hq, d] of probe steps
    probe_lse: List[np.ndarray] = field(default_factory=list)
    probe_pos: List[int] = field(default_factory=list)       # window offsets of probe steps
    n_packed: int = 0

    def _tail(self):
        if not self.tail_k:
            return None, None
        return np.stack(self.tail_k, axis=2), np.stack(self.tail_v, axis=2)

    def step(self, q, k_new, v_new, is_probe: bool, sm_scale=None):
        """One decode step: append k, v in full precision, attend over the
        whole cache, remember the step if it is a probe."""
        self.tail_k.append(np.asarray(k_new, F64))
        self.tail_v.append(np.asarray(v_new, F64))
        tk, tv = self._tail()
        Kc, Vc = cache_matrices(self.chunks_K, self.chunks_V, self.Hkv, tk, tv)
        out, lse, probs = decode_attention(q, Kc, Vc, sm_scale)
        if is_probe:
            self.probe_q.append(np.asarray(q, F64))
            self.probe_lse.append(lse)
            self.probe_pos.append(len(self.tail_k) - 1)
        return out, lse, probs

    def tail_scores(self, sm_scale=None):
        """Normalized score of each tail token from the window's probe steps:
        a probe taken at window offset j saw tail columns t <= j, with the
        log-normaliser of its own decode step."""
        tk, _ = self._tail()
        Qp = np.stack(self.probe_q, axis=2)                    # [B, Hq, P, d]
        lse = np.stack(self.probe_lse, axis=2)                 # [B, Hq, P]
        pos = np.asarray(self.probe_pos, np.int64)
        return saliency_scores(Qp, tk, pos, probe_rows=np.arange(len(pos)),
                               sm_scale=sm_scale, lse_ext=lse)[0]

    def flush(self, k: int, sm_scale=None):
        """Compress the tail as a new chunk with k salient tokens."""
        scores = self.tail_scores(sm_scale)
        tk, tv = self._tail()
        ck, cv, sal, reg = compress_prefill(tk, tv, scores, k, self.bits_hi, self.bits_lo,
                                            self.k_scheme, self.v_scheme)
        for c in (ck, cv):
            c.hi.idx = c.hi.idx + self.n_packed
            c.lo.idx = c.lo.idx + self.n_packed
        self.chunks_K.append(ck)
        self.chunks_V.append(cv)
        self.n_packed += tk.shape[2]
        self.tail_k, self.tail_v = [], []
        self.probe_q, self.probe_lse, self.probe_pos = [], [], []
        return scores, sal, reg


# --------------------------------------------------------------------------
# Algorithm 3 read literally: explicit attention rows of the probe steps,
# re-compression of everything but the newest `interval` tokens
# --------------------------------------------------------------------------

def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """x rounded to the nearest value of a storage type ("fp32", "fp16", "bf16";
    ties to even), returned as float64."""
    x = np.asarray(x, F64)
    if dtype == "fp32":
        return x.astype(np.float32).astype(F64)
    if dtype == "fp16":
        return x.astype(np.float16).astype(F64)
    if dtype == "bf16":
        # 8 significant bits: x = m 2^e with 1/2 <= |m| < 1, so m 2^8 is rounded to an integer
        # (numpy.rint: ties to even) directly on the float64 value - no detour through fp32,
        # which would round twice.  (Values below bf16's normal range, 2^-126, do not occur.)
        m, e = np.frexp(x)
        return np.ldexp(np.rint(m * 256.0) / 256.0, e)
    raise ValueError(dtype)


def cache_positions(chunks: List[QuantChunk], n_tail: int, tail_pos0: int) -> np.ndarray:
    """[B, N] original token position of every column of `cache_matrices`
    (chunk by chunk: salient subset, regular subset; then the tail)."""
    cols = []
    for ck in chunks:
        cols += [ck.hi.idx, ck.lo.idx]
    B = cols[0].shape[0] if cols else 1
    cols.append(np.tile(np.arange(tail_pos0, tail_pos0 + n_tail), (B, 1)))
    return np.concatenate(cols, axis=1).astype(np.int64)


def rows_saliency(rows: Sequence[np.ndarray], normalized: bool = True) -> np.ndarray:
    """Eq. 8 on explicit attention rows: rows[j] is [B, Hq, n_j], the probabilities of
    probe j over the n_j tokens it could see (token order), n_j non-decreasing.
    score[b, i] = mean over heads of (sum of rows that see token i) / (their number);
    a token no row sees scores 0.  Returns [B, n_max]."""
    n = max(r.shape[2] for r in rows)
    B, Hq = rows[0].shape[:2]
    tot = np.zeros((B, Hq, n), F64)
    cnt = np.zeros(n, F64)
    for r in rows:
        tot[:, :, :r.shape[2]] += np.asarray(r, F64)
        cnt[:r.shape[2]] += 1.0
    if normalized:
        tot = np.where(cnt > 0, tot / np.maximum(cnt, 1.0), 0.0)
    return tot.mean(axis=1)


@dataclass
class LiteralStreamingCache:
    """Algorithm 3 taken at its word.  Every decode step appends k, v in full precision and
    attends over the whole cache; a probe step also keeps its attention row a (Eq. 4's
    probabilities, in token order).  After every `interval` steps, everything except the
    newest `interval` tokens - "K[:-100]": the tokens compressed earlier, as they now are
    (de-quantized, rounded to the cache's storage type), and the full-precision tokens
    older than the window - is compressed again as one whole by Algorithm 2's
    compression part: normalized scores (Eq. 8) from this window's probe rows, Split at
    r %, ChannelQuant / CSTQuant per subset.  A token can so move between the salient
    and the regular subset, and every re-compression quantizes de-quantized values.
    The probe rows are dropped after each re-compression."""
    Hkv: int
    store_dtype: str = "fp32"
    bits_hi: int = 4
    bits_lo: int = 2
    k_scheme: str = "channel"
    v_scheme: str = "cst"
    interval: int = 100
    chunk_K: Optional[QuantChunk] = None        # the compressed part: one chunk, positions 0 .. n_packed-1
    chunk_V: Optional[QuantChunk] = None
    n_packed: int = 0
    fp_k: List[np.ndarray] = field(default_factory=list)    # full-precision tokens, positions n_packed ..
    fp_v: List[np.ndarray] = field(default_factory=list)
    rows: List[np.ndarray] = field(default_factory=list)    # probe rows [B, Hq, n_j], token order

    def _matrices(self):
        tk = np.stack(self.fp_k, axis=2) if self.fp_k else None
        tv = np.stack(self.fp_v, axis=2) if self.fp_v else None
        ck = [self.chunk_K] if self.chunk_K is not None else []
        cv = [self.chunk_V] if self.chunk_V is not None else []
        Kc, Vc = cache_matrices(ck, cv, self.Hkv, tk, tv)
        pos = cache_positions(ck, len(self.fp_k), self.n_packed)
        return Kc, Vc, pos

    def step(self, q, k_new, v_new, is_probe: bool, sm_scale=None):
        self.fp_k.append(np.asarray(k_new, F64))
        self.fp_v.append(np.asarray(v_new, F64))
        Kc, Vc, pos = self._matrices()
        out, lse, probs = decode_attention(q, Kc, Vc, sm_scale)
        row = np.zeros_like(probs)
        for b in range(probs.shape[0]):
            row[b][:, pos[b]] = probs[b]                      # token order
        if is_probe:
            self.rows.append(row)
        return out, lse, row

    def token_matrices(self):
        """The cache in token order as it would be compressed again: [B, Hkv, n, d] of
        de-quantized (and storage-rounded) packed tokens followed by the full-precision ones."""
        Kc, Vc, pos = self._matrices()
        B = Kc.shape[0]
        Kt, Vt = np.zeros_like(Kc), np.zeros_like(Vc)
        npk = self.n_packed
        for b in range(B):
            Kt[b][:, pos[b]] = Kc[b]
            Vt[b][:, pos[b]] = Vc[b]
        Kt[:, :, :npk] = round_to_dtype(Kt[:, :, :npk], self.store_dtype)
        Vt[:, :, :npk] = round_to_dtype(Vt[:, :, :npk], self.store_dtype)
        return Kt, Vt

    def recompress(self, salient_ratio: float):
        """The `i == 100` branch.  Returns (scores [B, m], salient, regular) over the
        m = n - interval tokens that were compressed."""
        Kt, Vt = self.token_matrices()
        n = Kt.shape[2]
        m = n - self.interval
        scores = rows_saliency(self.rows)[:, :m]
        k = int(np.floor(salient_ratio * m + 1e-9))
        ck, cv, sal, reg = compress_prefill(Kt[:, :, :m], Vt[:, :, :m], scores, k, self.bits_hi, self.bits_lo,
                                            self.k_scheme, self.v_scheme)
        self.chunk_K, self.chunk_V, self.n_packed = ck, cv, m
        self.fp_k, self.fp_v = self.fp_k[-self.interval:], self.fp_v[-self.interval:]
        self.rows = []
        return scores, sal, reg


# --------------------------------------------------------------------------
# Compression-ratio accounting (Appendix A, Table 1)
# --------------------------------------------------------------------------

def quant_param_count(granularity: str, b: int, hd: int, l: int, n: int = 32) -> float:
    """Number of quantization parameters for keys plus values (Table 1's
    "Quantization Parameters" column)."""
    if granularity == "groupwise":          # K and V groupwise: 2 * 2bhld/n
        return 4.0 * b * hd * l / n
    if granularity == "tokenwise":          # K and V tokenwise: 2 * 2bl
        return 4.0 * b * l
    if granularity == "channel+token":      # K channelwise (2hd), V tokenwise (2bl)
        return 2.0 * hd + 2.0 * b * l
    if granularity == "channel+cst":        # K channelwise (2hd), V CST (hd + 2bl)
        return 3.0 * hd + 2.0 * b * l
    raise ValueError(granularity)


def compression_ratio(granularity: str, b: int, hd: int, l: int, bits_hi: float = 4,
                      bits_lo: Optional[float] = None, salient_ratio: float = 1.0,
                      n: int = 32, param_bits: int = 16, subsets: int = 1) -> float:
    """Appendix A: 16-bit K and V over quantized codes plus parameters.
    With two bit-widths the code term uses the token-weighted mean width;
    `subsets` multiplies the per-channel parameter count (one set per subset)."""
    bits = bits_hi if bits_lo is None else salient_ratio * bits_hi + (1.0 - salient_ratio) * bits_lo
    elems = 2.0 * b * hd * l
    params = quant_param_count(granularity, b, hd, l, n)
    if subsets != 1 and granularity in ("channel+token", "channel+cst"):
        chan = params - 2.0 * b * l
        params = subsets * chan + 2.0 * b * l
    return elems * 16.0 / (elems * bits + params * param_bits)
