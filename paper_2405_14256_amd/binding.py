"""ctypes binding of libzipcache.so: argument marshalling only.

Every function has the name of the C entry point it calls.  Tensors are torch
tensors on the GPU (torch supplies device memory and the current HIP stream);
no arithmetic of the method happens here.  If the library has not been built
the import of any entry point fails loudly - there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libzipcache.so")

ZC_OK = 0
ZC_F32, ZC_F16, ZC_BF16 = 0, 1, 2
ZC_SCHEME_CHANNEL, ZC_SCHEME_CST, ZC_SCHEME_TOKEN = 0, 1, 2
ZC_LAYOUT_ROW, ZC_LAYOUT_TGROUP = 0, 1
ZC_SLOT_ALIGN = 64

SCHEMES = {"channel": ZC_SCHEME_CHANNEL, "cst": ZC_SCHEME_CST, "token": ZC_SCHEME_TOKEN}
_DTYPE = {torch.float32: ZC_F32, torch.float16: ZC_F16, torch.bfloat16: ZC_BF16}


class zc_tensor4(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("B", C.c_int64), ("H", C.c_int64), ("L", C.c_int64), ("D", C.c_int64),
                ("sB", C.c_int64), ("sH", C.c_int64), ("sL", C.c_int64)]


class zc_packed(C.Structure):
    _fields_ = [("layout", C.c_int32), ("scheme", C.c_int32), ("bits_hi", C.c_int32), ("bits_lo", C.c_int32),
                ("B", C.c_int64), ("H", C.c_int64), ("D", C.c_int64),
                ("cap_hi", C.c_int64), ("cap_lo", C.c_int64), ("n_hi", C.c_int64), ("n_lo", C.c_int64),
                ("codes_hi", C.c_void_p), ("codes_lo", C.c_void_p),
                ("tok_scale_hi", C.c_void_p), ("tok_zero_hi", C.c_void_p),
                ("tok_scale_lo", C.c_void_p), ("tok_zero_lo", C.c_void_p),
                ("pos_hi", C.c_void_p), ("pos_lo", C.c_void_p),
                ("chan_scale", C.c_void_p), ("chan_zero", C.c_void_p),
                ("chunk_table", C.c_void_p), ("chunk_table_host", C.c_void_p),
                ("n_chunks", C.c_int32), ("max_chunks", C.c_int32)]


class ZipCacheError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        msg = load().zc_status_string(status).decode()
        super().__init__(f"{fn} failed with status {status}: {msg}")


_lib = None


def load() -> C.CDLL:
    """Loads the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` to build the HIP library")
    lib = C.CDLL(LIB_PATH)
    P, I32, I64, F, SZ = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    T4, PK = C.POINTER(zc_tensor4), C.POINTER(zc_packed)
    lib.zc_probe_saliency_workspace.restype = SZ
    lib.zc_probe_saliency_workspace.argtypes = [I64, I64, I64, I64]
    lib.zc_probe_saliency.restype = C.c_int
    lib.zc_probe_saliency.argtypes = [T4, T4, P, P, I32, F, P, P, P, P, SZ, P]
    lib.zc_probe_accumulated.restype = C.c_int
    lib.zc_probe_accumulated.argtypes = [T4, T4, P, P, I32, F, P, P, P, P, SZ, P]
    lib.zc_prefill_attention.restype = C.c_int
    lib.zc_prefill_attention.argtypes = [T4, T4, T4, F, T4, P, P, I32, P, P]
    lib.zc_select_salient_workspace.restype = SZ
    lib.zc_select_salient_workspace.argtypes = [I64, I64]
    lib.zc_select_salient.restype = C.c_int
    lib.zc_select_salient.argtypes = [P, I64, I64, I64, P, P, P, P, SZ, P]
    lib.zc_quantize_pack_workspace.restype = SZ
    lib.zc_quantize_pack_workspace.argtypes = [I64, I64, I64, I64]
    lib.zc_quantize_pack.restype = C.c_int
    lib.zc_quantize_pack.argtypes = [T4, P, I64, P, I64, I64, PK, P, SZ, P]
    lib.zc_quantize_pack_kv_workspace.restype = SZ
    lib.zc_quantize_pack_kv_workspace.argtypes = [I64, I64, I64, I64]
    lib.zc_quantize_pack_kv.restype = C.c_int
    lib.zc_quantize_pack_kv.argtypes = [T4, T4, P, I64, P, I64, I64, PK, PK, P, SZ, P]
    lib.zc_decode_attention_workspace.restype = SZ
    lib.zc_decode_attention_workspace.argtypes = [I64, I64, I64]
    lib.zc_decode_attention.restype = C.c_int
    lib.zc_decode_attention.argtypes = [T4, PK, PK, T4, T4, I64, F, P, P, P, SZ, P]
    lib.zc_decode_attention_static.restype = C.c_int
    lib.zc_decode_attention_static.argtypes = [T4, PK, PK, T4, T4, I64, F, P, P, P]
    lib.zc_decode_probs.restype = C.c_int
    lib.zc_decode_probs.argtypes = [T4, PK, T4, I64, I64, F, P, P, I64, P]
    lib.zc_rows_saliency.restype = C.c_int
    lib.zc_rows_saliency.argtypes = [P, P, I32, I64, I64, I64, I64, I32, P, P]
    lib.zc_dequantize_cache.restype = C.c_int
    lib.zc_dequantize_cache.argtypes = [PK, T4, P]
    lib.zc_group_quantize.restype = C.c_int
    lib.zc_group_quantize.argtypes = [T4, P, I64, I32, I32, P, P, P, P, P]
    lib.zc_unpack.restype = C.c_int
    lib.zc_unpack.argtypes = [PK, I32, I32, P, P, P]
    lib.zc_arena_bytes.restype = SZ
    lib.zc_arena_bytes.argtypes = [I64, I64, I64, I64, I32]
    lib.zc_arena_slots.restype = I64
    lib.zc_arena_slots.argtypes = [I64, I64]
    lib.zc_status_string.restype = C.c_char_p
    lib.zc_status_string.argtypes = [C.c_int]
    lib.zc_version.restype = C.c_int
    lib.zc_version.argtypes = []
    _lib = lib
    return lib


def _check(fn: str, status: int) -> None:
    if status != ZC_OK:
        raise ZipCacheError(fn, status)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def tensor4(t: torch.Tensor) -> zc_tensor4:
    """Describes a [B, H, L, D] torch tensor (any strides, unit stride on D)."""
    assert t.dim() == 4 and t.stride(3) == 1, "need a 4-D tensor with contiguous last axis"
    return zc_tensor4(t.data_ptr(), _DTYPE[t.dtype], 0, t.shape[0], t.shape[1], t.shape[2], t.shape[3],
                      t.stride(0), t.stride(1), t.stride(2))


_ws_cache = {}


def _workspace(nbytes: int, device, tag: str = "scratch") -> torch.Tensor:
    """A scratch tensor per device, operation and stream (calls issued on different
    streams may run concurrently, so they must not share scratch memory), grown
    on demand and reused across calls."""
    key = (str(device), tag, _stream())
    cur = _ws_cache.get(key)
    if cur is None or cur.numel() < nbytes:
        cur = torch.zeros(max(int(nbytes), 256), dtype=torch.uint8, device=device)
        _ws_cache[key] = cur
    return cur


class PackedTensor:
    """Caller-side owner of the arrays of one zc_packed (K or V of a cache)."""

    def __init__(self, B: int, H: int, D: int, cap_hi: int, cap_lo: int, bits_hi: int, bits_lo: int,
                 scheme: str, layout: int, max_chunks: int = 8, device="cuda", store_pos: bool = True):
        lib = load()
        self.B, self.H, self.D = B, H, D
        al = ZC_SLOT_ALIGN
        cap_hi = (cap_hi + al - 1) // al * al
        cap_lo = (cap_lo + al - 1) // al * al
        dev = torch.device(device)
        W = H * D
        self.codes_hi = torch.zeros(max(lib.zc_arena_bytes(B, H, D, cap_hi, bits_hi), 16), dtype=torch.uint8, device=dev)
        self.codes_lo = torch.zeros(max(lib.zc_arena_bytes(B, H, D, cap_lo, bits_lo), 16), dtype=torch.uint8, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        self.tok_scale_hi = torch.zeros(B, max(cap_hi, 1), **f32)
        self.tok_zero_hi = torch.zeros(B, max(cap_hi, 1), **f32)
        self.tok_scale_lo = torch.zeros(B, max(cap_lo, 1), **f32)
        self.tok_zero_lo = torch.zeros(B, max(cap_lo, 1), **f32)
        self.pos_hi = torch.full((B, max(cap_hi, 1)), -1, dtype=torch.int32, device=dev) if store_pos else None
        self.pos_lo = torch.full((B, max(cap_lo, 1)), -1, dtype=torch.int32, device=dev) if store_pos else None
        self.chan_scale = torch.zeros(max_chunks, 2, B, W, **f32)
        self.chan_zero = torch.zeros(max_chunks, 2, B, W, **f32)
        self.chunk_table = torch.zeros(max_chunks, 4, dtype=torch.int32, device=dev)
        self.chunk_table_host = np.zeros((max_chunks, 4), np.int32)
        self.c = zc_packed(layout, SCHEMES[scheme], bits_hi, bits_lo, B, H, D, cap_hi, cap_lo, 0, 0,
                           _ptr(self.codes_hi), _ptr(self.codes_lo),
                           _ptr(self.tok_scale_hi), _ptr(self.tok_zero_hi),
                           _ptr(self.tok_scale_lo), _ptr(self.tok_zero_lo),
                           _ptr(self.pos_hi), _ptr(self.pos_lo),
                           _ptr(self.chan_scale), _ptr(self.chan_zero),
                           _ptr(self.chunk_table), self.chunk_table_host.ctypes.data, 0, max_chunks)
        self.scheme, self.layout = scheme, layout

    def reset(self) -> None:
        """Forget all chunks (the arrays are reused)."""
        self.c.n_hi = self.c.n_lo = 0
        self.c.n_chunks = 0

    def clone(self) -> "PackedTensor":
        """A copy with arrays of its own (same contents, same chunks)."""
        o = PackedTensor(self.B, self.H, self.D, self.c.cap_hi, self.c.cap_lo, self.c.bits_hi, self.c.bits_lo,
                         self.scheme, self.layout, max_chunks=self.c.max_chunks, device=self.chan_scale.device,
                         store_pos=self.pos_hi is not None)
        for name in ("codes_hi", "codes_lo", "tok_scale_hi", "tok_zero_hi", "tok_scale_lo", "tok_zero_lo",
                     "pos_hi", "pos_lo", "chan_scale", "chan_zero", "chunk_table"):
            src = getattr(self, name)
            if src is not None:
                getattr(o, name).copy_(src)
        o.chunk_table_host[:] = self.chunk_table_host
        o.c.n_hi, o.c.n_lo, o.c.n_chunks = self.c.n_hi, self.c.n_lo, self.c.n_chunks
        return o

    @property
    def chunks(self):
        return [tuple(int(v) for v in self.chunk_table_host[i]) for i in range(self.c.n_chunks)]


def zc_probe_saliency(q: torch.Tensor, k: torch.Tensor, probe_pos: torch.Tensor,
                      probe_rows: Optional[torch.Tensor] = None, sm_scale: float = 0.0,
                      lse_ext: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                      scores_per_head: Optional[torch.Tensor] = None, _entry: str = "zc_probe_saliency") -> torch.Tensor:
    lib = load()
    B, Hq, _, _ = q.shape
    Lk = k.shape[2]
    P = int(probe_pos.numel())
    if scores is None:
        scores = torch.empty(B, Lk, dtype=torch.float32, device=q.device)
    need = lib.zc_probe_saliency_workspace(B, Hq, Lk, P)
    ws = _workspace(need, q.device)
    tq, tk = tensor4(q), tensor4(k)
    _check(_entry,
           getattr(lib, _entry)(C.byref(tq), C.byref(tk), _ptr(probe_rows), _ptr(probe_pos), P, float(sm_scale),
                                _ptr(lse_ext), _ptr(scores), _ptr(scores_per_head), ws.data_ptr(), ws.numel(),
                                _stream()))
    return scores


def zc_probe_accumulated(q: torch.Tensor, k: torch.Tensor, probe_pos: torch.Tensor, **kw) -> torch.Tensor:
    """Eq. 7: as zc_probe_saliency, without the division by the unmasked count."""
    return zc_probe_saliency(q, k, probe_pos, _entry="zc_probe_accumulated", **kw)


def zc_prefill_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, sm_scale: float = 0.0,
                         out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                         probe_pos: Optional[torch.Tensor] = None, lse_probe: Optional[torch.Tensor] = None):
    """(out [B, Hq, L, D], lse [B, Hq, L], lse_probe [B, Hq, P] or None)."""
    lib = load()
    B, Hq, L, _ = q.shape
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty(B, Hq, L, dtype=torch.float32, device=q.device)
    P = int(probe_pos.numel()) if probe_pos is not None else 0
    if P and lse_probe is None:
        lse_probe = torch.empty(B, Hq, P, dtype=torch.float32, device=q.device)
    tq, tk, tv, to = tensor4(q), tensor4(k), tensor4(v), tensor4(out)
    _check("zc_prefill_attention",
           lib.zc_prefill_attention(C.byref(tq), C.byref(tk), C.byref(tv), float(sm_scale), C.byref(to), _ptr(lse),
                                    _ptr(probe_pos) if P else None, P, _ptr(lse_probe) if P else None, _stream()))
    return out, lse, lse_probe


def zc_select_salient(scores: torch.Tensor, k: int, salient_idx: Optional[torch.Tensor] = None,
                      regular_idx: Optional[torch.Tensor] = None, mask: Optional[torch.Tensor] = None):
    lib = load()
    B, L = scores.shape
    dev = scores.device
    if salient_idx is None:
        salient_idx = torch.empty(B, max(k, 0), dtype=torch.int32, device=dev)
    if regular_idx is None:
        regular_idx = torch.empty(B, max(L - k, 0), dtype=torch.int32, device=dev)
    _check("zc_select_salient",
           lib.zc_select_salient(scores.data_ptr(), B, L, k, _ptr(salient_idx), _ptr(regular_idx), _ptr(mask),
                                 None, 0, _stream()))
    return salient_idx, regular_idx


def zc_quantize_pack(x: torch.Tensor, salient_idx: torch.Tensor, regular_idx: torch.Tensor,
                     out: PackedTensor, pos_offset: int = 0) -> None:
    lib = load()
    B, H, _, D = x.shape
    k = int(salient_idx.shape[1]) if salient_idx is not None else 0
    n_reg = int(regular_idx.shape[1]) if regular_idx is not None else 0
    need = lib.zc_quantize_pack_workspace(B, H, k + n_reg, D)
    ws = _workspace(need, x.device, "quantize")
    tx = tensor4(x)
    _check("zc_quantize_pack",
           lib.zc_quantize_pack(C.byref(tx), _ptr(salient_idx) if k else None, k,
                                _ptr(regular_idx) if n_reg else None, n_reg, pos_offset,
                                C.byref(out.c), ws.data_ptr(), ws.numel(), _stream()))


def zc_quantize_pack_kv(xk: torch.Tensor, xv: torch.Tensor, salient_idx: torch.Tensor, regular_idx: torch.Tensor,
                        outK: PackedTensor, outV: PackedTensor, pos_offset: int = 0) -> None:
    """Keys and values of one cache in the same launches (the four quantizer calls of Algorithm 2)."""
    lib = load()
    B, H, _, D = xk.shape
    k = int(salient_idx.shape[1]) if salient_idx is not None else 0
    n_reg = int(regular_idx.shape[1]) if regular_idx is not None else 0
    need = lib.zc_quantize_pack_kv_workspace(B, H, k + n_reg, D)
    ws = _workspace(need, xk.device, "quantize_kv")
    tk, tv = tensor4(xk), tensor4(xv)
    _check("zc_quantize_pack_kv",
           lib.zc_quantize_pack_kv(C.byref(tk), C.byref(tv), _ptr(salient_idx) if k else None, k,
                                   _ptr(regular_idx) if n_reg else None, n_reg, pos_offset,
                                   C.byref(outK.c), C.byref(outV.c), ws.data_ptr(), ws.numel(), _stream()))


def zc_unpack(p: PackedTensor, which: int, chunk: int, codes: bool = True, dequant: bool = True):
    """(codes uint8 [B, len, W] or None, x_hat float32 [B, len, W] or None) of subset
    `which` (0 hi, 1 lo) of chunk `chunk`, token-major in slot order."""
    lib = load()
    row = p.chunks[chunk]
    n = int(row[2 * which + 1])
    W = p.H * p.D
    dev = p.chan_scale.device
    co = torch.empty(p.B, n, W, dtype=torch.uint8, device=dev) if codes else None
    dq = torch.empty(p.B, n, W, dtype=torch.float32, device=dev) if dequant else None
    _check("zc_unpack", lib.zc_unpack(C.byref(p.c), which, chunk, _ptr(co) if n else None, _ptr(dq) if n else None, _stream()))
    return co, dq


def zc_decode_attention(q: torch.Tensor, Kp: PackedTensor, Vp: PackedTensor,
                        tail_k: Optional[torch.Tensor] = None, tail_v: Optional[torch.Tensor] = None,
                        tail_len: int = 0, sm_scale: float = 0.0, out: Optional[torch.Tensor] = None,
                        lse_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """q: [B, Hq, D] or [B, Hq, 1, D]."""
    lib = load()
    if q.dim() == 3:
        q = q.unsqueeze(2)
    B, Hq, _, D = q.shape
    if out is None:
        out = torch.empty(B, Hq, D, dtype=q.dtype, device=q.device)
    need = lib.zc_decode_attention_workspace(B, Hq, D)
    ws = _workspace(need, q.device, "decode")
    tq = tensor4(q)
    ttk = tensor4(tail_k) if tail_len else None
    ttv = tensor4(tail_v) if tail_len else None
    _check("zc_decode_attention",
           lib.zc_decode_attention(C.byref(tq), C.byref(Kp.c), C.byref(Vp.c),
                                   C.byref(ttk) if tail_len else None, C.byref(ttv) if tail_len else None,
                                   tail_len, float(sm_scale), out.data_ptr(), _ptr(lse_out),
                                   ws.data_ptr(), ws.numel(), _stream()))
    return out


def zc_decode_attention_static(q: torch.Tensor, Kp: PackedTensor, Vp: PackedTensor,
                               tail_k: Optional[torch.Tensor] = None, tail_v: Optional[torch.Tensor] = None,
                               tail_len: int = 0, sm_scale: float = 0.0, *, out: torch.Tensor,
                               lse_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """zc_decode_attention on the library's own scratch buffer: nothing is allocated, here
    or in the library (`out` must be given)."""
    lib = load()
    if q.dim() == 3:
        q = q.unsqueeze(2)
    tq = tensor4(q)
    ttk = tensor4(tail_k) if tail_len else None
    ttv = tensor4(tail_v) if tail_len else None
    _check("zc_decode_attention_static",
           lib.zc_decode_attention_static(C.byref(tq), C.byref(Kp.c), C.byref(Vp.c),
                                          C.byref(ttk) if tail_len else None, C.byref(ttv) if tail_len else None,
                                          tail_len, float(sm_scale), out.data_ptr(), _ptr(lse_out), _stream()))
    return out


def zc_decode_probs(q: torch.Tensor, Kp: PackedTensor, tail_k: Optional[torch.Tensor], tail_len: int, tail_pos0: int,
                    lse: torch.Tensor, probs_out: torch.Tensor, sm_scale: float = 0.0) -> torch.Tensor:
    """probs_out [B, Hq, N] (token order) of one decode step; lse from zc_decode_attention."""
    lib = load()
    if q.dim() == 3:
        q = q.unsqueeze(2)
    assert probs_out.dim() == 3 and probs_out.is_contiguous() and probs_out.dtype == torch.float32
    tq = tensor4(q)
    ttk = tensor4(tail_k) if tail_len else None
    _check("zc_decode_probs",
           lib.zc_decode_probs(C.byref(tq), C.byref(Kp.c), C.byref(ttk) if tail_len else None, tail_len, tail_pos0,
                               float(sm_scale), lse.data_ptr(), probs_out.data_ptr(), probs_out.shape[2], _stream()))
    return probs_out


def zc_rows_saliency(rows: torch.Tensor, row_len: torch.Tensor, n_out: int, normalize: bool = True,
                     scores: Optional[torch.Tensor] = None) -> torch.Tensor:
    """rows [P, B, Hq, N] float32, row_len int32 [P] -> scores [B, n_out]."""
    lib = load()
    P, B, Hq, N = rows.shape
    assert rows.is_contiguous() and rows.dtype == torch.float32 and row_len.dtype == torch.int32
    if scores is None:
        scores = torch.empty(B, n_out, dtype=torch.float32, device=rows.device)
    _check("zc_rows_saliency",
           lib.zc_rows_saliency(rows.data_ptr(), row_len.data_ptr(), P, B, Hq, N, n_out, int(normalize),
                                scores.data_ptr(), _stream()))
    return scores


def zc_dequantize_cache(p: PackedTensor, out: torch.Tensor) -> torch.Tensor:
    """Scatters x_hat of every token of `p` to out[b, h, position, :]."""
    lib = load()
    to = tensor4(out)
    _check("zc_dequantize_cache", lib.zc_dequantize_cache(C.byref(p.c), C.byref(to), _stream()))
    return out


def zc_group_quantize(x: torch.Tensor, bits: int, group: int = 32, idx: Optional[torch.Tensor] = None,
                      codes: bool = True, dequant: bool = True):
    """Groupwise quantization of the token rows `idx` [B, n] (default: all) of x [B, H, L, D]:
    (codes uint8 [B, n, W], scale [B, n, W/group], zero, x_hat float32 [B, n, W])."""
    lib = load()
    B, H, L, D = x.shape
    n = int(idx.shape[1]) if idx is not None else L
    W = H * D
    dev = x.device
    co = torch.empty(B, n, W, dtype=torch.uint8, device=dev) if codes else None
    sc = torch.empty(B, n, W // group, dtype=torch.float32, device=dev)
    ze = torch.empty(B, n, W // group, dtype=torch.float32, device=dev)
    dq = torch.empty(B, n, W, dtype=torch.float32, device=dev) if dequant else None
    tx = tensor4(x)
    _check("zc_group_quantize", lib.zc_group_quantize(C.byref(tx), _ptr(idx), n, bits, group, _ptr(co), _ptr(sc), _ptr(ze),
                                                      _ptr(dq), _stream()))
    return co, sc, ze, dq
