"""CPU-only checks of the C-ABI library: it loads, exports every function the
header declares, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2405_14256_amd import binding as zb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "zipcache.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(zc_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = zb.load()
    names = declared_functions()
    assert {"zc_probe_saliency", "zc_select_salient", "zc_quantize_pack", "zc_decode_attention", "zc_unpack",
            "zc_probe_accumulated"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in zipcache.h but not exported"
    assert lib.zc_version() >= 1
    assert lib.zc_status_string(0) == b"ok"
    assert b"workspace" in lib.zc_status_string(-3)


def test_traced_library_exports_both_headers():
    """libzipcache_trace.so (bench.py --decode-timeline) is the library with time stamps in the
    bf16 decode kernels: everything zipcache.h declares, plus zc_trace.h."""
    src = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "zc_trace.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(zc_trace_[a-z_]+)\s*\(", src)))
    assert names == ["zc_trace_fetch"]
    lib = C.CDLL(os.path.join(ROOT, "paper_2405_14256_amd", "libzipcache_trace.so"))
    for n in names + declared_functions():
        assert hasattr(lib, n), f"{n} is not exported by the traced library"
    assert not hasattr(zb.load(), "zc_trace_fetch")          # the library proper records nothing
    lib.zc_trace_fetch.argtypes = [C.c_void_p, C.c_size_t, C.c_int]
    slots = 16 * 8192 + 4 * 2048
    assert re.search(r"#define ZC_TRACE_SLOTS 16\b", src) and re.search(r"#define ZC_TRACE_WAVES 8192\b", src) \
        and re.search(r"#define ZC_TRACE_HEADS 2048\b", src)
    assert lib.zc_trace_fetch(None, slots + 1, 0) == -1      # refused on the host: larger than the buffer
    assert lib.zc_trace_fetch(None, 8, 0) == -1              # ... no destination


def test_peak_probe_library_exports_its_header_and_checks_arguments():
    """The machine-peak probes of bench.py --peaks live in a library of their own."""
    src = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "zc_peaks.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(zc_peak_[a-z_]+)\s*\(", src)))
    assert names == ["zc_peak_chase", "zc_peak_copy", "zc_peak_empty", "zc_peak_mfma", "zc_peak_read", "zc_peak_touch"]
    lib = C.CDLL(os.path.join(ROOT, "paper_2405_14256_amd", "libzc_peaks.so"))
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in zc_peaks.h but not exported"
    lib.zc_peak_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.zc_peak_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.zc_peak_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    # host-side refusals (nothing is launched): null, misaligned, overlapping, bad type
    assert lib.zc_peak_read(None, 16, 0x1000, None) == -1
    assert lib.zc_peak_read(0x1008, 16, 0x1000, None) == -1
    assert lib.zc_peak_read(0x1000, 24, 0x1000, None) == -1
    assert lib.zc_peak_copy(0x1000, 0x1010, 32, None) == -1
    assert lib.zc_peak_copy(0x1000, None, 32, None) == -1
    assert lib.zc_peak_mfma(0, 1, 1, 0x1000, None) == -1
    assert lib.zc_peak_mfma(2, 0, 1, 0x1000, None) == -1
    assert lib.zc_peak_mfma(2, 1, 1, None, None) == -1
    lib.zc_peak_empty.argtypes = [C.c_int, C.c_void_p]
    lib.zc_peak_touch.argtypes = [C.c_void_p, C.c_size_t, C.c_size_t, C.c_int, C.c_uint32, C.c_void_p, C.c_void_p]
    lib.zc_peak_chase.argtypes = [C.c_void_p, C.c_size_t, C.c_uint32, C.c_int, C.c_void_p, C.c_void_p]
    assert lib.zc_peak_empty(0, None) == -1
    assert lib.zc_peak_touch(None, 64, 16, 1, 0, 0x1000, None) == -1
    assert lib.zc_peak_touch(0x1000, 24, 16, 1, 0, 0x2000, None) == -1
    assert lib.zc_peak_touch(0x1000, 64, 16, 0, 0, 0x2000, None) == -1
    assert lib.zc_peak_chase(0x1000, 16, 16, 1, 0x2000, None) == -1          # start outside the table
    assert lib.zc_peak_chase(0x1000, 16, 0, -1, 0x2000, None) == -1


def test_struct_sizes_match_header_layout():
    # 8-byte alignment, no hidden padding surprises
    assert C.sizeof(zb.zc_tensor4) == 8 + 4 + 4 + 7 * 8
    assert C.sizeof(zb.zc_packed) == 4 * 4 + 7 * 8 + 12 * 8 + 2 * 4


def test_sizes_and_workspaces():
    lib = zb.load()
    assert lib.zc_arena_bytes(1, 8, 128, 1664, 4) == 8 * 128 * 1664 // 2
    assert lib.zc_arena_bytes(2, 8, 128, 64, 2) == 2 * 8 * 128 * 64 // 4
    assert lib.zc_arena_slots(1638, 1) % zb.ZC_SLOT_ALIGN == 0 and lib.zc_arena_slots(1638, 1) >= 1638
    assert lib.zc_arena_slots(100, 2) >= 128
    assert lib.zc_quantize_pack_workspace(1, 8, 4096, 128) >= 2 * 1024 * 16 + (4096 // 16) * 1024 * 8
    assert lib.zc_probe_saliency_workspace(1, 32, 4096, 410) >= 4 * (32 * 410 + 32 * 4096)
    assert lib.zc_decode_attention_workspace(1, 32, 128) >= 32 * 130 * 4
    assert lib.zc_select_salient_workspace(1, 4096) == 0


def _t4(ptr=0x1000, dtype=zb.ZC_BF16, B=1, H=8, L=64, D=128):
    return zb.zc_tensor4(ptr, dtype, 0, B, H, L, D, H * L * D, L * D, D)


def test_select_rejects_bad_arguments_before_launch():
    lib = zb.load()
    assert lib.zc_select_salient(None, 1, 16, 4, 0x1000, 0x2000, None, None, 0, None) == -1
    assert lib.zc_select_salient(0x1000, 1, 16, 17, 0x1000, 0x2000, None, None, 0, None) == -1   # k > L
    assert lib.zc_select_salient(0x1000, 1, 16, -1, 0x1000, 0x2000, None, None, 0, None) == -1
    assert lib.zc_select_salient(0x1001, 1, 16, 4, 0x1000, 0x2000, None, None, 0, None) == -1   # misaligned
    assert lib.zc_select_salient(0x1000, 0, 16, 4, 0x1000, 0x2000, None, None, 0, None) == 0    # empty batch: no-op


def test_probe_rejects_bad_arguments_before_launch():
    lib = zb.load()
    q, k = _t4(H=32), _t4(H=8)
    ws = 1 << 24
    call = lambda q_, k_, pos=0x3000, P=4, sc=0x4000, w=0x5000, wsz=ws: lib.zc_probe_saliency(
        C.byref(q_), C.byref(k_), None, pos, P, 0.0, None, sc, None, w, wsz, None)
    assert call(q, k, P=0) == -1
    assert call(q, k, pos=None) == -1
    assert call(q, k, sc=None) == -1
    assert call(q, k, w=None) == -3
    assert call(q, k, wsz=16) == -3
    assert call(_t4(H=32, dtype=zb.ZC_F16), k) == -1            # dtype mismatch
    assert call(_t4(H=32, D=96), _t4(H=8, D=96)) == -2           # head dim not built
    assert call(_t4(H=30), k) == -1                              # Hq not a multiple of Hkv
    assert call(_t4(H=32, ptr=0x1004), k) == -1                  # misaligned
    bad = _t4(H=32); bad.sL = 100
    assert call(bad, k) == -1                                    # stride not a multiple of 8 / < D
    # one (batch, head) slab of q or k beyond what a 32-bit byte offset reaches: refused, not wrapped
    huge = 1 << 24                                               # 16 M tokens x 128 x 2 bytes = 4 GiB per slab
    big_ws = lib.zc_probe_saliency_workspace(1, 32, huge, 4)
    assert call(_t4(H=32, L=huge), _t4(H=8, L=huge), wsz=big_ws) == -2
    assert lib.zc_probe_accumulated(C.byref(q), C.byref(k), None, None, 4, 0.0, None, 0x4000, None, 0x5000, ws, None) == -1


def _packed(layout, scheme=zb.ZC_SCHEME_CST, cap=128, n_chunks=0, max_chunks=2, table=None):
    table = table if table is not None else np.zeros((max_chunks, 4), np.int32)
    return zb.zc_packed(layout, scheme, 4, 2, 1, 8, 128, cap, cap, 0, 0, 0x10000, 0x20000,
                        0x30000, 0x40000, 0x50000, 0x60000, None, None, 0x70000, 0x80000, 0x90000,
                        table.ctypes.data, n_chunks, max_chunks), table


def test_quantize_rejects_bad_arguments_before_launch():
    lib = zb.load()
    x = _t4()
    ws = 1 << 20
    call = lambda p, k=16, n=48, sal=0x1000, reg=0x2000, w=0xA0000, wsz=ws, x_=x: lib.zc_quantize_pack(
        C.byref(x_), sal, k, reg, n, 0, C.byref(p), w, wsz, None)
    p, _t = _packed(zb.ZC_LAYOUT_TGROUP)
    assert call(p, k=40, n=40) == -1                 # k + n_reg > L
    assert call(p, sal=None) == -1
    assert call(p, w=None) == -3
    assert call(p, wsz=64) == -3
    p2, _t2 = _packed(zb.ZC_LAYOUT_TGROUP, cap=64)
    p2.n_hi = 64
    assert call(p2) == -4                            # hi arena full
    p3, _t3 = _packed(zb.ZC_LAYOUT_TGROUP, n_chunks=2)
    assert call(p3) == -4                            # chunk table full
    p4, _t4_ = _packed(zb.ZC_LAYOUT_TGROUP, cap=100)
    assert call(p4) == -1                            # capacity not a multiple of the slot alignment
    p5, _t5 = _packed(7)
    assert call(p5) == -2                            # unknown layout
    p6, _t6 = _packed(zb.ZC_LAYOUT_ROW); p6.bits_lo = 3
    assert call(p6) == -2
    p7, _t7 = _packed(zb.ZC_LAYOUT_ROW); p7.tok_scale_hi = None
    assert call(p7) == -1                            # tokenwise scheme needs token parameter arrays
    assert call(p, x_=_t4(H=4)) == -1                # shape mismatch with the cache
    # a failed call leaves the host bookkeeping untouched
    assert p.n_chunks == 0 and p.n_hi == 0 and p.n_lo == 0


def test_decode_rejects_bad_arguments_before_launch():
    lib = zb.load()
    q = _t4(H=32, L=1)
    Kp, tk = _packed(zb.ZC_LAYOUT_ROW, scheme=zb.ZC_SCHEME_CHANNEL)
    Vp, tv = _packed(zb.ZC_LAYOUT_TGROUP)
    ws = 1 << 22
    call = lambda q_=q, K=Kp, V=Vp, tail=0, out=0xB0000, w=0xC0000, wsz=ws: lib.zc_decode_attention(
        C.byref(q_), C.byref(K), C.byref(V), None, None, tail, 0.0, out, None, w, wsz, None)
    assert call(q_=_t4(H=32, L=2)) == -1             # not a single query
    assert call(K=Vp) == -1                          # keys must use the ROW layout
    assert call(V=Kp) == -1
    assert call(out=None) == -1
    assert call(w=None) == -3
    assert call(tail=5) == -1                        # tail length without tail tensors
    assert call(q_=_t4(H=36, L=1)) == -2             # Hq not a multiple of Hkv
    Vq, _ = _packed(zb.ZC_LAYOUT_TGROUP); Vq.bits_hi = 8
    assert call(V=Vq) == -1                          # K and V caches disagree
    # chunk tables that disagree
    ta = np.array([[0, 10, 0, 20], [0, 0, 0, 0]], np.int32)
    tb = np.array([[0, 10, 0, 21], [0, 0, 0, 0]], np.int32)
    Ka, _ = _packed(zb.ZC_LAYOUT_ROW, scheme=zb.ZC_SCHEME_CHANNEL, n_chunks=1, table=ta)
    Vb, _ = _packed(zb.ZC_LAYOUT_TGROUP, n_chunks=1, table=tb)
    Ka.n_hi = Ka.n_lo = Vb.n_hi = Vb.n_lo = 64
    assert call(K=Ka, V=Vb) == -1


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(zb, "_lib", None)
    monkeypatch.setattr(zb, "LIB_PATH", "/nonexistent/libzipcache.so")
    with pytest.raises(ImportError):
        zb.load()


def test_static_scratch_entry_point_refuses_oversize_problems_on_the_host():
    """zc_decode_attention_static: a problem whose split-K partials exceed the library's
    static buffer is refused before anything touches the GPU (so this runs without one)."""
    lib = zb.load()
    B, Hq, Hkv, D = 64, 32, 8, 128
    assert lib.zc_decode_attention_workspace(B, Hq, D) > (8 << 20)
    host = np.zeros((1, 4), np.int32)
    def packed(layout, scheme):
        return zb.zc_packed(layout, scheme, 4, 2, B, Hkv, D, 64, 64, 0, 0, 0x10000, 0x20000, 0x30000, 0x40000, 0x50000,
                            0x60000, None, None, 0x70000, 0x80000, 0x90000, host.ctypes.data, 0, 1)
    q = zb.zc_tensor4(0x1000, zb.ZC_BF16, 0, B, Hq, 1, D, Hq * D, D, D)
    kp, vp = packed(zb.ZC_LAYOUT_ROW, zb.ZC_SCHEME_CHANNEL), packed(zb.ZC_LAYOUT_TGROUP, zb.ZC_SCHEME_CST)
    rc = lib.zc_decode_attention_static(C.byref(q), C.byref(kp), C.byref(vp), None, None, 0, 0.0, 0x2000, None, None)
    assert rc == -6 and b"static" in lib.zc_status_string(rc)
