"""zc_decode_attention_static (the decode entry point for callers that cannot
allocate: its split-K partials live in a buffer inside the library's device
image) against zc_decode_attention, through the C ABI, on two calls in a row,
the second on a smaller input - the shared buffer keeps the first call's
contents, and nothing of them may show in the second result."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import zipcache_oracle as zo
from paper_2405_14256_amd import binding as zb

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _cache(B, Hq, Hkv, d, L, k, T, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    K = torch.randn(B, Hkv, L + T, d, generator=g).to(dtype)
    V = torch.randn(B, Hkv, L + T, d, generator=g).to(dtype)
    q = torch.randn(B, Hq, 1, d, generator=g).to(dtype)
    lib = zb.load()
    sal, reg = zb.zc_select_salient(torch.rand(B, L, generator=g).to(DEV), k)
    cap_hi, cap_lo = lib.zc_arena_slots(k, 1), lib.zc_arena_slots(L - k, 1)
    Kp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, 4, 2, "channel", zb.ZC_LAYOUT_ROW, max_chunks=1, device=DEV)
    Vp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=1, device=DEV)
    Kd, Vd = K.to(DEV), V.to(DEV)
    zb.zc_quantize_pack(Kd[:, :, :L], sal, reg, Kp)
    zb.zc_quantize_pack(Vd[:, :, :L], sal, reg, Vp)
    return q.to(DEV), Kp, Vp, Kd[:, :, L:], Vd[:, :, L:], (K, V, q)


def _call_both(q, Kp, Vp, tk, tv, T):
    """(out, lse) of the workspace entry point and of the static one, both through the C ABI."""
    lib = zb.load()
    B, Hq, _, d = q.shape
    st = torch.cuda.current_stream().cuda_stream
    tq, ttk, ttv = zb.tensor4(q), zb.tensor4(tk), zb.tensor4(tv)
    res = []
    for static in (False, True):
        out = torch.full((B, Hq, d), float("nan"), dtype=q.dtype, device=DEV)
        lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
        args = [C.byref(tq), C.byref(Kp.c), C.byref(Vp.c), C.byref(ttk), C.byref(ttv), T, 0.0, out.data_ptr(), lse.data_ptr()]
        if static:
            rc = lib.zc_decode_attention_static(*args, st)
        else:
            need = lib.zc_decode_attention_workspace(B, Hq, d)
            ws = torch.empty(need, dtype=torch.uint8, device=DEV)
            rc = lib.zc_decode_attention(*args, ws.data_ptr(), need, st)
        assert rc == 0, (static, lib.zc_status_string(rc))
        torch.cuda.synchronize()
        res.append((out, lse))
    return res


def test_static_scratch_entry_point_matches_the_workspace_one():
    from tests.pipeline_check import packed_to_chunks
    # first a cache that is split over many workgroups per head (many partials in the buffer),
    # then a smaller one (fewer heads, fewer and shorter partials), then the first again
    big = _cache(2, 16, 4, 128, 3000, 1200, 50, torch.bfloat16, 1)
    small = _cache(1, 8, 8, 64, 500, 200, 7, torch.float32, 2)
    for name, (q, Kp, Vp, tk, tv, cpu), T in (("big", big, 50), ("small", small, 7), ("big again", big, 33)):
        (o_ws, l_ws), (o_st, l_st) = _call_both(q, Kp, Vp, tk, tv, T)
        assert torch.equal(o_ws, o_st) and torch.equal(l_ws, l_st), name       # same kernels, same split: bit for bit
        K, V, qc = cpu
        B, L = q.shape[0], K.shape[2] - tk.shape[2]
        bsel = list(range(B))
        Kc, Vc = zo.cache_matrices(packed_to_chunks(Kp, bsel), packed_to_chunks(Vp, bsel), Kp.H,
                                   K[:, :, L:L + T].double().numpy(), V[:, :, L:L + T].double().numpy())
        ref, lse_o, _ = zo.decode_attention(qc[:, :, 0].double().numpy(), Kc, Vc)
        atol = 1e-4 if q.dtype == torch.float32 else 2e-2
        assert np.abs(o_st.cpu().double().numpy() - ref).max() <= atol, name
        assert np.abs(l_st.cpu().numpy() - lse_o).max() <= max(atol, 1e-3), name


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    lib = zb.load()
    B, Hq, Hkv, d = 64, 32, 8, 128                    # 2048 query heads: 9 partials each of 130 floats > 8 MiB
    assert lib.zc_decode_attention_workspace(B, Hq, d) > (8 << 20)
    q = torch.zeros(B, Hq, 1, d, dtype=torch.bfloat16, device=DEV)
    Kp = zb.PackedTensor(B, Hkv, d, 64, 64, 4, 2, "channel", zb.ZC_LAYOUT_ROW, max_chunks=1, device=DEV)
    Vp = zb.PackedTensor(B, Hkv, d, 64, 64, 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=1, device=DEV)
    out = torch.zeros(B, Hq, d, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(zb.ZipCacheError) as e:
        zb.zc_decode_attention_static(q, Kp, Vp, out=out)
    assert e.value.status == -6 and "static" in str(e.value)
