"""GPU parity of Algorithm 3's re-compression branch taken at its word (explicit probe rows,
re-ranking and re-compression of everything but the newest window) against the oracle's
LiteralStreamingCache: the attention rows zc_decode_probs emits, Eq. 8 on them
(zc_rows_saliency), the de-quantized token buffer (zc_dequantize_cache), the split and the
re-quantized cache, and every decode output, over two windows."""
import numpy as np
import pytest
import torch

from oracle import zipcache_oracle as zo
from paper_2405_14256_amd import binding as zb
from paper_2405_14256_amd import probes
from paper_2405_14256_amd.workloads import WORKLOADS, make_decode_step, make_prefill, scaled, to_f64
from tests.pipeline_check import CODE_COUNTS, assert_code_budgets, check_index_sets, compare_subset, packed_to_chunks

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run_literal(w, interval, windows, extra_steps=3):
    dev = torch.device(DEV)
    lib = zb.load()
    B, Hq, Hkv, d, L = w.B, w.Hq, w.Hkv, w.d, w.L
    bsel = list(range(B))
    steps = windows * interval + extra_steps
    Nmax = L + steps
    fp32 = w.dtype == "fp32"
    atol = 1e-4 if fp32 else 2e-2
    inp = make_prefill(w)
    Qg, Kg, Vg = (inp[n].to(dev) for n in ("Q", "K", "V"))
    pos_np = probes.probe_positions(L, w.probe_ratio, w.seed)
    scores0 = zb.zc_probe_saliency(Qg, Kg, torch.from_numpy(pos_np).to(dev))
    k0 = w.k_salient
    sal, reg = zb.zc_select_salient(scores0, k0)
    m_max = L + (windows - 1) * interval
    k_max = int(np.floor(w.salient_ratio * m_max + 1e-9))
    cap_hi, cap_lo = lib.zc_arena_slots(k_max, 1), lib.zc_arena_slots(m_max - min(k0, k_max), 1)
    def mk(scheme, layout):
        return zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, w.bits_hi, w.bits_lo, scheme, layout, max_chunks=1, device=DEV)
    caches = [(mk("channel", zb.ZC_LAYOUT_ROW), mk("cst", zb.ZC_LAYOUT_TGROUP)) for _ in range(2)]
    Kp, Vp = caches[0]
    zb.zc_quantize_pack(Kg, sal, reg, Kp)
    zb.zc_quantize_pack(Vg, sal, reg, Vp)
    torch.cuda.synchronize()
    # the token buffers: positions [0, n_packed) are filled by zc_dequantize_cache when a window
    # closes, [n_packed, n) are the full-precision tokens (the decode calls' tail)
    Xk = torch.zeros(B, Hkv, Nmax, d, dtype=w.torch_dtype, device=dev)
    Xv = torch.zeros_like(Xk)
    n_packed = L
    oracle = zo.LiteralStreamingCache(Hkv=Hkv, store_dtype=w.dtype, bits_hi=w.bits_hi, bits_lo=w.bits_lo, interval=interval,
                                      chunk_K=packed_to_chunks(Kp, bsel)[0], chunk_V=packed_to_chunks(Vp, bsel)[0], n_packed=L)
    probe_off = set(probes.decode_probe_offsets(interval, seed=w.seed).tolist())
    n_probe = len(probe_off)
    rows_g = torch.zeros(n_probe, B, Hq, Nmax, dtype=torch.float32, device=dev)
    row_len = []
    rep = {"out": 0.0, "lse": 0.0, "row": 0.0, "score": 0.0, "score_e2e": 0.0, "dequant_mismatch": 0.0}
    totals = {key: 0 for key in CODE_COUNTS}
    prev_sal = set(sal[0].cpu().tolist())
    changed = 0
    for j in range(steps):
        d_in = make_decode_step(w, j)
        n = L + j                                      # position of the new token
        Xk[:, :, n] = d_in["k_new"].to(dev)
        Xv[:, :, n] = d_in["v_new"].to(dev)
        T = n + 1 - n_packed
        qg = d_in["q"].to(dev)
        lse_g = torch.empty(B, Hq, dtype=torch.float32, device=dev)
        out_g = zb.zc_decode_attention(qg, Kp, Vp, Xk[:, :, n_packed:], Xv[:, :, n_packed:], T, lse_out=lse_g)
        is_probe = j < windows * interval and (j % interval) in probe_off
        out_o, lse_o, row_o = oracle.step(to_f64(d_in["q"]), to_f64(d_in["k_new"]), to_f64(d_in["v_new"]), is_probe)
        rep["out"] = max(rep["out"], float(np.abs(to_f64(out_g) - out_o).max()))
        rep["lse"] = max(rep["lse"], float(np.abs(lse_g.cpu().numpy() - lse_o).max()))
        assert rep["out"] <= atol and rep["lse"] <= max(atol, 1e-3), (j, rep)
        if is_probe:
            jp = len(row_len)
            zb.zc_decode_probs(qg, Kp, Xk[:, :, n_packed:], T, n_packed, lse_g, rows_g[jp])
            row_len.append(n + 1)
            got = rows_g[jp, :, :, :n + 1].cpu().numpy().astype(np.float64)
            assert float(rows_g[jp, :, :, n + 1:].abs().sum()) == 0.0           # nothing past the row's tokens
            assert np.allclose(got.sum(-1), 1.0, atol=2e-3 if not fp32 else 1e-5)
            if fp32:
                err = float((np.abs(got - row_o) / np.maximum(row_o, 1e-6 * row_o.max())).max())
                assert err <= 1e-4, (j, err)
            else:
                err = float(np.abs(got - row_o).max())
                assert err <= 2e-3, (j, err)
            rep["row"] = max(rep["row"], err)
        if (j + 1) % interval == 0 and j < windows * interval:
            m = n + 1 - interval
            k = int(np.floor(w.salient_ratio * m + 1e-9))
            rl = torch.tensor(row_len, dtype=torch.int32, device=dev)
            sc_g = zb.zc_rows_saliency(rows_g[:len(row_len)].contiguous(), rl, m)
            # (a) Eq. 8 on the rows the GPU produced; (b) end to end against the oracle's own rows
            sc_dec = zo.rows_saliency([rows_g[i, :, :, :row_len[i]].cpu().numpy().astype(np.float64) for i in range(len(row_len))])[:, :m]
            sg = sc_g.cpu().numpy().astype(np.float64)
            srel = float((np.abs(sg - sc_dec) / np.maximum(sc_dec, 1e-6 * sc_dec.max())).max())
            assert srel <= 1e-5, srel
            Kt_o, Vt_o = oracle.token_matrices()
            sc_o, sal_o, reg_o = oracle.recompress(w.salient_ratio)
            erel = float((np.abs(sg - sc_o) / np.maximum(sc_o, 1e-6 * sc_o.max())).max())
            assert erel <= (1e-4 if fp32 else 3e-3) + 2.0 * rep["lse"], erel
            rep["score"], rep["score_e2e"] = max(rep["score"], srel), max(rep["score_e2e"], erel)
            sal_g, reg_g = zb.zc_select_salient(sc_g, k)
            sal_np, reg_np = sal_g.cpu().numpy(), reg_g.cpu().numpy()
            for b in bsel:
                s_ex, r_ex = zo.select_salient(sc_g[b].cpu().numpy(), k)
                assert np.array_equal(s_ex, sal_np[b]) and np.array_equal(r_ex, reg_np[b])
                if fp32:
                    check_index_sets(sc_o[b], sal_np[b], k, f"window {j // interval} b={b}")
            # the compressed tokens as they now are, at their positions
            zb.zc_dequantize_cache(Kp, Xk)
            zb.zc_dequantize_cache(Vp, Xv)
            torch.cuda.synchronize()
            for Xg, Xo in ((Xk, Kt_o), (Xv, Vt_o)):
                got = to_f64(Xg[:, :, :n + 1])
                ulp = {"fp32": 2.0 ** -22, "fp16": 2.0 ** -10, "bf16": 2.0 ** -7}[w.dtype]
                assert np.all(np.abs(got - Xo) <= ulp * np.abs(Xo) + 1e-30)
                rep["dequant_mismatch"] = max(rep["dequant_mismatch"], float((got != Xo).mean()))
                assert np.array_equal(got[:, :, n_packed:], Xo[:, :, n_packed:])         # the full-precision tokens are untouched
            # (16-bit storage: the kernel's fp32 evaluation and the oracle's fp64 one round to the same
            # stored value except at a rounding boundary; fp32 storage keeps the fp32 evaluation itself)
            assert fp32 or rep["dequant_mismatch"] <= 1e-3
            # re-compression into the other pair of packed tensors
            Kp2, Vp2 = caches[((j + 1) // interval) % 2]
            Kp2.reset(); Vp2.reset()
            zb.zc_quantize_pack(Xk[:, :, :m], sal_g, reg_g, Kp2)
            zb.zc_quantize_pack(Xv[:, :, :m], sal_g, reg_g, Vp2)
            torch.cuda.synchronize()
            ck_g, cv_g = packed_to_chunks(Kp2, bsel)[0], packed_to_chunks(Vp2, bsel)[0]
            ok_ = zo.compress_tensor(to_f64(Xk[:, :, :m]), sal_np, reg_np, w.bits_hi, w.bits_lo, "channel")
            ov_ = zo.compress_tensor(to_f64(Xv[:, :, :m]), sal_np, reg_np, w.bits_hi, w.bits_lo, "cst")
            for name, g_, o_ in (("K.hi", ck_g.hi, ok_.hi), ("K.lo", ck_g.lo, ok_.lo), ("V.hi", cv_g.hi, ov_.hi), ("V.lo", cv_g.lo, ov_.lo)):
                c = compare_subset(g_, o_, f"window {j // interval} {name}")
                print(f"[literal]   {name}: " + " ".join(f"{key}={c[key]}" for key in CODE_COUNTS), flush=True)
                for key in CODE_COUNTS:
                    totals[key] += c[key]
            # the oracle goes on with the cache the GPU holds
            oracle.chunk_K, oracle.chunk_V, oracle.n_packed = ck_g, cv_g, m
            Kp, Vp, n_packed = Kp2, Vp2, m
            rows_g.zero_()
            row_len = []
            now_sal = set(sal_np[0].tolist())
            promoted = len([p for p in now_sal - prev_sal if p < m - interval or j < interval])    # were compressed as regular before
            demoted = len(prev_sal - now_sal)
            changed += promoted + demoted
            prev_sal = now_sal
            print(f"[literal] window {j // interval}: m={m} k={k} row err {rep['row']:.2e} score rel {srel:.1e} / {erel:.1e} end to end; "
                  f"b=0: {promoted} tokens promoted to salient, {demoted} demoted to regular", flush=True)
    # Re-compression quantizes values that sit on the previous quantization grid.  With fp32
    # storage that grid survives exactly, so x / s hits n + 1/2 structurally (a channel whose new
    # range spans an even number of old steps puts every odd old level on a tie), give or take
    # the 1e-7 rounding noise of the stored x_hat; the fp32 kernel rounds the quotient to fp32
    # before it rounds to an integer and so sees a tie where exact arithmetic sees +-1e-7.  Every
    # such element is still one step apart at its rounding boundary (compare_subset); only the
    # budget is wider here.  16-bit storage rounds x_hat off the grid: the usual budget holds.
    rep.update(assert_code_budgets(totals, w.name, level_budget=1e-3 if fp32 else 1e-4))
    print("[literal]", w.name, rep, flush=True)
    assert changed > 0          # the literal reading's signature: tokens change subsets
    return rep


def test_literal_recompression_fp32_two_windows():
    w = scaled(WORKLOADS["tiny"], B=2, Hq=8, Hkv=4, L=150)
    run_literal(w, interval=40, windows=2)


def test_literal_recompression_bf16_grouped_heads_two_windows():
    w = scaled(WORKLOADS["llama3_8b_4k"], B=1, Hq=8, Hkv=2, L=300)
    run_literal(w, interval=100, windows=2)


def test_literal_recompression_fp16_mha():
    w = scaled(WORKLOADS["llama2_13b_4k_b16"], B=2, Hq=4, Hkv=4, L=130)
    run_literal(w, interval=64, windows=2)


def test_decode_probs_over_many_chunks_and_schemes():
    """zc_decode_probs on a chunk-local cache (several chunks, CST keys too): the row sums to one
    and equals the oracle's probabilities in token order."""
    B, Hq, Hkv, d = 2, 8, 2, 64
    g = torch.Generator().manual_seed(21)
    sizes = [150, 70, 33]
    T = 19
    Ltot = sum(sizes) + T
    for dtype, k_scheme in ((torch.float32, "cst"), (torch.bfloat16, "channel"), (torch.float16, "token")):
        K = torch.randn(B, Hkv, Ltot, d, generator=g).to(dtype)
        V = torch.randn(B, Hkv, Ltot, d, generator=g).to(dtype)
        q = torch.randn(B, Hq, d, generator=g).to(dtype)
        lib = zb.load()
        ks = [60, 20, 0]
        cap_hi, cap_lo = lib.zc_arena_slots(sum(ks), 3), lib.zc_arena_slots(sum(sizes) - sum(ks), 3)
        Kp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, 4, 2, k_scheme, zb.ZC_LAYOUT_ROW, max_chunks=3, device=DEV)
        Vp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=3, device=DEV)
        Kd, Vd = K.to(DEV), V.to(DEV)
        n0 = 0
        for n_new, k_new in zip(sizes, ks):
            sal, reg = zb.zc_select_salient(torch.rand(B, n_new, generator=g).to(DEV), k_new)
            zb.zc_quantize_pack(Kd[:, :, n0:n0 + n_new], sal, reg, Kp, pos_offset=n0)
            zb.zc_quantize_pack(Vd[:, :, n0:n0 + n_new], sal, reg, Vp, pos_offset=n0)
            n0 += n_new
        lse = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
        zb.zc_decode_attention(q.to(DEV), Kp, Vp, Kd[:, :, n0:], Vd[:, :, n0:], T, lse_out=lse)
        row = torch.zeros(B, Hq, Ltot + 5, dtype=torch.float32, device=DEV)
        zb.zc_decode_probs(q.to(DEV), Kp, Kd[:, :, n0:], T, n0, lse, row)
        bsel = [0, 1]
        chunks_k, chunks_v = packed_to_chunks(Kp, bsel), packed_to_chunks(Vp, bsel)
        Kc, Vc = zo.cache_matrices(chunks_k, chunks_v, Hkv, K[:, :, n0:].double().numpy(), V[:, :, n0:].double().numpy())
        _, _, probs = zo.decode_attention(q.double().numpy(), Kc, Vc)
        pos = zo.cache_positions(chunks_k, T, n0)
        want = np.zeros((B, Hq, Ltot + 5))
        for b in range(B):
            want[b][:, pos[b]] = probs[b]
        got = row.cpu().numpy().astype(np.float64)
        tol = 1e-4 if dtype == torch.float32 else 2e-3
        if dtype == torch.float32:
            assert (np.abs(got - want) / np.maximum(want, 1e-6 * want.max())).max() <= tol, (dtype, k_scheme)
        else:
            assert np.abs(got - want).max() <= tol, (dtype, k_scheme)
        assert np.all(got[:, :, Ltot:] == 0.0)
