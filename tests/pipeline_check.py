"""GPU-versus-oracle parity harness for the whole hot path.

`run_pipeline_check` drives the four C-ABI entry points on a seeded workload
(probe saliency -> select -> quantize-pack K, V -> decode steps, optionally with
the streaming tail flush) and compares every stage with the float64 oracle under
these rules:

  scores      relative error <= SCORE_RTOL against the oracle
  index sets  |S| = k; every token scoring above tau*(1+delta) is selected and
              none below tau*(1-delta) is (tau = oracle's k-th score); given the
              GPU's own fp32 scores the selection is exact
  codes       >= 99.99 % identical; a mismatch is one step and sits at a
              rounding boundary of the oracle (or follows a zero-point that does)
  scales      within 1e-6 relative of the oracle value
  attention   <= 2e-2 absolute (fp16 / bf16), <= 1e-4 (fp32), against the oracle
              run on the codes the GPU produced (isolates the decode kernel);
              also against the oracle's own codes when no code differs
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import zipcache_oracle as zo
from paper_2405_14256_amd import binding as zb
from paper_2405_14256_amd import probes
from paper_2405_14256_amd.workloads import Workload, make_decode_step, make_prefill, needle_positions, to_f64
from tests import packfmt

SCORE_RTOL = 1e-4
BAND = 1e-4
CODE_MISMATCH_BUDGET = 1e-4
SCALE_RTOL = 1e-6


def out_atol(dtype: str) -> float:
    return 1e-4 if dtype == "fp32" else 2e-2


# ---------------------------------------------------------------------------
# reading a packed tensor back into oracle structures
# ---------------------------------------------------------------------------

def packed_to_chunks(P: zb.PackedTensor, bsel: Sequence[int]) -> List[zo.QuantChunk]:
    """The GPU cache's chunks, for batch elements `bsel`, as oracle QuantChunks."""
    B, H, D = P.B, P.H, P.D
    W = H * D
    dec = packfmt.decode_row if P.layout == zb.ZC_LAYOUT_ROW else packfmt.decode_tgroup
    out = []
    arenas = {}
    for name, codes, cap, bits in (("hi", P.codes_hi, P.c.cap_hi, P.c.bits_hi), ("lo", P.codes_lo, P.c.cap_lo, P.c.bits_lo)):
        per_b = cap * H * D * bits // 8
        flat = codes[: B * per_b].view(B, per_b)[list(bsel)].cpu().numpy()
        arenas[name] = packfmt.to_token_rows(dec(flat.reshape(-1), len(bsel), H, D, cap, bits)) if cap else None
    ts = {"hi": (P.tok_scale_hi, P.tok_zero_hi, P.pos_hi), "lo": (P.tok_scale_lo, P.tok_zero_lo, P.pos_lo)}
    cs_all = P.chan_scale.cpu().numpy().astype(np.float64)
    cz_all = P.chan_zero.cpu().numpy().astype(np.float64)
    tokwise = P.scheme != "channel"
    for ci, (b_hi, n_hi, b_lo, n_lo) in enumerate(P.chunks):
        subs = []
        for si, (name, beg, n, bits) in enumerate((("hi", b_hi, n_hi, P.c.bits_hi), ("lo", b_lo, n_lo, P.c.bits_lo))):
            codes = arenas[name][:, beg:beg + n, :].astype(np.float64) if n else np.zeros((len(bsel), 0, W))
            tsc, tze, pos = ts[name]
            if tokwise and n:
                s = tsc[list(bsel), beg:beg + n].cpu().numpy().astype(np.float64)
                z = tze[list(bsel), beg:beg + n].cpu().numpy().astype(np.float64)
            else:
                s = np.ones((len(bsel), n)); z = np.zeros((len(bsel), n))
            idx = pos[list(bsel), beg:beg + n].cpu().numpy().astype(np.int64) if pos is not None else np.zeros((len(bsel), n), np.int64)
            subs.append(zo.QuantSubset(P.scheme, bits, idx, codes, cs_all[ci, si][list(bsel)], cz_all[ci, si][list(bsel)], s, z))
        out.append(zo.QuantChunk(*subs))
    return out


def compare_subset(g: zo.QuantSubset, o: zo.QuantSubset, what: str) -> Dict[str, float]:
    """Codes, scales and zero-points of one subset: GPU (g) against oracle (o)."""
    assert g.codes.shape == o.codes.shape, (what, g.codes.shape, o.codes.shape)
    rep = {"n_codes": int(g.codes.size), "n_mismatch": 0}
    if g.codes.size == 0:
        return rep
    assert np.array_equal(g.idx, o.idx), f"{what}: stored positions differ"
    tokwise = o.scheme != "channel"

    def rel(a, b):
        return float(np.max(np.abs(a - b) / np.maximum(np.abs(b), 1e-30)))
    f32 = lambda x: x.astype(np.float32).astype(np.float64)
    rep["chan_scale_rel"] = rel(g.chan_scale, f32(o.chan_scale))
    assert rep["chan_scale_rel"] <= SCALE_RTOL, f"{what}: channel scale off by {rep['chan_scale_rel']:.3e}"
    if tokwise:
        rep["tok_scale_rel"] = rel(g.tok_scale, f32(o.tok_scale))
        assert rep["tok_scale_rel"] <= SCALE_RTOL, f"{what}: token scale off by {rep['tok_scale_rel']:.3e}"
        zg, zo_ = g.tok_zero[:, :, None], o.tok_zero[:, :, None]
    else:
        zg, zo_ = g.chan_zero[:, None, :], o.chan_zero[:, None, :]
    # Eq. 5 defines x_hat = (code - z) s: a row (or channel) whose zero point came out one
    # step apart on the two sides, with every code shifted along, is the same quantization.
    # What is unique is the level code - z: mismatches are counted on levels, and a differing
    # zero point must sit at its own rounding boundary, z = -round(min / s) with min / s
    # within 1e-3 of n + 1/2 (fp32 on one side, fp64 on the other).
    zdiff = np.broadcast_to(zg != zo_, g.codes.shape)
    assert np.all(np.abs(zg - zo_) <= 1), f"{what}: zero-point differs by more than one step"
    if np.any(zg != zo_):
        zpre = -o.pre_round.min(axis=2 if tokwise else 1)            # -min / s of every row / channel
        zpre = zpre[:, :, None] if tokwise else zpre[:, None, :]
        zfrac = np.abs(zpre - np.floor(zpre) - 0.5)
        assert np.all(zfrac[zg != zo_] < 1e-3), f"{what}: a zero point differs away from its rounding boundary"
    mism = (g.codes - zg) != (o.codes - zo_)
    rep["n_mismatch"] = int(mism.sum())
    rep["n_zero_mismatch"] = int((zg != zo_).sum())
    if rep["n_mismatch"]:
        d = np.abs((g.codes - zg) - (o.codes - zo_))[mism]
        assert np.all(d == 1), f"{what}: a level differs by more than one step"
        frac = np.abs(o.pre_round[mism] - np.floor(o.pre_round[mism]) - 0.5)
        # (where the zero points differ, the clipped ends of the code range move by one level)
        at_boundary = (frac < 1e-3) | zdiff[mism]
        assert np.all(at_boundary), f"{what}: {int((~at_boundary).sum())} mismatches away from a rounding boundary"
    return rep


def check_index_sets(scores_o: np.ndarray, sal_g: np.ndarray, k: int, what: str) -> None:
    L = scores_o.shape[0]
    assert len(sal_g) == k and len(set(sal_g.tolist())) == k, f"{what}: salient set has wrong size"
    if k == 0 or k == L:
        return
    tau = np.sort(scores_o)[::-1][k - 1]
    chosen = np.zeros(L, bool)
    chosen[sal_g] = True
    must = scores_o > tau * (1 + BAND)
    must_not = scores_o < tau * (1 - BAND)
    assert np.all(chosen[must]), f"{what}: {int((~chosen[must]).sum())} clearly salient tokens were not selected"
    assert not np.any(chosen[must_not]), f"{what}: {int(chosen[must_not].sum())} clearly regular tokens were selected"


# ---------------------------------------------------------------------------
# the pipeline
# ---------------------------------------------------------------------------

def run_pipeline_check(w: Workload, decode_steps: Optional[int] = None, bsel: Optional[Sequence[int]] = None,
                       k_scheme: str = "channel", v_scheme: str = "cst", flush_interval: Optional[int] = None,
                       verbose: bool = False, device: str = "cuda") -> Dict[str, float]:
    """Runs the hot path on the GPU for workload `w` and checks it against the
    oracle on batch elements `bsel` (default: all).  Raises AssertionError on the
    first violated rule; returns a report of the observed errors."""
    log = (lambda *a: print("[pipeline]", *a, flush=True)) if verbose else (lambda *a: None)
    dev = torch.device(device)
    bsel = list(range(w.B)) if bsel is None else list(bsel)
    steps = w.decode_steps if decode_steps is None else decode_steps
    rep: Dict[str, float] = {"workload": w.name}
    G = w.Hq // w.Hkv

    inp = make_prefill(w)
    Qg, Kg, Vg = (inp[n].to(dev) for n in ("Q", "K", "V"))
    Qo, Ko, Vo = (to_f64(inp[n][bsel]) for n in ("Q", "K", "V"))
    pos_np = probes.probe_positions(w.L, w.probe_ratio, w.seed)
    pos_g = torch.from_numpy(pos_np).to(dev)
    k = w.k_salient
    log(f"{w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} d={w.d} L={w.L} {w.dtype} P={len(pos_np)} k={k}")

    # ---- probe saliency ---------------------------------------------------------
    per_head_g = torch.empty(w.B, w.Hq, w.L, dtype=torch.float32, device=dev)
    scores_g = zb.zc_probe_saliency(Qg, Kg, pos_g, scores_per_head=per_head_g)
    torch.cuda.synchronize()
    scores_o, per_head_o = zo.saliency_scores(Qo, Ko, pos_np)
    sg = scores_g[bsel].cpu().numpy().astype(np.float64)
    floor = 1e-6 * scores_o.max()
    rel = np.abs(sg - scores_o) / np.maximum(scores_o, floor)
    rep["score_max_rel"] = float(rel.max())
    log(f"scores: max rel err {rep['score_max_rel']:.3e}")
    assert rep["score_max_rel"] <= SCORE_RTOL, f"scores off by {rep['score_max_rel']:.3e}"
    phg = per_head_g[bsel].cpu().numpy().astype(np.float64)
    assert np.abs(phg - per_head_o).max() <= SCORE_RTOL * per_head_o.max() + 1e-12
    cnt = zo.unmasked_count(pos_np, w.L)
    cons = (phg * cnt).sum(-1)                         # every probe row sums to 1
    assert np.allclose(cons, len(pos_np), rtol=1e-4), f"column sums do not add up to P: {cons.min()}..{cons.max()}"

    # ---- select ------------------------------------------------------------------
    sal_g, reg_g = zb.zc_select_salient(scores_g, k)
    torch.cuda.synchronize()
    sal_np, reg_np = sal_g.cpu().numpy(), reg_g.cpu().numpy()
    sg32 = scores_g.cpu().numpy()
    for i, b in enumerate(bsel):
        check_index_sets(scores_o[i], sal_np[b], k, f"select b={b}")
        s_ex, r_ex = zo.select_salient(sg32[b], k)      # exact on the GPU's own fp32 scores
        assert np.array_equal(s_ex, sal_np[b]) and np.array_equal(r_ex, reg_np[b]), f"select b={b}: not exact"
    rep["salient_overlap"] = float(np.mean([len(set(sal_np[b]) & set(zo.select_salient(scores_o[i], k)[0])) / max(k, 1)
                                            for i, b in enumerate(bsel)]))
    log(f"select: exact on fp32 scores; overlap with oracle set {rep['salient_overlap']:.5f}")
    # the structure the inputs were given must come out as salient, in the oracle and on the GPU:
    # the attention sink (token 0) and every needle (keys aligned with the recent queries)
    must = ([0] if w.sink else []) + [int(p) for p in needle_positions(w)]
    for i, b in enumerate(bsel):
        sal_o = set(zo.select_salient(scores_o[i], k)[0].tolist())
        sal_b = set(sal_np[b].tolist())
        missing = [p for p in must if p not in sal_o or p not in sal_b]
        assert not missing, f"b={b}: tokens {missing} should be salient (sink / needles)"
    if must:
        log(f"select: sink / needle tokens salient in the oracle and on the GPU ({len(must)} of them)")

    # ---- quantize + pack -----------------------------------------------------------
    n_flush = (steps // flush_interval) if flush_interval else 0
    k_tail = int(np.floor(w.salient_ratio * flush_interval + 1e-9)) if flush_interval else 0
    cap_hi = zb.load().zc_arena_slots(k + n_flush * k_tail, 1 + n_flush)
    cap_lo = zb.load().zc_arena_slots(w.L - k + n_flush * ((flush_interval or 0) - k_tail), 1 + n_flush)
    Kp = zb.PackedTensor(w.B, w.Hkv, w.d, cap_hi, cap_lo, w.bits_hi, w.bits_lo, k_scheme, zb.ZC_LAYOUT_ROW,
                         max_chunks=1 + n_flush, device=device)
    Vp = zb.PackedTensor(w.B, w.Hkv, w.d, cap_hi, cap_lo, w.bits_hi, w.bits_lo, v_scheme, zb.ZC_LAYOUT_TGROUP,
                         max_chunks=1 + n_flush, device=device)
    zb.zc_quantize_pack(Kg, sal_g, reg_g, Kp)
    zb.zc_quantize_pack(Vg, sal_g, reg_g, Vp)
    torch.cuda.synchronize()
    assert Kp.chunks == Vp.chunks and np.array_equal(Kp.chunk_table.cpu().numpy()[:1], Kp.chunk_table_host[:1])

    def check_chunk(ci: int, Xo_k, Xo_v, sal_sel, reg_sel, pos_offset: int):
        chunks_gk, chunks_gv = packed_to_chunks(Kp, bsel), packed_to_chunks(Vp, bsel)
        ok_ = zo.compress_tensor(Xo_k, sal_sel, reg_sel, w.bits_hi, w.bits_lo, k_scheme, pos_offset)
        ov_ = zo.compress_tensor(Xo_v, sal_sel, reg_sel, w.bits_hi, w.bits_lo, v_scheme, pos_offset)
        tot = mis = 0
        for name, g_, o_ in (("K.hi", chunks_gk[ci].hi, ok_.hi), ("K.lo", chunks_gk[ci].lo, ok_.lo),
                             ("V.hi", chunks_gv[ci].hi, ov_.hi), ("V.lo", chunks_gv[ci].lo, ov_.lo)):
            r = compare_subset(g_, o_, f"chunk {ci} {name}")
            tot += r["n_codes"]; mis += r["n_mismatch"]
            for key in ("chan_scale_rel", "tok_scale_rel"):
                if key in r:
                    rep[key] = max(rep.get(key, 0.0), r[key])
        frac = mis / max(tot, 1)
        assert frac <= CODE_MISMATCH_BUDGET, f"chunk {ci}: {frac:.3e} of the codes differ"
        rep["code_mismatch_frac"] = max(rep.get("code_mismatch_frac", 0.0), frac)
        rep["codes_checked"] = rep.get("codes_checked", 0) + tot
        log(f"chunk {ci}: {tot} codes, {mis} mismatches (all at rounding boundaries)")
        return chunks_gk, chunks_gv, ok_, ov_, mis

    chunks_gk, chunks_gv, ok0, ov0, mis0 = check_chunk(0, Ko, Vo, sal_np[bsel], reg_np[bsel], 0)
    any_mismatch = mis0 > 0

    # ---- decode --------------------------------------------------------------------
    T_cap = max(flush_interval or steps, 1)
    tail_k = torch.zeros(w.B, w.Hkv, T_cap, w.d, dtype=w.torch_dtype, device=dev)
    tail_v = torch.zeros_like(tail_k)
    cache = zo.StreamingCache(Hkv=w.Hkv, bits_hi=w.bits_hi, bits_lo=w.bits_lo, k_scheme=k_scheme, v_scheme=v_scheme,
                              interval=flush_interval or (steps + 1), chunks_K=list(chunks_gk), chunks_V=list(chunks_gv),
                              n_packed=w.L)
    own = zo.StreamingCache(Hkv=w.Hkv, chunks_K=[ok0], chunks_V=[ov0], n_packed=w.L)
    lse_g = torch.empty(w.B, w.Hq, dtype=torch.float32, device=dev)
    probe_off = probes.decode_probe_offsets(flush_interval, seed=w.seed) if flush_interval else np.zeros(0, np.int32)
    probe_q, probe_lse = [], []
    atol = out_atol(w.dtype)
    rep["out_max_abs"] = rep["lse_max_abs"] = 0.0
    T = 0
    for step in range(steps):
        d_in = make_decode_step(w, step)
        qg = d_in["q"].to(dev)
        tail_k[:, :, T] = d_in["k_new"].to(dev)
        tail_v[:, :, T] = d_in["v_new"].to(dev)
        T += 1
        out_g = zb.zc_decode_attention(qg, Kp, Vp, tail_k, tail_v, T, lse_out=lse_g)
        torch.cuda.synchronize()
        is_probe = bool(flush_interval) and (T - 1) in set(probe_off.tolist())
        qo, kno, vno = to_f64(d_in["q"][bsel]), to_f64(d_in["k_new"][bsel]), to_f64(d_in["v_new"][bsel])
        out_o, lse_o, _ = cache.step(qo, kno, vno, is_probe)
        err = float(np.abs(to_f64(out_g[bsel]) - out_o).max())
        lerr = float(np.abs(lse_g[bsel].cpu().numpy() - lse_o).max())
        rep["out_max_abs"] = max(rep["out_max_abs"], err)
        rep["lse_max_abs"] = max(rep["lse_max_abs"], lerr)
        assert err <= atol, f"decode step {step}: output off by {err:.3e} (> {atol})"
        assert lerr <= max(atol, 1e-3), f"decode step {step}: lse off by {lerr:.3e}"
        if not any_mismatch and not flush_interval:
            out_own, _, _ = own.step(qo, kno, vno, False)
            e2 = float(np.abs(to_f64(out_g[bsel]) - out_own).max())
            assert e2 <= atol, f"decode step {step}: output off by {e2:.3e} against the oracle's own codes"
        if is_probe:
            probe_q.append(qg)
            probe_lse.append(lse_g.clone())
        if flush_interval and T == flush_interval:
            # ---- streaming flush: score the window, split it, append a chunk ----
            Qp = torch.stack(probe_q, dim=2).contiguous()                 # [B, Hq, P', d]
            lse_p = torch.stack(probe_lse, dim=2).contiguous()            # [B, Hq, P']
            ppos = torch.from_numpy(probe_off).to(dev)
            prow = torch.arange(len(probe_off), dtype=torch.int32, device=dev)
            sc_g = zb.zc_probe_saliency(Qp, tail_k, ppos, probe_rows=prow, lse_ext=lse_p)
            sal_t, reg_t = zb.zc_select_salient(sc_g, k_tail)
            zb.zc_quantize_pack(tail_k, sal_t, reg_t, Kp, pos_offset=cache.n_packed)
            zb.zc_quantize_pack(tail_v, sal_t, reg_t, Vp, pos_offset=cache.n_packed)
            torch.cuda.synchronize()
            sc_o = cache.tail_scores()
            srel = float((np.abs(sc_g[bsel].cpu().numpy() - sc_o) / np.maximum(sc_o, 1e-6 * sc_o.max())).max())
            rep["flush_score_max_rel"] = max(rep.get("flush_score_max_rel", 0.0), srel)
            assert srel <= 1e-3, f"flush scores off by {srel:.3e}"
            sal_tn, reg_tn = sal_t.cpu().numpy(), reg_t.cpu().numpy()
            for i, b in enumerate(bsel):
                check_index_sets(sc_o[i], sal_tn[b], k_tail, f"flush select b={b}")
            tk_o = np.stack(cache.tail_k, axis=2)
            tv_o = np.stack(cache.tail_v, axis=2)
            ci = len(cache.chunks_K)
            cgk, cgv, _, _, mis = check_chunk(ci, tk_o, tv_o, sal_tn[bsel], reg_tn[bsel], cache.n_packed)
            cache.chunks_K.append(cgk[ci]); cache.chunks_V.append(cgv[ci])
            cache.n_packed += T
            cache.tail_k, cache.tail_v = [], []
            cache.probe_q, cache.probe_lse, cache.probe_pos = [], [], []
            probe_q, probe_lse = [], []
            T = 0
            log(f"flush after step {step}: chunk {ci} appended, flush score rel err {srel:.2e}")
    log(f"decode: {steps} steps, max |out err| {rep['out_max_abs']:.3e}, max |lse err| {rep['lse_max_abs']:.3e}")
    return rep
