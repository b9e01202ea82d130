"""GPU-versus-oracle parity harness for the whole hot path.

A pass of the hot path (probe saliency -> select -> quantize-pack K, V -> decode
steps, optionally with the streaming tail flush) is recorded - by
`run_pipeline_check`, which drives the four C-ABI entry points call by call, or
from the benchmark's own `HotPath` object after a step - and `verify_record`
compares every stage with the float64 oracle under these rules:

  scores      relative error <= SCORE_RTOL against the oracle (the flush windows too,
              given the log-sum-exps of the GPU's decode steps; end to end they
              inherit the decode stage's lse error on top)
  index sets  |S| = k; every token scoring above tau*(1+delta) is selected and
              none below tau*(1-delta) is (tau = oracle's k-th score); given the
              GPU's own fp32 scores the selection is exact
  codes       over the pass: >= 99.99 % of the stored codes identical to the
              oracle's; <= 1e-4 of the levels code - z different, each by one step
              at the element's own rounding boundary (or, in a group whose zero point
              differs, at an end of the code range); <= 1e-4 of the zero points
              different, each by one step at its own rounding boundary
  scales      within 1e-6 relative of the oracle value
  attention   <= 2e-2 absolute (fp16 / bf16), <= 1e-4 (fp32), against the oracle
              run on the codes the GPU produced (isolates the decode kernel);
              also against the oracle's own codes when no code differs
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

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
ZERO_MISMATCH_BUDGET = 1e-4
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
            idx = pos[list(bsel), beg:beg + n].cpu().numpy().astype(np.int64) if pos is not None else None   # not stored
            subs.append(zo.QuantSubset(P.scheme, bits, idx, codes, cs_all[ci, si][list(bsel)], cz_all[ci, si][list(bsel)], s, z))
        out.append(zo.QuantChunk(*subs))
    return out


def compare_subset(g: zo.QuantSubset, o: zo.QuantSubset, what: str) -> Dict[str, float]:
    """Codes, scales and zero-points of one subset: GPU (g) against oracle (o).

    Returned counts: n_codes, n_raw_mismatch (stored codes that are not identical),
    n_raw_unshifted (those of them in groups whose zero points agree), n_mismatch
    (levels code - z that are not identical), n_groups (token rows or channels,
    whichever carries the zero point) and n_zero_mismatch (groups whose zero point
    differs).  The budgets over a whole workload are asserted by the caller
    (`assert_code_budgets`)."""
    assert g.codes.shape == o.codes.shape, (what, g.codes.shape, o.codes.shape)
    rep = {"n_codes": int(g.codes.size), "n_mismatch": 0, "n_raw_mismatch": 0, "n_raw_unshifted": 0, "n_groups": 0,
           "n_zero_mismatch": 0}
    if g.codes.size == 0:
        return rep
    assert g.idx is None or np.array_equal(g.idx, o.idx), f"{what}: stored positions differ"
    tokwise = o.scheme != "channel"
    grouped = o.scheme == "group"
    qmax = float(2 ** o.bits - 1)

    def rel(a, b):
        return float(np.max(np.abs(a - b) / np.maximum(np.abs(b), 1e-30)))
    f32 = lambda x: x.astype(np.float32).astype(np.float64)
    rep["chan_scale_rel"] = rel(g.chan_scale, f32(o.chan_scale))
    assert rep["chan_scale_rel"] <= SCALE_RTOL, f"{what}: channel scale off by {rep['chan_scale_rel']:.3e}"
    if grouped:
        gsz = o.codes.shape[2] // o.grp_scale.shape[2]
        rep["tok_scale_rel"] = rel(g.grp_scale, f32(o.grp_scale))
        assert rep["tok_scale_rel"] <= SCALE_RTOL, f"{what}: group scale off by {rep['tok_scale_rel']:.3e}"
        zg, zo_ = np.repeat(g.grp_zero, gsz, axis=2), np.repeat(o.grp_zero, gsz, axis=2)
    elif tokwise:
        rep["tok_scale_rel"] = rel(g.tok_scale, f32(o.tok_scale))
        assert rep["tok_scale_rel"] <= SCALE_RTOL, f"{what}: token scale off by {rep['tok_scale_rel']:.3e}"
        zg, zo_ = g.tok_zero[:, :, None], o.tok_zero[:, :, None]
    else:
        zg, zo_ = g.chan_zero[:, None, :], o.chan_zero[:, None, :]
    rep["n_groups"] = int(o.grp_zero.size) if grouped else int(zg.size)
    rep["n_raw_mismatch"] = int((g.codes != o.codes).sum())
    # Eq. 5 defines x_hat = (code - z) s: a row (or channel) whose zero point came out one
    # step apart on the two sides, with every code shifted along, is the same quantization.
    # What is unique is the level code - z.  A differing zero point must sit at its own
    # rounding boundary, z = -round(min / s) with min / s within 1e-3 of n + 1/2 (fp32 on
    # one side, fp64 on the other), and such groups have a budget of their own.
    zdiff = np.broadcast_to(zg != zo_, g.codes.shape)
    rep["n_raw_unshifted"] = int(((g.codes != o.codes) & ~zdiff).sum())
    assert np.all(np.abs(zg - zo_) <= 1), f"{what}: zero-point differs by more than one step"
    if np.any(zg != zo_):
        if grouped:
            B_, n_, W_ = o.codes.shape
            zpre = np.repeat(-o.pre_round.reshape(B_, n_, W_ // gsz, gsz).min(axis=3), gsz, axis=2)
        else:
            zpre = -o.pre_round.min(axis=2 if tokwise else 1)        # -min / s of every row / channel
            zpre = zpre[:, :, None] if tokwise else zpre[:, None, :]
        zfrac = np.abs(zpre - np.floor(zpre) - 0.5)
        assert np.all(zfrac[zg != zo_] < 1e-3), f"{what}: a zero point differs away from its rounding boundary"
    mism = (g.codes - zg) != (o.codes - zo_)
    rep["n_mismatch"] = int(mism.sum())
    rep["n_zero_mismatch"] = int((g.grp_zero != o.grp_zero).sum()) if grouped else int((zg != zo_).sum())
    if rep["n_mismatch"]:
        d = np.abs((g.codes - zg) - (o.codes - zo_))[mism]
        assert np.all(d == 1), f"{what}: a level differs by more than one step"
        frac = np.abs(o.pre_round[mism] - np.floor(o.pre_round[mism]) - 0.5)
        # level = clip(round(x / s), -z, 2^k - 1 - z): where the zero points differ, the two
        # sides clip at different levels, so exactly the elements whose code sits at an end
        # of the code range (0 or 2^k - 1) on one side may move by one level; every other
        # mismatch must be the element's own rounding tie
        gm, om = g.codes[mism], o.codes[mism]
        clipped_end = zdiff[mism] & ((gm == 0) | (gm == qmax) | (om == 0) | (om == qmax))
        at_boundary = (frac < 1e-3) | clipped_end
        assert np.all(at_boundary), f"{what}: {int((~at_boundary).sum())} mismatches away from a rounding boundary"
    return rep


CODE_COUNTS = ("n_codes", "n_mismatch", "n_raw_mismatch", "n_raw_unshifted", "n_groups", "n_zero_mismatch")


def assert_code_budgets(tot: Dict[str, int], what: str, level_budget: float = CODE_MISMATCH_BUDGET) -> Dict[str, float]:
    """The budgets of the code rule over everything `tot` has summed up (CODE_COUNTS).
    At most 1e-4 of the levels differ; at most 1e-4 of the zero points differ (one of
    them when there are fewer than 10^4 groups: a single tie must not fail a small
    case); stored codes: at least 99.99 % identical in the groups whose zero points
    agree, and - once a case is large enough for the zero-point budget to be a
    fraction (10^4 groups) - at least 99.99 % identical over all codes, the shifted
    groups included."""
    n = max(tot["n_codes"], 1)
    out = {"raw_identical_frac": 1.0 - tot["n_raw_mismatch"] / n, "code_mismatch_frac": tot["n_mismatch"] / n,
           "zero_mismatch_frac": tot["n_zero_mismatch"] / max(tot["n_groups"], 1)}
    assert out["code_mismatch_frac"] <= level_budget, f"{what}: {out['code_mismatch_frac']:.3e} of the levels differ"
    assert tot["n_raw_unshifted"] / n <= level_budget, f"{what}: {tot['n_raw_unshifted']} stored codes differ"
    assert tot["n_zero_mismatch"] <= max(1, int(np.floor(ZERO_MISMATCH_BUDGET * tot["n_groups"]))), \
        f"{what}: {tot['n_zero_mismatch']} of {tot['n_groups']} zero points differ"
    if tot["n_groups"] >= 1.0 / ZERO_MISMATCH_BUDGET:
        assert out["raw_identical_frac"] >= 1.0 - level_budget, \
            f"{what}: only {out['raw_identical_frac']:.6f} of the stored codes are identical"
    return out


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

@dataclass
class PathRecord:
    """Everything one pass of the hot path left behind on the GPU, plus the inputs it ran
    on: what `verify_record` compares with the oracle.  Filled by `run_pipeline_check`
    (eager calls, buffers of its own) and by `record_of_hot_path` (the benchmark's
    HotPath object after one step, eager or replayed from its HIP graphs)."""
    w: Workload
    k_scheme: str
    v_scheme: str
    steps: int
    flush_interval: Optional[int]
    prefill: Dict[str, torch.Tensor]            # CPU tensors Q, K, V
    decode_inputs: Callable[[int], Dict[str, torch.Tensor]]
    pos_np: np.ndarray
    scores: torch.Tensor                        # [B, L]
    sal: torch.Tensor
    reg: torch.Tensor
    Kp: zb.PackedTensor
    Vp: zb.PackedTensor
    out: List[torch.Tensor]                     # per step [B, Hq, d]
    lse: Dict[int, torch.Tensor]                # step -> [B, Hq]; at least the probe steps
    probe_off: np.ndarray
    flushes: List[Dict[str, torch.Tensor]] = field(default_factory=list)   # scores [B, FI], sal, reg per flush
    per_head: Optional[torch.Tensor] = None
    sm_scale: float = 0.0


def verify_record(r: PathRecord, bsel: Sequence[int], verbose: bool = False) -> Dict[str, float]:
    """Compares a recorded pass with the oracle, stage by stage, on batch elements `bsel`.
    Raises AssertionError on the first violated rule; returns the observed errors."""
    log = (lambda *a: print("[pipeline]", *a, flush=True)) if verbose else (lambda *a: None)
    w, bsel = r.w, list(bsel)
    rep: Dict[str, float] = {"workload": w.name}
    sm = r.sm_scale or None
    Qo, Ko, Vo = (to_f64(r.prefill[n][bsel]) for n in ("Q", "K", "V"))
    pos_np, k = r.pos_np, int(r.sal.shape[1])
    log(f"{w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} d={w.d} L={w.L} {w.dtype} P={len(pos_np)} k={k} "
        f"steps={r.steps} flush={r.flush_interval} checking b={bsel}")

    # ---- probe saliency ---------------------------------------------------------
    scores_o, per_head_o = zo.saliency_scores(Qo, Ko, pos_np, sm_scale=sm)
    sg = r.scores[bsel].cpu().numpy().astype(np.float64)
    floor = 1e-6 * scores_o.max()
    rel = np.abs(sg - scores_o) / np.maximum(scores_o, floor)
    rep["score_max_rel"] = float(rel.max())
    log(f"scores: max rel err {rep['score_max_rel']:.3e}")
    assert rep["score_max_rel"] <= SCORE_RTOL, f"scores off by {rep['score_max_rel']:.3e}"
    if r.per_head is not None:
        phg = r.per_head[bsel].cpu().numpy().astype(np.float64)
        assert np.abs(phg - per_head_o).max() <= SCORE_RTOL * per_head_o.max() + 1e-12
        cnt = zo.unmasked_count(pos_np, w.L)
        cons = (phg * cnt).sum(-1)                         # every probe row sums to 1
        assert np.allclose(cons, len(pos_np), rtol=1e-4), f"column sums do not add up to P: {cons.min()}..{cons.max()}"

    # ---- select ------------------------------------------------------------------
    sal_np, reg_np = r.sal.cpu().numpy(), r.reg.cpu().numpy()
    sg32 = r.scores.cpu().numpy()
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

    # ---- quantize + pack: every chunk the pass appended ------------------------------
    Kp, Vp = r.Kp, r.Vp
    FI = r.flush_interval
    n_flush = (r.steps // FI) if FI else 0
    assert Kp.chunks == Vp.chunks and len(Kp.chunks) == 1 + n_flush
    assert np.array_equal(Kp.chunk_table.cpu().numpy()[:1 + n_flush], Kp.chunk_table_host[:1 + n_flush])
    chunks_gk, chunks_gv = packed_to_chunks(Kp, bsel), packed_to_chunks(Vp, bsel)
    totals = {key: 0 for key in CODE_COUNTS}

    def check_chunk(ci: int, Xo_k, Xo_v, sal_sel, reg_sel, pos_offset: int):
        ok_ = zo.compress_tensor(Xo_k, sal_sel, reg_sel, w.bits_hi, w.bits_lo, r.k_scheme, pos_offset)
        ov_ = zo.compress_tensor(Xo_v, sal_sel, reg_sel, w.bits_hi, w.bits_lo, r.v_scheme, pos_offset)
        mis = 0
        for name, g_, o_ in (("K.hi", chunks_gk[ci].hi, ok_.hi), ("K.lo", chunks_gk[ci].lo, ok_.lo),
                             ("V.hi", chunks_gv[ci].hi, ov_.hi), ("V.lo", chunks_gv[ci].lo, ov_.lo)):
            c = compare_subset(g_, o_, f"chunk {ci} {name}")
            for key in CODE_COUNTS:
                totals[key] += c[key]
            mis += c["n_raw_mismatch"]
            for key in ("chan_scale_rel", "tok_scale_rel"):
                if key in c:
                    rep[key] = max(rep.get(key, 0.0), c[key])
        log(f"chunk {ci}: {mis} stored codes differ from the oracle's")
        return ok_, ov_, mis

    ok0, ov0, mis0 = check_chunk(0, Ko, Vo, sal_np[bsel], reg_np[bsel], 0)
    any_mismatch = mis0 > 0

    # ---- decode, step by step, with the streaming flushes -------------------------------
    cache = zo.StreamingCache(Hkv=w.Hkv, bits_hi=w.bits_hi, bits_lo=w.bits_lo, k_scheme=r.k_scheme, v_scheme=r.v_scheme,
                              interval=FI or (r.steps + 1), chunks_K=[chunks_gk[0]], chunks_V=[chunks_gv[0]], n_packed=w.L)
    own = zo.StreamingCache(Hkv=w.Hkv, chunks_K=[ok0], chunks_V=[ov0], n_packed=w.L)
    probe_set = set(r.probe_off.tolist()) if FI else set()
    atol = out_atol(w.dtype)
    rep["out_max_abs"] = rep["lse_max_abs"] = 0.0
    rep["decode_steps_checked"] = 0
    lse_gpu_window: List[np.ndarray] = []
    for step in range(r.steps):
        f, T = divmod(step, FI) if FI else (0, step)
        d_in = r.decode_inputs(step)
        is_probe = bool(FI) and f < n_flush and T in probe_set
        qo, kno, vno = to_f64(d_in["q"][bsel]), to_f64(d_in["k_new"][bsel]), to_f64(d_in["v_new"][bsel])
        out_o, lse_o, _ = cache.step(qo, kno, vno, is_probe, sm_scale=sm)
        err = float(np.abs(to_f64(r.out[step][bsel]) - out_o).max())
        rep["out_max_abs"] = max(rep["out_max_abs"], err)
        assert err <= atol, f"decode step {step}: output off by {err:.3e} (> {atol})"
        if step in r.lse:
            lg = r.lse[step][bsel].cpu().numpy().astype(np.float64)
            lerr = float(np.abs(lg - lse_o).max())
            rep["lse_max_abs"] = max(rep["lse_max_abs"], lerr)
            assert lerr <= max(atol, 1e-3), f"decode step {step}: lse off by {lerr:.3e}"
            if is_probe:
                lse_gpu_window.append(lg)
        else:
            assert not is_probe, f"decode step {step} is a probe step but its log-sum-exp was not recorded"
        if not any_mismatch and not FI:
            out_own, _, _ = own.step(qo, kno, vno, False, sm_scale=sm)
            e2 = float(np.abs(to_f64(r.out[step][bsel]) - out_own).max())
            assert e2 <= atol, f"decode step {step}: output off by {e2:.3e} against the oracle's own codes"
        rep["decode_steps_checked"] += 1
        if FI and f < n_flush and T == FI - 1:
            # ---- streaming flush: the window's scores, its split, the chunk it appended ----
            fl = r.flushes[f]
            sc_g = fl["scores"][bsel].cpu().numpy().astype(np.float64)
            # (a) the probe stage alone: the oracle scores the window with the log-sum-exps the
            #     GPU's decode steps produced (what zc_probe_saliency was given)
            oracle_lse = cache.probe_lse
            cache.probe_lse = lse_gpu_window
            sc_o = cache.tail_scores(sm_scale=sm)
            cache.probe_lse = oracle_lse
            srel = float((np.abs(sc_g - sc_o) / np.maximum(sc_o, 1e-6 * sc_o.max())).max())
            rep["flush_score_max_rel"] = max(rep.get("flush_score_max_rel", 0.0), srel)
            assert srel <= SCORE_RTOL, f"flush {f}: scores off by {srel:.3e}"
            # (b) end to end: against the oracle's own log-sum-exps; a probability is
            #     exp(logit - lse), so the scores inherit the decode stage's lse error
            sc_e = cache.tail_scores(sm_scale=sm)
            erel = float((np.abs(sc_g - sc_e) / np.maximum(sc_e, 1e-6 * sc_e.max())).max())
            rep["flush_score_end_to_end_rel"] = max(rep.get("flush_score_end_to_end_rel", 0.0), erel)
            assert erel <= SCORE_RTOL + 2.0 * rep["lse_max_abs"], f"flush {f}: scores off by {erel:.3e} end to end"
            sal_tn, reg_tn = fl["sal"].cpu().numpy(), fl["reg"].cpu().numpy()
            k_tail = sal_tn.shape[1]
            sg_t = fl["scores"].cpu().numpy()
            for i, b in enumerate(bsel):
                check_index_sets(sc_o[i], sal_tn[b], k_tail, f"flush {f} select b={b}")
                s_ex, r_ex = zo.select_salient(sg_t[b], k_tail)
                assert np.array_equal(s_ex, sal_tn[b]) and np.array_equal(r_ex, reg_tn[b]), f"flush {f} select b={b}: not exact"
            tk_o = np.stack(cache.tail_k, axis=2)
            tv_o = np.stack(cache.tail_v, axis=2)
            ci = f + 1
            check_chunk(ci, tk_o, tv_o, sal_tn[bsel], reg_tn[bsel], cache.n_packed)
            cache.chunks_K.append(chunks_gk[ci]); cache.chunks_V.append(chunks_gv[ci])
            cache.n_packed += FI
            cache.tail_k, cache.tail_v = [], []
            cache.probe_q, cache.probe_lse, cache.probe_pos = [], [], []
            lse_gpu_window = []
            log(f"flush {f} after step {step}: chunk {ci} appended, score rel err {srel:.2e} (end to end {erel:.2e})")
    rep.update(assert_code_budgets(totals, w.name))
    rep["codes_checked"] = totals["n_codes"]
    rep["n_zero_mismatch"] = totals["n_zero_mismatch"]
    log(f"codes: {totals['n_codes']} checked, {totals['n_raw_mismatch']} stored codes differ "
        f"(identical {rep['raw_identical_frac']:.6f}), {totals['n_mismatch']} levels differ, "
        f"{totals['n_zero_mismatch']} of {totals['n_groups']} zero points differ")
    log(f"decode: {r.steps} steps, max |out err| {rep['out_max_abs']:.3e}, max |lse err| {rep['lse_max_abs']:.3e}")
    return rep


def run_pipeline_check(w: Workload, decode_steps: Optional[int] = None, bsel: Optional[Sequence[int]] = None,
                       k_scheme: str = "channel", v_scheme: str = "cst", flush_interval: Optional[int] = None,
                       verbose: bool = False, device: str = "cuda", sm_scale: float = 0.0,
                       store_pos: bool = True) -> Dict[str, float]:
    """Runs the hot path on the GPU for workload `w`, call by call through the binding,
    and checks it against the oracle on batch elements `bsel` (default: all)."""
    dev = torch.device(device)
    bsel = list(range(w.B)) if bsel is None else list(bsel)
    steps = w.decode_steps if decode_steps is None else decode_steps
    inp = make_prefill(w)
    Qg, Kg, Vg = (inp[n].to(dev) for n in ("Q", "K", "V"))
    pos_np = probes.probe_positions(w.L, w.probe_ratio, w.seed)
    pos_g = torch.from_numpy(pos_np).to(dev)
    k = w.k_salient

    per_head_g = torch.empty(w.B, w.Hq, w.L, dtype=torch.float32, device=dev)
    scores_g = zb.zc_probe_saliency(Qg, Kg, pos_g, scores_per_head=per_head_g, sm_scale=sm_scale)
    sal_g, reg_g = zb.zc_select_salient(scores_g, k)

    n_flush = (steps // flush_interval) if flush_interval else 0
    k_tail = int(np.floor(w.salient_ratio * flush_interval + 1e-9)) if flush_interval else 0
    cap_hi = zb.load().zc_arena_slots(k + n_flush * k_tail, 1 + n_flush)
    cap_lo = zb.load().zc_arena_slots(w.L - k + n_flush * ((flush_interval or 0) - k_tail), 1 + n_flush)
    Kp = zb.PackedTensor(w.B, w.Hkv, w.d, cap_hi, cap_lo, w.bits_hi, w.bits_lo, k_scheme, zb.ZC_LAYOUT_ROW,
                         max_chunks=1 + n_flush, device=device, store_pos=store_pos)
    Vp = zb.PackedTensor(w.B, w.Hkv, w.d, cap_hi, cap_lo, w.bits_hi, w.bits_lo, v_scheme, zb.ZC_LAYOUT_TGROUP,
                         max_chunks=1 + n_flush, device=device, store_pos=store_pos)
    zb.zc_quantize_pack(Kg, sal_g, reg_g, Kp)
    zb.zc_quantize_pack(Vg, sal_g, reg_g, Vp)
    torch.cuda.synchronize()

    T_cap = max(flush_interval or steps, 1)
    tail_k = torch.zeros(w.B, w.Hkv, T_cap, w.d, dtype=w.torch_dtype, device=dev)
    tail_v = torch.zeros_like(tail_k)
    probe_off = probes.decode_probe_offsets(flush_interval, seed=w.seed) if flush_interval else np.zeros(0, np.int32)
    rec = PathRecord(w=w, k_scheme=k_scheme, v_scheme=v_scheme, steps=steps, flush_interval=flush_interval,
                     prefill=inp, decode_inputs=lambda j: make_decode_step(w, j), pos_np=pos_np, scores=scores_g,
                     sal=sal_g, reg=reg_g, Kp=Kp, Vp=Vp, out=[], lse={}, probe_off=probe_off, per_head=per_head_g,
                     sm_scale=sm_scale)
    probe_q, probe_lse = [], []
    T = n_packed = 0
    for step in range(steps):
        d_in = make_decode_step(w, step)
        qg = d_in["q"].to(dev)
        tail_k[:, :, T] = d_in["k_new"].to(dev)
        tail_v[:, :, T] = d_in["v_new"].to(dev)
        T += 1
        lse_g = torch.empty(w.B, w.Hq, dtype=torch.float32, device=dev)
        rec.out.append(zb.zc_decode_attention(qg, Kp, Vp, tail_k, tail_v, T, lse_out=lse_g, sm_scale=sm_scale))
        rec.lse[step] = lse_g
        if flush_interval and step < n_flush * flush_interval and (T - 1) in set(probe_off.tolist()):
            probe_q.append(qg)
            probe_lse.append(lse_g)
        if flush_interval and T == flush_interval:
            Qp = torch.stack(probe_q, dim=2).contiguous()                 # [B, Hq, P', d]
            lse_p = torch.stack(probe_lse, dim=2).contiguous()            # [B, Hq, P']
            ppos = torch.from_numpy(probe_off).to(dev)
            prow = torch.arange(len(probe_off), dtype=torch.int32, device=dev)
            sc_g = zb.zc_probe_saliency(Qp, tail_k, ppos, probe_rows=prow, lse_ext=lse_p, sm_scale=sm_scale)
            sal_t, reg_t = zb.zc_select_salient(sc_g, k_tail)
            zb.zc_quantize_pack(tail_k, sal_t, reg_t, Kp, pos_offset=w.L + n_packed)
            zb.zc_quantize_pack(tail_v, sal_t, reg_t, Vp, pos_offset=w.L + n_packed)
            torch.cuda.synchronize()                                      # the tail buffers are reused
            rec.flushes.append({"scores": sc_g, "sal": sal_t, "reg": reg_t})
            n_packed += T
            probe_q, probe_lse = [], []
            T = 0
    torch.cuda.synchronize()
    return verify_record(rec, bsel, verbose)


def record_of_hot_path(hp) -> PathRecord:
    """The record of a `bench.HotPath` object after one whole step (eager or replayed)."""
    import bench
    w = hp.w
    FI = bench.FLUSH_INTERVAL
    lse = {}
    for f in range(hp.n_flush):
        for i, off in enumerate(hp.probe_off_np.tolist()):
            lse[f * FI + off] = hp.lse_probe[f][i]
    flushes = [{"scores": hp.tail_scores[f], "sal": hp.sal_t[f], "reg": hp.reg_t[f]} for f in range(hp.n_flush)]
    return PathRecord(w=w, k_scheme=hp.Kp.scheme, v_scheme=hp.Vp.scheme, steps=hp.S, flush_interval=FI,
                      prefill=hp.cpu_inputs, decode_inputs=lambda j: hp.cpu_decode[j], pos_np=hp.pos_np,
                      scores=hp.scores, sal=hp.sal, reg=hp.reg, Kp=hp.Kp, Vp=hp.Vp,
                      out=[hp.out[j] for j in range(hp.S)], lse=lse, probe_off=hp.probe_off_np, flushes=flushes)
