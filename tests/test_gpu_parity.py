"""GPU parity tests: every stage of the hot path, called through the C ABI,
against the float64 oracle on the same seeded inputs."""
import os

import numpy as np
import pytest
import torch

from oracle import zipcache_oracle as zo
from paper_2405_14256_amd import binding as zb
from paper_2405_14256_amd.workloads import WORKLOADS, scaled
from tests.pipeline_check import record_of_hot_path, run_pipeline_check, verify_record

pytestmark = pytest.mark.gpu

DEV = "cuda"


def test_extension_is_loaded():
    lib = zb.load()
    assert lib.zc_version() >= 1 and torch.cuda.is_available()


# ---- whole pipeline, reduced and full sizes ---------------------------------------

def test_tiny_full():
    rep = run_pipeline_check(WORKLOADS["tiny"], verbose=True)
    assert rep["codes_checked"] == 2 * 256 * 512


@pytest.mark.parametrize("k_scheme,v_scheme", [("cst", "cst"), ("token", "token"), ("channel", "channel")])
def test_tiny_other_schemes(k_scheme, v_scheme):
    run_pipeline_check(WORKLOADS["tiny"], decode_steps=3, k_scheme=k_scheme, v_scheme=v_scheme, verbose=True)


@pytest.mark.parametrize("bits_hi,bits_lo", [(8, 4), (8, 8), (4, 4), (2, 2), (8, 2)])
def test_other_bit_widths(bits_hi, bits_lo):
    # 8-bit subsets take the generic decode kernel, equal widths the matrix-core one
    run_pipeline_check(scaled(WORKLOADS["tiny"], bits_hi=bits_hi, bits_lo=bits_lo), decode_steps=3, verbose=True)
    w = scaled(WORKLOADS["llama3_8b_4k"], L=700, decode_steps=2, bits_hi=bits_hi, bits_lo=bits_lo)
    run_pipeline_check(w, verbose=True)


def test_llama3_shape_ragged():
    # several 128-column tiles, 64-row probe tiles and 32/64-slot blocks, all with ragged tails
    w = scaled(WORKLOADS["llama3_8b_4k"], L=1237, decode_steps=5)
    run_pipeline_check(w, verbose=True)


def _timed_step_against_oracle(name, bsel, graphs=True):
    """The benchmark's own object and launch sequence (bench.HotPath: every buffer, view and
    call of the step bench.py times, replayed from its HIP graphs), at the workload's full
    size and full number of decode steps, flushes included; afterwards everything the step
    left behind - prefill scores and split, every chunk of the packed cache, the output of
    every decode step, the log-sum-exp of every probe step, every flush window's scores and
    split - is compared with the oracle on the batch elements `bsel`."""
    import bench
    w = WORKLOADS[name]
    hp = bench.HotPath(w)
    hp.step()
    if graphs:
        runners, _, _ = hp.launch_units(hp.stages(), graph=True)
        for t in [hp.scores, hp.out, hp.Kp.codes_hi, hp.Kp.codes_lo, hp.Vp.codes_hi, hp.Vp.codes_lo] + hp.tail_scores:
            t.zero_()                                # what the check reads was written by the replay
        torch.cuda.synchronize()
        for r in runners:
            r()
    torch.cuda.synchronize()
    rep = verify_record(record_of_hot_path(hp), bsel, verbose=True)
    assert rep["decode_steps_checked"] == w.decode_steps
    return rep


def test_timed_step_llama3_8b_4k_all_128_steps_and_the_flush():
    rep = _timed_step_against_oracle("llama3_8b_4k", [0])
    assert "flush_score_max_rel" in rep and rep["codes_checked"] == 2 * 1024 * (4096 + 100)


def test_mha_fp16_with_streaming_flush():
    # LLaMA2-13B-like layer, reduced: MHA, fp16, tail grows token by token and is
    # re-compressed every 100 steps (two flushes, then 10 more tail tokens)
    w = scaled(WORKLOADS["llama2_13b_4k_b16"], B=2, Hq=8, Hkv=8, L=700, decode_steps=210)
    rep = run_pipeline_check(w, flush_interval=100, verbose=True)
    assert "flush_score_max_rel" in rep


def test_mistral_shape_batch():
    w = scaled(WORKLOADS["mistral_7b_8k_b8"], B=3, L=2048, decode_steps=4)
    run_pipeline_check(w, bsel=[0, 2], verbose=True)


def test_needles_are_selected():
    w = scaled(WORKLOADS["llama3_8b_32k"], L=4096, decode_steps=2)
    rep = run_pipeline_check(w, verbose=True)
    assert rep["salient_overlap"] > 0.99


# ---- the other configurations at their full sizes and lengths ----------------------------
# The GPU runs the whole batch in the launch configuration the benchmark times, all decode
# steps with the cache growing through its flushes; the oracle checks one batch element:
# every stage, element by element, every decode step.

@pytest.mark.timeout(600)
def test_timed_step_mistral_7b_8k_b8_all_256_steps_two_flushes():
    rep = _timed_step_against_oracle("mistral_7b_8k_b8", [5])
    assert rep["codes_checked"] == 2 * 1024 * (8192 + 200)


@pytest.mark.timeout(900)
def test_timed_step_llama2_13b_4k_b16_all_512_steps_five_flushes():
    rep = _timed_step_against_oracle("llama2_13b_4k_b16", [11])
    assert rep["codes_checked"] == 2 * 5120 * (4096 + 500)


@pytest.mark.timeout(600)
def test_timed_step_llama3_8b_32k_all_64_steps():
    rep = _timed_step_against_oracle("llama3_8b_32k", [0])
    assert rep["salient_overlap"] > 0.99


def test_timed_step_tiny():
    _timed_step_against_oracle("tiny", [0])


def test_softmax_scale_override_and_no_position_arrays():
    """sm_scale != 0 on the probe, accumulated-score and decode entry points (the oracle takes
    the same override), with a streaming flush so that the decode-time probes use it too; the
    packed tensors carry no position arrays (pos_hi = pos_lo = NULL)."""
    w = scaled(WORKLOADS["llama3_8b_4k"], L=777, decode_steps=110, Hq=8, Hkv=2, B=2)
    rep = run_pipeline_check(w, flush_interval=100, sm_scale=0.05, store_pos=False, verbose=True)
    assert "flush_score_max_rel" in rep
    w = scaled(WORKLOADS["tiny"], decode_steps=4)
    run_pipeline_check(w, sm_scale=0.2, store_pos=False, k_scheme="cst", verbose=True)
    from paper_2405_14256_amd import probes
    from paper_2405_14256_amd.workloads import make_prefill
    inp = make_prefill(w)
    pos = probes.probe_positions(w.L, w.probe_ratio, 3)
    got = zb.zc_probe_accumulated(inp["Q"].to(DEV), inp["K"].to(DEV), torch.from_numpy(pos).to(DEV), sm_scale=0.2)
    ref, _ = zo.saliency_scores(inp["Q"].double().numpy(), inp["K"].double().numpy(), pos, sm_scale=0.2, normalized=False)
    assert np.abs(got.cpu().double().numpy() - ref).max() <= 1e-4 * np.abs(ref).max()


# ---- edge cases ---------------------------------------------------------------------

def _rand_scores(B, L, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.rand(B, L, generator=g)


def test_probe_more_rows_than_the_position_table():
    """4200 probe rows: more than the kernels keep in LDS, so the binary searches and the
    row addresses of the column sweep take their path through memory; also a sequence
    length that is no multiple of any tile and head_dim 64."""
    from paper_2405_14256_amd import probes
    L, d = 21013, 64
    g = torch.Generator().manual_seed(77)
    Q = torch.randn(1, 1, L, d, generator=g).to(torch.bfloat16)
    K = torch.randn(1, 1, L, d, generator=g).to(torch.bfloat16)
    K[:, :, 0] += 2.0
    pos = probes.probe_positions(L, 0.2, seed=5)
    assert len(pos) > 4096
    per_head = torch.empty(1, 1, L, dtype=torch.float32, device=DEV)
    sc = zb.zc_probe_saliency(Q.to(DEV), K.to(DEV), torch.from_numpy(pos).to(DEV), scores_per_head=per_head)
    ref, ref_ph = zo.saliency_scores(Q.double().numpy(), K.double().numpy(), pos)
    got = sc.cpu().double().numpy()
    assert np.abs(got - ref).max() <= 1e-4 * np.abs(ref).max()
    assert np.abs(per_head.cpu().double().numpy() - ref_ph).max() <= 1e-4 * np.abs(ref_ph).max()
    # each probe row's probabilities sum to one: the column sums times their counts add up to P per head
    cnt = zo.unmasked_count(pos.astype(np.int64), L)
    assert np.allclose((per_head.cpu().double().numpy() * cnt).sum(-1), len(pos), rtol=1e-4)


def test_probe_randomized_shapes():
    """Sixteen seeded draws of (batch, heads, group size, head_dim, dtype, key length, probe set):
    normalized scores against the oracle; every other case takes the decode-time form
    (probe queries in rows of their own, external log-normalisers)."""
    rng = np.random.Generator(np.random.PCG64(424242))
    for case in range(16):
        d = int(rng.choice([64, 128]))
        G = int(rng.choice([1, 2, 4]))
        Hkv = int(rng.choice([1, 2, 3]))
        B = int(rng.choice([1, 2, 5]))
        dtype = [torch.bfloat16, torch.float16, torch.float32][int(rng.integers(3))]
        Lk = int(rng.integers(1, 1500))
        P = int(rng.integers(1, min(Lk, 400) + 1))
        pos = np.sort(rng.choice(Lk, size=P, replace=False)).astype(np.int32)
        g = torch.Generator().manual_seed(5000 + case)
        K = torch.randn(B, Hkv, Lk, d, generator=g).to(dtype)
        kw, kwo = {}, {}
        if case % 2:
            Q = torch.randn(B, Hkv * G, P + 3, d, generator=g).to(dtype)        # probe queries in rows of their own
            rows = rng.permutation(P + 3)[:P].astype(np.int32)
            # log-normalisers of a softmax that also covered tokens outside k: anything >= the window's own
            own = np.stack([[zo.probe_attention(Q[b, h, rows].double().numpy(), pos, K[b, h // G].double().numpy())[1]
                             for h in range(Hkv * G)] for b in range(B)])
            ext = own + rng.random(own.shape) * 2.0
            kw = dict(probe_rows=torch.from_numpy(rows).to(DEV), lse_ext=torch.from_numpy(ext).float().to(DEV))
            kwo = dict(probe_rows=rows, lse_ext=ext.astype(np.float32).astype(np.float64))
        else:
            Q = torch.randn(B, Hkv * G, Lk, d, generator=g).to(dtype)
        got = zb.zc_probe_saliency(Q.to(DEV), K.to(DEV), torch.from_numpy(pos).to(DEV), **kw).cpu().double().numpy()
        ref, _ = zo.saliency_scores(Q.double().numpy(), K.double().numpy(), pos, **kwo)
        what = (case, B, Hkv, G, d, str(dtype), Lk, P)
        assert np.abs(got - ref).max() <= 1e-4 * max(np.abs(ref).max(), 1e-30), what


def test_accumulated_scores_and_probe_strategies():
    """Eq. 7 (no division by the unmasked count) and the probe choices of the strategy
    comparison (Section 4.3): every variant against the oracle on the same probes; with
    every token as a probe the normalized score is Eq. 8 on the full matrix, and the
    accumulated score of token 0 exceeds one (the bias the normalization removes)."""
    from paper_2405_14256_amd import probes
    from paper_2405_14256_amd.workloads import make_prefill
    w = scaled(WORKLOADS["llama3_8b_4k"], L=901, Hq=8, Hkv=2)
    inp = make_prefill(w)
    Q, K = inp["Q"].to(DEV), inp["K"].to(DEV)
    Qo, Ko = inp["Q"].double().numpy(), inp["K"].double().numpy()
    k = w.k_salient
    picked = {}
    for strategy in probes.STRATEGIES:
        pos = probes.probe_positions(w.L, w.probe_ratio, seed=11, strategy=strategy)
        pos_d = torch.from_numpy(pos).to(DEV)
        for normalized, fn in ((True, zb.zc_probe_saliency), (False, zb.zc_probe_accumulated)):
            got = fn(Q, K, pos_d).cpu().double().numpy()
            ref, _ = zo.saliency_scores(Qo, Ko, pos, normalized=normalized)
            assert np.abs(got - ref).max() <= 1e-4 * np.abs(ref).max(), (strategy, normalized)
            if strategy == "all" and not normalized:
                assert got[0, 0] > 1.0 and abs(got[0].sum() - w.L) <= 1e-3 * w.L     # every row of A sums to one
            if normalized:
                sal, _ = zb.zc_select_salient(torch.from_numpy(got).float().to(DEV), k)
                picked[strategy] = set(sal[0].cpu().tolist())
    # what each strategy selects, against what the full attention matrix selects (Table 2's question)
    overlap = {s: len(picked[s] & picked["all"]) / k for s in picked}
    print("overlap with the full-matrix salient set:", overlap)
    assert overlap["all"] == 1.0 and all(0.0 <= v <= 1.0 for v in overlap.values())


@pytest.mark.parametrize("L,k", [(1, 0), (1, 1), (7, 3), (1000, 0), (1000, 1000), (1024, 1), (5000, 4999), (40000, 4000)])
def test_select_edges(L, k):
    sc = _rand_scores(2, L, L + k)
    sc[:, ::3] = 0.5                                   # massive ties, some straddling the k-th place
    sal, reg = zb.zc_select_salient(sc.to(DEV), k)
    for b in range(2):
        s_o, r_o = zo.select_salient(sc[b].numpy(), k)
        assert np.array_equal(sal[b].cpu().numpy(), s_o) and np.array_equal(reg[b].cpu().numpy(), r_o)


def test_select_value_distributions_and_row_alignments():
    """The cached select kernel starts its radix passes at the first bit in which two keys of the
    row differ, loads rows with 16-byte words when they are aligned and writes the mask a word
    at a time when it can: rows of mixed sign (no common bit), of one value (no undecided bit),
    of two adjacent floats (one undecided bit), of one octave, of many octaves, with ties across
    the k-th place; row lengths around the piece sizes (4, 256, a wave's run) and the largest
    cached row, with B > 1 so that odd lengths leave rows and mask rows misaligned."""
    rng = np.random.default_rng(77)
    def rows(kind, B, L):
        if kind == "mixed":
            x = rng.standard_normal((B, L)).astype(np.float32)
        elif kind == "const":
            x = np.full((B, L), 0.375, np.float32)
        elif kind == "adjacent":
            x = np.where(rng.random((B, L)) < 0.5, np.float32(1.0), np.nextafter(np.float32(1.0), np.float32(2.0))).astype(np.float32)
        elif kind == "octave":
            x = (1.0 + rng.random((B, L))).astype(np.float32) / np.float32(L)
        elif kind == "wide":
            x = np.exp(rng.uniform(-30, 3, (B, L))).astype(np.float32)
        elif kind == "special":                     # infinities of both signs (-inf has the lowest key of all) and subnormals
            x = rng.random((B, L), dtype=np.float32)
            x[:, ::7] = np.inf; x[:, 1::11] = -np.inf; x[:, 2::13] = 1e-42
        else:                                       # ties: few distinct values
            x = rng.integers(0, 5, (B, L)).astype(np.float32) * np.float32(0.25)
        return x
    cases = [(1, 1), (3, 2), (3, 5), (2, 255), (2, 256), (3, 257), (2, 4095), (1, 4096), (2, 4100), (3, 12289),
             (1, 34816), (2, 34815), (1, 34817)]
    for B, L in cases:
        for kind in ("mixed", "const", "adjacent", "octave", "wide", "ties", "special"):
            x = rows(kind, B, L)
            for k in sorted({0, 1, L // 3, L - 1, L} & set(range(L + 1))):
                mask = torch.full((B, L), 7, dtype=torch.uint8, device=DEV)
                sal, reg = zb.zc_select_salient(torch.from_numpy(x).to(DEV), k, mask=mask)
                sal, reg, mk = sal.cpu().numpy(), reg.cpu().numpy(), mask.cpu().numpy()
                for b in range(B):
                    s_o, r_o = zo.select_salient(x[b].astype(np.float64), k)
                    assert np.array_equal(sal[b], s_o) and np.array_equal(reg[b], r_o), (kind, B, L, k, b)
                    m_o = np.zeros(L, np.uint8); m_o[s_o] = 1
                    assert np.array_equal(mk[b], m_o), (kind, B, L, k, b)


def test_select_negative_and_mask():
    sc = torch.tensor([[-1.0, -0.0, 0.0, 3.0, -7.5, 3.0, 1e-30, -1e-30]])
    mask = torch.zeros(1, 8, dtype=torch.uint8, device=DEV)
    sal, reg = zb.zc_select_salient(sc.to(DEV), 3, mask=mask)
    s_o, _ = zo.select_salient(sc[0].numpy().astype(np.float64), 3)
    # -0.0 and 0.0 compare equal in the oracle; the kernel orders -0.0 below 0.0, so index 2 wins either way
    assert sal[0].cpu().tolist() == [3, 5, 6] == list(s_o)
    assert mask[0].cpu().tolist() == [0, 0, 0, 1, 0, 1, 1, 0]


def test_quantize_empty_subsets_and_degenerate_rows():
    B, H, L, D = 1, 8, 96, 64
    g = torch.Generator().manual_seed(5)
    X = torch.randn(B, H, L, D, generator=g)
    X[:, :, 10] = 1.25                      # a constant token row: max == min for the tokenwise schemes
    X[:, 2, :, 7] = 0.0                     # an all-zero channel: c := 1
    X[:, 3, :, 9] = -2.0                    # a constant channel: s := 1 for the channelwise scheme
    Xg = X.to(DEV)
    from tests.pipeline_check import compare_subset, packed_to_chunks
    for k in (0, L, 40):
        sal = torch.arange(0, k, dtype=torch.int32)[None]
        reg = torch.arange(k, L, dtype=torch.int32)[None]
        for scheme, layout in (("cst", zb.ZC_LAYOUT_TGROUP), ("channel", zb.ZC_LAYOUT_ROW), ("token", zb.ZC_LAYOUT_ROW)):
            P = zb.PackedTensor(B, H, D, 128, 128, 4, 2, scheme, layout, max_chunks=1, device=DEV)
            zb.zc_quantize_pack(Xg, sal.to(DEV), reg.to(DEV), P)
            torch.cuda.synchronize()
            got = packed_to_chunks(P, [0])[0]
            ref = zo.compress_tensor(X.double().numpy(), sal.numpy(), reg.numpy(), 4, 2, scheme)
            for name, a, b in (("hi", got.hi, ref.hi), ("lo", got.lo, ref.lo)):
                r = compare_subset(a, b, f"{scheme} k={k} {name}")
                assert r["n_mismatch"] == 0
                assert np.all(np.isfinite(a.dequant()))
            assert P.chunks == [(0, k, 0, L - k)]


def test_quantize_randomized_shapes():
    """Seeded random shapes of zc_quantize_pack against the oracle: row widths from a
    fraction of a wave to ten waves (teams with a ragged last wave included), all three
    schemes, both layouts, every bit-width pair, all three input types, ragged subsets."""
    from tests.pipeline_check import compare_subset, packed_to_chunks
    rng = np.random.default_rng(20240521)
    total = mism = 0
    for case in range(24):
        D = int(rng.choice([64, 128]))
        H = int(rng.choice([1, 2, 3, 5, 8, 12, 40] if D == 128 else [1, 3, 8, 9, 16]))
        B = int(rng.integers(1, 4)) if H * D <= 2048 else 1
        L = int(rng.integers(1, 300))
        k = int(rng.integers(0, L + 1))
        dtype = [torch.float32, torch.float16, torch.bfloat16][case % 3]
        bits_hi, bits_lo = [(4, 2), (8, 4), (2, 2), (8, 2)][int(rng.integers(0, 4))]
        scheme, layout = [("cst", zb.ZC_LAYOUT_TGROUP), ("channel", zb.ZC_LAYOUT_ROW), ("token", zb.ZC_LAYOUT_ROW),
                          ("cst", zb.ZC_LAYOUT_ROW), ("channel", zb.ZC_LAYOUT_TGROUP)][case % 5]
        g = torch.Generator().manual_seed(1000 + case)
        X = (torch.randn(B, H, L, D, generator=g) * (1 + 9 * (torch.rand(1, H, 1, D, generator=g) > 0.9))).to(dtype)
        perm = torch.stack([torch.randperm(L, generator=g) for _ in range(B)])
        sal = perm[:, :k].sort(dim=1).values.to(torch.int32)
        reg = perm[:, k:].sort(dim=1).values.to(torch.int32)
        cap = zb.load().zc_arena_slots(L, 1)
        P = zb.PackedTensor(B, H, D, cap, cap, bits_hi, bits_lo, scheme, layout, max_chunks=1, device=DEV)
        what = f"case {case}: B={B} H={H} D={D} L={L} k={k} {dtype} {bits_hi}/{bits_lo} {scheme} layout={layout}"
        print(what, flush=True)
        zb.zc_quantize_pack(X.to(DEV), sal.to(DEV), reg.to(DEV), P)
        torch.cuda.synchronize()
        got = packed_to_chunks(P, list(range(B)))[0]
        ref = zo.compress_tensor(X.double().numpy(), sal.numpy(), reg.numpy(), bits_hi, bits_lo, scheme)
        for name, a, b in (("hi", got.hi, ref.hi), ("lo", got.lo, ref.lo)):
            r = compare_subset(a, b, f"{what} {name}")
            total += r["n_codes"]
            mism += r["n_mismatch"]
    assert mism <= 1e-4 * total, (mism, total)


def test_quantize_pack_kv_equals_two_calls():
    """zc_quantize_pack_kv leaves exactly what two zc_quantize_pack calls leave: every array of
    both packed tensors, bit for bit - the merged launches of the paper's configuration and the
    per-tensor fallbacks (other schemes / layouts, rows wider than one workgroup), two chunks."""
    rng = np.random.default_rng(5150)
    cases = [("channel", zb.ZC_LAYOUT_ROW, "cst", zb.ZC_LAYOUT_TGROUP, 8, 128, torch.bfloat16),      # merged
             ("channel", zb.ZC_LAYOUT_ROW, "cst", zb.ZC_LAYOUT_TGROUP, 3, 64, torch.float32),        # merged, ragged wave
             ("channel", zb.ZC_LAYOUT_ROW, "cst", zb.ZC_LAYOUT_TGROUP, 40, 128, torch.float16),      # wide rows: per-tensor packs
             ("cst", zb.ZC_LAYOUT_ROW, "cst", zb.ZC_LAYOUT_TGROUP, 4, 128, torch.bfloat16),
             ("token", zb.ZC_LAYOUT_ROW, "token", zb.ZC_LAYOUT_TGROUP, 2, 64, torch.float16),
             ("channel", zb.ZC_LAYOUT_ROW, "channel", zb.ZC_LAYOUT_TGROUP, 5, 64, torch.float32)]
    for ks, kl, vs, vl, H, D, dtype in cases:
        B = 2
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        sizes = [int(rng.integers(1, 400)), int(rng.integers(1, 120))]
        caps = zb.load().zc_arena_slots(sum(sizes), 2)
        packs = [[zb.PackedTensor(B, H, D, caps, caps, 4, 2, s_, l_, max_chunks=2, device=DEV) for s_, l_ in ((ks, kl), (vs, vl))]
                 for _ in range(2)]
        n0 = 0
        for n in sizes:
            K = torch.randn(B, H, n, D, generator=g).to(dtype).to(DEV)
            V = torch.randn(B, H, n, D, generator=g).to(dtype).to(DEV)
            kk = int(rng.integers(0, n + 1))
            sal, reg = zb.zc_select_salient(torch.rand(B, n, generator=g).to(DEV), kk)
            zb.zc_quantize_pack(K, sal, reg, packs[0][0], pos_offset=n0)
            zb.zc_quantize_pack(V, sal, reg, packs[0][1], pos_offset=n0)
            zb.zc_quantize_pack_kv(K, V, sal, reg, packs[1][0], packs[1][1], pos_offset=n0)
            n0 += n
        torch.cuda.synchronize()
        for a, b in zip(packs[0], packs[1]):
            assert a.chunks == b.chunks and (a.c.n_hi, a.c.n_lo, a.c.n_chunks) == (b.c.n_hi, b.c.n_lo, b.c.n_chunks)
            for name in ("codes_hi", "codes_lo", "tok_scale_hi", "tok_zero_hi", "tok_scale_lo", "tok_zero_lo", "pos_hi", "pos_lo",
                         "chan_scale", "chan_zero", "chunk_table"):
                assert torch.equal(getattr(a, name), getattr(b, name)), (ks, vs, H, D, dtype, name)


def test_plain_tokenwise_codes_are_tie_exact():
    """Without channel normalization (scheme "token", c = 1) 16-bit inputs sit on a grid where
    x / s lands on n + 1/2 exactly about once in 10^4 elements: the codes must still be the
    oracle's (round half to even on the exact quotient), for both 16-bit types and layouts."""
    from tests.pipeline_check import compare_subset, packed_to_chunks
    B, H, L, D, k = 2, 4, 1500, 64, 600
    total = 0
    for dtype, layout in ((torch.bfloat16, zb.ZC_LAYOUT_ROW), (torch.float16, zb.ZC_LAYOUT_TGROUP), (torch.bfloat16, zb.ZC_LAYOUT_TGROUP)):
        g = torch.Generator().manual_seed(31)
        X = torch.randn(B, H, L, D, generator=g).to(dtype)
        perm = torch.stack([torch.randperm(L, generator=g) for _ in range(B)])
        sal = perm[:, :k].sort(dim=1).values.to(torch.int32)
        reg = perm[:, k:].sort(dim=1).values.to(torch.int32)
        cap = zb.load().zc_arena_slots(L, 1)
        P = zb.PackedTensor(B, H, D, cap, cap, 4, 2, "token", layout, max_chunks=1, device=DEV)
        zb.zc_quantize_pack(X.to(DEV), sal.to(DEV), reg.to(DEV), P)
        torch.cuda.synchronize()
        got = packed_to_chunks(P, list(range(B)))[0]
        ref = zo.compress_tensor(X.double().numpy(), sal.numpy(), reg.numpy(), 4, 2, "token")
        for name, a, b in (("hi", got.hi, ref.hi), ("lo", got.lo, ref.lo)):
            r = compare_subset(a, b, f"token {dtype} layout={layout} {name}")
            assert r["n_mismatch"] == 0, (dtype, layout, name, r)
            total += r["n_codes"]
    assert total == 3 * B * L * H * D


@pytest.mark.parametrize("bits_hi,bits_lo", [(4, 2), (8, 4), (2, 2)])
def test_unpack_inverts_the_packing(bits_hi, bits_lo):
    # zc_unpack against the reference decoder written from the header (tests/packfmt.py)
    # and the oracle's de-quantization; two chunks, ragged lengths, both layouts, all schemes
    from tests.pipeline_check import packed_to_chunks
    B, H, L, D = 2, 4, 150, 64
    g = torch.Generator().manual_seed(11)
    X = torch.randn(B, H, L, D, generator=g).to(torch.bfloat16)
    X2 = torch.randn(B, H, 70, D, generator=g).to(torch.bfloat16)
    perm = torch.stack([torch.randperm(L, generator=g) for _ in range(B)])
    sal = perm[:, :61].sort(dim=1).values.to(torch.int32)
    reg = perm[:, 61:].sort(dim=1).values.to(torch.int32)
    sal2 = torch.arange(0, 70, 3, dtype=torch.int32)[None].repeat(B, 1)
    reg2 = torch.tensor([i for i in range(70) if i % 3], dtype=torch.int32)[None].repeat(B, 1)
    for scheme, layout in (("cst", zb.ZC_LAYOUT_TGROUP), ("channel", zb.ZC_LAYOUT_ROW), ("token", zb.ZC_LAYOUT_TGROUP), ("channel", zb.ZC_LAYOUT_TGROUP)):
        P = zb.PackedTensor(B, H, D, 256, 256, bits_hi, bits_lo, scheme, layout, max_chunks=2, device=DEV)
        zb.zc_quantize_pack(X.to(DEV), sal.to(DEV), reg.to(DEV), P)
        zb.zc_quantize_pack(X2.to(DEV), sal2.to(DEV), reg2.to(DEV), P, pos_offset=L)
        torch.cuda.synchronize()
        ref = packed_to_chunks(P, list(range(B)))
        for ci in range(2):
            for which, sub in ((0, ref[ci].hi), (1, ref[ci].lo)):
                codes, xhat = zb.zc_unpack(P, which, ci)
                torch.cuda.synchronize()
                assert np.array_equal(codes.cpu().numpy().astype(np.float64), sub.codes), (scheme, layout, ci, which)
                want = sub.dequant()
                got = xhat.cpu().numpy().astype(np.float64)
                assert np.allclose(got, want, rtol=2e-6, atol=1e-6 * np.abs(want).max()), (scheme, layout, ci, which)


def test_decode_tail_only_and_no_tail():
    w = scaled(WORKLOADS["tiny"], L=64)
    B, Hq, Hkv, d = 1, 8, 8, 64
    g = torch.Generator().manual_seed(9)
    q = torch.randn(B, Hq, d, generator=g)
    tk = torch.randn(B, Hkv, 37, d, generator=g)
    tv = torch.randn(B, Hkv, 37, d, generator=g)
    Kp = zb.PackedTensor(B, Hkv, d, 64, 64, 4, 2, "channel", zb.ZC_LAYOUT_ROW, max_chunks=1, device=DEV)
    Vp = zb.PackedTensor(B, Hkv, d, 64, 64, 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=1, device=DEV)
    lse = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
    out = zb.zc_decode_attention(q.to(DEV), Kp, Vp, tk.to(DEV), tv.to(DEV), 37, lse_out=lse)
    ref, lse_o, _ = zo.decode_attention(q.double().numpy(), tk.double().numpy(), tv.double().numpy())
    assert np.abs(out.cpu().double().numpy() - ref).max() < 1e-4
    assert np.abs(lse.cpu().numpy() - lse_o).max() < 1e-4


@pytest.mark.parametrize("B,Hq,Hkv,d,dtype,L0,bsel", [
    (2, 8, 2, 128, torch.bfloat16, 500, (0, 1)),      # grouped heads, few workgroups: one tail unit per wave
    (2, 4, 4, 128, torch.float16, 333, (0, 1)),       # one query head per KV head
    (1, 8, 8, 64, torch.float32, 257, (0,)),          # fp32: split weights, normalized codes
    (40, 8, 8, 64, torch.float16, 300, (0, 39)),      # more (batch, KV head) pairs than CUs: the tail shares waves by cost
])
def test_decode_many_chunks_and_tails(B, Hq, Hkv, d, dtype, L0, bsel):
    """A streaming cache of up to seven chunks (a prefill and six 100-token flushes, so
    most segments are a few half-blocks long) with tails from nothing to 700 tokens:
    every split of the packed cost line and of the tail over the waves is exercised,
    against the oracle's attention over the de-quantized GPU codes."""
    from tests.pipeline_check import packed_to_chunks
    g = torch.Generator().manual_seed(1234 + B + d)
    n_flush, T_max = 6, 700
    L_all = L0 + 100 * n_flush + T_max
    K = torch.randn(B, Hkv, L_all, d, generator=g).to(dtype)
    V = torch.randn(B, Hkv, L_all, d, generator=g).to(dtype)
    K[:, :, :, 3] *= 12.0                                        # an outlier channel
    Kd, Vd = K.to(DEV), V.to(DEV)
    lib = zb.load()
    k0, kt = int(0.4 * L0), 40
    cap_hi = lib.zc_arena_slots(k0 + n_flush * kt, 1 + n_flush)
    cap_lo = lib.zc_arena_slots(L0 - k0 + n_flush * (100 - kt), 1 + n_flush)
    Kp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, 4, 2, "channel", zb.ZC_LAYOUT_ROW, max_chunks=1 + n_flush, device=DEV)
    Vp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=1 + n_flush, device=DEV)
    atol = 1e-4 if dtype == torch.float32 else 2e-2
    n_packed = 0
    for c in range(1 + n_flush):
        n_new, k_new = (L0, k0) if c == 0 else (100, kt)
        sc = torch.rand(B, n_new, generator=g).to(DEV)
        sal, reg = zb.zc_select_salient(sc, k_new)
        sl = slice(n_packed, n_packed + n_new)
        zb.zc_quantize_pack(Kd[:, :, sl], sal, reg, Kp, pos_offset=n_packed)
        zb.zc_quantize_pack(Vd[:, :, sl], sal, reg, Vp, pos_offset=n_packed)
        n_packed += n_new
        if c not in (0, 1, n_flush):
            continue
        chunks_k, chunks_v = packed_to_chunks(Kp, bsel), packed_to_chunks(Vp, bsel)
        for T in (0, 1, 16, 17, 100, 300, 700):
            q = torch.randn(B, Hq, d, generator=g).to(dtype)
            lse = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
            tk, tv = Kd[:, :, n_packed:n_packed + T_max], Vd[:, :, n_packed:n_packed + T_max]
            out = zb.zc_decode_attention(q.to(DEV), Kp, Vp, tk if T else None, tv if T else None, T, lse_out=lse)
            sel = list(bsel)
            tko = K[sel, :, n_packed:n_packed + T].double().numpy() if T else None
            tvo = V[sel, :, n_packed:n_packed + T].double().numpy() if T else None
            Kc, Vc = zo.cache_matrices(chunks_k, chunks_v, Hkv, tko, tvo)
            ref, lse_o, _ = zo.decode_attention(q[sel].double().numpy(), Kc, Vc)
            err = np.abs(out[sel].cpu().double().numpy() - ref).max()
            lerr = np.abs(lse[sel].cpu().numpy() - lse_o).max()
            assert err <= atol and lerr <= max(atol, 1e-3) * 0.5, (c + 1, T, err, lerr)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_decode_more_chunks_than_travel_in_the_arguments(dtype):
    """Up to twelve chunk-table rows travel in the kernel arguments; a cache of 15 chunks
    makes the kernel read the table from device memory instead."""
    from tests.pipeline_check import packed_to_chunks
    B, Hq, Hkv, d, L0 = 2, 8, 4, 128, 230
    g = torch.Generator().manual_seed(77)
    sizes = [L0] + [int(torch.randint(5, 70, (1,), generator=g)) for _ in range(14)]
    T_max = 40
    L_all = sum(sizes) + T_max
    K = torch.randn(B, Hkv, L_all, d, generator=g).to(dtype)
    V = torch.randn(B, Hkv, L_all, d, generator=g).to(dtype)
    Kd, Vd = K.to(DEV), V.to(DEV)
    lib = zb.load()
    ks = [int(0.4 * n) for n in sizes]
    cap_hi = lib.zc_arena_slots(sum(ks), len(sizes))
    cap_lo = lib.zc_arena_slots(sum(sizes) - sum(ks), len(sizes))
    Kp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, 4, 2, "channel", zb.ZC_LAYOUT_ROW, max_chunks=len(sizes), device=DEV)
    Vp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=len(sizes), device=DEV)
    atol = 1e-4 if dtype == torch.float32 else 2e-2
    n_packed = 0
    bsel = [0, 1]
    for c, (n_new, k_new) in enumerate(zip(sizes, ks)):
        sal, reg = zb.zc_select_salient(torch.rand(B, n_new, generator=g).to(DEV), k_new)
        sl = slice(n_packed, n_packed + n_new)
        zb.zc_quantize_pack(Kd[:, :, sl], sal, reg, Kp, pos_offset=n_packed)
        zb.zc_quantize_pack(Vd[:, :, sl], sal, reg, Vp, pos_offset=n_packed)
        n_packed += n_new
        if c + 1 not in (12, 13, 15):                 # the last inline table, the first and a longer one in memory
            continue
        chunks_k, chunks_v = packed_to_chunks(Kp, bsel), packed_to_chunks(Vp, bsel)
        for T in (0, 23):
            q = torch.randn(B, Hq, d, generator=g).to(dtype)
            lse = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
            tk, tv = Kd[:, :, n_packed:n_packed + T_max], Vd[:, :, n_packed:n_packed + T_max]
            out = zb.zc_decode_attention(q.to(DEV), Kp, Vp, tk if T else None, tv if T else None, T, lse_out=lse)
            tko = K[:, :, n_packed:n_packed + T].double().numpy() if T else None
            tvo = V[:, :, n_packed:n_packed + T].double().numpy() if T else None
            Kc, Vc = zo.cache_matrices(chunks_k, chunks_v, Hkv, tko, tvo)
            ref, lse_o, _ = zo.decode_attention(q.double().numpy(), Kc, Vc)
            err = np.abs(out.cpu().double().numpy() - ref).max()
            lerr = np.abs(lse.cpu().numpy() - lse_o).max()
            assert err <= atol and lerr <= max(atol, 1e-3) * 0.5, (c + 1, T, err, lerr)


def test_decode_arena_full_to_its_capacity():
    """Arenas with no slack: the salient arena holds 100 tokens in 128 slots and the regular
    one 228 in 256, so the last 4-bit block ends exactly where the (batch) row of every
    per-slot array ends - the kernel must not depend on anything past it."""
    from tests.pipeline_check import packed_to_chunks
    B, Hq, Hkv, d, L, k = 3, 8, 4, 128, 328, 100
    g = torch.Generator().manual_seed(99)
    K = torch.randn(B, Hkv, L, d, generator=g).to(torch.float16)
    V = torch.randn(B, Hkv, L, d, generator=g).to(torch.float16)
    q = torch.randn(B, Hq, d, generator=g).to(torch.float16)
    sal, reg = zb.zc_select_salient(torch.rand(B, L, generator=g).to(DEV), k)
    for k_scheme in ("cst", "channel"):
        Kp = zb.PackedTensor(B, Hkv, d, 128, 256, 4, 2, k_scheme, zb.ZC_LAYOUT_ROW, max_chunks=1, device=DEV)
        Vp = zb.PackedTensor(B, Hkv, d, 128, 256, 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=1, device=DEV)
        assert Kp.c.cap_hi == 128 and Kp.tok_scale_hi.numel() == B * 128
        zb.zc_quantize_pack(K.to(DEV), sal, reg, Kp)
        zb.zc_quantize_pack(V.to(DEV), sal, reg, Vp)
        lse = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
        out = zb.zc_decode_attention(q.to(DEV), Kp, Vp, lse_out=lse)
        bsel = [0, 1, 2]
        Kc, Vc = zo.cache_matrices(packed_to_chunks(Kp, bsel), packed_to_chunks(Vp, bsel), Hkv)
        ref, lse_o, _ = zo.decode_attention(q.double().numpy(), Kc, Vc)
        assert np.abs(out.cpu().double().numpy() - ref).max() <= 2e-2
        assert np.abs(lse.cpu().numpy() - lse_o).max() <= 1e-3


def test_decode_randomized_shapes():
    """Thirty seeded draws of (batch, heads, group size, head_dim, dtype, bit widths, K scheme,
    prefill length, number and size of flushed chunks, tail length): the decode entry
    point against the oracle's attention over the de-quantized GPU codes."""
    from tests.pipeline_check import packed_to_chunks
    rng = np.random.Generator(np.random.PCG64(20240514))
    lib = zb.load()
    for case in range(30):
        d = int(rng.choice([64, 128]))
        G = int(rng.choice([1, 2, 4, 8]))
        Hkv = int(rng.choice([1, 2, 4, 8]))
        B = int(rng.choice([1, 2, 3, 37])) if Hkv * G <= 16 else int(rng.choice([1, 2]))
        dtype = [torch.bfloat16, torch.float16, torch.float32][int(rng.integers(3))]
        bits_hi, bits_lo = [(4, 2), (4, 4), (2, 2)][int(rng.integers(3))]
        k_scheme = ["channel", "cst"][int(rng.integers(2))]
        L0 = int(rng.integers(1, 700))
        n_flush = int(rng.integers(0, 4))
        T = int(rng.choice([0, 1, 15, 16, 33, 100, 257]))
        sizes = [L0] + [int(rng.integers(1, 130)) for _ in range(n_flush)]
        ks = [int(rng.integers(0, n + 1)) for n in sizes]
        g = torch.Generator().manual_seed(1000 + case)
        L_all = sum(sizes) + max(T, 1)
        K = torch.randn(B, Hkv, L_all, d, generator=g).to(dtype)
        V = torch.randn(B, Hkv, L_all, d, generator=g).to(dtype)
        Kd, Vd = K.to(DEV), V.to(DEV)
        cap_hi = lib.zc_arena_slots(sum(ks), len(sizes))
        cap_lo = lib.zc_arena_slots(sum(sizes) - sum(ks), len(sizes))
        Kp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, bits_hi, bits_lo, k_scheme, zb.ZC_LAYOUT_ROW, max_chunks=len(sizes), device=DEV)
        Vp = zb.PackedTensor(B, Hkv, d, cap_hi, cap_lo, bits_hi, bits_lo, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=len(sizes), device=DEV)
        n_packed = 0
        for n_new, k_new in zip(sizes, ks):
            sal, reg = zb.zc_select_salient(torch.rand(B, n_new, generator=g).to(DEV), k_new)
            sl = slice(n_packed, n_packed + n_new)
            zb.zc_quantize_pack(Kd[:, :, sl], sal, reg, Kp, pos_offset=n_packed)
            zb.zc_quantize_pack(Vd[:, :, sl], sal, reg, Vp, pos_offset=n_packed)
            n_packed += n_new
        bsel = sorted({0, B - 1})
        q = torch.randn(B, Hkv * G, d, generator=g).to(dtype)
        lse = torch.empty(B, Hkv * G, dtype=torch.float32, device=DEV)
        tk, tv = Kd[:, :, n_packed:], Vd[:, :, n_packed:]
        out = zb.zc_decode_attention(q.to(DEV), Kp, Vp, tk if T else None, tv if T else None, T, lse_out=lse)
        tko = K[bsel, :, n_packed:n_packed + T].double().numpy() if T else None
        tvo = V[bsel, :, n_packed:n_packed + T].double().numpy() if T else None
        Kc, Vc = zo.cache_matrices(packed_to_chunks(Kp, bsel), packed_to_chunks(Vp, bsel), Hkv, tko, tvo)
        ref, lse_o, _ = zo.decode_attention(q[bsel].double().numpy(), Kc, Vc)
        atol = 1e-4 if dtype == torch.float32 else 2e-2
        what = (case, B, Hkv, G, d, str(dtype), bits_hi, bits_lo, k_scheme, sizes, ks, T)
        assert np.abs(out[bsel].cpu().double().numpy() - ref).max() <= atol, what
        assert np.abs(lse[bsel].cpu().numpy() - lse_o).max() <= max(atol, 1e-3) * 0.5, what


@pytest.mark.parametrize("L", [600, 2000, 2700, 3300, 4300, 5600, 7000, 9000])
def test_decode_every_instance_of_the_reduce_kernel(L):
    """One prompt, two KV heads: the number of workgroups per head grows with the cache (about one
    per eight half-blocks, up to 32), and the reduce kernel has an instance for up to 8, 16, 24
    and 32 of them; without a tail the count is the cache's alone.  Every length against the
    oracle's attention over the de-quantized GPU codes, output and log-sum-exp."""
    from tests.pipeline_check import packed_to_chunks
    Hq, Hkv, d = 8, 2, 128
    g = torch.Generator().manual_seed(9000 + L)
    K = torch.randn(1, Hkv, L, d, generator=g).to(torch.bfloat16)
    V = torch.randn(1, Hkv, L, d, generator=g).to(torch.bfloat16)
    q = torch.randn(1, Hq, d, generator=g).to(torch.bfloat16)
    lib = zb.load()
    k = int(0.4 * L)
    sal, reg = zb.zc_select_salient(torch.rand(1, L, generator=g).to(DEV), k)
    Kp = zb.PackedTensor(1, Hkv, d, lib.zc_arena_slots(k, 1), lib.zc_arena_slots(L - k, 1), 4, 2, "channel", zb.ZC_LAYOUT_ROW, max_chunks=1, device=DEV)
    Vp = zb.PackedTensor(1, Hkv, d, lib.zc_arena_slots(k, 1), lib.zc_arena_slots(L - k, 1), 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=1, device=DEV)
    zb.zc_quantize_pack(K.to(DEV), sal, reg, Kp)
    zb.zc_quantize_pack(V.to(DEV), sal, reg, Vp)
    lse = torch.empty(1, Hq, dtype=torch.float32, device=DEV)
    out = zb.zc_decode_attention(q.to(DEV), Kp, Vp, None, None, 0, lse_out=lse)
    Kc, Vc = zo.cache_matrices(packed_to_chunks(Kp, [0]), packed_to_chunks(Vp, [0]), Hkv, None, None)
    ref, lse_o, _ = zo.decode_attention(q.double().numpy(), Kc, Vc)
    assert np.abs(out.cpu().double().numpy() - ref).max() <= 2e-2
    assert np.abs(lse.cpu().numpy() - lse_o).max() <= 1e-3


def test_decode_same_answer_under_any_split():
    """The same sequence alone (few workgroups: many waves per head, a workgroup per tail
    unit) and replicated 48 times (more heads than CUs: two or three workgroups per
    head, the tail sharing waves): the split of the cost line must not show in the
    result beyond the rounding of the partial sums."""
    Hq, Hkv, d, L, T = 16, 8, 128, 3000, 77
    g = torch.Generator().manual_seed(4242)
    K1 = torch.randn(1, Hkv, L + T, d, generator=g).to(torch.bfloat16)
    V1 = torch.randn(1, Hkv, L + T, d, generator=g).to(torch.bfloat16)
    q1 = torch.randn(1, Hq, d, generator=g).to(torch.bfloat16)
    sc1 = torch.rand(1, L, generator=g)
    lib = zb.load()
    k = 1200
    outs, lses = [], []
    for B in (1, 48):
        Kd, Vd = K1.expand(B, -1, -1, -1).contiguous().to(DEV), V1.expand(B, -1, -1, -1).contiguous().to(DEV)
        sal, reg = zb.zc_select_salient(sc1.expand(B, -1).contiguous().to(DEV), k)
        Kp = zb.PackedTensor(B, Hkv, d, lib.zc_arena_slots(k, 1), lib.zc_arena_slots(L - k, 1), 4, 2, "channel", zb.ZC_LAYOUT_ROW, max_chunks=1, device=DEV)
        Vp = zb.PackedTensor(B, Hkv, d, lib.zc_arena_slots(k, 1), lib.zc_arena_slots(L - k, 1), 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=1, device=DEV)
        zb.zc_quantize_pack(Kd[:, :, :L], sal, reg, Kp)
        zb.zc_quantize_pack(Vd[:, :, :L], sal, reg, Vp)
        lse = torch.empty(B, Hq, dtype=torch.float32, device=DEV)
        out = zb.zc_decode_attention(q1.expand(B, -1, -1).contiguous().to(DEV), Kp, Vp, Kd[:, :, L:], Vd[:, :, L:], T, lse_out=lse)
        outs.append(out.float().cpu())
        lses.append(lse.cpu())
    assert torch.equal(outs[1], outs[1][:1].expand_as(outs[1]))          # every replica alike (deterministic)
    assert (lses[1] - lses[0]).abs().max() <= 2e-5
    assert (outs[1] - outs[0]).abs().max() <= 2.0 ** -7 * outs[0].abs().max()    # one bf16 rounding step at most


def test_machine_peak_probes_run_and_copy_exactly():
    """The probes of bench.py --peaks: the copy is exact (ragged size, loop tail included), the
    read and the matrix-instruction loop launch and finish."""
    import ctypes as C
    import os
    lib = C.CDLL(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                              "paper_2405_14256_amd", "libzc_peaks.so"))
    lib.zc_peak_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.zc_peak_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.zc_peak_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    st = torch.cuda.current_stream().cuda_stream
    n = (37 << 20) + 16 * 12345                      # bytes: not a multiple of the grid's stride
    src = torch.randint(0, 2 ** 31 - 1, (n // 4,), dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    sink = torch.zeros(16, dtype=torch.float32, device=DEV)
    assert lib.zc_peak_copy(dst.data_ptr(), src.data_ptr(), n, st) == 0
    assert lib.zc_peak_read(src.data_ptr(), n, sink.data_ptr(), st) == 0
    assert lib.zc_peak_mfma(2, 64, 8, sink.data_ptr(), st) == 0
    assert lib.zc_peak_mfma(1, 64, 8, sink.data_ptr(), st) == 0
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert float(sink.abs().sum()) == 0.0
    # latency probes: the touch kernel adds up the words it read, the chase ends where the table says
    lib.zc_peak_empty.argtypes = [C.c_int, C.c_void_p]
    lib.zc_peak_touch.argtypes = [C.c_void_p, C.c_size_t, C.c_size_t, C.c_int, C.c_uint32, C.c_void_p, C.c_void_p]
    lib.zc_peak_chase.argtypes = [C.c_void_p, C.c_size_t, C.c_uint32, C.c_int, C.c_void_p, C.c_void_p]
    assert lib.zc_peak_empty(256, st) == 0
    words = torch.arange(4096, dtype=torch.int32, device=DEV)
    got = torch.zeros(8, dtype=torch.int32, device=DEV)
    assert lib.zc_peak_touch(words.data_ptr(), 4096 * 4, 4096, 8, 5, got.data_ptr(), st) == 0
    table = ((torch.arange(1000, dtype=torch.int64) * 7 + 3) % 1000).to(torch.int32)
    end = torch.zeros(1, dtype=torch.int32, device=DEV)
    assert lib.zc_peak_chase(table.to(DEV).data_ptr(), 1000, 11, 25, end.data_ptr(), st) == 0
    torch.cuda.synchronize()
    assert got.tolist() == [4 * (1024 * i % 4096) + 6 + 5 for i in range(8)]
    i = 11
    for _ in range(25):
        i = int(table[i])
    assert int(end[0]) == i


def test_pipeline_randomized_configurations():
    """Seeded draws over what the single-purpose tests fix: input law (all five workloads,
    scaled down), batch, heads and group size, K / V scheme (channelwise, CST, plain
    tokenwise), bit-width pair, input type, with and without streaming flushes (interval 64
    or 100) - the whole path against the oracle, every stage, at the usual bars."""
    rng = np.random.default_rng(11)
    names = ["tiny", "llama3_8b_4k", "mistral_7b_8k_b8", "llama2_13b_4k_b16", "llama3_8b_32k"]
    for case in range(12):
        base = WORKLOADS[names[int(rng.integers(len(names)))]]
        G = int(rng.choice([1, 2, 4, 8])); Hkv = int(rng.choice([1, 2, 4])); B = int(rng.choice([1, 2, 3]))
        L = int(rng.integers(120, 900))
        fi = int(rng.choice([0, 100, 100, 64]))
        steps = int(rng.integers(1, 12)) if not fi else int(fi * rng.integers(1, 3) + rng.integers(0, 20))
        ks, vs = [("channel", "cst"), ("cst", "cst"), ("channel", "token"), ("token", "cst")][int(rng.integers(4))]
        bh, bl = [(4, 2), (4, 2), (8, 4), (2, 2), (4, 4), (8, 2)][int(rng.integers(6))]
        dt = ["bf16", "fp16", "fp32"][int(rng.integers(3))]
        w = scaled(base, bits_hi=bh, bits_lo=bl, dtype=dt, B=B, Hq=Hkv * G, Hkv=Hkv, L=L, decode_steps=steps,
                   index=base.index + 100 + case, needles=min(base.needles, 4))
        print(f"case {case}: {base.name} B={B} Hq={Hkv * G} Hkv={Hkv} d={w.d} L={L} steps={steps} flush={fi} "
              f"{ks}/{vs} bits={bh}/{bl} {dt}", flush=True)
        run_pipeline_check(w, k_scheme=ks, v_scheme=vs, flush_interval=fi or None)


def test_graph_replays_reproduce_the_eager_step():
    """bench.py times replayed HIP graphs: the step of a scaled workload with a streaming
    flush, captured stage by stage as the benchmark does, must leave exactly what the eager
    step leaves - scores, index lists, every packed array, all decode outputs and the flush's
    scores - on each of three replays, with eager work and synchronizations in between."""
    import bench
    w = scaled(WORKLOADS["llama2_13b_4k_b16"], B=2, Hq=8, Hkv=8, L=520, decode_steps=130)
    hp = bench.HotPath(w)

    def snapshot():
        torch.cuda.synchronize()
        parts = [hp.scores, hp.sal, hp.reg, hp.out] + hp.tail_scores + hp.sal_t + hp.reg_t
        for P in (hp.Kp, hp.Vp):
            parts += [P.codes_hi, P.codes_lo, P.tok_scale_hi, P.tok_zero_hi, P.tok_scale_lo, P.tok_zero_lo,
                      P.chan_scale, P.chan_zero, P.chunk_table]
        return [t.clone() for t in parts], (hp.Kp.chunks, hp.Vp.chunks)

    hp.step()
    want, want_chunks = snapshot()
    hp.step()                                            # eager again: the step is repeatable
    again, _ = snapshot()
    assert all(torch.equal(a, b) for a, b in zip(want, again))
    stages = hp.stages()
    graphs = []
    for _, fn, _, _ in stages:                           # captured in execution order
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        graphs.append(g)
    assert (hp.Kp.chunks, hp.Vp.chunks) == want_chunks   # capture advanced the host bookkeeping like a step
    for rep in range(3):
        for t in [hp.scores, hp.out, hp.Kp.codes_lo, hp.Vp.codes_hi] + hp.tail_scores:
            t.zero_()                                    # eager work between the replays
        torch.cuda.synchronize()
        for g in graphs:
            g.replay()
        got, _ = snapshot()
        for i, (a, b) in enumerate(zip(want, got)):
            assert torch.equal(a, b), f"replay {rep}: array {i} differs from the eager step"


def test_results_are_deterministic():
    w = scaled(WORKLOADS["llama3_8b_4k"], L=900)
    from paper_2405_14256_amd import probes
    from paper_2405_14256_amd.workloads import make_decode_step, make_prefill
    inp = make_prefill(w)
    Q, K, V = (inp[n].to(DEV) for n in ("Q", "K", "V"))
    pos = torch.from_numpy(probes.probe_positions(w.L, w.probe_ratio, 1)).to(DEV)
    outs = []
    for _ in range(2):
        sc = zb.zc_probe_saliency(Q, K, pos)
        sal, reg = zb.zc_select_salient(sc, w.k_salient)
        Kp = zb.PackedTensor(w.B, w.Hkv, w.d, 448, 576, 4, 2, "channel", zb.ZC_LAYOUT_ROW, max_chunks=1, device=DEV)
        Vp = zb.PackedTensor(w.B, w.Hkv, w.d, 448, 576, 4, 2, "cst", zb.ZC_LAYOUT_TGROUP, max_chunks=1, device=DEV)
        zb.zc_quantize_pack(K, sal, reg, Kp)
        zb.zc_quantize_pack(V, sal, reg, Vp)
        o = zb.zc_decode_attention(make_decode_step(w, 0)["q"].to(DEV), Kp, Vp)
        torch.cuda.synchronize()
        outs.append((sc.clone(), sal.clone(), Kp.codes_lo.clone(), Vp.codes_hi.clone(), Vp.tok_scale_lo.clone(), o.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_decode_timeline_mode_of_the_benchmark():
    """bench.py --decode-timeline: the traced build of the library runs a decode call and its
    time stamps come out in order (entry <= arguments <= operand <= first block <= half-blocks
    done <= folded <= barrier <= stored; the reduce kernel after the first kernel's last store)."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--decode-timeline"], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr[-2000:]
    d = json.loads([ln for ln in out.stdout.splitlines() if ln.startswith("{")][-1])
    m = d["k_decode_mfma"]
    order = ["entry", "arguments in registers", "query operand built", "first block in LDS", "half-blocks done",
             "segments folded", "at the merge barrier", "result stored"]
    med = [m[k]["median"] for k in order]
    assert all(a <= b for a, b in zip(med, med[1:])), med
    assert m["entry"]["min"] == 0.0 and m["result stored"]["max"] < 50.0
    r = d["k_decode_reduce"]
    assert m["result stored"]["max"] <= r["entry"]["min"] <= r["partials landed"]["median"] <= r["end"]["median"]
    assert 1.0 < d["call_period_us"] < 100.0
