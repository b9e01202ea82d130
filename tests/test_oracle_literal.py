"""Pins of the oracle's literal reading of Algorithm 3 (explicit probe rows, re-compression
of everything but the newest window).  The paper's text is ambiguous here, so nothing it
prints pins this reading ("parity unpinned" by the paper); what is pinned is that each piece
is what it says it is: Eq. 8 on explicit rows equals Eq. 8 through the probe-attention path,
the re-compression equals Algorithm 2's compression of the token-ordered cache, rounding to
a storage type equals a library conversion, and at 16 bits the cache loses nothing."""
import numpy as np
import pytest
import torch

from oracle import zipcache_oracle as zo


def test_round_to_storage_types_matches_library_conversions():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(50000) * rng.choice([1e-4, 1.0, 300.0], 50000)).astype(np.float32).astype(np.float64)
    x = np.concatenate([x, [0.0, -0.0, 1.0, 1.00390625, 1.01171875, -2.5, 65280.0]])
    for name, tt in (("bf16", torch.bfloat16), ("fp16", torch.float16), ("fp32", torch.float32)):
        want = torch.from_numpy(x).float().to(tt).double().numpy()
        keep = np.isfinite(want)
        assert np.array_equal(zo.round_to_dtype(x, name)[keep], want[keep]), name
    # a float64 value just past a bf16 midpoint goes to the far neighbour (a detour through fp32,
    # which rounds it onto the midpoint first, would send it to the even one)
    assert zo.round_to_dtype(np.array([-0.73632815]), "bf16")[0] == -0.73828125
    # exact ties go to the even significand
    assert zo.round_to_dtype(np.array([1.00390625]), "bf16")[0] == 1.0            # 1 + 2^-8: tie, even below
    assert zo.round_to_dtype(np.array([1.01171875]), "bf16")[0] == 1.015625       # 1 + 3 * 2^-8: tie, even above


def test_saliency_from_explicit_rows_is_eq8():
    """rows_saliency on the rows of A_probe equals saliency_scores (which never forms them as
    an argument): Eq. 8 either way; and the unnormalized variant is Eq. 7."""
    rng = np.random.default_rng(4)
    B, Hq, Hkv, L, d = 2, 4, 2, 23, 8
    Q = rng.standard_normal((B, Hq, L, d)); K = rng.standard_normal((B, Hkv, L, d))
    pos = np.array([3, 9, 15, 21, 22])
    want, _ = zo.saliency_scores(Q, K, pos)
    want_acc, _ = zo.saliency_scores(Q, K, pos, normalized=False)
    rows = []
    for p in pos:
        r = np.zeros((B, Hq, p + 1))
        for b in range(B):
            for h in range(Hq):
                r[b, h] = zo.probe_attention(Q[b, h, [p]], np.array([p]), K[b, h // 2])[0][0, :p + 1]
        rows.append(r)
    got = zo.rows_saliency(rows)
    assert np.allclose(got[:, :L], want[:, :23], rtol=1e-12, atol=1e-15)
    assert np.allclose(zo.rows_saliency(rows, normalized=False), want_acc, rtol=1e-12, atol=1e-15)
    # hand-worked: two rows over 2 and 3 tokens, one head
    r1 = np.array([[[0.25, 0.75]]]); r2 = np.array([[[0.5, 0.25, 0.25]]])
    assert np.allclose(zo.rows_saliency([r1, r2]), [[0.375, 0.5, 0.25]])


def _run(cache, rng, B, Hq, Hkv, d, steps, probe_every, ratio):
    outs = []
    for j in range(steps):
        q = rng.standard_normal((B, Hq, d)); k = rng.standard_normal((B, Hkv, d)); v = rng.standard_normal((B, Hkv, d))
        out, lse, row = cache.step(q, k, v, is_probe=(j % cache.interval) % probe_every == probe_every - 1)
        outs.append((q, out, lse, row))
        if (j + 1) % cache.interval == 0:
            outs.append(cache.recompress(ratio))
    return outs


def test_literal_recompression_is_algorithm2_on_the_token_ordered_cache():
    rng = np.random.default_rng(5)
    B, Hq, Hkv, d, L, I = 2, 4, 2, 8, 30, 10
    K0 = rng.standard_normal((B, Hkv, L, d)); V0 = rng.standard_normal((B, Hkv, L, d))
    sc0 = rng.random((B, L))
    ck, cv, _, _ = zo.compress_prefill(K0, V0, sc0, 12)
    cache = zo.LiteralStreamingCache(Hkv=Hkv, interval=I, chunk_K=ck, chunk_V=cv, n_packed=L, store_dtype="fp32")
    fed_k, fed_v = [], []
    for j in range(2 * I):
        q = rng.standard_normal((B, Hq, d)); k = rng.standard_normal((B, Hkv, d)); v = rng.standard_normal((B, Hkv, d))
        fed_k.append(k); fed_v.append(v)
        out, lse, row = cache.step(q, k, v, is_probe=j % 3 == 2)
        n = L + j + 1
        assert row.shape == (B, Hq, n) and np.allclose(row.sum(-1), 1.0)
        # the row is in token order: its last entry belongs to the token just appended
        Kt, Vt = cache.token_matrices()
        assert np.allclose(Kt[:, :, -1], k) and np.allclose(Vt[:, :, -1], v)
        logits = np.einsum("bhd,bhnd->bhn", q, np.repeat(Kt, Hq // Hkv, axis=1)) / np.sqrt(d)
        # (token_matrices rounds the packed part to the storage type: fp32 here, a 1e-7 effect)
        want = np.exp(logits - logits.max(-1, keepdims=True)); want /= want.sum(-1, keepdims=True)
        assert np.allclose(row, want, atol=1e-6)
        assert np.allclose(out, np.einsum("bhn,bhnd->bhd", want, np.repeat(Vt, Hq // Hkv, axis=1)), atol=1e-6)
        if (j + 1) % I == 0:
            rows = list(cache.rows)
            m = n - I
            scores, sal, reg = cache.recompress(0.4)
            # brute force of the same step: Eq. 8 over the window's rows, Algorithm 2's split and
            # quantizers on the m oldest tokens of the token-ordered cache
            want_sc = zo.rows_saliency(rows)[:, :m]
            assert np.array_equal(scores, want_sc) and scores.shape == (B, m)
            k_sal = int(np.floor(0.4 * m + 1e-9))
            for b in range(B):
                s_o, r_o = zo.select_salient(want_sc[b], k_sal)
                assert np.array_equal(sal[b], s_o) and np.array_equal(reg[b], r_o)
            ref_k = zo.compress_tensor(Kt[:, :, :m], sal, reg, 4, 2, "channel")
            ref_v = zo.compress_tensor(Vt[:, :, :m], sal, reg, 4, 2, "cst")
            for got, ref in ((cache.chunk_K, ref_k), (cache.chunk_V, ref_v)):
                assert np.array_equal(got.hi.codes, ref.hi.codes) and np.array_equal(got.lo.codes, ref.lo.codes)
                assert np.array_equal(got.hi.idx, sal) and np.array_equal(got.lo.idx, reg)
            # every token is in exactly one place: m compressed, the newest window in full precision
            assert cache.n_packed == m and len(cache.fp_k) == I and not cache.rows
            assert np.array_equal(np.stack(cache.fp_k, 2), np.stack(fed_k[-I:], 2))
            allpos = np.sort(np.concatenate([cache.chunk_K.hi.idx, cache.chunk_K.lo.idx], axis=1), axis=1)
            assert np.array_equal(allpos, np.tile(np.arange(m), (B, 1)))


def test_literal_cache_at_16_bits_is_unquantized_attention():
    rng = np.random.default_rng(6)
    B, Hq, Hkv, d, L, I = 1, 2, 2, 8, 20, 8
    K0 = rng.standard_normal((B, Hkv, L, d)); V0 = rng.standard_normal((B, Hkv, L, d))
    ck, cv, _, _ = zo.compress_prefill(K0, V0, rng.random((B, L)), 8, 16, 16)
    cache = zo.LiteralStreamingCache(Hkv=Hkv, interval=I, bits_hi=16, bits_lo=16, chunk_K=ck, chunk_V=cv, n_packed=L,
                                     store_dtype="fp32")
    Kall, Vall = [K0], [V0]
    for j in range(3 * I):
        q = rng.standard_normal((B, Hq, d)); k = rng.standard_normal((B, Hkv, d)); v = rng.standard_normal((B, Hkv, d))
        Kall.append(k[:, :, None]); Vall.append(v[:, :, None])
        out, _, _ = cache.step(q, k, v, is_probe=j % 2 == 1)
        ref, _, _ = zo.decode_attention(q, np.concatenate(Kall, 2), np.concatenate(Vall, 2))
        assert np.abs(out - ref).max() < 2e-3          # three rounds of 16-bit re-quantization
        if (j + 1) % I == 0:
            cache.recompress(0.5)


def test_a_token_can_change_subsets_under_the_literal_reading():
    """What distinguishes the literal reading: a token compressed as regular can later become
    salient (and the other way round), because every window re-ranks the whole older cache."""
    rng = np.random.default_rng(7)
    B, Hq, Hkv, d, L, I = 1, 2, 1, 8, 16, 4
    K0 = rng.standard_normal((B, Hkv, L, d)); V0 = rng.standard_normal((B, Hkv, L, d))
    sc0 = np.linspace(1.0, 0.0, L)[None]                       # prefill: the first tokens are salient
    ck, cv, sal0, _ = zo.compress_prefill(K0, V0, sc0, 4)
    cache = zo.LiteralStreamingCache(Hkv=Hkv, interval=I, chunk_K=ck, chunk_V=cv, n_packed=L)
    target = K0[0, 0, L - 1] * 4.0                             # queries that look at the last prefill token
    for j in range(I):
        q = np.tile(target, (B, Hq, 1))
        cache.step(q, rng.standard_normal((B, Hkv, d)) * 0.1, rng.standard_normal((B, Hkv, d)), is_probe=True)
    _, sal1, _ = cache.recompress(0.25)
    assert L - 1 not in sal0[0] and L - 1 in sal1[0]
