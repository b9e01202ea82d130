"""Pins for the oracle's decode attention (Eq. 4) over the de-quantized cache
and for the streaming (Algorithm 3) bookkeeping."""
import math

import numpy as np
from scipy.special import softmax as scipy_softmax

from oracle import zipcache_oracle as zo


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _setup(seed=30, B=2, Hq=4, Hkv=2, L=24, d=8):
    Q, K, V = _rand((B, Hq, L, d), seed), _rand((B, Hkv, L, d), seed + 1), _rand((B, Hkv, L, d), seed + 2)
    K[..., 1] *= 8
    return Q, K, V


def test_decode_is_library_softmax_attention():
    B, Hq, Hkv, N, d = 2, 4, 2, 13, 8
    q, Kc, Vc = _rand((B, Hq, d), 31), _rand((B, Hkv, N, d), 32), _rand((B, Hkv, N, d), 33)
    out, lse, probs = zo.decode_attention(q, Kc, Vc)
    for b in range(B):
        for h in range(Hq):
            logits = Kc[b, h // 2] @ q[b, h] / math.sqrt(d)
            a = scipy_softmax(logits)
            assert np.allclose(probs[b, h], a, atol=1e-14)
            assert np.allclose(out[b, h], a @ Vc[b, h // 2], atol=1e-13)
            assert np.isclose(lse[b, h], math.log(np.exp(logits).sum()))
    # decode at position N-1 is the last row of prefill attention
    Qf = _rand((N, d), 34)
    A = zo.causal_attention(Qf, Kc[0, 0])
    _, _, p = zo.decode_attention(Qf[None, None, -1], Kc[:1, :1], Vc[:1, :1])
    assert np.allclose(p[0, 0], A[-1], atol=1e-14)


def test_sixteen_bit_cache_equals_unquantized_attention():
    Q, K, V = _setup()
    B, Hq, L, d = Q.shape
    scores, _ = zo.saliency_scores(Q, K, np.arange(L))
    ck, cv, sal, reg = zo.compress_prefill(K, V, scores, 10, bits_hi=16, bits_lo=16)
    Kc, Vc = zo.cache_matrices([ck], [cv], 2)
    q = _rand((B, Hq, d), 35)
    out, _, _ = zo.decode_attention(q, Kc, Vc)
    # reference: unquantized, tokens in the cache's order (salient first, then regular)
    order = np.concatenate([sal, reg], axis=1)
    Kp = np.stack([K[b][:, order[b]] for b in range(B)])
    Vp = np.stack([V[b][:, order[b]] for b in range(B)])
    ref, _, _ = zo.decode_attention(q, Kp, Vp)
    assert np.allclose(out, ref, rtol=1e-4, atol=1e-4)
    ref_nat, _, _ = zo.decode_attention(q, K, V)          # permutation invariance of attention
    assert np.allclose(ref, ref_nat, atol=1e-12)


def test_cache_order_and_dequant_bound():
    Q, K, V = _setup(40)
    B, Hq, L, d = Q.shape
    scores, _ = zo.saliency_scores(Q, K, np.array([5, 11, 22, 23]))
    ck, cv, sal, reg = zo.compress_prefill(K, V, scores, 9)
    assert sal.shape == (B, 9) and reg.shape == (B, L - 9)
    for b in range(B):
        assert sorted(set(sal[b]) | set(reg[b])) == list(range(L)) and not set(sal[b]) & set(reg[b])
        assert list(sal[b]) == sorted(sal[b]) and list(reg[b]) == sorted(reg[b])
        top = sorted(range(L), key=lambda i: (-scores[b, i], i))[:9]
        assert sorted(top) == list(sal[b])
    Kc, Vc = zo.cache_matrices([ck], [cv], 2)
    # slot j of the cache holds token order[j]; error bounded by half a step
    order = np.concatenate([sal, reg], axis=1)
    RV = zo.token_rows(V)
    step_hi = cv.hi.chan_scale[:, None, :] * cv.hi.tok_scale[:, :, None]
    step_lo = cv.lo.chan_scale[:, None, :] * cv.lo.tok_scale[:, :, None]
    step = np.concatenate([step_hi, step_lo], axis=1)
    for b in range(B):
        got = zo.token_rows(Vc)[b]
        assert np.all(np.abs(got - RV[b, order[b]]) <= step[b] / 2 + 1e-12)
    # 4-bit salient tokens are reconstructed better than 2-bit regular ones
    e_hi = np.abs(cv.hi.dequant() - np.stack([RV[b, sal[b]] for b in range(B)])).mean()
    e_lo = np.abs(cv.lo.dequant() - np.stack([RV[b, reg[b]] for b in range(B)])).mean()
    assert e_hi < e_lo


def test_streaming_flush_equals_compressing_the_window():
    """A flush of the tail is a prefill-style compression of those tokens with
    the window's scores; decode over (chunks + tail) sees every token once."""
    B, Hq, Hkv, d, L = 1, 2, 1, 8, 16
    Q, K, V = _rand((B, Hq, L, d), 50), _rand((B, Hkv, L, d), 51), _rand((B, Hkv, L, d), 52)
    scores, _ = zo.saliency_scores(Q, K, np.array([7, 14, 15]))
    ck, cv, _, _ = zo.compress_prefill(K, V, scores, 6)
    cache = zo.StreamingCache(Hkv=Hkv, interval=10, chunks_K=[ck], chunks_V=[cv], n_packed=L)
    probes = {3, 8, 9}
    steps = []
    for j in range(10):
        q, kn, vn = _rand((B, Hq, d), 60 + j), _rand((B, Hkv, d), 80 + j), _rand((B, Hkv, d), 100 + j)
        out, lse, probs = cache.step(q, kn, vn, j in probes)
        steps.append((q, probs))
        assert probs.shape[-1] == L + j + 1 and np.allclose(probs.sum(-1), 1.0)
    tk = np.stack(cache.tail_k, axis=2); tv = np.stack(cache.tail_v, axis=2)
    sc = cache.tail_scores()
    # brute force: window part of the recorded probability rows
    for t in range(10):
        vis = [j for j in sorted(probes) if j >= t]
        ref = np.mean([[steps[j][1][0, h, L + t] for j in vis] for h in range(Hq)], axis=0).sum() / len(vis)
        assert np.isclose(sc[0, t], ref, atol=1e-14)
    scores_f, sal, reg = cache.flush(4)
    ck2, cv2, sal2, reg2 = zo.compress_prefill(tk, tv, sc, 4)
    assert np.array_equal(sal, sal2) and np.array_equal(cache.chunks_V[1].hi.codes, cv2.hi.codes)
    assert np.array_equal(cache.chunks_K[1].lo.codes, ck2.lo.codes)
    assert np.array_equal(cache.chunks_K[1].hi.idx, sal2 + L)
    assert cache.n_packed == L + 10 and not cache.tail_k
    Kc, _ = zo.cache_matrices(cache.chunks_K, cache.chunks_V, Hkv)
    assert Kc.shape[2] == L + 10
