"""Pins for the oracle's attention, saliency and selection functions.

Each pin ties the oracle to something other than its own code: a brute-force
loop over the printed definition (Eq. 2, 7, 8, 9), a closed form, a library
routine on a special case, or a structural fact the paper states.
"""
import math

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import zipcache_oracle as zo


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def brute_attention(q, k):
    """Eq. 2 written as scalar loops (causal)."""
    L, d = q.shape
    A = [[0.0] * L for _ in range(L)]
    for p in range(L):
        logits = [sum(q[p][c] * k[i][c] for c in range(d)) / math.sqrt(d) for i in range(p + 1)]
        mx = max(logits)
        ex = [math.exp(v - mx) for v in logits]
        Z = sum(ex)
        for i in range(p + 1):
            A[p][i] = ex[i] / Z
    return np.array(A)


def test_causal_attention_matches_brute_force_and_library():
    q, k = _rand((9, 4), 1), _rand((9, 4), 2)
    A = zo.causal_attention(q, k)
    assert np.allclose(A, brute_attention(q, k), atol=1e-14)
    # library softmax row by row on the visible prefix
    for p in range(9):
        ref = scipy_softmax((k[: p + 1] @ q[p]) / 2.0)
        assert np.allclose(A[p, : p + 1], ref, atol=1e-14)
        assert np.all(A[p, p + 1:] == 0.0)
    assert np.allclose(A.sum(1), 1.0)
    assert A[0, 0] == 1.0


def test_operands_not_transposed():
    # q and k play different roles: swapping them must change the result.
    q, k = _rand((6, 3), 3), _rand((6, 3), 4)
    assert not np.allclose(zo.causal_attention(q, k), zo.causal_attention(k, q))
    # one-hot construction: q_p = e_0 * t, keys k_i = e_0 * i  -> logits grow with i
    q = np.zeros((4, 2)); q[:, 0] = 2.0
    k = np.zeros((4, 2)); k[:, 0] = np.arange(4)
    A = zo.causal_attention(q, k)
    assert A[3, 3] > A[3, 2] > A[3, 1] > A[3, 0]


def test_uniform_attention_closed_form():
    """Q = 0 gives A[p, i] = 1/(p+1); accumulated score = H_n - H_i and the
    normalized score divides by n - i (Section 4.2's bias argument)."""
    n, d = 17, 4
    Q = np.zeros((1, 1, n, d)); K = _rand((1, 1, n, d), 5)
    H = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, n + 1))])
    acc, _ = zo.saliency_scores(Q, K, np.arange(n), normalized=False)
    nrm, _ = zo.saliency_scores(Q, K, np.arange(n))
    exp_acc = H[n] - H[np.arange(n)]
    assert np.allclose(acc[0], exp_acc, atol=1e-13)
    assert np.allclose(nrm[0], exp_acc / (n - np.arange(n)), atol=1e-13)
    assert acc[0, 0] > 1.0 and np.isclose(acc[0, -1], 1.0 / n)
    # probe subset
    R = np.array([3, 8, 16])
    sub, _ = zo.saliency_scores(Q, K, R)
    for i in range(n):
        vis = R[R >= i]
        assert np.isclose(sub[0, i], sum(1.0 / (p + 1) for p in vis) / len(vis))


def test_unmasked_count_is_n_minus_i_with_all_rows():
    n = 23
    assert np.array_equal(zo.unmasked_count(np.arange(n), n), n - np.arange(n))
    # the first token accumulates l values, the last accumulates one
    assert zo.unmasked_count(np.arange(n), n)[0] == n
    assert zo.unmasked_count(np.arange(n), n)[-1] == 1
    assert np.array_equal(zo.unmasked_count(np.array([2, 5]), 7), [2, 2, 2, 1, 1, 1, 0])


def test_scores_all_rows_equal_full_matrix_definition():
    """With every row a probe, Eq. 9 substituted in Eq. 8 is Eq. 8 on the full
    matrix: brute force per head, mean over query heads, GQA head mapping."""
    B, Hq, Hkv, L, d = 2, 4, 2, 11, 4
    Q, K = _rand((B, Hq, L, d), 6), _rand((B, Hkv, L, d), 7)
    s, per_head = zo.saliency_scores(Q, K, np.arange(L))
    for b in range(B):
        tot = np.zeros(L)
        for h in range(Hq):
            A = brute_attention(Q[b, h], K[b, h // 2])
            col = np.array([sum(A[p][i] for p in range(L)) / (L - i) for i in range(L)])
            assert np.allclose(per_head[b, h], col, atol=1e-13)
            tot += col
        assert np.allclose(s[b], tot / Hq, atol=1e-13)


def test_probe_rows_are_rows_of_full_matrix():
    L, d = 14, 8
    q, k = _rand((L, d), 8), _rand((L, d), 9)
    A = zo.causal_attention(q, k)
    pos = np.array([2, 7, 13])
    Ap, lse = zo.probe_attention(q[pos], pos, k)
    assert np.allclose(Ap, A[pos], atol=1e-14)
    # single probe: score_i = A[p, i] on visible columns, 0 beyond (no probe sees them)
    s, _ = zo.saliency_scores(q[None, None], k[None, None], np.array([7]))
    assert np.allclose(s[0, :8], A[7, :8], atol=1e-14)
    assert np.all(s[0, 8:] == 0.0)
    # conservation: every probe row sums to 1, so the accumulated scores sum to P
    acc, _ = zo.saliency_scores(q[None, None], k[None, None], pos, normalized=False)
    assert np.isclose(acc.sum(), len(pos))
    # log-normaliser is the log of the row's partition function
    S = (q[pos] @ k.T) / math.sqrt(d)
    for r, p in enumerate(pos):
        assert np.isclose(lse[r], math.log(sum(math.exp(v) for v in S[r, : p + 1])))


def test_external_normaliser():
    """A probe whose softmax also covered other tokens: probabilities on the
    window are exp(logit - lse_total)."""
    d = 4
    q = _rand((3, d), 10); k_old = _rand((5, d), 11); k_win = _rand((3, d), 12)
    pos = np.array([0, 1, 2])
    lse_tot = []
    for j in range(3):
        logits = np.concatenate([k_old @ q[j], k_win[: j + 1] @ q[j]]) / math.sqrt(d)
        lse_tot.append(math.log(np.exp(logits).sum()))
    A, _ = zo.probe_attention(q, pos, k_win, lse=np.array(lse_tot))
    for j in range(3):
        full = scipy_softmax(np.concatenate([k_old @ q[j], k_win[: j + 1] @ q[j]]) / math.sqrt(d))
        assert np.allclose(A[j, : j + 1], full[5:], atol=1e-14)
        assert np.all(A[j, j + 1:] == 0)


def test_sm_scale_default_and_override():
    q, k = _rand((5, 16), 13), _rand((5, 16), 14)
    assert np.allclose(zo.causal_attention(q, k), zo.causal_attention(q, k, 0.25))
    assert not np.allclose(zo.causal_attention(q, k), zo.causal_attention(q, k, 1.0))


@pytest.mark.parametrize("k", [0, 1, 5, 12])
def test_select_matches_sorted_brute_force(k):
    rng = np.random.default_rng(15)
    score = rng.integers(0, 4, 12).astype(np.float64)  # many ties
    sal, reg = zo.select_salient(score, k)
    brute = sorted(range(12), key=lambda i: (-score[i], i))[:k]
    assert list(sal) == sorted(brute)
    assert list(reg) == sorted(set(range(12)) - set(brute))
    # stable library sort agrees
    lib = np.argsort(-score, kind="stable")[:k]
    assert set(lib) == set(sal)


def test_select_tie_goes_to_lower_index():
    sal, reg = zo.select_salient(np.array([1.0, 3.0, 3.0, 3.0, 0.5]), 2)
    assert list(sal) == [1, 2] and list(reg) == [0, 3, 4]


def test_prefill_attention_against_a_scalar_loop_and_library_routines():
    """Algorithm 2's attention output and row normalisers: a scalar-loop evaluation of
    o_p = sum_{i<=p} softmax_i(q_p . k_i / sqrt(d)) v_i with the grouped-head mapping,
    scipy's logsumexp for the normaliser, and the special cases that have closed forms
    (first row copies v_0; equal values are reproduced; Q = 0 gives running means)."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(12)
    B, Hq, Hkv, L, d = 2, 4, 2, 9, 8
    Q = rng.standard_normal((B, Hq, L, d)); K = rng.standard_normal((B, Hkv, L, d)); V = rng.standard_normal((B, Hkv, L, d))
    O, lse = zo.prefill_attention(Q, K, V)
    G = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            for p in range(L):
                logits = [sum(Q[b, h, p, c] * K[b, h // G, i, c] for c in range(d)) / math.sqrt(d) for i in range(p + 1)]
                mx = max(logits)
                w = [math.exp(x - mx) for x in logits]
                for c in range(d):
                    want = sum(w[i] * V[b, h // G, i, c] for i in range(p + 1)) / sum(w)
                    assert abs(O[b, h, p, c] - want) < 1e-12
                assert abs(lse[b, h, p] - logsumexp(logits)) < 1e-12
    assert np.allclose(O[:, :, 0], np.repeat(V[:, :, 0], G, axis=1))             # the first token sees only itself
    assert np.allclose(zo.prefill_attention(Q, K, np.ones_like(V) * 2.5)[0], 2.5)   # a convex combination
    O0, lse0 = zo.prefill_attention(np.zeros_like(Q), K, V)                      # uniform attention: running means
    means = np.cumsum(V, axis=2) / np.arange(1, L + 1)[None, None, :, None]
    assert np.allclose(O0, np.repeat(means, G, axis=1)) and np.allclose(lse0, np.log(np.arange(1, L + 1)))
    # the probe rows of Eq. 9 are rows of the same matrix: re-normalising with these log-normalisers
    # reproduces them
    pos = np.array([2, 5, 8])
    A_rows, lse_rows = zo.probe_attention(Q[1, 3, pos], pos, K[1, 1])
    assert np.allclose(lse_rows, lse[1, 3, pos])
    assert np.allclose(A_rows @ V[1, 1], O[1, 3, pos])
    # an override of the softmax scale is honoured
    O2, _ = zo.prefill_attention(Q, K, V, sm_scale=0.3)
    assert np.allclose(O2[0, 1], zo.causal_attention(Q[0, 1], K[0, 0], 0.3) @ V[0, 0]) and not np.allclose(O2, O)
