"""Pins for the oracle's quantizers (Eq. 5, Eq. 6, Algorithm 1) and the
compression-ratio accounting (Appendix A, Table 1)."""
import os

import numpy as np
import pytest

from oracle import zipcache_oracle as zo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(path):
    with open(os.path.join(GOLDEN, path)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---- Eq. 5 -----------------------------------------------------------------

def test_hand_worked_example():
    # x = [-1, 0, 0.5, 2], 2 bits: s = 3/3 = 1, z = -round(-1) = 1,
    # codes = clip(round(x)+1) = [0, 1, 1 (0.5 rounds to even 0), 3]
    x = np.array([-1.0, 0.0, 0.5, 2.0])
    s, z = zo.quant_params(x.min(), x.max(), 2)
    assert s == 1.0 and z == 1.0
    codes, _ = zo.quantize(x, x.min(), x.max(), 2)
    assert list(codes) == [0, 1, 1, 3]
    assert list(zo.dequantize(codes, s, z)) == [-1.0, 0.0, 0.0, 2.0]
    # half-to-even: 1.5 -> 2, 2.5 -> 2 (extrema 0 and 15 at 4 bits give s = 1, z = 0)
    assert list(zo.quantize(np.array([1.5, 2.5]), 0.0, 15.0, 4)[0]) == [2, 2]
    # round first, then add z (Eq. 5): with z odd the order decides a tie.
    # x in [-3, 12], 4 bits: s = 1, z = 3; 0.5 -> round(0.5) + 3 = 3, not round(3.5) = 4
    assert list(zo.quantize(np.array([0.5, 1.5]), -3.0, 12.0, 4)[0]) == [3, 5]


def test_exact_ties_survive_a_coarse_grid():
    """Inputs on a dyadic grid that sit exactly halfway between two codes must
    round half-to-even even when s = (max - min) / (2^k - 1) is not representable.
    Range 0.625 at 4 bits: s = 1/24, x / s = 24 x, z = -round(-0.25 * 24) = 6."""
    lo, hi = -0.25, 0.375
    x = np.array([1, 3, 5, -1, -3]) / 16.0          # 24 x = 1.5, 4.5, 7.5, -1.5, -4.5
    codes, pre = zo.quantize(x, lo, hi, 4)
    assert zo.quant_params(lo, hi, 4)[1] == 6.0
    assert list(codes) == [2 + 6, 4 + 6, 8 + 6, -2 + 6, -4 + 6]
    # a family of ranges 5 * 2^-e * m (s not representable): ties at x = (2n+1) R / 30
    for m in (3, 7, 11, 13):
        R = 5.0 * m / 64
        xs = np.array([(2 * n + 1) * R / 30 for n in (1, 4, 7)])        # exact dyadic values
        c, _ = zo.quantize(xs, 0.0, R, 4)
        assert list(c) == [2, 4, 8]


def test_mirror_image_row_has_an_exact_zero_point():
    """max = -min makes min/s exactly -(2^k-1)/2 in real arithmetic, whatever
    the float products round to: z = 8 (half-to-even) at 4 bits, 2 at 2 bits."""
    for v in (1.0 / 3.0, 0.1, 2.7182818284590451, 1e-3 / 7):
        x = np.array([-v, 0.25 * v, v])
        assert zo.quant_params(x.min(), x.max(), 4)[1] == 8.0
        assert zo.quant_params(x.min(), x.max(), 2)[1] == 2.0
        codes, _ = zo.quantize(x, x.min(), x.max(), 4)
        assert codes[0] == 0 and codes[2] == 15


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_error_bound_half_scale(bits):
    x = _rand((200, 64), 20 + bits) * 3 + 0.7
    s, z = zo.quant_params(x.min(1, keepdims=True), x.max(1, keepdims=True), bits)
    codes, _ = zo.quantize(x, x.min(1, keepdims=True), x.max(1, keepdims=True), bits)
    assert codes.min() >= 0 and codes.max() <= 2 ** bits - 1
    assert np.all(codes == np.rint(codes))
    err = np.abs(zo.dequantize(codes, s, z) - x)
    assert np.all(err <= s / 2 + 1e-12)
    # without the "- z" the bound fails (the printed Eq. 5 is shorthand)
    assert np.any(np.abs(codes * s - x) > s / 2 + 1e-9)
    # min maps to code 0 and max to the top code, up to one step at a rounding tie
    assert np.all(codes.min(1) <= 1) and np.all(codes.max(1) >= 2 ** bits - 2)


@pytest.mark.parametrize("bits", [2, 4])
def test_integers_on_grid_are_their_own_codes(bits):
    top = 2 ** bits - 1
    x = np.random.default_rng(3).integers(0, top + 1, (50, 32)).astype(float)
    x[:, 0], x[:, 1] = 0, top
    s, z = zo.quant_params(x.min(1, keepdims=True), x.max(1, keepdims=True), bits)
    assert np.all(s == 1) and np.all(z == 0)
    assert np.array_equal(zo.quantize(x, x.min(1, keepdims=True), x.max(1, keepdims=True), bits)[0], x)
    # data already on an affine grid round-trips exactly
    y = 0.25 * x - 1.5
    s, z = zo.quant_params(y.min(1, keepdims=True), y.max(1, keepdims=True), bits)
    yc, _ = zo.quantize(y, y.min(1, keepdims=True), y.max(1, keepdims=True), bits)
    assert np.allclose(zo.dequantize(yc, s, z), y, atol=1e-12)


def test_degenerate_groups():
    x = np.full((1, 3, 4), 2.3)
    for scheme in ("channel", "cst", "token"):
        q = zo.quantize_rows(x, 4, scheme)
        assert np.all(np.isfinite(q.dequant())) and np.all(q.codes >= 0)
    z = zo.quantize_rows(np.zeros((1, 3, 4)), 2, "cst")
    assert np.all(z.chan_scale == 1.0) and np.all(z.dequant() == 0.0)
    e = zo.quantize_rows(np.zeros((2, 0, 4)), 2, "cst")
    assert e.codes.shape == (2, 0, 4) and np.all(e.chan_scale == 1.0)


# ---- granularities -----------------------------------------------------------

def test_channelwise_axis_and_params():
    X = _rand((2, 30, 12), 21)
    X[:, :, 3] *= 20  # outlier channel
    q = zo.quantize_rows(X, 4, "channel")
    assert q.chan_scale.shape == (2, 12) and np.all(q.tok_scale == 1) and np.all(q.tok_zero == 0)
    for b in range(2):
        for w in range(12):
            col = X[b, :, w]
            s = (col.max() - col.min()) / 15
            assert np.isclose(q.chan_scale[b, w], s)
            assert q.chan_zero[b, w] == -np.rint(col.min() / s)
            assert np.all(np.abs(q.dequant()[b, :, w] - col) <= s / 2 + 1e-12)


def test_cst_steps_match_algorithm_1():
    X = _rand((1, 10, 6), 22)
    X[0, 4, 1] = -9.0   # max |.| = 9 -> c = 3
    X[0, 2, 5] = 4.0    # c = 2 if nothing larger
    X[0, :, 5] = np.clip(X[0, :, 5], -4, 4)
    q = zo.quantize_rows(X, 4, "cst")
    assert q.chan_scale[0, 1] == 3.0 and q.chan_scale[0, 5] == 2.0   # square root, not max
    assert np.all(q.chan_zero == 0)
    Xn = X[0] / q.chan_scale[0]
    for t in range(10):
        s = (Xn[t].max() - Xn[t].min()) / 15
        assert np.isclose(q.tok_scale[0, t], s)
        assert q.tok_zero[0, t] == -np.rint(Xn[t].min() / s)
        ref = np.clip(np.rint(Xn[t] / s) + q.tok_zero[0, t], 0, 15)
        assert np.array_equal(q.codes[0, t], ref)
    err = np.abs(q.dequant() - X)
    assert np.all(err <= q.chan_scale[:, None, :] * q.tok_scale[:, :, None] / 2 + 1e-12)


def test_cst_with_unit_channels_is_tokenwise():
    X = _rand((2, 9, 8), 23)
    X = X / np.abs(X).max(axis=1, keepdims=True)       # every channel has max |x| = 1 -> c = 1
    a, b = zo.quantize_rows(X, 2, "cst"), zo.quantize_rows(X, 2, "token")
    assert np.allclose(a.chan_scale, 1.0)
    assert np.array_equal(a.codes, b.codes) and np.allclose(a.dequant(), b.dequant())


def test_cst_beats_tokenwise_on_outlier_channels():
    X = _rand((1, 64, 128), 24)
    X[:, :, :6] *= 15
    e_tok = np.abs(zo.quantize_rows(X, 4, "token").dequant() - X)[:, :, 6:].mean()
    e_cst = np.abs(zo.quantize_rows(X, 4, "cst").dequant() - X)[:, :, 6:].mean()
    assert e_cst < 0.5 * e_tok


def test_token_rows_layout():
    X = np.arange(2 * 3 * 4 * 5, dtype=float).reshape(2, 3, 4, 5)
    R = zo.token_rows(X)
    assert R.shape == (2, 4, 15)
    assert R[1, 2, 1 * 5 + 3] == X[1, 1, 2, 3]
    assert np.array_equal(zo.head_rows(R, 3), X)


def test_compress_splits_by_subset():
    K = _rand((2, 2, 12, 4), 25)
    sal = np.array([[1, 4, 7], [0, 2, 11]])
    reg = np.array([[i for i in range(12) if i not in s] for s in sal])
    ch = zo.compress_tensor(K, sal, reg, 4, 2, "channel")
    R = zo.token_rows(K)
    assert ch.hi.bits == 4 and ch.lo.bits == 2 and ch.hi.codes.max() <= 15 and ch.lo.codes.max() <= 3
    for b in range(2):
        sub = R[b, sal[b]]
        assert np.allclose(ch.hi.chan_scale[b], (sub.max(0) - sub.min(0)) / 15)  # stats of the subset only
        assert np.all(np.abs(ch.hi.dequant()[b] - sub) <= ch.hi.chan_scale[b] / 2 + 1e-12)
        assert np.all(np.abs(ch.lo.dequant()[b] - R[b, reg[b]]) <= ch.lo.chan_scale[b] / 2 + 1e-12)


# ---- Appendix A / Table 1 ------------------------------------------------------

def test_appendix_a_printed_ratios():
    for name, gran, printed, dec in _rows("appendix_a_ratios.txt"):
        r = zo.compression_ratio(gran, b=8, hd=4096, l=4096, bits_hi=4, n=32)
        assert round(r, int(dec)) == float(printed), (name, r)


def test_table1_parameter_counts():
    b, hd, l, n = 8, 4096, 4096, 32
    for gran, c_g, c_bl, c_hd in _rows("table1_param_counts.txt"):
        expect = int(c_g) * b * hd * l / n + int(c_bl) * b * l + int(c_hd) * hd
        assert zo.quant_param_count(gran, b, hd, l, n) == expect


def test_published_mixed_ratios_are_bracketed():
    for ratio, l, printed in _rows("published_mixed_ratios.txt"):
        vals = [zo.compression_ratio("channel+cst", 8, 4096, int(l), 4, 2, float(ratio), subsets=s)
                for s in (1, 2)]
        assert min(abs(v - float(printed)) for v in vals) <= 0.025, (ratio, l, vals)


def test_groupwise_quantization_pins():
    """Groupwise quantization (Table 1's first row, Appendix A Eq. A): every group of n channels
    of a token row is Eq. 5 on its own - checked group by group against the scalar quantizer, by
    the half-step error bound per group, by its two limits (one group per row = tokenwise; the
    parameter count 2 l h d / n per tensor) and by data already on a group's grid."""
    rng = np.random.default_rng(8)
    B, n, W, g = 2, 5, 64, 32
    X = rng.standard_normal((B, n, W)) * (1 + 9 * (rng.random((1, 1, W)) > 0.9))
    q = zo.quantize_rows(X, 4, "group", group=g)
    assert q.grp_scale.shape == (B, n, W // g) and q.codes.min() >= 0 and q.codes.max() <= 15
    xh = q.dequant()
    for b in range(B):
        for t in range(n):
            for j in range(W // g):
                grp = X[b, t, j * g:(j + 1) * g]
                s, z = zo.quant_params(grp.min(), grp.max(), 4)
                codes, _ = zo.quantize(grp, grp.min(), grp.max(), 4)
                assert np.array_equal(q.codes[b, t, j * g:(j + 1) * g], codes)
                assert q.grp_scale[b, t, j] == s and q.grp_zero[b, t, j] == z
                assert np.all(np.abs(xh[b, t, j * g:(j + 1) * g] - grp) <= s / 2 + 1e-12)
    # outlier channels only hurt their own group: error of a group without outliers is far below tokenwise
    tok = zo.quantize_rows(X, 4, "token")
    assert np.abs(xh - X).mean() < np.abs(tok.dequant() - X).mean()
    # one group per row is plain tokenwise quantization
    one = zo.quantize_rows(X, 4, "group", group=W)
    assert np.array_equal(one.codes, tok.codes) and np.allclose(one.dequant(), tok.dequant())
    # parameters: 2 (s, z) per group; keys and values together 4 b h d l / n (Table 1)
    assert 2 * (q.grp_scale.size + q.grp_zero.size) == zo.quant_param_count("groupwise", B, W, n, g)
    # integers 0..3 in every group round-trip exactly at 2 bits
    Xi = np.tile(np.arange(4.0), (B, n, W // 4))
    qi = zo.quantize_rows(Xi, 2, "group", group=8)
    assert np.array_equal(qi.codes, Xi) and np.all(qi.grp_scale == 1.0) and np.all(qi.grp_zero == 0.0)
