"""CPU checks of the host-side logic: probe choice, workload generators, the
packed-format reader/writer used by the parity tests."""
import numpy as np
import pytest
import torch

from paper_2405_14256_amd import probes
from paper_2405_14256_amd.workloads import WORKLOADS, make_decode_step, make_prefill, needle_positions, scaled
from tests import packfmt


@pytest.mark.parametrize("L,ratio", [(256, 0.10), (4096, 0.10), (4096, 0.05), (8192, 0.10), (100, 0.10), (7, 0.10)])
def test_probe_positions(L, ratio):
    pos = probes.probe_positions(L, ratio, seed=3)
    n_rec, n_rand = probes.probe_counts(L, ratio)
    assert len(pos) == n_rec + n_rand and pos.dtype == np.int32
    assert np.all(np.diff(pos) > 0)                          # sorted, unique
    assert list(pos[-n_rec:]) == list(range(L - n_rec, L))    # the most recent tokens
    assert pos[-1] == L - 1 and pos.min() >= 0
    assert np.array_equal(pos, probes.probe_positions(L, ratio, seed=3))
    if n_rand > 1:
        assert not np.array_equal(pos, probes.probe_positions(L, ratio, seed=4))


def test_probe_strategies_take_the_same_number_of_probes():
    L, ratio = 4096, 0.10
    hybrid = probes.probe_positions(L, ratio, seed=2)
    recent = probes.probe_positions(L, ratio, seed=2, strategy="recent")
    rand = probes.probe_positions(L, ratio, seed=2, strategy="random")
    every = probes.probe_positions(L, ratio, seed=2, strategy="all")
    assert len(recent) == len(rand) == len(hybrid) == 410
    assert list(recent) == list(range(L - 410, L))
    assert np.all(np.diff(rand) > 0) and rand.min() >= 0 and rand.max() < L
    assert not np.array_equal(rand, hybrid)
    assert list(every) == list(range(L))
    for p in (hybrid, recent, rand, every):
        assert p.dtype == np.int32
    with pytest.raises(ValueError):
        probes.probe_positions(L, ratio, strategy="special")


def test_probe_counts_match_the_five_configs():
    assert probes.probe_counts(256, 0.10) == (13, 13)
    assert probes.probe_counts(4096, 0.10) == (205, 205)
    assert probes.probe_counts(8192, 0.10) == (410, 410)
    assert probes.probe_counts(4096, 0.05) == (102, 102)
    assert probes.probe_counts(32768, 0.10) == (1638, 1638)


def test_decode_probe_offsets():
    off = probes.decode_probe_offsets(100, seed=1)
    assert list(off[-5:]) == [95, 96, 97, 98, 99] and np.all(np.diff(off) > 0)
    assert off[-1] == 99                                       # every tail column is seen by a probe
    assert np.array_equal(off, probes.decode_probe_offsets(100, seed=1))


def test_workloads_are_seeded_and_sliceable():
    w = scaled(WORKLOADS["mistral_7b_8k_b8"], B=3, L=64)
    a, b = make_prefill(w), make_prefill(w)
    assert all(torch.equal(a[k], b[k]) for k in a)
    one = make_prefill(w, batch=2)
    assert torch.equal(one["K"][0], a["K"][2]) and torch.equal(one["Q"][0], a["Q"][2])
    assert a["Q"].shape == (3, 32, 64, 128) and a["K"].shape == (3, 8, 64, 128) and a["K"].dtype == torch.bfloat16
    # outlier channels: a few key channels per head are much larger than the rest
    mag = a["K"].float().abs().amax(dim=(0, 2))               # [Hkv, d]
    assert ((mag > 15).sum(dim=1) == w.outlier_channels).all()
    d0, d1 = make_decode_step(w, 0), make_decode_step(w, 1)
    assert d0["q"].shape == (3, 32, 128) and not torch.equal(d0["q"], d1["q"])


def test_workload_table():
    w = WORKLOADS["llama3_8b_4k"]
    assert (w.B, w.Hq, w.Hkv, w.d, w.L, w.dtype) == (1, 32, 8, 128, 4096, "bf16")
    assert w.k_salient == 1638 and w.W == 1024 and w.n_recent == 205
    assert WORKLOADS["mistral_7b_8k_b8"].k_salient == 1638
    assert WORKLOADS["llama3_8b_32k"].k_salient == 3276
    assert WORKLOADS["tiny"].k_salient == 102
    assert len(needle_positions(WORKLOADS["llama3_8b_32k"])) == 32


def test_sink_and_needles_structure():
    w = scaled(WORKLOADS["llama3_8b_4k"], L=128)
    x = make_prefill(w)
    assert x["K"][0, :, 0].float().mean() > 2.0                  # token 0 offset
    w5 = scaled(WORKLOADS["llama3_8b_32k"], L=512, needles=4)
    x5 = make_prefill(w5)
    pos = needle_positions(w5)
    q = x5["Q"][0, 0, -1].float(); kk = x5["K"][0, 0, pos].float()
    cos = (kk @ q) / (kk.norm(dim=1) * q.norm())
    assert (cos > 0.8).all()


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_packfmt_roundtrip(bits):
    rng = np.random.default_rng(bits)
    B, H, D, cap = 2, 3, 64, 128
    codes = rng.integers(0, 2 ** bits, (B, H, cap, D))
    for enc, dec in ((packfmt.encode_row, packfmt.decode_row), (packfmt.encode_tgroup, packfmt.decode_tgroup)):
        arena = enc(codes, bits)
        assert arena.dtype == np.uint8 and arena.size == B * H * cap * D * bits // 8
        assert np.array_equal(dec(arena, B, H, D, cap, bits), codes)


def test_packfmt_bit_positions_follow_the_header():
    # ROW, 4 bits: channel 2j in the low nibble of byte j
    codes = np.zeros((1, 1, 64, 64), np.int64); codes[0, 0, 0, 0] = 0x3; codes[0, 0, 0, 1] = 0xA
    assert packfmt.encode_row(codes, 4)[0] == 0xA3
    # TGROUP, 4 bits: field e of word [blk][kg][c] holds slot 16*(e/4) + 4*kg + e%4
    codes = np.zeros((1, 1, 64, 64), np.int64); codes[0, 0, 16 + 4 * 2 + 1, 5] = 0xF     # j=1, kg=2, v=1 -> e=5
    w = packfmt.encode_tgroup(codes, 4).view(np.uint32).reshape(2, 4, 64)
    assert w[0, 2, 5] == 0xF << 20 and w.sum() == 0xF << 20
    # TGROUP, 2 bits: field groups 0,1,2,3 address slot tiles 0,2,1,3
    codes = np.zeros((1, 1, 64, 64), np.int64); codes[0, 0, 32 + 4 * 1 + 3, 7] = 0x3     # tile 2, kg=1, v=3 -> e=4*1+3
    w = packfmt.encode_tgroup(codes, 2).view(np.uint32).reshape(1, 4, 64)
    assert w[0, 1, 7] == 0x3 << 14 and w.sum() == 0x3 << 14


def test_parity_rule_counts_levels_and_polices_zero_point_differences():
    """The code comparison of the GPU tests, exercised on the CPU with planted differences in
    copies of the oracle's own result: a zero point one step apart with every code shifted
    along is the same quantization (Eq. 5: x_hat = (code - z) s) if and only if -min / s sat
    at a rounding boundary; anywhere else it must be rejected, and so must a shifted level."""
    import copy
    import pytest
    from oracle import zipcache_oracle as zo
    from tests.pipeline_check import compare_subset
    rng = np.random.default_rng(5)
    X = rng.standard_normal((1, 40, 64))
    # plant a near-tie in row 3: make -min/s = n + 1/2 + 1e-6 by moving the row's minimum
    ref = zo.quantize_rows(X, 4, "token")
    row = X[0, 3].copy()
    hi, j = row.max(), int(row.argmin())
    # min / s = 15 min / (hi - min) = -(n + 0.5) - eps  =>  min = -(n + .5 + eps) hi / (15 - (n + .5 + eps))
    n = 6
    t = n + 0.5 + 1e-6
    row[j] = -t * hi / (15 - t)
    row[np.arange(64) != j] = np.maximum(row[np.arange(64) != j], row[j] * 0.99)
    X[0, 3] = row
    ref = zo.quantize_rows(X, 4, "token")
    assert abs(-ref.pre_round[0, 3].min() - (n + 0.5)) < 1e-5
    same = compare_subset(copy.deepcopy(ref), ref, "identical")
    assert same["n_mismatch"] == 0 and same["n_zero_mismatch"] == 0
    # the other side rounded that zero point the other way: all codes of the row shift, the clipped end moves a level
    other = copy.deepcopy(ref)
    dz = -1.0 if ref.tok_zero[0, 3] == np.round(t) else 1.0
    other.tok_zero[0, 3] += dz
    other.codes[0, 3] = np.clip(ref.codes[0, 3] + dz, 0, 15)
    rep = compare_subset(other, ref, "zero point at its boundary")
    assert rep["n_zero_mismatch"] == 1 and rep["n_mismatch"] <= 2          # only clipped ends differ in level
    # the same shift in a row that is nowhere near a boundary is an error
    r2 = next(r for r in range(40) if r != 3 and abs((-ref.pre_round[0, r].min()) % 1 - 0.5) > 0.1)
    bad = copy.deepcopy(ref)
    bad.tok_zero[0, r2] += 1.0
    bad.codes[0, r2] = np.clip(ref.codes[0, r2] + 1.0, 0, 15)
    with pytest.raises(AssertionError, match="zero point differs away"):
        compare_subset(bad, ref, "zero point off")
    # and so is a level that differs away from a rounding boundary of its element
    r3, c3 = next((r, c) for r in range(40) for c in range(64)
                  if abs(ref.pre_round[0, r, c] % 1 - 0.5) > 0.2 and 1 <= ref.codes[0, r, c] <= 14)
    bad = copy.deepcopy(ref)
    bad.codes[0, r3, c3] += 1.0
    with pytest.raises(AssertionError, match="away from a rounding boundary"):
        compare_subset(bad, ref, "level off")
    # inside the row whose zero point legitimately differs, only the clipped ends may move:
    # a level off by one in the middle of the code range, away from its own tie, is an error
    c4 = next(c for c in range(64) if abs(ref.pre_round[0, 3, c] % 1 - 0.5) > 0.2 and 2 <= other.codes[0, 3, c] <= 13)
    bad = copy.deepcopy(other)
    bad.codes[0, 3, c4] += 1.0
    with pytest.raises(AssertionError, match="away from a rounding boundary"):
        compare_subset(bad, ref, "level off inside a shifted row")
    # budgets over a pass: raw identical codes, levels, zero points
    from tests.pipeline_check import CODE_COUNTS, assert_code_budgets
    tot = {k: rep[k] for k in CODE_COUNTS}
    assert rep["n_raw_mismatch"] >= 60 and rep["n_raw_unshifted"] == 0          # the whole shifted row differs as stored
    assert tot["n_mismatch"] == 1                                               # the clipped end of that row: 1 level in 2560,
    tot["n_codes"] *= 10                                                        # within budget in a case ten times the size
    out = assert_code_budgets(tot, "one tie in a small case")                   # 40 rows: one tie is tolerated
    assert out["raw_identical_frac"] < 0.999
    big = dict(tot, n_groups=20000, n_codes=20000 * 64)                         # a whole workload: budgets are fractions
    assert_code_budgets(big, "one tie in 20000 rows")
    with pytest.raises(AssertionError, match="zero points differ"):
        assert_code_budgets(dict(big, n_zero_mismatch=3), "three ties in 20000 rows")
    with pytest.raises(AssertionError, match="stored codes are identical"):
        assert_code_budgets(dict(big, n_raw_mismatch=200), "too many stored codes differ")
    with pytest.raises(AssertionError, match="levels differ"):
        assert_code_budgets(dict(big, n_mismatch=200, n_raw_mismatch=100), "too many levels differ")
