"""GPU parity of zc_group_quantize (groupwise quantization, Table 1's baseline granularity)
against the oracle, and a smoke run of bench.py's error-versus-ratio report."""
import numpy as np
import pytest
import torch

from oracle import zipcache_oracle as zo
from paper_2405_14256_amd import binding as zb
from tests.pipeline_check import CODE_COUNTS, assert_code_budgets, compare_subset

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_groupwise_quantize_randomized_shapes():
    rng = np.random.default_rng(77)
    totals = {key: 0 for key in CODE_COUNTS}
    for case in range(18):
        D = int(rng.choice([64, 128]))
        H = int(rng.choice([1, 2, 5, 8, 40]))
        B = int(rng.integers(1, 3))
        L = int(rng.integers(1, 200))
        n = int(rng.integers(1, L + 1))
        bits = int(rng.choice([2, 4, 8]))
        group = int(rng.choice([g for g in (8, 16, 32, 64, 128) if (H * D) % g == 0]))
        dtype = [torch.float32, torch.float16, torch.bfloat16][case % 3]
        g = torch.Generator().manual_seed(300 + case)
        X = (torch.randn(B, H, L, D, generator=g) * (1 + 9 * (torch.rand(1, H, 1, D, generator=g) > 0.9))).to(dtype)
        if case % 4 == 0:
            X[:, :, 0] = 0.75                              # a constant row: every group has max == min
        idx = torch.stack([torch.randperm(L, generator=g)[:n].sort().values for _ in range(B)]).to(torch.int32)
        what = f"case {case}: B={B} H={H} D={D} L={L} n={n} bits={bits} group={group} {dtype}"
        print(what, flush=True)
        use_idx = case % 5 != 1
        co, sc, ze, dq = zb.zc_group_quantize(X.to(DEV), bits, group, idx.to(DEV) if use_idx else None)
        torch.cuda.synchronize()
        rows = zo.token_rows(X.double().numpy())
        sel = idx.numpy().astype(np.int64) if use_idx else np.tile(np.arange(L), (B, 1))
        ref = zo.quantize_rows(np.stack([rows[b, sel[b]] for b in range(B)]), bits, "group", sel, group=group)
        got = zo.QuantSubset("group", bits, sel, co.cpu().numpy().astype(np.float64), ref.chan_scale, ref.chan_zero,
                             ref.tok_scale, ref.tok_zero, None, sc.cpu().numpy().astype(np.float64), ze.cpu().numpy().astype(np.float64))
        c = compare_subset(got, ref, what)
        for key in CODE_COUNTS:
            totals[key] += c[key]
        # the de-quantized values are (code - z) s of the kernel's own codes and parameters
        want = got.dequant()
        assert np.allclose(dq.cpu().numpy().astype(np.float64), want, rtol=2e-6, atol=1e-6 * max(np.abs(want).max(), 1e-30)), what
    rep = assert_code_budgets(totals, "groupwise")
    print(rep, totals)


def test_error_report_runs_and_orders_the_granularities():
    """bench.py --error-report on the tiny workload: every row is finite, a finer granularity
    never reconstructs worse than the coarse ones it refines, and the ratios are Appendix A's."""
    import bench
    rep = bench.error_report("tiny", decode_queries=8)
    rows = {(r["k_scheme"], r["v_scheme"], r["bits"]): r for r in rep["granularities"]}
    for r in rep["granularities"]:
        assert np.isfinite([r["k_rel_mse"], r["v_rel_mse"], r["attn_out_rel_err"], r["compression_ratio"]]).all(), r
    g4, t4, cst4 = rows[("group", "group", "4/4")], rows[("token", "token", "4/4")], rows[("channel", "cst", "4/4")]
    assert g4["k_rel_mse"] < t4["k_rel_mse"] and g4["v_rel_mse"] <= t4["v_rel_mse"] * 1.001
    assert cst4["k_rel_mse"] < t4["k_rel_mse"]                     # outlier channels: channelwise keys beat tokenwise keys
    assert g4["compression_ratio"] < t4["compression_ratio"]       # 4 b h d l / n parameters against 4 b l
    assert {s["metric"] for s in rep["saliency_metrics"]} == {"normalized (Eq. 8)", "accumulated (Eq. 7)"}
