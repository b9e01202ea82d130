"""GPU parity of zc_prefill_attention (Algorithm 2's attention line) against the oracle,
and of the probe stage fed with its row normalisers."""
import numpy as np
import pytest
import torch

from oracle import zipcache_oracle as zo
from paper_2405_14256_amd import binding as zb
from paper_2405_14256_amd import probes
from paper_2405_14256_amd.workloads import WORKLOADS, make_prefill, scaled

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _check_heads(w, inp, out, lse, heads, b=0, sm_scale=None, what=""):
    """Output and log-normaliser of the given query heads of batch element b, all rows."""
    G = w.Hq // w.Hkv
    atol = 1e-4 if w.dtype == "fp32" else 2e-2
    ltol = 1e-4 if w.dtype == "fp32" else 1e-3
    worst = [0.0, 0.0]
    for h in heads:
        Q = inp["Q"][b:b + 1, h:h + 1].double().numpy()
        K = inp["K"][b:b + 1, h // G:h // G + 1].double().numpy()
        V = inp["V"][b:b + 1, h // G:h // G + 1].double().numpy()
        O_o, lse_o = zo.prefill_attention(Q, K, V, sm_scale)
        e = np.abs(out[b, h].double().cpu().numpy() - O_o[0, 0]).max()
        le = np.abs(lse[b, h].double().cpu().numpy() - lse_o[0, 0]).max()
        worst = [max(worst[0], e), max(worst[1], le)]
        assert e <= atol, (what, b, h, e)
        assert le <= ltol, (what, b, h, le)
    print(f"[prefill] {what or w.name}: heads {list(heads)} of b={b}: max |out err| {worst[0]:.3e}, max |lse err| {worst[1]:.3e}", flush=True)


def test_prefill_tiny_fp32_every_head():
    w = WORKLOADS["tiny"]
    inp = make_prefill(w)
    out, lse, _ = zb.zc_prefill_attention(inp["Q"].to(DEV), inp["K"].to(DEV), inp["V"].to(DEV))
    _check_heads(w, inp, out, lse, range(w.Hq))


def test_prefill_llama3_8b_4k_sampled_heads():
    w = WORKLOADS["llama3_8b_4k"]
    inp = make_prefill(w)
    out, lse, _ = zb.zc_prefill_attention(inp["Q"].to(DEV), inp["K"].to(DEV), inp["V"].to(DEV))
    _check_heads(w, inp, out, lse, [0, 13, 31])


@pytest.mark.parametrize("name,kw,heads", [
    ("llama3_8b_32k", dict(L=3000, needles=8), [0, 5, 31]),                 # long-context law, ragged against every tile
    ("llama2_13b_4k_b16", dict(B=2, Hq=4, Hkv=4, L=701), [0, 3]),           # fp16, one query head per KV head
    ("mistral_7b_8k_b8", dict(B=2, Hq=8, Hkv=2, L=129), [1, 6]),            # one row past a row block
    ("tiny", dict(L=63, Hq=4, Hkv=2), [0, 3]),                              # fp32, grouped heads, less than one tile
    ("tiny", dict(L=1), [0]),
    ("llama3_8b_4k", dict(L=520, dtype="fp32", Hq=4, Hkv=2), [0, 3]),       # fp32 at head_dim 128
    ("llama3_8b_4k", dict(L=300, dtype="fp16", Hq=2, Hkv=1), [0, 1]),
])
def test_prefill_shapes_and_types(name, kw, heads):
    w = scaled(WORKLOADS[name], **kw)
    inp = make_prefill(w)
    out, lse, _ = zb.zc_prefill_attention(inp["Q"].to(DEV), inp["K"].to(DEV), inp["V"].to(DEV))
    for b in sorted({0, w.B - 1}):
        _check_heads(w, inp, out, lse, heads, b=b, what=f"{name} {kw}")


def test_prefill_strided_views_and_scale_override():
    """Inputs and output as strided views of larger buffers (a fused QKV projection's layout),
    and a softmax scale of the caller's."""
    w = scaled(WORKLOADS["llama3_8b_4k"], L=333, Hq=8, Hkv=2, B=2)
    inp = make_prefill(w)
    big = torch.zeros(w.B, w.L, (w.Hq + 2 * w.Hkv) * w.d + 64, dtype=w.torch_dtype, device=DEV)

    def view(h0, H):
        return big[:, :, h0 * w.d:(h0 + H) * w.d].view(w.B, w.L, H, w.d).permute(0, 2, 1, 3)
    Qv, Kv, Vv = view(0, w.Hq), view(w.Hq, w.Hkv), view(w.Hq + w.Hkv, w.Hkv)
    Qv.copy_(inp["Q"]); Kv.copy_(inp["K"]); Vv.copy_(inp["V"])
    obuf = torch.zeros(w.B, w.L, w.Hq * w.d + 32, dtype=w.torch_dtype, device=DEV)
    Ov = obuf[:, :, :w.Hq * w.d].view(w.B, w.L, w.Hq, w.d).permute(0, 2, 1, 3)
    out, lse, _ = zb.zc_prefill_attention(Qv, Kv, Vv, sm_scale=0.05, out=Ov)
    _check_heads(w, inp, out, lse, [0, 7], b=1, sm_scale=0.05, what="strided views")
    assert float(obuf[:, :, w.Hq * w.d:].abs().sum()) == 0.0              # nothing written past the rows


def test_probe_saliency_from_the_prefill_normalisers():
    """The probe stage given the prefill pass's log-normalisers (one sweep instead of two): the
    scores must be those of the two-sweep path and of the oracle, and select the same tokens."""
    w = scaled(WORKLOADS["llama3_8b_4k"], L=2500)
    inp = make_prefill(w)
    Q, K, V = (inp[n].to(DEV) for n in ("Q", "K", "V"))
    pos_np = probes.probe_positions(w.L, w.probe_ratio, w.seed)
    pos = torch.from_numpy(pos_np).to(DEV)
    _, lse, lse_p = zb.zc_prefill_attention(Q, K, V, probe_pos=pos)
    assert torch.equal(lse_p, lse[:, :, pos.long()])
    one = zb.zc_probe_saliency(Q, K, pos, lse_ext=lse_p)
    two = zb.zc_probe_saliency(Q, K, pos)
    ref, _ = zo.saliency_scores(inp["Q"].double().numpy(), inp["K"].double().numpy(), pos_np)
    got = one.cpu().double().numpy()
    rel = np.abs(got - ref) / np.maximum(ref, 1e-6 * ref.max())
    assert rel.max() <= 1e-4, rel.max()
    assert (one - two).abs().max() <= 1e-4 * two.abs().max()
    s1, _ = zb.zc_select_salient(one, w.k_salient)
    from tests.pipeline_check import check_index_sets
    check_index_sets(ref[0], s1[0].cpu().numpy(), w.k_salient, "split on one-sweep scores")
