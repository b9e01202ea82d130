"""Seeded synthetic workloads shaped like the paper's LLaMA / Mistral layers.

This module only draws random inputs; it holds none of the method's
arithmetic, so both the GPU path and the CPU oracle may take their inputs from
it.  Tensors are produced on the CPU with torch generators and rounded once to
the configuration's dtype; the same bytes are then handed to either side.

The value structure follows what the paper describes for real activations
(Section 4.1: outlier channels in keys; Section 1: a few dominant tokens and an
attention sink; Section 4.2: salient tokens may sit anywhere in the prompt).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

BASE_SEED = 20240514

_DTYPES = {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    B: int
    Hq: int
    Hkv: int
    d: int
    L: int
    dtype: str
    probe_ratio: float
    salient_ratio: float
    bits_hi: int
    bits_lo: int
    decode_steps: int
    outlier_channels: int      # per KV head
    outlier_gain: float
    sink: bool = False         # token 0 key offset + query mean shift
    needles: int = 0           # injected keys aligned with the recent queries
    growing_tail: bool = False  # decode appends tokens and flushes every 100

    @property
    def torch_dtype(self):
        return _DTYPES[self.dtype]

    @property
    def W(self) -> int:
        return self.Hkv * self.d

    @property
    def k_salient(self) -> int:
        return int(np.floor(self.salient_ratio * self.L + 1e-9))

    @property
    def n_recent(self) -> int:
        return max(1, int(round(self.probe_ratio / 2 * self.L)))

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    Workload("tiny", 1, B=1, Hq=8, Hkv=8, d=64, L=256, dtype="fp32", probe_ratio=0.10,
             salient_ratio=0.40, bits_hi=4, bits_lo=2, decode_steps=8,
             outlier_channels=4, outlier_gain=10.0),
    Workload("llama3_8b_4k", 2, B=1, Hq=32, Hkv=8, d=128, L=4096, dtype="bf16", probe_ratio=0.10,
             salient_ratio=0.40, bits_hi=4, bits_lo=2, decode_steps=128,
             outlier_channels=6, outlier_gain=15.0, sink=True),
    Workload("mistral_7b_8k_b8", 3, B=8, Hq=32, Hkv=8, d=128, L=8192, dtype="bf16", probe_ratio=0.10,
             salient_ratio=0.20, bits_hi=4, bits_lo=2, decode_steps=256,
             outlier_channels=6, outlier_gain=15.0),
    Workload("llama2_13b_4k_b16", 4, B=16, Hq=40, Hkv=40, d=128, L=4096, dtype="fp16", probe_ratio=0.05,
             salient_ratio=0.40, bits_hi=4, bits_lo=2, decode_steps=512,
             outlier_channels=8, outlier_gain=20.0, growing_tail=True),
    Workload("llama3_8b_32k", 5, B=1, Hq=32, Hkv=8, d=128, L=32768, dtype="bf16", probe_ratio=0.10,
             salient_ratio=0.10, bits_hi=4, bits_lo=2, decode_steps=64,
             outlier_channels=6, outlier_gain=15.0, needles=32),
]}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some sizes changed (reduced-size parity cases
    keep the value structure of the full configuration)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


def _gen(seed: int, *stream: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    s = seed
    for x in stream:
        s = (s * 1000003 + x + 1) % (2 ** 62)
    g.manual_seed(s)
    return g


def outlier_channel_gain(w: Workload) -> torch.Tensor:
    """[Hkv, d] per-channel gain of the keys: `outlier_channels` seeded channels
    of every KV head are multiplied by `outlier_gain`."""
    g = _gen(w.seed, 11)
    gain = torch.ones(w.Hkv, w.d)
    for h in range(w.Hkv):
        ch = torch.randperm(w.d, generator=g)[: w.outlier_channels]
        gain[h, ch] = w.outlier_gain
    return gain


def needle_positions(w: Workload) -> np.ndarray:
    if not w.needles:
        return np.zeros(0, np.int64)
    g = _gen(w.seed, 13)
    return np.sort(torch.randperm(w.L - w.n_recent, generator=g)[: w.needles].numpy())


def _needle_dirs(w: Workload) -> torch.Tensor:
    g = _gen(w.seed, 17)
    u = torch.randn(w.Hkv, w.d, generator=g)
    return u / u.norm(dim=1, keepdim=True)


def make_prefill(w: Workload, batch: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """Q [B, Hq, L, d], K and V [B, Hkv, L, d] in the workload dtype (CPU).
    With `batch` given, only that batch element is produced (leading dim 1);
    it is identical to the same slice of the full tensors."""
    bs = range(w.B) if batch is None else [batch]
    gain = outlier_channel_gain(w)
    G = w.Hq // w.Hkv
    Qs, Ks, Vs = [], [], []
    for b in bs:
        g = _gen(w.seed, 1, b)
        Q = torch.randn(w.Hq, w.L, w.d, generator=g)
        K = torch.randn(w.Hkv, w.L, w.d, generator=g) * gain[:, None, :]
        V = torch.randn(w.Hkv, w.L, w.d, generator=g)
        if w.sink:
            Q += 0.25
            K[:, 0, :] += 3.0
        if w.needles:
            u = _needle_dirs(w)                                   # [Hkv, d]
            a = 5.0 * np.sqrt(w.d)
            Q[:, w.L - w.n_recent:, :] += a * u.repeat_interleave(G, dim=0)[:, None, :]
            rho = K.norm(dim=2).mean(dim=1)                       # [Hkv]
            pos = torch.from_numpy(needle_positions(w))
            r = torch.randn(w.Hkv, len(pos), w.d, generator=g)
            r = r - (r * u[:, None, :]).sum(-1, keepdim=True) * u[:, None, :]
            r = r / r.norm(dim=2, keepdim=True)
            K[:, pos, :] = rho[:, None, None] * (0.9 * u[:, None, :] + np.sqrt(0.19) * r)
        Qs.append(Q.to(w.torch_dtype))
        Ks.append(K.to(w.torch_dtype))
        Vs.append(V.to(w.torch_dtype))
    return {"Q": torch.stack(Qs), "K": torch.stack(Ks), "V": torch.stack(Vs)}


def make_decode_step(w: Workload, step: int) -> Dict[str, torch.Tensor]:
    """q [B, Hq, d], k_new and v_new [B, Hkv, d] of decode step `step`."""
    g = _gen(w.seed, 1000 + step)
    gain = outlier_channel_gain(w)
    q = torch.randn(w.B, w.Hq, w.d, generator=g)
    k = torch.randn(w.B, w.Hkv, w.d, generator=g) * gain[None]
    v = torch.randn(w.B, w.Hkv, w.d, generator=g)
    if w.sink:
        q += 0.25
    return {"q": q.to(w.torch_dtype), "k_new": k.to(w.torch_dtype), "v_new": v.to(w.torch_dtype)}


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact float64 image of a stored tensor (every fp16/bf16/fp32 value is
    representable)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
