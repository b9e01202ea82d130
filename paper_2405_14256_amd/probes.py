"""Host-side choice of probe tokens (Section 4.3, "random+recent" strategy).

The probe positions are an input of the library: they are drawn here, on the
host, from a seeded generator and handed to `zc_probe_saliency` (and to
whatever checks it) as a sorted int32 list.
"""
from __future__ import annotations

import numpy as np


def probe_counts(L: int, probe_ratio: float):
    """Half of the probes are the most recent tokens, half are random ones
    (5 % + 5 % by default).  A fractional count is rounded to nearest; there is
    always at least one recent probe, so the last token is always a probe and
    every column is seen by at least one probe row."""
    n_recent = max(1, int(round(probe_ratio / 2 * L)))
    n_recent = min(n_recent, L)
    n_random = min(int(round(probe_ratio / 2 * L)), L - n_recent)
    return n_recent, n_random


STRATEGIES = ("random+recent", "recent", "random", "all")


def probe_positions(L: int, probe_ratio: float = 0.10, seed: int = 0, strategy: str = "random+recent") -> np.ndarray:
    """Sorted unique probe positions.

    "random+recent" (the method's choice): the last n_recent tokens plus
    n_random tokens drawn without replacement from the remaining ones.
    The alternatives of the probe-strategy comparison (Section 4.3, Table 2) take
    the same number of probes: "recent" the last ones only, "random" a uniform
    draw over the whole sequence, "all" every token (the full attention matrix).
    A column after the last probe is seen by no probe and scores 0: only "random"
    can leave such columns."""
    if strategy not in STRATEGIES:
        raise ValueError(f"unknown probe strategy {strategy!r}")
    n_recent, n_random = probe_counts(L, probe_ratio)
    rng = np.random.Generator(np.random.PCG64(seed))
    if strategy == "all":
        return np.arange(L, dtype=np.int32)
    if strategy == "recent":
        return np.arange(L - min(L, n_recent + n_random), L, dtype=np.int32)
    if strategy == "random":
        return np.sort(rng.choice(L, size=min(L, n_recent + n_random), replace=False)).astype(np.int32)
    rand = rng.choice(L - n_recent, size=n_random, replace=False) if n_random else np.zeros(0, np.int64)
    pos = np.concatenate([np.sort(rand), np.arange(L - n_recent, L)])
    return pos.astype(np.int32)


def decode_probe_offsets(interval: int = 100, recent: int = 5, p_random: float = 0.05,
                         seed: int = 0) -> np.ndarray:
    """Window offsets (0-based) of the decode steps that act as probes inside
    one re-compression window (Algorithm 3): the last `recent` steps of the
    window and, before them, each step with probability `p_random`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    draw = rng.random(interval) < p_random
    off = [j for j in range(interval) if j >= interval - recent or draw[j]]
    return np.asarray(off, np.int32)
