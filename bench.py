#!/usr/bin/env python3
"""Benchmark of the ZipCache hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch of the
LLaMA3-8B-shaped layer at 4k context (the configuration the metric is quoted
on): probe saliency -> salient split -> quantize-pack K and V -> the
configuration's decode steps over the packed cache, the full-precision tail
growing one token per step and being re-compressed after 100 tokens
(probe saliency with the decode-time normalisers, split, quantize-pack).
All inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is decode tokens per second of the whole step
(compression included).  `roofline` describes the dominant kernel (packed
decode attention): algorithmic bytes per launch over the average launch
duration measured with HIP events.  `cpu_baseline` times the float64 oracle on
the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2405_14256_amd import binding as zb          # noqa: E402
from paper_2405_14256_amd import probes                 # noqa: E402
from paper_2405_14256_amd.workloads import WORKLOADS, make_decode_step, make_prefill, to_f64  # noqa: E402

HBM_PEAK_GBPS = 8000.0
FLUSH_INTERVAL = 100


def measured_decode_traffic(workload: str):
    """HBM bytes per decode call from rocprofv3 counter runs of this script (FETCH_SIZE, then
    WRITE_SIZE, each scaled by what the same counter reads for a plain 256 MiB copy): not
    measurable from inside a run, so it is read from the summary of those runs,
    profiles/decode_traffic_<workload>.txt (its last line, "# decode entry point ...: N bytes").
    None when no summary exists for the workload."""
    path = os.path.join(ROOT, "profiles", f"decode_traffic_{workload}.txt")
    try:
        for line in reversed(open(path).read().splitlines()):
            if line.startswith("# decode entry point"):
                return {"bytes_per_launch": float(line.split(":")[1].split()[0]), "source": os.path.relpath(path, ROOT)}
    except (OSError, ValueError, IndexError):
        pass
    return None


class HotPath:
    """Pre-allocated buffers and the call sequence of one step."""

    def __init__(self, w, device="cuda", k_scheme="channel", v_scheme="cst"):
        self.w = w
        dev = torch.device(device)
        inp = make_prefill(w)
        self.cpu_inputs = inp
        self.Q, self.K, self.V = (inp[n].to(dev) for n in ("Q", "K", "V"))
        self.pos_np = probes.probe_positions(w.L, w.probe_ratio, w.seed)
        self.pos = torch.from_numpy(self.pos_np).to(dev)
        self.k = w.k_salient
        S = w.decode_steps
        self.S = S
        dec = [make_decode_step(w, j) for j in range(S)]
        self.cpu_decode = dec
        # q of all steps as one [B, Hq, S, d] view; new keys / values of all steps laid out
        # where the tail view will find them: [B, Hkv, S, d]
        self.q_all = torch.stack([d["q"] for d in dec], dim=2).contiguous().to(dev)
        self.tail_k = torch.stack([d["k_new"] for d in dec], dim=2).contiguous().to(dev)
        self.tail_v = torch.stack([d["v_new"] for d in dec], dim=2).contiguous().to(dev)
        self.n_flush = S // FLUSH_INTERVAL
        self.k_tail = int(np.floor(w.salient_ratio * FLUSH_INTERVAL + 1e-9))
        lib = zb.load()
        cap_hi = lib.zc_arena_slots(self.k + self.n_flush * self.k_tail, 1 + self.n_flush)
        cap_lo = lib.zc_arena_slots(w.L - self.k + self.n_flush * (FLUSH_INTERVAL - self.k_tail), 1 + self.n_flush)
        mk = lambda scheme, layout: zb.PackedTensor(w.B, w.Hkv, w.d, cap_hi, cap_lo, w.bits_hi, w.bits_lo, scheme,
                                                    layout, max_chunks=1 + self.n_flush, device=device, store_pos=True)
        self.Kp, self.Vp = mk(k_scheme, zb.ZC_LAYOUT_ROW), mk(v_scheme, zb.ZC_LAYOUT_TGROUP)
        f32 = dict(dtype=torch.float32, device=dev)
        i32 = dict(dtype=torch.int32, device=dev)
        self.scores = torch.empty(w.B, w.L, **f32)
        self.sal = torch.empty(w.B, self.k, **i32)
        self.reg = torch.empty(w.B, w.L - self.k, **i32)
        self.out = torch.empty(S, w.B, w.Hq, w.d, dtype=w.torch_dtype, device=dev)
        self.probe_off_np = probes.decode_probe_offsets(FLUSH_INTERVAL, seed=w.seed)
        self.probe_off = torch.from_numpy(self.probe_off_np).to(dev)
        # every flush keeps its window's scores and index lists (a few KB each), so that a
        # whole step can be checked against the oracle after the fact
        self.tail_scores = [torch.empty(w.B, FLUSH_INTERVAL, **f32) for _ in range(self.n_flush)]
        self.sal_t = [torch.empty(w.B, self.k_tail, **i32) for _ in range(self.n_flush)]
        self.reg_t = [torch.empty(w.B, FLUSH_INTERVAL - self.k_tail, **i32) for _ in range(self.n_flush)]
        self.lse_p = torch.empty(w.B, w.Hq, len(self.probe_off_np), **f32)
        # the log-sum-exp of a probe step goes straight to its row of lse_probe[f] (the other
        # steps do not ask for it): the flush then needs one transposing copy, no gather
        self.lse_probe = [torch.empty(len(self.probe_off_np), w.B, w.Hq, **f32) for _ in range(self.n_flush)]
        self.lse_slot = {}
        for f in range(self.n_flush):
            for i, off in enumerate(self.probe_off_np.tolist()):
                self.lse_slot[f * FLUSH_INTERVAL + off] = self.lse_probe[f][i]
        self.flush_rows = []
        for f in range(self.n_flush):
            r = (self.probe_off + f * FLUSH_INTERVAL).to(torch.int32)
            self.flush_rows.append((r, r.long()))
        self.decode_events = None     # filled by step(timed=True)
        self.stage_events = None

    # -- algorithmic traffic ---------------------------------------------------------
    def decode_bytes(self, n_hi: int, n_lo: int, n_chunks: int, tail_len: int) -> float:
        w = self.w
        eb = 4 if w.dtype == "fp32" else 2
        codes = 2 * w.B * w.W * (w.bits_hi * n_hi + w.bits_lo * n_lo) / 8          # K and V codes
        tok = 8 * w.B * (n_hi + n_lo)                                              # (s, z) per token of V
        chan = n_chunks * 2 * w.B * w.W * (8 + 4)                                  # K: s, z; V: c (per subset)
        tail = 2 * eb * w.B * tail_len * w.W
        qo = 2 * w.B * w.Hq * w.d * eb
        return codes + tok + chan + tail + qo

    def quant_bytes(self) -> float:
        """Compulsory bytes of the prefill quantize-pack of K and V: read each
        tensor once, write codes, token parameters (V) and channel parameters."""
        w = self.w
        eb = 4 if w.dtype == "fp32" else 2
        read = 2 * eb * w.B * w.L * w.W
        codes = 2 * w.B * w.W * (w.bits_hi * self.k + w.bits_lo * (w.L - self.k)) / 8
        tok = 8 * w.B * w.L
        chan = 2 * w.B * w.W * (8 + 4)
        return read + codes + tok + chan

    def probe_flops(self) -> float:
        w = self.w
        return 2.0 * w.d * float((self.pos_np.astype(np.int64) + 1).sum()) * w.Hq * w.B

    # -- one pass of the hot path, as a list of stages -------------------------------------
    def stages(self):
        """[(name, fn, n_decode_calls, decode_bytes)] in execution order.  Calling the
        functions in order performs one whole step (host bookkeeping of the packed
        cache included), so they can be run eagerly or captured one by one."""
        w = self
        out = []

        def probe():
            self.Kp.reset(); self.Vp.reset()
            zb.zc_probe_saliency(self.Q, self.K, self.pos, scores=self.scores)

        def select():
            zb.zc_select_salient(self.scores, self.k, self.sal, self.reg)

        def quantize():
            zb.zc_quantize_pack_kv(self.K, self.V, self.sal, self.reg, self.Kp, self.Vp)

        out += [("probe", probe, 0, 0.0), ("select", select, 0, 0.0), ("quantize", quantize, 0, 0.0)]

        def decode_range(j0, j1, base):
            def fn():
                nbytes = 0.0
                for j in range(j0, j1):
                    T = j - base + 1
                    zb.zc_decode_attention(self.q_all[:, :, j:j + 1], self.Kp, self.Vp, self.tail_k[:, :, base:],
                                           self.tail_v[:, :, base:], T, out=self.out[j], lse_out=self.lse_slot.get(j))    # only probe steps need it (Alg. 3)
                    hi = sum(c[1] for c in self.Kp.chunks); lo = sum(c[3] for c in self.Kp.chunks)
                    nbytes += self.decode_bytes(hi, lo, self.Kp.c.n_chunks, T)
                fn.nbytes = nbytes
            return fn

        def flush_at(f):
            def fn():
                base = f * FLUSH_INTERVAL
                rows, rows_long = self.flush_rows[f]
                self.lse_p.copy_(self.lse_probe[f].permute(1, 2, 0))
                tk = self.tail_k[:, :, base:base + FLUSH_INTERVAL]
                tv = self.tail_v[:, :, base:base + FLUSH_INTERVAL]
                zb.zc_probe_saliency(self.q_all, tk, self.probe_off, probe_rows=rows, lse_ext=self.lse_p,
                                     scores=self.tail_scores[f])
                zb.zc_select_salient(self.tail_scores[f], self.k_tail, self.sal_t[f], self.reg_t[f])
                n_packed = self.w.L + base
                zb.zc_quantize_pack_kv(tk, tv, self.sal_t[f], self.reg_t[f], self.Kp, self.Vp, pos_offset=n_packed)
            return fn

        j = 0
        for f in range(self.n_flush):
            out.append(("decode", decode_range(j, (f + 1) * FLUSH_INTERVAL, f * FLUSH_INTERVAL), FLUSH_INTERVAL, None))
            out.append(("flush", flush_at(f), 0, 0.0))
            j = (f + 1) * FLUSH_INTERVAL
        if j < self.S:
            out.append(("decode", decode_range(j, self.S, self.n_flush * FLUSH_INTERVAL), self.S - j, None))
        return out

    def step(self):
        for _, fn, _, _ in self.stages():
            fn()

    def launch_units(self, stages, graph: bool = True):
        """The launch units of the timed region - the three compression stages of the prefill
        as one unit, every decode range and every flush a unit of its own (so that HIP events
        can bracket exactly the decode launches) - and, for the split of the first unit, one
        unit per stage.  With `graph` every unit is captured into a HIP graph and the
        callables replay it.  Returns (units, their names, per-stage units)."""
        groups = []
        for i, (name, _, _, _) in enumerate(stages):
            if name in ("select", "quantize") and groups and stages[groups[-1][-1]][0] in ("probe", "select"):
                groups[-1].append(i)
            else:
                groups.append([i])
        group_name = ["compress" if len(gr) > 1 else stages[gr[0]][0] for gr in groups]
        if not graph:
            def run_unit(unit):
                return lambda: [stages[i][1]() for i in unit]
            self.step()
            return [run_unit(gr) for gr in groups], group_name, [fn for _, fn, _, _ in stages]

        def capture(units):
            out = []
            for unit in units:                      # captured in execution order: the host-side
                g = torch.cuda.CUDAGraph()          # cache bookkeeping advances as in a real step
                with torch.cuda.graph(g):
                    for i in unit:
                        stages[i][1]()
                out.append(g.replay)
            torch.cuda.synchronize()
            for r in out:
                r()
            torch.cuda.synchronize()
            return out

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        return capture(groups), group_name, capture([[i] for i in range(len(stages))])

    def prefill_components(self, reps: int):
        """Outside the step: the prefill attention of Algorithm 2 on the same inputs
        (zc_prefill_attention, which also hands the probe rows' log-normalisers over) and the
        probe stage run on those normalisers (one sweep instead of two); milliseconds, mean /
        median / min over `reps` launches, HIP events around each."""
        w = self.w
        out = torch.empty_like(self.Q)
        lse = torch.empty(w.B, w.Hq, w.L, dtype=torch.float32, device=self.Q.device)
        lse_p = torch.empty(w.B, w.Hq, len(self.pos_np), dtype=torch.float32, device=self.Q.device)
        scores = torch.empty_like(self.scores)

        def timed(fn):
            fn(); fn()
            torch.cuda.synchronize()
            ts = []
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); fn(); e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            ts.sort()
            return {"mean": round(sum(ts) / len(ts), 5), "median": round(ts[len(ts) // 2], 5), "min": round(ts[0], 5)}

        pf = timed(lambda: zb.zc_prefill_attention(self.Q, self.K, self.V, out=out, lse=lse, probe_pos=self.pos, lse_probe=lse_p))
        pr = timed(lambda: zb.zc_probe_saliency(self.Q, self.K, self.pos, lse_ext=lse_p, scores=scores))
        flops = 4.0 * w.d * (w.L * (w.L + 1) / 2.0) * w.Hq * w.B          # unmasked (row, key) pairs, two products
        rel = float(((scores - self.scores).abs().max() / self.scores.abs().max()).item())
        assert rel <= 1e-4, f"one-sweep probe scores differ from the step's by {rel:.2e}"
        return {"prefill_attention_ms": pf, "prefill_attention_TFLOPs": flops / (pf["mean"] * 1e-3) / 1e12,
                "probe_saliency_given_prefill_lse_ms": pr,
                "probe_saliency_given_prefill_lse_TFLOPs": self.probe_flops() / (pr["mean"] * 1e-3) / 1e12}

    def decode_cold(self, reps: int):
        """Decode calls on the cache as the step leaves it, rotating through copies of it
        that together exceed 512 MiB, so that no call finds its lines in the last-level
        cache: microseconds per call (mean / median / min over `reps` replays of a graph
        that holds one call per copy) and the algorithmic bytes of such a call."""
        w = self.w
        hi = sum(c[1] for c in self.Kp.chunks); lo = sum(c[3] for c in self.Kp.chunks)
        base = self.n_flush * FLUSH_INTERVAL
        T = self.S - base
        nbytes = self.decode_bytes(hi, lo, self.Kp.c.n_chunks, T)
        copies = int(min(max(4, -(-(512 << 20) // int(nbytes))), 192))
        caches = [(self.Kp.clone(), self.Vp.clone(), self.tail_k[:, :, base:].clone(), self.tail_v[:, :, base:].clone())
                  for _ in range(copies)]
        q = self.q_all[:, :, self.S - 1:self.S]
        out = torch.empty_like(self.out[0])
        for Kp, Vp, tk, tv in caches[:2]:
            zb.zc_decode_attention(q, Kp, Vp, tk, tv, T, out=out)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for Kp, Vp, tk, tv in caches:
                zb.zc_decode_attention(q, Kp, Vp, tk, tv, T, out=out)
        gr.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); gr.replay(); e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3 / copies)
        ts.sort()
        assert torch.equal(out, self.out[self.S - 1]), "a copy of the cache decodes differently"
        return {"mean": round(sum(ts) / len(ts), 3), "median": round(ts[len(ts) // 2], 3), "min": round(ts[0], 3),
                "copies": copies, "bytes_per_launch": nbytes, "tail_len": T}


def cpu_baseline(hp: HotPath, decode_sample: int = 4):
    """The oracle, as it stands, on the host cores: the whole prefill part of one step
    plus `decode_sample` decode steps, stage by stage, extrapolated to the step's decode
    count; once with the thread count numpy's BLAS chooses by itself and once limited to
    one thread (batch elements are independent: one is timed and the result scaled)."""
    from oracle import zipcache_oracle as zo
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits = None
        cores = os.cpu_count() or 1
    w = hp.w
    nb = 1
    Q, K, V = (to_f64(hp.cpu_inputs[n][:nb]) for n in ("Q", "K", "V"))
    n = min(decode_sample, hp.S)

    def one_pass():
        t = [time.perf_counter()]
        scores, _ = zo.saliency_scores(Q, K, hp.pos_np)
        t.append(time.perf_counter())
        sal, reg = zip(*(zo.select_salient(scores[b], hp.k) for b in range(nb)))
        sal, reg = np.stack(sal), np.stack(reg)
        t.append(time.perf_counter())
        ck = zo.compress_tensor(K, sal, reg, w.bits_hi, w.bits_lo, "channel")
        cv = zo.compress_tensor(V, sal, reg, w.bits_hi, w.bits_lo, "cst")
        t.append(time.perf_counter())
        cache = zo.StreamingCache(Hkv=w.Hkv, chunks_K=[ck], chunks_V=[cv], n_packed=w.L)
        for j in range(n):
            d = hp.cpu_decode[j]
            cache.step(to_f64(d["q"][:nb]), to_f64(d["k_new"][:nb]), to_f64(d["v_new"][:nb]), False)
        t.append(time.perf_counter())
        st = {"probe_s": t[1] - t[0], "select_s": t[2] - t[1], "quantize_s": t[3] - t[2], "decode_step_s": (t[4] - t[3]) / n}
        st["step_s"] = (st["probe_s"] + st["select_s"] + st["quantize_s"] + st["decode_step_s"] * hp.S) * (w.B / nb)
        return st

    multi = one_pass()
    single = None
    if threadpool_limits is not None and multi["step_s"] * nb / w.B < 40.0:
        with threadpool_limits(limits=1):
            single = one_pass()
    out = {"value": w.B * hp.S / multi["step_s"], "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": f"float64 numpy oracle on {nb} of {w.B} batch elements: probe scores, split and quantize of the "
                     f"{w.name} prefill and {n} of {hp.S} decode steps, extrapolated to one whole step of the whole batch",
           "stages_s": {k: round(v, 4) for k, v in multi.items()}}
    if single is not None:
        out["single_thread"] = {"value": w.B * hp.S / single["step_s"], "stages_s": {k: round(v, 4) for k, v in single.items()}}
    return out


def machine_peaks(args):
    """What the GPU attains on the simplest code: a streaming read and a streaming copy of
    2 GiB (eight times the Infinity Cache, so every byte comes from HBM) and a register-only
    loop of 32x32x16 matrix instructions; best and median of `--steps` launches each."""
    import ctypes as C
    lib = C.CDLL(os.path.join(ROOT, "paper_2405_14256_amd", "libzc_peaks.so"))
    lib.zc_peak_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.zc_peak_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.zc_peak_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    st = torch.cuda.current_stream().cuda_stream
    nbytes = 2 << 30
    src = torch.randint(0, 2 ** 31 - 1, (nbytes // 4,), dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    iters, wgs = 512, n_cu * 8
    flops = wgs * 4 * iters * 8 * 2 * 32 * 32 * 16

    def timed(fn):
        for _ in range(max(args.warmup, 1)):
            assert fn() == 0
        ts = []
        for _ in range(max(args.steps, 3)):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            assert fn() == 0
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e-3)
        ts.sort()
        return ts[0], ts[len(ts) // 2]

    rd = timed(lambda: lib.zc_peak_read(src.data_ptr(), nbytes, sink.data_ptr(), st))
    cp = timed(lambda: lib.zc_peak_copy(dst.data_ptr(), src.data_ptr(), nbytes, st))
    assert torch.equal(dst[-4096:], src[-4096:]) and torch.equal(dst[:4096], src[:4096])
    mb = timed(lambda: lib.zc_peak_mfma(2, wgs, iters, sink.data_ptr(), st))
    mh = timed(lambda: lib.zc_peak_mfma(1, wgs, iters, sink.data_ptr(), st))
    print(json.dumps({
        "machine_peaks": {
            "read_TBps": {"best": nbytes / rd[0] / 1e12, "median": nbytes / rd[1] / 1e12, "bytes": nbytes},
            "copy_TBps_read_plus_write": {"best": 2 * nbytes / cp[0] / 1e12, "median": 2 * nbytes / cp[1] / 1e12, "bytes": 2 * nbytes},
            "mfma_bf16_PFLOPs": {"best": flops / mb[0] / 1e15, "median": flops / mb[1] / 1e15},
            "mfma_f16_PFLOPs": {"best": flops / mh[0] / 1e15, "median": flops / mh[1] / 1e15},
            "data_sheet": {"hbm_TBps": 8.0, "mfma_16bit_PFLOPs": 2.5},
            "compute_units": n_cu, "launches_timed": max(args.steps, 3),
        }}))


def latency_floor(args):
    """What a launch costs on this GPU before it does any work - the terms a latency-bound call
    (one decode step at batch 1 moves 3 MB: 0.4 us at the HBM peak) is made of.  Each line is
    the median and minimum over `--steps` repetitions, HIP events around each repetition:
      empty_eager        an empty kernel of 256 workgroups, 200 launches back to back, per launch
      empty_graph_node   the same 200 launches as nodes of one HIP graph, per node
      touch_graph_node   nodes that each make one trip to cold memory per workgroup and store a word
      dependent_pair     two such kernels, the second reading what the first stored (a producer
                         and its reduction), per pair, inside a graph
      memory_trip        one wave chasing dependent loads through a 1 GiB table: microseconds per hop"""
    import ctypes as C
    lib = C.CDLL(os.path.join(ROOT, "paper_2405_14256_amd", "libzc_peaks.so"))
    V, SZ, U32 = C.c_void_p, C.c_size_t, C.c_uint32
    lib.zc_peak_empty.argtypes = [C.c_int, V]
    lib.zc_peak_touch.argtypes = [V, SZ, SZ, C.c_int, U32, V, V]
    lib.zc_peak_chase.argtypes = [V, SZ, U32, C.c_int, V, V]
    dev = torch.device("cuda")
    st = lambda: torch.cuda.current_stream().cuda_stream
    WG, N = 256, 200
    big = torch.randint(0, 2 ** 31 - 1, ((1 << 30) // 4,), dtype=torch.int32, device=dev)     # 1 GiB: beyond the last-level cache
    nbytes = big.numel() * 4
    d1 = torch.zeros(4096, dtype=torch.int32, device=dev)
    d2 = torch.zeros(4096, dtype=torch.int32, device=dev)
    # a permutation whose successor is always far away: i -> (i + 1 + 2^22 + odd offset) mod n is one cycle
    n_tab = big.numel()
    step = (1 << 22) + 12345
    table = ((torch.arange(n_tab, dtype=torch.int64, device=dev) + step) % n_tab).to(torch.int32)
    reps = max(args.steps, 5)

    def graph_of(fn):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        torch.cuda.synchronize()
        return g.replay

    def timed(run, per):
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); run(); b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / per)
        ts.sort()
        return {"median_us": round(ts[len(ts) // 2], 3), "min_us": round(ts[0], 3)}

    salt = [0]

    def empties():
        for _ in range(N):
            assert lib.zc_peak_empty(WG, st()) == 0

    def touches():
        for i in range(N):      # every node reads lines no earlier node of this replay has read
            assert lib.zc_peak_touch(big.data_ptr() + (i * 4096 * WG) % (nbytes // 2), nbytes // 2, 4096, WG, i, d1.data_ptr(), st()) == 0

    def pairs():
        for i in range(N // 2):
            assert lib.zc_peak_touch(big.data_ptr() + (i * 4096 * WG) % (nbytes // 2), nbytes // 2, 4096, WG, i, d1.data_ptr(), st()) == 0
            assert lib.zc_peak_touch(d1.data_ptr(), 4096 * 4, 16, 32, i, d2.data_ptr(), st()) == 0

    out = {"empty_eager": timed(empties, N), "empty_graph_node": timed(graph_of(empties), N),
           "touch_graph_node": timed(graph_of(touches), N), "dependent_pair": timed(graph_of(pairs), N // 2)}
    hop = {}
    for hops in (1, 33):
        def chase(h=hops):
            salt[0] = (salt[0] + 7919) % n_tab
            assert lib.zc_peak_chase(table.data_ptr(), n_tab, salt[0], h, d2.data_ptr(), st()) == 0
        hop[hops] = timed(chase, 1)
    out["memory_trip"] = {"median_us": round((hop[33]["median_us"] - hop[1]["median_us"]) / 32, 3),
                          "min_us": round((hop[33]["min_us"] - hop[1]["min_us"]) / 32, 3),
                          "kernel_with_1_hop_us": hop[1], "kernel_with_33_hops_us": hop[33]}
    print(json.dumps({"latency_floor": out, "workgroups_per_kernel": WG, "launches_per_repetition": N, "repetitions": reps}))


def error_report(workload: str, decode_queries: int = 16, max_batch: int = 2):
    """Reconstruction and attention error against compression ratio for the quantization
    granularities of Table 1 (groupwise n = 32, tokenwise, channelwise keys with tokenwise or
    channel-separable tokenwise values) and for the two saliency metrics (Eq. 7 accumulated,
    Eq. 8 normalized) on a synthetic workload - what stands in for the paper's accuracy
    columns, which need datasets and weights.  Everything is computed by the library on the
    GPU: zc_quantize_pack + zc_unpack (zc_group_quantize for groupwise) for x_hat,
    zc_decode_attention over the packed cache (over x_hat as a full-precision tail for
    groupwise) against zc_decode_attention over the unquantized tensors for the attention
    error; torch only takes norms of differences.  Batch elements beyond `max_batch` are left
    out (the errors are per-token statistics)."""
    import dataclasses
    from oracle import zipcache_oracle as zo          # Appendix A's accounting formulas only
    w0 = WORKLOADS[workload]
    w = dataclasses.replace(w0, B=min(w0.B, max_batch))
    dev = torch.device("cuda")
    lib = zb.load()
    inp = make_prefill(w)
    Q, K, V = (inp[n].to(dev) for n in ("Q", "K", "V"))
    pos = torch.from_numpy(probes.probe_positions(w.L, w.probe_ratio, w.seed)).to(dev)
    qs = torch.stack([make_decode_step(w, j)["q"] for j in range(decode_queries)], dim=0).to(dev)    # [n, B, Hq, d]
    f32 = dict(dtype=torch.float32, device=dev)

    def empty_cache():
        mk = lambda s, l: zb.PackedTensor(w.B, w.Hkv, w.d, 64, 64, 4, 2, s, l, max_chunks=1, device="cuda")
        return mk("channel", zb.ZC_LAYOUT_ROW), mk("cst", zb.ZC_LAYOUT_TGROUP)

    def attend_tail(Kt, Vt):
        Ke, Ve = empty_cache()
        return torch.stack([zb.zc_decode_attention(qs[j], Ke, Ve, Kt, Vt, w.L).float() for j in range(decode_queries)])

    def attend_packed(Kp, Vp):
        return torch.stack([zb.zc_decode_attention(qs[j], Kp, Vp).float() for j in range(decode_queries)])

    o_ref = attend_tail(K, V)

    def rel_mse(xh, X):
        X = X.float()
        return float(((xh - X) ** 2).sum() / (X ** 2).sum())

    def x_hat(P):
        """[B, H, L, d] de-quantized tensor of a packed cache (token order)."""
        out = torch.zeros(w.B, w.Hkv, w.L, w.d, **f32)
        zb.zc_dequantize_cache(P, out)
        return out

    def pack(scheme_k, scheme_v, bits_hi, bits_lo, sal, reg):
        cap_hi, cap_lo = lib.zc_arena_slots(sal.shape[1], 1), lib.zc_arena_slots(reg.shape[1], 1)
        Kp = zb.PackedTensor(w.B, w.Hkv, w.d, cap_hi, cap_lo, bits_hi, bits_lo, scheme_k, zb.ZC_LAYOUT_ROW, max_chunks=1, device="cuda")
        Vp = zb.PackedTensor(w.B, w.Hkv, w.d, cap_hi, cap_lo, bits_hi, bits_lo, scheme_v, zb.ZC_LAYOUT_TGROUP, max_chunks=1, device="cuda")
        zb.zc_quantize_pack(K, sal, reg, Kp)
        zb.zc_quantize_pack(V, sal, reg, Vp)
        return Kp, Vp

    def out_err(o):
        return float((o - o_ref).norm() / o_ref.norm())

    scores = zb.zc_probe_saliency(Q, K, pos)
    sal, reg = zb.zc_select_salient(scores, w.k_salient)
    all_idx, none_idx = zb.zc_select_salient(scores, w.L)
    hd, ratio = w.W, w.salient_ratio
    rows = []
    for bits_hi, bits_lo, s_idx, r_idx, label in ((4, 4, all_idx, none_idx, "4/4"), (w.bits_hi, w.bits_lo, sal, reg, f"{w.bits_hi}/{w.bits_lo}")):
        mixed = label != "4/4"
        for ks, vs, gran in (("group", "group", "groupwise"), ("token", "token", "tokenwise"),
                             ("channel", "token", "channel+token"), ("channel", "cst", "channel+cst")):
            if ks == "group":
                parts_k, parts_v = torch.zeros(w.B, w.L, w.W, **f32), torch.zeros(w.B, w.L, w.W, **f32)
                for idx, bits in ((s_idx, bits_hi), (r_idx, bits_lo)):
                    if idx.shape[1] == 0:
                        continue
                    for X, dst in ((K, parts_k), (V, parts_v)):
                        _, _, _, dq = zb.zc_group_quantize(X, bits, 32, idx, codes=False)
                        dst.scatter_(1, idx.long()[:, :, None].expand(-1, -1, w.W), dq)
                Kh = parts_k.view(w.B, w.L, w.Hkv, w.d).permute(0, 2, 1, 3).contiguous()
                Vh = parts_v.view(w.B, w.L, w.Hkv, w.d).permute(0, 2, 1, 3).contiguous()
                o = attend_tail(Kh.to(w.torch_dtype), Vh.to(w.torch_dtype))
            else:
                Kp, Vp = pack(ks, vs, bits_hi, bits_lo, s_idx, r_idx)
                Kh, Vh = x_hat(Kp), x_hat(Vp)
                o = attend_packed(Kp, Vp)
            cr = zo.compression_ratio(gran, w.B, hd, w.L, bits_hi, bits_lo if mixed else None, ratio if mixed else 1.0,
                                      subsets=2 if mixed else 1)
            rows.append({"k_scheme": ks, "v_scheme": vs, "bits": label, "k_rel_mse": rel_mse(Kh, K), "v_rel_mse": rel_mse(Vh, V),
                         "attn_out_rel_err": out_err(o), "compression_ratio": cr})
    # Eq. 7 against Eq. 8: which tokens get the high bit width, and what that does to the output
    sal_rows = []
    full = torch.arange(w.L, dtype=torch.int32, device=dev)
    for name, fn in (("normalized (Eq. 8)", zb.zc_probe_saliency), ("accumulated (Eq. 7)", zb.zc_probe_accumulated)):
        sc = fn(Q, K, pos)
        s_i, r_i = zb.zc_select_salient(sc, w.k_salient)
        Kp, Vp = pack("channel", "cst", w.bits_hi, w.bits_lo, s_i, r_i)
        sc_full = fn(Q, K, full)                        # the same metric from the full attention matrix
        s_full, _ = zb.zc_select_salient(sc_full, w.k_salient)
        overlap = float(np.mean([len(set(s_i[b].tolist()) & set(s_full[b].tolist())) / max(w.k_salient, 1) for b in range(w.B)]))
        sal_rows.append({"metric": name, "attn_out_rel_err": out_err(attend_packed(Kp, Vp)),
                         "mean_salient_position": float(s_i.float().mean()) / w.L,
                         "overlap_with_full_matrix_selection": overlap})
    torch.cuda.synchronize()
    return {"error_report": workload, "batch_elements": w.B, "seq_len": w.L, "decode_queries": decode_queries,
            "salient_ratio": ratio, "granularities": rows, "saliency_metrics": sal_rows}


def decode_sweep(args):
    """Decode entry point alone at the metric's layer shape, batch 1 -> 64: each size is
    timed "warm" (the same packed cache every call: it stays in the last-level cache) and
    "cold" (calls rotate through copies of the cache that together exceed 512 MiB, so no
    call finds its lines cached).  A least-squares line t = t0 + bytes / BW over the cold
    points gives the fixed cost of a call and the asymptotic bandwidth."""
    import dataclasses
    w0 = WORKLOADS[args.workload]
    lib = zb.load()
    dev = torch.device("cuda")
    rows = []
    for B in (1, 2, 4, 8, 16, 32, 64):
        w = dataclasses.replace(w0, B=B)
        g = torch.Generator(device=dev).manual_seed(w.seed)
        K = torch.randn(B, w.Hkv, w.L, w.d, device=dev, generator=g).to(w.torch_dtype)
        V = torch.randn(B, w.Hkv, w.L, w.d, device=dev, generator=g).to(w.torch_dtype)
        q = torch.randn(B, w.Hq, 1, w.d, device=dev, generator=g).to(w.torch_dtype)
        scores = torch.rand(B, w.L, device=dev, generator=g)
        k = w.k_salient
        sal, reg = zb.zc_select_salient(scores, k)
        eb = 4 if w.dtype == "fp32" else 2
        nbytes = (2 * B * w.W * (w.bits_hi * k + w.bits_lo * (w.L - k)) / 8 + 8 * B * w.L
                  + 2 * B * w.W * 12 + 2 * B * w.Hq * w.d * eb)
        copies = int(min(max(4, -(-(512 << 20) // int(nbytes))), 192))
        caches = []
        for _ in range(copies):
            mk = lambda scheme, layout: zb.PackedTensor(B, w.Hkv, w.d, lib.zc_arena_slots(k, 1),
                                                        lib.zc_arena_slots(w.L - k, 1), w.bits_hi, w.bits_lo,
                                                        scheme, layout, max_chunks=1, device="cuda", store_pos=False)
            Kp, Vp = mk("channel", zb.ZC_LAYOUT_ROW), mk("cst", zb.ZC_LAYOUT_TGROUP)
            zb.zc_quantize_pack(K, sal, reg, Kp)
            zb.zc_quantize_pack(V, sal, reg, Vp)
            caches.append((Kp, Vp))
        del K, V
        out = torch.empty(B, w.Hq, w.d, dtype=w.torch_dtype, device=dev)
        torch.cuda.synchronize()

        def timed(seq, reps):
            for Kp, Vp in seq[:2]:
                zb.zc_decode_attention(q, Kp, Vp, out=out)
            torch.cuda.synchronize()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                for Kp, Vp in seq:
                    zb.zc_decode_attention(q, Kp, Vp, out=out)
            gr.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                gr.replay()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / (reps * len(seq))

        reps = max(2, 400 // copies)
        cold_us = timed(caches, reps)
        warm_us = timed([caches[0]] * min(copies, 32), max(2, 400 // min(copies, 32)))
        rows.append({"batch": B, "bytes_per_call": nbytes, "copies": copies, "cold_us": cold_us, "warm_us": warm_us,
                     "cold_GBps": nbytes / cold_us * 1e-3, "warm_GBps": nbytes / warm_us * 1e-3,
                     "cold_frac_of_peak": nbytes / cold_us * 1e-3 / HBM_PEAK_GBPS})
        del caches
        torch.cuda.empty_cache()
    x = np.array([r["bytes_per_call"] for r in rows]); y = np.array([r["cold_us"] for r in rows])
    slope, t0 = np.polyfit(x, y, 1)
    print(json.dumps({"sweep": "zc_decode_attention alone, batch 1..64 at the layer shape of " + w0.name,
                      "fit_cold": {"t0_us": float(t0), "asymptotic_GBps": float(1e-3 / slope)}, "rows": rows}))


TIMELINE_MARKS = ["entry", "arguments in registers", "query operand built", "first block in LDS", "half-blocks done",
                  "segments folded", "at the merge barrier", "result stored", "tail units done"]


def decode_timeline(args):
    """One decode call in slow motion.  Loads the traced build of the library, compresses the
    workload's prompt, replays a graph of eight decode calls a few times and reads the time
    stamps of the last call: per mark the minimum, median and maximum over the waves that
    reached it, in microseconds after the first wave's entry; the reduce kernel likewise; and
    the period of a call from the same graph's HIP events."""
    import ctypes as C
    trace_lib = os.path.join(os.path.dirname(zb.LIB_PATH), "libzipcache_trace.so")
    if not os.path.exists(trace_lib):
        raise SystemExit(f"{trace_lib} is missing: run `python __graft_entry__.py`")
    zb.LIB_PATH = trace_lib
    lib = zb.load()
    lib.zc_trace_fetch.restype = C.c_int
    lib.zc_trace_fetch.argtypes = [C.c_void_p, C.c_size_t, C.c_int]
    w = WORKLOADS[args.workload]
    if w.dtype != "bf16":
        raise SystemExit("--decode-timeline: only the bf16 kernels of the traced build carry time stamps")
    hp = HotPath(w)
    for _, fn, _, _ in hp.stages()[:3]:               # probe, select, quantize
        fn()
    T = min(args.tail_len, hp.tail_k.shape[2])
    calls = 8

    def call(j):
        zb.zc_decode_attention(hp.q_all[:, :, j:j + 1], hp.Kp, hp.Vp, hp.tail_k, hp.tail_v, T, out=hp.out[j])

    for j in range(3):
        call(j)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for j in range(calls):
            call(j)
    SLOTS, WAVES, HEADS = 16, 8192, 2048
    buf = np.zeros(WAVES * SLOTS + HEADS * 4, np.uint64)
    assert lib.zc_trace_fetch(None, 0, 1) == 0        # clear what the eager calls left
    periods = []
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); g.replay(); e1.record()
        torch.cuda.synchronize()
        periods.append(e0.elapsed_time(e1) * 1e3 / calls)
    assert lib.zc_trace_fetch(buf.ctypes.data, buf.size, 0) == 0
    waves = buf[:WAVES * SLOTS].reshape(WAVES, SLOTS).astype(np.int64)
    waves = waves[waves[:, 0] != 0]
    heads = buf[WAVES * SLOTS:].reshape(HEADS, 4).astype(np.int64)
    heads = heads[heads[:, 0] != 0]
    t0 = waves[:, 0].min()

    def stats(col):
        col = (col[col != 0] - t0) * 0.01             # 100 MHz counter -> microseconds
        return None if col.size == 0 else {"waves": int(col.size), "min": round(float(col.min()), 2),
                                           "median": round(float(np.median(col)), 2), "max": round(float(col.max()), 2)}

    out = {"mode": "decode-timeline", "workload": w.name, "tail_len": int(T), "unit": "us after the first wave's entry",
           "call_period_us": round(sorted(periods)[len(periods) // 2], 3),
           "k_decode_mfma": {name: stats(waves[:, i]) for i, name in enumerate(TIMELINE_MARKS)},
           "k_decode_reduce": {name: stats(heads[:, i]) for i, name in enumerate(["entry", "partials landed", "end"])},
           "note": "time stamps of the last of eight calls in a replayed graph; the traced kernels are a little slower "
                   "than the library's (a mark costs a scalar memory instruction and a store)"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b_4k")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the passes after the timed region (cold-cache decode, prefill attention and the one-sweep probe)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, run three plain copies of 256 MiB (a kernel of known traffic, "
                         "for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--peaks", action="store_true",
                    help="instead of the step: time the machine-peak probes (streaming read, streaming copy, a loop "
                         "of matrix instructions) and print what this GPU attains as one JSON line")
    ap.add_argument("--latency-floor", action="store_true",
                    help="instead of the step: time what a launch costs before it does any work (empty kernels, "
                         "graph nodes, a dependent pair, one trip to memory) and print it as one JSON line")
    ap.add_argument("--error-report", action="store_true",
                    help="instead of the step: reconstruction and attention error against compression ratio for the "
                         "granularities of Table 1 and the two saliency metrics, one JSON line per workload given")
    ap.add_argument("--decode-sweep", action="store_true",
                    help="instead of the step: time the decode entry point alone at batch 1..64 of the "
                         "workload's layer shape, cold and warm caches, and print that table as one JSON line")
    ap.add_argument("--decode-timeline", action="store_true",
                    help="instead of the step: what one decode call's latency is made of - time stamps the decode "
                         "kernels of the traced build of the library (libzipcache_trace.so, bf16 workloads) write at "
                         "their phase boundaries; medians over the waves of a call, one JSON line")
    ap.add_argument("--tail-len", type=int, default=50, help="--decode-timeline: tokens in the full-precision tail")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if args.decode_timeline:
        decode_timeline(args)
        return
    zb.load()
    if args.peaks:
        machine_peaks(args)
        return
    if args.latency_floor:
        latency_floor(args)
        return
    if args.error_report:
        print(json.dumps(error_report(args.workload)))
        return
    if args.decode_sweep:
        decode_sweep(args)
        return
    w = WORKLOADS[args.workload]
    hp = HotPath(w)

    # ---- warm-up (eager), then capture every stage of the step in its own HIP graph ----------
    for _ in range(max(args.warmup, 1)):
        hp.step()
    torch.cuda.synchronize()
    stages = hp.stages()
    runners, group_name, stage_runners = hp.launch_units(stages, graph=not args.no_graph)
    dec_bytes_step = sum(getattr(fn, "nbytes", 0.0) for name, fn, _, _ in stages if name == "decode")
    n_dec = sum(nc for name, _, nc, _ in stages if name == "decode")

    # ---- timed region: exactly K steps; HIP events between the launch units ----------------
    def timed(rs):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(rs) + 1)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            ev[k][0].record()
            for i, r in enumerate(rs):
                r()
                ev[k][i + 1].record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # [step][unit] milliseconds
        return dt, [[ev[k][i].elapsed_time(ev[k][i + 1]) for i in range(len(rs))] for k in range(args.steps)]

    def stats(xs):
        xs = sorted(xs)
        return {"mean": sum(xs) / len(xs), "median": xs[len(xs) // 2], "min": xs[0]}

    def per_step(ms, names, key):
        """One value per timed step: the sum of the units called `key` in that step."""
        return [sum(v for n, v in zip(names, row) if n == key) for row in ms]

    dt, unit_ms = timed(runners)
    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = w.B * hp.S * args.steps / dt
    st_ms = {n: stats(per_step(unit_ms, group_name, n)) for n in dict.fromkeys(group_name)}
    # the split of the compression graph into its stages: a second pass over the same step,
    # one graph per stage (outside the timed region; `value` does not depend on it)
    _, stage_ms = timed(stage_runners)
    names = [name for name, _, _, _ in stages]
    for n in ("probe", "select", "quantize"):
        st_ms[n] = stats(per_step(stage_ms, names, n))
    st_ms.setdefault("flush", {"mean": 0.0, "median": 0.0, "min": 0.0})
    dec_us = {k: v / n_dec * 1e3 for k, v in st_ms["decode"].items()}      # per launch, the step's average
    dec_avg_bytes = dec_bytes_step / n_dec
    achieved = dec_avg_bytes / (dec_us["mean"] * 1e-6) / 1e9
    quant_gbps = hp.quant_bytes() / (st_ms["quantize"]["mean"] * 1e-3) / 1e9
    probe_tflops = hp.probe_flops() / (st_ms["probe"]["mean"] * 1e-3) / 1e12
    cold = None if args.no_cold else hp.decode_cold(max(args.steps, 5))
    prefill = None if args.no_cold else hp.prefill_components(max(args.steps, 5))
    traffic = measured_decode_traffic(w.name)

    result = {
        "metric": "KV quantize-pack GB/s + packed decode-attn tokens/s, LLaMA3-8B shape @4k",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp16": "f16", "fp32": "f32"}[w.dtype], "data": "synthetic",
        "config": {"workload": w.name, "batch": w.B, "q_heads": w.Hq, "kv_heads": w.Hkv, "head_dim": w.d,
                   "seq_len": w.L, "probe_rows": int(len(hp.pos_np)), "salient_tokens": hp.k,
                   "bits": f"{w.bits_hi}/{w.bits_lo}", "decode_steps": hp.S, "flush_interval": FLUSH_INTERVAL,
                   "k_scheme": "channel", "v_scheme": "cst",
                   "launch": "eager" if args.no_graph else "hipgraph replay: one graph for probe + select + quantize, one per decode range, one per flush"},
        "components": {
            "quantize_pack_GBps": quant_gbps, "quantize_pack_ms": st_ms["quantize"]["mean"],
            "decode_attention_tokens_per_s": w.B / (dec_us["mean"] * 1e-6), "decode_attention_us_per_launch": dec_us["mean"],
            "probe_saliency_TFLOPs": probe_tflops, "probe_saliency_ms": st_ms["probe"]["mean"],
            "select_ms": st_ms["select"]["mean"], "flush_ms": st_ms["flush"]["mean"],
            "compress_ms": st_ms.get("compress", {"mean": 0.0})["mean"],
            "per_step_ms": {n: {k: round(v, 5) for k, v in d.items()} for n, d in st_ms.items()},
            "decode_us_per_launch": {"warm": {k: round(v, 3) for k, v in dec_us.items()}, "cold": cold},
            "prefill": prefill,
            "timing": "HIP events between the graphs inside the timed region (decode, flush, compress = probe + select + "
                      "quantize as one graph), mean / median / min over the timed steps; probe / select / quantize alone "
                      "from a second pass with one graph per stage; decode 'warm' is the timed region itself (one layer: "
                      "every call re-reads the cache the previous call read, so it is served from the last-level "
                      "cache), 'cold' a separate pass in which the calls rotate through copies of the final cache that "
                      "together exceed 512 MiB (every call reads HBM)"},
        "roofline": {"bound": "hbm", "kernel": "zc_decode_attention (k_decode_mfma + k_decode_reduce)",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "bytes_per_launch": dec_avg_bytes, "avg_launch_us": dec_us["mean"],
                     "cache_state": "warm (timed region)",
                     "traffic": traffic["bytes_per_launch"] if traffic else None,
                     "traffic_source": traffic["source"] if traffic else None},
    }
    if cold:
        result["roofline"]["cold"] = {"achieved": cold["bytes_per_launch"] / (cold["mean"] * 1e-6) / 1e9,
                                      "frac": cold["bytes_per_launch"] / (cold["mean"] * 1e-6) / 1e9 / HBM_PEAK_GBPS}
    if w.name != "llama3_8b_4k":
        result["metric"] += f" (supplementary workload {w.name})"
    if args.calibrate_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(hp)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
