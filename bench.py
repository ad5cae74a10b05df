#!/usr/bin/env python3
"""Benchmark of the denoise step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5]

A "step" is one pass of the whole hot path over one batch of synthetic
input that is already resident in HBM: shared-prefix block attention,
confidence-threshold unmask over the vocabulary, and the K/V refresh of the
committed positions (done by the unmask call itself); every 8 steps the N rollouts are re-forked from one
parent block state (a new block starts), which is the fork bookkeeping, and
the prefix V is laid out once for the attention kernel (fdd_prefix_pack).
The default workload is the long multi-camera configuration (N=16 rollouts,
B=64, prefix L=16384, V=152064, bf16).

Prints ONE JSON line: whole-step throughput in rollout-tokens/s (N*B block
positions per step, scaffold included), the roofline of the dominant kernel
(attention on the matrix cores) from HIP events recorded around that kernel
inside the timed region, the HBM roofline of the vocabulary reduction, the
N=1 prefix-stream figures, and the fp64 CPU oracle timed on one full
repetition of the same step on this machine's host cores.

Before the timed region the same step runs untimed until 80 ms of GPU time
have passed (`preheat_ms`), whatever --warmup says: the shader clock needs
about 30 ms of load to settle, and a cold start reads 10..15 % low.  The
attention kernel is timed on at least 20 launches: when --steps gives fewer
samples inside the timed region, a post-pass of the same step supplies the
rest (`launches_timed` / `launches_timed_in_region`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Published MI355X peaks
PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0
PEAK_VALU_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12      # one 32-bit vector operation per lane and clock
SAMPLER_OPS_PER_ENTRY = 64                         # Philox share 20, uniform 4, two log2 36, key and compare 4
STEPS_PER_BLOCK = 8
# HBM bytes per launch, measured offline with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs of this file),
# each scaled by what the same counter reads for a 1 GiB device copy (`--copy-probe`; 0.5x and 1.0x).  The
# counters cannot be read from inside this process, so the line quotes the figure and says where it is from.
# (read MiB, write MiB) per launch.
MEASURED_TRAFFIC_MIB = {"cfg5": {"attn_bf16_kernel": (48.7, 15.3), "vocab_reduce_kernel": (192.9, 0.1)}}
TRAFFIC_SOURCE = "profiles/bench_cfg5_denoise_step.md (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; build of commit 41205d4)"
PREHEAT_MS = 80.0          # untimed GPU load before the timed region: the shader clock takes about 30 ms to settle
MIN_ATTN_SAMPLES = 20      # the attention kernel is timed on at least this many launches


def dev(a):
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def attn_flops(w):
    return 4.0 * w.N * w.B * w.Hq * (w.L + w.B) * w.D


def attn_bytes(w, es=2):
    prefix = 2 * w.L * w.Hkv * w.D * es
    block = 2 * w.N * w.B * w.Hkv * w.D * es
    qo = 2 * w.N * w.B * w.Hq * w.D * es
    return prefix, prefix + block + qo


EVENT_STRIDE = 5      # supplements: every this many calls carry the pair of timing events around the main kernel


class Events:
    """Pairs of timing events, created and recorded once so their handles exist."""

    def __init__(self, n):
        import torch
        self.pairs = []
        for _ in range(n):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            b.record()
            self.pairs.append((a, b))
        torch.cuda.synchronize()

    def mean_ms(self, used):
        return float(np.mean([a.elapsed_time(b) for a, b in self.pairs[:used]]))


def time_attention_only(F, w, steps, warmup, n_buffers, prepacked=False):
    """Attention alone on `n_buffers` distinct prefix buffers used in rotation
    (cold caches when their total size exceeds the 256 MB last-level cache).
    `prepacked`: the caller has laid the prefix V out beforehand (fdd_prefix_pack)."""
    import torch
    import fdd_workloads as W
    d = W.attention_inputs(w)
    q, bk, bv = dev(d["q"]), dev(d["block_k"]), dev(d["block_v"])
    pk0, pv0 = dev(d["prefix_k"]), dev(d["prefix_v"])
    pks = [pk0] + [pk0.clone() for _ in range(n_buffers - 1)]
    pvs = [pv0] + [pv0.clone() for _ in range(n_buffers - 1)]
    packs = [F.fdd_prefix_pack(v) if prepacked else None for v in pvs]
    out = torch.empty_like(q)
    ws_bytes = F.fdd_block_attn_workspace(q, pk0, pv0, bk, bv, prefix_v_packed=packs[0])
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    n_ev = (steps + EVENT_STRIDE - 1) // EVENT_STRIDE       # the kernel is timed on a sample of the calls (see main)
    ev = Events(n_ev)
    for i in range(warmup):
        F.fdd_block_attn(q, pks[i % n_buffers], pvs[i % n_buffers], bk, bv, out=out, workspace=ws,
                         prefix_v_packed=packs[i % n_buffers])
    torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    t0.record()
    for i in range(steps):
        F.fdd_profile_attn_events(*(ev.pairs[i // EVENT_STRIDE] if i % EVENT_STRIDE == 0 else (None, None)))
        F.fdd_block_attn(q, pks[i % n_buffers], pvs[i % n_buffers], bk, bv, out=out, workspace=ws,
                         prefix_v_packed=packs[i % n_buffers])
    t1.record()
    torch.cuda.synchronize()
    F.fdd_profile_attn_events(None, None)
    call_ms = t0.elapsed_time(t1) / steps
    kern_ms = ev.mean_ms(n_ev)
    prefix, total = attn_bytes(w)
    return {
        "workload": f"N={w.N} B={w.B} L={w.L} Hq={w.Hq} Hkv={w.Hkv} D={w.D} bf16, {n_buffers} rotating prefix buffers"
                    + (", prefix V laid out beforehand" if prepacked else ""),
        "call_us": round(call_ms * 1e3, 2), "kernel_us": round(kern_ms * 1e3, 2),
        "prefix_bytes": prefix, "prefix_GBs_kernel": round(prefix / (kern_ms * 1e-3) / 1e9, 1),
        "prefix_GBs_call": round(prefix / (call_ms * 1e-3) / 1e9, 1),
        "frac_peak_hbm_kernel": round(prefix / (kern_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        "frac_peak_hbm_call": round(prefix / (call_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        "rollout_tokens_per_s": round(w.N * w.B / (call_ms * 1e-3), 1),
        "tflops_kernel": round(attn_flops(w) / (kern_ms * 1e-3) / 1e12, 1),
        "frac_peak_mfma_kernel": round(attn_flops(w) / (kern_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "frac_peak_mfma_call": round(attn_flops(w) / (call_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
    }


def time_spec_verify(F, w, d, g, logits, steps, warmup):
    """Verify pass of scaffold speculative decoding at the bench workload:
    causal in-block attention, then the accept scan over the AR logits.  The
    mask state is restored by a fork before every pass (inside the timing)."""
    import torch
    scaffold = dev(d["scaffold_mask"])
    parent = {k: dev(d[k][0]) for k in ("block_k", "block_v", "tokens", "mask")}
    st = {k: torch.empty((w.N,) + tuple(parent[k].shape), dtype=parent[k].dtype, device="cuda") for k in parent}
    rng = np.random.default_rng([w.seed, 77])
    draft = dev(rng.integers(0, w.V, size=(w.N, w.B)).astype(np.int32))
    out = torch.empty_like(g["q"])
    nacc = torch.empty((w.N,), dtype=torch.int32, device="cuda")
    acc = torch.empty((w.N, w.B), dtype=torch.uint8, device="cuda")
    packed_v = F.fdd_prefix_pack(g["prefix_v"])
    ws_a = torch.empty(max(256, F.fdd_block_attn_workspace(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"],
                                                           st["block_v"], prefix_v_packed=packed_v)),
                       dtype=torch.uint8, device="cuda")
    ws_u = torch.empty(max(256, F.fdd_verify_workspace(logits[0]), F.fdd_verify_workspace(logits[0], temperature=1.0)),
                       dtype=torch.uint8, device="cuda")
    n_ev = (steps + EVENT_STRIDE - 1) // EVENT_STRIDE       # the event pairs sit on a sample of the passes (see main)
    ev = Events(n_ev)
    v0 = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev)]
    v1 = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev)]
    n_v = 0

    def one(i, timed):
        nonlocal n_v
        for k in ("tokens", "mask"):
            F.fdd_fork_block(parent[k], w.N, dst=st[k])
        F.fdd_profile_attn_events(*(ev.pairs[i // EVENT_STRIDE] if timed and i % EVENT_STRIDE == 0 else (None, None)))
        F.fdd_block_attn(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"], scaffold, out=out,
                         workspace=ws_a, prefix_v_packed=packed_v, causal_block=True)
        v_timed = timed and i % EVENT_STRIDE == EVENT_STRIDE // 2 and n_v < n_ev
        if v_timed:
            v0[n_v].record()
        F.fdd_verify_step(logits[i % 2], st["mask"], scaffold, draft, st["tokens"], nacc, acc, workspace=ws_u)
        if v_timed:
            v1[n_v].record()
            n_v += 1

    for k in ("block_k", "block_v"):
        F.fdd_fork_block(parent[k], w.N, dst=st[k])
    for i in range(warmup):
        one(i, False)
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for i in range(steps):
        one(i, True)
    t1.record()
    torch.cuda.synchronize()
    F.fdd_profile_attn_events(None, None)
    ms = t0.elapsed_time(t1) / steps
    attn_ms = ev.mean_ms(n_ev)
    ver_ms = float(np.mean([a.elapsed_time(b) for a, b in zip(v0[:n_v], v1[:n_v])]))
    # the sampled verifier of the trajectory section on the same rows
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_samp = max(4, steps // 5)
    for i in range(n_samp + 2):
        for k in ("tokens", "mask"):
            F.fdd_fork_block(parent[k], w.N, dst=st[k])
        if i == 2:
            s0.record()
        F.fdd_verify_step(logits[i % 2], st["mask"], scaffold, draft, st["tokens"], nacc, acc, workspace=ws_u,
                          temperature=1.0, seed=1000 + i)
    s1.record()
    torch.cuda.synchronize()
    samp_ms = s0.elapsed_time(s1) / n_samp
    elig = int(((d["mask"][0] == 1) & (d["scaffold_mask"][0] == 0)).sum()) * w.N
    byt = elig * w.V * 2
    # causal tail: position b sees L + b + 1 keys
    flops = 4.0 * w.N * w.Hq * w.D * sum(w.L + b + 1 for b in range(w.B))
    return {
        "workload": f"{w.name}: causal in-block attention + accept scan, N={w.N} B={w.B} L={w.L} V={w.V} bf16",
        "pass_us": round(ms * 1e3, 2), "rollout_tokens_per_s": round(w.N * w.B / (ms * 1e-3), 1),
        "attn_kernel_us": round(attn_ms * 1e3, 2), "attn_tflops": round(flops / (attn_ms * 1e-3) / 1e12, 1),
        "attn_frac_peak_mfma": round(flops / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "verify_call_us": round(ver_ms * 1e3, 2), "verify_rows": elig,
        "verify_GBs": round(byt / (ver_ms * 1e-3) / 1e9, 1),
        "verify_frac_peak_hbm": round(byt / (ver_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        # Gumbel-max sampling is bound by the vector ALUs: 64 vector operations per vocabulary entry by the
        # sampler's definition, against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
        "sampled_verify_call_us": round(samp_ms * 1e3, 2),
        "sampled_verify": {"bound": "alu", "unit": "Tops/s", "peak": PEAK_VALU_TOPS,
                           "achieved": round(elig * w.V * SAMPLER_OPS_PER_ENTRY / (samp_ms * 1e-3) / 1e12, 2),
                           "frac": round(elig * w.V * SAMPLER_OPS_PER_ENTRY / (samp_ms * 1e-3) / 1e12 / PEAK_VALU_TOPS, 4),
                           "entries_per_call": elig * w.V, "ops_per_entry": SAMPLER_OPS_PER_ENTRY},
    }


def time_layer_sweep_graph(F, w, n_layers, replays):
    """One decode step's worth of attention at N=1: `n_layers` calls on distinct
    prefix buffers (as the layers of a step are), recorded once into a HIP graph
    and replayed, which takes the per-call launch work off the host."""
    import torch
    import fdd_workloads as W
    d = W.attention_inputs(w)
    q, bk, bv = dev(d["q"]), dev(d["block_k"]), dev(d["block_v"])
    pk0, pv0 = dev(d["prefix_k"]), dev(d["prefix_v"])
    pks = [pk0] + [pk0.clone() for _ in range(n_layers - 1)]
    pvs = [pv0] + [pv0.clone() for _ in range(n_layers - 1)]
    packs = [F.fdd_prefix_pack(v) for v in pvs]
    outs = [torch.empty_like(q) for _ in range(n_layers)]
    ws = torch.empty(max(256, F.fdd_block_attn_workspace(q, pk0, pv0, bk, bv, prefix_v_packed=packs[0])), dtype=torch.uint8,
                     device="cuda")

    def sweep():
        for l in range(n_layers):
            F.fdd_block_attn(q, pks[l], pvs[l], bk, bv, out=outs[l], workspace=ws, prefix_v_packed=packs[l])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sweep()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sweep()
    times = {}
    for name, fn in (("eager", sweep), ("graph", graph.replay)):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record()
        for _ in range(replays):
            fn()
        t1.record()
        torch.cuda.synchronize()
        times[name] = t0.elapsed_time(t1) / replays / n_layers
    prefix, _ = attn_bytes(w)
    return {"workload": f"N={w.N} B={w.B} L={w.L} Hq={w.Hq} Hkv={w.Hkv} D={w.D} bf16, {n_layers} layers back to back "
                        f"on distinct prefix buffers, prefix V laid out beforehand",
            "eager_us_per_layer": round(times["eager"] * 1e3, 2), "graph_us_per_layer": round(times["graph"] * 1e3, 2),
            "prefix_GBs_graph": round(prefix / (times["graph"] * 1e-3) / 1e9, 1),
            "frac_peak_hbm_graph": round(prefix / (times["graph"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "rollout_tokens_per_s_graph": round(w.N * w.B / (times["graph"] * 1e-3), 1)}


def time_batched(F, w, P, reps):
    """P independent N=1 problems (each with its own prefix) in ONE launch: the prefix stream without the
    per-launch latencies that bound a single small problem."""
    import torch
    import fdd_workloads as W
    d = W.attention_inputs(w)
    rep = lambda a: dev(a).unsqueeze(0).repeat(P, *([1] * a.ndim)).contiguous()
    q, pk, pv, bk, bv = (rep(d[k]) for k in ("q", "prefix_k", "prefix_v", "block_k", "block_v"))
    pk += torch.randn(P, 1, 1, 1, device="cuda").to(pk.dtype) * 0.01       # the prefixes differ
    packed = torch.stack([F.fdd_prefix_pack(pv[i]) for i in range(P)])
    out = torch.empty_like(q)
    ws = torch.empty(max(256, F.fdd_block_attn_batched_workspace(q, pk, pv, bk, bv, prefix_v_packed=packed)),
                     dtype=torch.uint8, device="cuda")
    # rotate over copies of the prefixes so that they come from HBM, not from the last-level cache
    n_sets = max(2, int(600e6 // (2 * pk.numel() * 2)) + 1)
    sets = [(pk, packed)] + [(pk.clone(), packed.clone()) for _ in range(n_sets - 1)]
    n_ev = (reps + EVENT_STRIDE - 1) // EVENT_STRIDE
    ev = Events(n_ev)
    for i in range(3):
        F.fdd_block_attn_batched(q, sets[i % n_sets][0], pv, bk, bv, out=out, workspace=ws, prefix_v_packed=sets[i % n_sets][1])
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for i in range(reps):
        F.fdd_profile_attn_events(*(ev.pairs[i // EVENT_STRIDE] if i % EVENT_STRIDE == 0 else (None, None)))
        F.fdd_block_attn_batched(q, sets[i % n_sets][0], pv, bk, bv, out=out, workspace=ws, prefix_v_packed=sets[i % n_sets][1])
    t1.record()
    torch.cuda.synchronize()
    F.fdd_profile_attn_events(None, None)
    call_ms, kern_ms = t0.elapsed_time(t1) / reps, ev.mean_ms(n_ev)
    prefix = attn_bytes(w)[0] * P
    flops = attn_flops(w) * P
    return {"workload": f"{P} independent problems of N={w.N} B={w.B} L={w.L} Hq={w.Hq} Hkv={w.Hkv} D={w.D} bf16 in one "
                        f"launch, {n_sets} sets of prefixes in rotation, prefix V laid out beforehand",
            "call_us": round(call_ms * 1e3, 2), "kernel_us": round(kern_ms * 1e3, 2), "prefix_bytes": prefix,
            "prefix_GBs_kernel": round(prefix / (kern_ms * 1e-3) / 1e9, 1), "prefix_GBs_call": round(prefix / (call_ms * 1e-3) / 1e9, 1),
            "frac_peak_hbm_kernel": round(prefix / (kern_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "frac_peak_hbm_call": round(prefix / (call_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "tflops_kernel": round(flops / (kern_ms * 1e-3) / 1e12, 1),
            "frac_peak_mfma_kernel": round(flops / (kern_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "rollout_tokens_per_s": round(P * w.N * w.B / (call_ms * 1e-3), 1)}


def time_extension(F, w, d, g, steps, warmup):
    """Third block of the trajectory section: every rollout has committed two
    blocks of its own since the fork (E = 2B extension rows), plus the commit."""
    import torch
    st = {k: dev(d[k]) for k in ("block_k", "block_v")}
    E = 2 * w.B
    rng = np.random.default_rng([w.seed, 78])
    import fdd_workloads as W
    ext = [dev(W.to_storage(rng.standard_normal((w.N, 3 * w.B, w.Hkv, w.D)).astype(np.float32), w.dtype)) for _ in range(2)]
    out = torch.empty_like(g["q"])
    packed_v = F.fdd_prefix_pack(g["prefix_v"])
    ws = torch.empty(max(256, F.fdd_block_attn_workspace(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"],
                                                         prefix_v_packed=packed_v, ext_k=ext[0], ext_v=ext[1], E=E),
                         F.fdd_block_attn_workspace(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"],
                                                    prefix_v_packed=packed_v)),
                     dtype=torch.uint8, device="cuda")
    def loop(**kw):
        ev = Events(steps)
        for i in range(warmup + steps):
            if i >= warmup:
                F.fdd_profile_attn_events(*ev.pairs[i - warmup])
            F.fdd_block_attn(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"], out=out, workspace=ws,
                             prefix_v_packed=packed_v, **kw)
        torch.cuda.synchronize()
        F.fdd_profile_attn_events(None, None)
        return ev.mean_ms(steps)
    # (attention calls back to back run at a lower clock than inside a step, where the memory-bound unmask
    # pass gives the chip a rest: the plain call is timed the same way for comparison)
    base_ms = loop()
    attn_ms = loop(ext_k=ext[0], ext_v=ext[1], E=E)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for i in range(20):
        F.fdd_block_commit(st["block_k"], st["block_v"], ext[0], ext[1], E)
    c1.record()
    torch.cuda.synchronize()
    flops = 4.0 * w.N * w.B * w.Hq * (w.L + E + w.B) * w.D
    return {"workload": f"{w.name} with E={E} private extension rows per rollout",
            "attn_kernel_us": round(attn_ms * 1e3, 2), "attn_tflops": round(flops / (attn_ms * 1e-3) / 1e12, 1),
            "attn_frac_peak_mfma": round(flops / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "attn_kernel_us_without_extension_same_loop": round(base_ms * 1e3, 2),
            "commit_call_us": round(c0.elapsed_time(c1) / 20 * 1e3, 2),
            "commit_bytes": 4 * w.N * w.B * w.Hkv * w.D * 2}


def time_scaffold_skip(F, w, d, g, steps, warmup):
    """The last layer of a step: only non-scaffold positions need an output row."""
    import torch
    import fdd_workloads as W
    st = {k: dev(d[k]) for k in ("block_k", "block_v")}
    scaffold = W.scaffold_positions(w, np.random.default_rng(w.seed))
    pos = torch.from_numpy(np.flatnonzero(scaffold.reshape(-1) == 0).astype(np.int32)).cuda()
    out = torch.zeros_like(g["q"])
    packed_v = F.fdd_prefix_pack(g["prefix_v"])
    ws = torch.empty(max(256, F.fdd_block_attn_workspace(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"],
                                                         prefix_v_packed=packed_v, n_q_positions=pos.numel()),
                         F.fdd_block_attn_workspace(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"],
                                                    prefix_v_packed=packed_v)),
                     dtype=torch.uint8, device="cuda")
    def loop(**kw):
        ev = Events(steps)
        for i in range(warmup + steps):
            if i >= warmup:
                F.fdd_profile_attn_events(*ev.pairs[i - warmup])
            F.fdd_block_attn(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"], out=out, workspace=ws,
                             prefix_v_packed=packed_v, **kw)
        torch.cuda.synchronize()
        F.fdd_profile_attn_events(None, None)
        return ev.mean_ms(steps)
    base_ms = loop()                    # all positions, timed the same way (calls back to back)
    ms = loop(q_positions=pos)
    flops = 4.0 * pos.numel() * w.Hq * (w.L + w.B) * w.D
    return {"workload": f"{w.name}, query rows of the {pos.numel()} non-scaffold positions of {w.N * w.B}",
            "attn_kernel_us": round(ms * 1e3, 2), "attn_tflops": round(flops / (ms * 1e-3) / 1e12, 1),
            "attn_frac_peak_mfma": round(flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "attn_kernel_us_all_positions_same_loop": round(base_ms * 1e3, 2)}


def cpu_baseline(w, d, logits):
    """The fp64 oracle as it stands on ONE full, unscaled repetition of the step: attention on every output
    row, then the unmask on every block (the K/V refresh is a copy of a few rows and is left out)."""
    import oracle
    t = time.perf_counter()
    oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"])
    t_attn = time.perf_counter() - t
    t_un = 0.0
    if logits is not None:
        t = time.perf_counter()
        oracle.unmask_step(logits, d["mask"], d["scaffold_mask"], d["tokens"], float(np.float32(w.tau)))
        t_un = time.perf_counter() - t
    t_step = t_attn + t_un
    return {
        "value": round(w.N * w.B / t_step, 2), "unit": "rollout-tokens/s", "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"one full step of {w.name}, unscaled: attention on all {w.N * w.B * w.Hq} output rows "
                  f"({t_attn:.2f} s) and unmask on all {w.N} blocks ({t_un:.2f} s); {t_step:.2f} s per step",
        "host_cpu_count": os.cpu_count(),
    }


def copy_probe(mib, reps):
    """A plain device-to-device copy of known size, for calibrating the HBM byte counters: run under
    `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE); each copy dispatch reads `mib` MiB and writes `mib` MiB,
    so (counter reading in KiB) / (mib * 1024) is the factor other kernels' readings are divided by."""
    import torch
    n = mib << 20
    x = torch.empty(n, dtype=torch.uint8, device="cuda")
    x.random_(0, 255)
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    for _ in range(reps):
        y.copy_(x)
    torch.cuda.synchronize()
    print(json.dumps({"copy_probe": {"mib": mib, "reps": reps, "bytes_read_per_dispatch": n, "bytes_written_per_dispatch": n}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)   # the shader clock takes about 30 ms of load to settle
    ap.add_argument("--workload", default="cfg5", choices=["cfg3", "cfg4", "cfg5"])
    ap.add_argument("--event-stride", type=int, default=5,
                    help="every this many timed steps carry the timing events the rooflines are measured with")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-supplements", action="store_true")
    ap.add_argument("--n1-only", action="store_true",
                    help="run only the N=1 layer sweeps (for profiling them) and print their figures")
    ap.add_argument("--attn-only", default=None, metavar="WORKLOAD",
                    help="run only the attention call of this workload (cfg2, cfg3, n1_L16384) for profiling it")
    ap.add_argument("--prepacked", action="store_true", help="with --attn-only: lay the prefix V out beforehand")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="run only a device copy of this many MiB, five times (calibration of the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1")

    import torch
    import fdd_workloads as W
    import paper_2605_23163_amd as F

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    F.load_library()
    torch.cuda.set_device(0)

    if args.copy_probe > 0:
        copy_probe(args.copy_probe, 5)
        return
    if args.attn_only:
        wl = dict(W.CONFIGS)
        wl["n1_L16384"] = W.Workload("n1_L16384", N=1, B=32, L=16384, Hq=28, Hkv=4, D=128, dtype=W.BF16, seed=12)
        wa = wl[args.attn_only]
        nbuf = max(1, int(600e6 // attn_bytes(wa)[0]))      # rotate over more than the last-level cache holds
        print(json.dumps({args.attn_only: time_attention_only(F, wa, args.steps, args.warmup, min(nbuf, 128),
                                                              prepacked=args.prepacked)}))
        return
    if args.n1_only:
        n1 = W.CONFIGS["cfg2"]
        n1_long = W.Workload("n1_L16384", N=1, B=32, L=16384, Hq=28, Hkv=4, D=128, dtype=W.BF16, seed=12)
        print(json.dumps({"n1_layer_sweep": time_layer_sweep_graph(F, n1, 28, 20),
                          "n1_layer_sweep_L16384": time_layer_sweep_graph(F, n1_long, 28, 10),
                          "n1_batched": time_batched(F, n1, 28, 50),
                          "n1_batched_L16384": time_batched(F, n1_long, 8, 30)}))
        return

    w = W.CONFIGS[args.workload]
    d = W.full_step_inputs(w, n_logit_steps=2)
    g = {k: dev(d[k]) for k in ("q", "prefix_k", "prefix_v")}
    scaffold = dev(d["scaffold_mask"])
    has_unmask = w.V > 0
    logits_h = None
    if has_unmask:
        # two distinct logits buffers in rotation (> 256 MB together at the default workload)
        lrng = [np.random.default_rng([w.seed, 1000 + s]) for s in range(2)]
        logits_h = W.step_logits(w, d["mask"], lrng[0])
        logits = [dev(logits_h), dev(W.step_logits(w, d["mask"], lrng[1]))]
        tk, tv = dev(d["table_k"]), dev(d["table_v"])
    # parent block state the rollouts are forked from at the start of every block
    parent = {k: dev(d[k][0]) for k in ("block_k", "block_v", "tokens", "mask")}
    st = {k: torch.empty((w.N,) + tuple(parent[k].shape), dtype=parent[k].dtype, device="cuda") for k in parent}
    out = torch.empty_like(g["q"])
    conf = torch.empty((w.N, w.B), dtype=torch.float32, device="cuda")
    nun = torch.empty((w.N,), dtype=torch.int32, device="cuda")
    com = torch.empty((w.N, w.B), dtype=torch.uint8, device="cuda")
    packed_v = torch.empty(max(256, F.fdd_prefix_pack_bytes(g["prefix_v"])), dtype=torch.uint8, device="cuda")
    ws_a = torch.empty(max(256, F.fdd_block_attn_workspace(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"],
                                                           st["block_v"], prefix_v_packed=packed_v)),
                       dtype=torch.uint8, device="cuda")
    ws_u = torch.empty(max(256, F.fdd_unmask_workspace(logits[0]) if has_unmask else 256), dtype=torch.uint8,
                       device="cuda")
    tau = float(np.float32(w.tau))

    # Kernel timings for the rooflines are taken live in the timed region, on a sample of its steps: a pair
    # of timing events costs a few microseconds of idle GPU around the kernel it brackets, so only every
    # `stride`-th step carries the pair around the attention kernel and another one the pair around the
    # unmask call.  The stride is odd: the samples cover the 8 steps of a block evenly.
    stride = max(1, min(args.event_stride, args.steps // 2 if args.steps >= 2 else 1))   # both pairs get samples
    n_samples = (args.steps + stride - 1) // stride
    ev = Events(n_samples)
    un_ev = Events(n_samples)

    def step(i, attn_pair=None, un_pair=None, set_hook=False):
        if set_hook:
            F.fdd_profile_attn_events(*(attn_pair if attn_pair else (None, None)))
        if i % STEPS_PER_BLOCK == 0:
            # a new block: fork the rollouts and lay the (unchanged) prefix V out for the kernel once
            for k in parent:
                F.fdd_fork_block(parent[k], w.N, dst=st[k])
            F.fdd_prefix_pack(g["prefix_v"], packed=packed_v)
        F.fdd_block_attn(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"], scaffold, out=out,
                         workspace=ws_a, prefix_v_packed=packed_v)
        if has_unmask:
            if un_pair:
                un_pair[0].record()
            # (the K/V refresh of the committed positions is done by the unmask call's own select kernel)
            F.fdd_unmask_step(logits[i % 2], st["mask"], scaffold, tau, st["tokens"], conf, nun, com, workspace=ws_u,
                              refresh=(tk, tv, st["block_k"], st["block_v"]))
            if un_pair:
                un_pair[1].record()

    def sampled(i, i_rel, pairs_a, pairs_u):
        # step i of the block cycle, the i_rel-th step of a sampled stretch: every `stride`-th step carries the
        # pair around the attention kernel, another one the pair around the unmask call
        a = pairs_a[i_rel // stride] if i_rel % stride == 0 else None
        u = pairs_u[i_rel // stride] if (i_rel % stride == stride // 2 and i_rel // stride < len(pairs_u)) else None
        step(i, a, u, set_hook=True)
        return u is not None

    # Untimed pre-heat, whatever --warmup says: whole blocks of the same step until PREHEAT_MS of GPU time have
    # passed, so that the timed region starts at the clock the chip sustains under this load.
    h0, h1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    h0.record()
    preheat_ms, preheat_steps = 0.0, 0
    while preheat_ms < PREHEAT_MS:
        for i in range(2 * STEPS_PER_BLOCK):
            step(i)
        preheat_steps += 2 * STEPS_PER_BLOCK
        h1.record()
        h1.synchronize()
        preheat_ms = h0.elapsed_time(h1)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    t0.record()
    n_un = 0
    for i in range(args.steps):
        n_un += sampled(i, i, ev.pairs, un_ev.pairs)
    t1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    F.fdd_profile_attn_events(None, None)
    ms_step = t0.elapsed_time(t1) / args.steps
    attn_samples = [a.elapsed_time(b) for a, b in ev.pairs[:n_samples]]
    un_samples = [a.elapsed_time(b) for a, b in un_ev.pairs[:n_un]]
    n_in_region = n_samples
    # Post-pass outside the headline timing: the same step goes on until both kernels have been timed on
    # MIN_ATTN_SAMPLES launches in all (a short --steps run has too few samples inside the timed region).
    if n_in_region < MIN_ATTN_SAMPLES:
        extra = MIN_ATTN_SAMPLES - n_in_region
        ev2, un2 = Events(extra), Events(extra)
        i0 = ((args.steps + STEPS_PER_BLOCK - 1) // STEPS_PER_BLOCK) * STEPS_PER_BLOCK    # a new block starts here
        n2 = 0
        for j in range(extra * stride):
            n2 += sampled(i0 + j, j, ev2.pairs, un2.pairs)
        torch.cuda.synchronize()
        F.fdd_profile_attn_events(None, None)
        attn_samples += [a.elapsed_time(b) for a, b in ev2.pairs]
        un_samples += [a.elapsed_time(b) for a, b in un2.pairs[:n2]]
    attn_ms = float(np.mean(attn_samples))
    tokens_per_s = w.N * w.B / (ms_step * 1e-3)

    flops = attn_flops(w)
    res = {
        "metric": "rollout-tokens/sec per denoise step", "value": round(tokens_per_s, 1), "unit": "rollout-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "preheat_ms": round(preheat_ms, 1),
        "preheat_steps": preheat_steps, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: one denoise step (block attention + unmask + K/V refresh), N={w.N} "
                               f"rollouts, B={w.B}, shared prefix L={w.L}, Hq={w.Hq}, Hkv={w.Hkv}, D={w.D}, V={w.V}, "
                               f"bf16, re-forked every {STEPS_PER_BLOCK} steps",
                   "N": w.N, "B": w.B, "L": w.L, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "V": w.V,
                   "scaffold_frac": w.scaffold_frac, "tau": w.tau},
        "wall_ms_per_step": round(wall * 1e3 / args.steps, 4),
        "ms_per_block_of_8_steps": round(ms_step * STEPS_PER_BLOCK, 4),
        "roofline": {"kernel": "attn_bf16_kernel", "bound": "mfma", "achieved": round(flops / (attn_ms * 1e-3) / 1e12, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(flops / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                     "traffic": (round(sum(MEASURED_TRAFFIC_MIB[w.name]["attn_bf16_kernel"]) * 2 ** 20)
                                 if w.name in MEASURED_TRAFFIC_MIB else None),
                     "algorithmic_bytes": attn_bytes(w)[1],
                     "traffic_source": TRAFFIC_SOURCE if w.name in MEASURED_TRAFFIC_MIB else None,
                     "flops_per_launch": flops, "avg_launch_us": round(attn_ms * 1e3, 2),
                     "min_launch_us": round(min(attn_samples) * 1e3, 2), "max_launch_us": round(max(attn_samples) * 1e3, 2),
                     "launches_timed": len(attn_samples), "launches_timed_in_region": n_in_region,
                     "event_stride": stride},
    }
    if has_unmask:
        un_ms = float(np.mean(un_samples))
        # eligible rows shrink by the commits of each step; average over the steps of a block
        elig0 = int(((d["mask"] == 1) & (d["scaffold_mask"] == 0)).sum())
        st_host = st["mask"].cpu().numpy()
        res["roofline_unmask"] = {
            "kernel": "vocab_reduce_kernel+block_select_kernel (with the K/V refresh)", "bound": "hbm", "unit": "GB/s", "peak": PEAK_HBM_GBS,
            "avg_call_us": round(un_ms * 1e3, 2), "calls_timed": len(un_samples), "eligible_rows_at_block_start": elig0,
            "eligible_rows_now": int(((st_host == 1) & (d["scaffold_mask"] == 0)).sum()),
        }
        # forced single commit per block per step at these logit statistics: rows = elig0 - N * (step in block)
        avg_rows = elig0 - w.N * (STEPS_PER_BLOCK - 1) / 2.0
        byt = avg_rows * w.V * 2
        res["roofline_unmask"].update({"traffic": (round(sum(MEASURED_TRAFFIC_MIB[w.name]["vocab_reduce_kernel"]) * 2 ** 20)
                                                   if w.name in MEASURED_TRAFFIC_MIB else None),
                                       "traffic_source": TRAFFIC_SOURCE if w.name in MEASURED_TRAFFIC_MIB else None,
                                       "achieved": round(byt / (un_ms * 1e-3) / 1e9, 1),
                                       "frac": round(byt / (un_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                       "bytes_per_call": byt})
    if not args.no_supplements:
        n1 = W.CONFIGS["cfg2"]
        res["n1_prefix_stream"] = time_attention_only(F, n1, 400, 40, 128)
        res["n1_prefix_stream_warm"] = time_attention_only(F, n1, 200, 20, 1)      # one buffer: served from the caches
        n1_long = W.Workload("n1_L16384", N=1, B=32, L=16384, Hq=28, Hkv=4, D=128, dtype=W.BF16, seed=12)
        res["n1_prefix_stream_L16384"] = time_attention_only(F, n1_long, 200, 20, 20)
        res["cfg3_attention"] = time_attention_only(F, W.CONFIGS["cfg3"], 200, 40, 40, prepacked=True)
        res["cfg3_attention_plain_call"] = time_attention_only(F, W.CONFIGS["cfg3"], 200, 40, 40)
        res["n1_layer_sweep"] = time_layer_sweep_graph(F, n1, 28, 20)
        res["n1_layer_sweep_L16384"] = time_layer_sweep_graph(F, n1_long, 28, 10)
        res["n1_batched"] = time_batched(F, n1, 28, 50)
        res["n1_batched_L16384"] = time_batched(F, n1_long, 8, 30)
        if has_unmask:
            res["spec_verify"] = time_spec_verify(F, w, d, g, logits, 100, 100)
        res["extension_block"] = time_extension(F, w, d, g, 50, 100)
        res["scaffold_skip"] = time_scaffold_skip(F, w, d, g, 50, 100)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, d, logits_h)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
