#!/usr/bin/env python3
"""Benchmark of the CQIL hot path on one MI355X.

Headline workload (the one the metric is quoted on): ONE LLaMA-33B-shaped group of P=4 input-aligned layers, bf16,
batch 1, single-token decode steps with the KV cache growing from 512 tokens (the decode phase of the full-model
configuration), bypass distance 1.  A "step" is one whole group step: all six kernels (QKV+rotary+append, attention,
O, gate/up, down, merge).

Prints ONE JSON line.  Its top level is the headline: step latency (the metric), the achieved fraction of the HBM
roofline for the dominant kernel measured live with HIP events, the CPU oracle timed on a bounded sample of the same
workload, the same four layers run one after another.  Under "configs" the same run also times the other named
configurations (7B group, 13B batch-8 ragged group, 13B prefill, whole 33B-shaped model), each with its own roofline
block, under "sweeps" the batch sweep (grouped against sequential for B = 1..256) and the bypass-distance sweep, and
under "stream_read" the rate of a plain read-only stream on this GPU measured in the same process.

`--only headline` prints the headline alone; `--shape/--P/--batch/--kv-start/--kv-hi`, `--prefill T` and `--model`
time one other configuration as the top-level line (used for the profiles).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by
# what the same counters read for a plain copy kernel (profiles/decode_step_33b_P4_B1_hbm_traffic.md).  Only valid
# for the workload it was measured on; other workloads report null.
MEASURED_TRAFFIC = {("33b", 4, "gateup"): 1_909_973_138}


def kernel_bytes(shape, P, lens, es=2):
    """Algorithmic HBM bytes of each decode kernel for one step of B = len(lens) sequences: every packed weight
    byte once, every valid KV byte once, activations once (lens = cached tokens per sequence before the step)."""
    dm, f, B = shape.d_model, shape.d_ffn, len(lens)
    ues = 4 if B == 1 else 2   # SwiGLU outputs: fp32 for one token, storage type for a batch
    return {
        "qkv_rope": P * 3 * dm * dm * es + B * dm * es + P * dm * es + B * P * dm * 4 + 2 * B * P * dm * es,
        "attn_decode": sum(2 * P * (S + 1) * dm * es for S in lens) + 2 * B * P * dm * 4,
        "oproj": P * dm * dm * es + 2 * B * P * dm * 4,
        "gateup": 2 * P * f * dm * es + B * dm * es + B * P * dm * 4 + P * dm * es + B * P * f * ues,
        "down": P * dm * f * es + B * P * f * ues,
        "merge": 2 * B * dm * es + B * P * dm * 4,
    }


class Ctx:
    """Modules and settings shared by the legs of one run."""

    def __init__(self, args):
        import numpy as np
        import torch

        from paper_2404_06709_amd import binding as cq
        from paper_2404_06709_amd import runtime as rt
        from paper_2404_06709_amd import synth
        self.args, self.np, self.torch, self.cq, self.rt, self.synth = args, np, torch, cq, rt, synth

    def free(self):
        # Drops the tensors of a finished leg but keeps their device memory in torch's allocator for the next leg.
        # Memory that was handed back to the driver and allocated again streams 4-5 % slower on this machine than
        # memory allocated once (measured: the same 33B single-layer step 185.6 us on kept blocks, 194.7 us after
        # empty_cache(), in every later leg of the process); a server allocates once, and so does this run.
        import gc
        gc.collect()


def timed(ctx, fn, steps, warmup):
    """fn(n) enqueues n steps.  Returns (wall-clock mean in us over exactly `steps` steps bracketed by device
    synchronisation, median and minimum in us of a second pass of `steps` steps timed one by one with HIP events on
    the launch stream)."""
    torch = ctx.torch
    fn(warmup, None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fn(steps, None)
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / steps * 1e6
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    fn(steps, ev)
    torch.cuda.synchronize()
    per = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    return wall_us, per[len(per) // 2], per[0]


def decode_leg(ctx, shape_name, P, B, kv_start, kv_hi, kv_span, steps, warmup, bypass, seed, per_kernel=True,
               sequential=True, cpu_steps=0, cpu_single_steps=0, want_stream=False):
    """Decode steps of one group: B sequences, one new token each, caches growing from their start lengths and
    wrapping every kv_span steps.  Returns the result dictionary of this configuration."""
    torch, cq, rt, synth, np = ctx.torch, ctx.cq, ctx.rt, ctx.synth, ctx.np
    shape = synth.SHAPES[shape_name]
    dtype = torch.bfloat16
    if B > 1:
        lens0 = [int(v) for v in synth.kv_lengths(B, kv_start, max(kv_hi, kv_start), seed=1003)]
    else:
        lens0 = [kv_start]
    max_seq = max(lens0) + kv_span + 8
    dims = cq.make_dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, max_seq, dtype)
    # synthetic inputs: weights N(0, 0.02), gains 1, KV fill and hidden state N(0, 1)
    layers = synth.make_layers(P, shape, dtype, seed=seed, device="cuda")
    group = rt.Group(dims, layers, b_max=B, device="cuda")
    gen = synth.generator(seed + 1000, "cuda")
    Smax = max(lens0)
    group.k[:, :, :, :Smax] = synth.normal((P, B, shape.n_heads, Smax, shape.head_dim), 1.0, dtype, gen)
    group.v[:, :, :, :Smax] = synth.normal((P, B, shape.n_heads, Smax, shape.head_dim), 1.0, dtype, gen)
    x = synth.normal((B, 1, shape.d_model), 1.0, dtype, gen)
    y = torch.empty_like(x)
    ws = group.workspace(B, 1)
    lens_dev = torch.tensor(lens0, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def reset(g):
        # device-to-device copy of the start lengths: no host synchronisation inside the timed region
        g.kv_len[:B].copy_(lens_dev)
        g.kv.max_kv_len = Smax

    def run(n, ev):
        for i in range(n):
            if i % kv_span == 0:
                reset(group)
            if ev:
                ev[i][0].record()
            cq.cqil_group_forward(dims, P, bypass, group.packed, group.kv, x, y, B, 1, True, ws)
            if ev:
                ev[i][1].record()

    wall_us, med_us, min_us = timed(ctx, run, steps, warmup)
    grown = [i % kv_span for i in range(steps)]
    mean_growth = sum(grown) / len(grown)
    lens_mean = [S + mean_growth for S in lens0]
    kb = kernel_bytes(shape, P, lens_mean)
    step_bytes = sum(kb.values())
    names = cq.DECODE_KERNELS
    res = {
        "workload": f"llama{shape_name}_shape_group_P{P}_decode_B{B}_kv{min(lens0)}-{max(lens0) + max(grown) + 1}",
        "us_per_step": round(wall_us, 2), "us_per_token": round(wall_us / B, 2),
        "event_us": {"median": round(med_us, 2), "min": round(min_us, 2)},
        "tokens_per_s": round(B * 1e6 / wall_us, 1), "steps": steps, "warmup": warmup,
        "kv_len_start": lens0, "bypass_d": bypass,
        "step_hbm": {"bytes": int(step_bytes), "gbps": round(step_bytes / (wall_us * 1e-6) / 1e9, 1),
                     "frac": round(step_bytes / (wall_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
    }
    if B == 1 and per_kernel:
        # per-kernel durations, HIP events on the launch stream, at the mean cache length
        group.set_kv_len([int(round(v)) for v in lens_mean])
        prof_n = 64
        acc = np.zeros(6)
        for i in range(prof_n + 8):
            ms = cq.cqil_decode_step_profile(dims, P, bypass, group.packed, group.kv, x, y, ws, B)
            if i >= 8:
                acc += np.array(ms)
        k_us = acc / prof_n * 1e3
        res["kernels"] = {n: {"us": round(float(k_us[i]), 2), "bytes": int(kb[n]),
                              "gbps": round(kb[n] / (k_us[i] * 1e-6) / 1e9, 1)} for i, n in enumerate(names)}
        dom = max(names, key=lambda n: kb[n])
        achieved = kb[dom] / (k_us[names.index(dom)] * 1e-6) / 1e9
        traffic = MEASURED_TRAFFIC.get((shape_name, P, dom))
    else:
        # a batch runs the token-parallel kernels: the roofline figure is that of the whole step
        dom, achieved, traffic = "whole group step", step_bytes / (wall_us * 1e-6) / 1e9, None
    res["roofline"] = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                       "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic}

    if want_stream:
        # a plain read-only stream over this group's packed weights, same process, same box
        sink = torch.empty(16384, dtype=torch.uint8, device="cuda")
        nbytes = group.packed.numel() // 16 * 16
        buf = group.packed[:nbytes]

        def stream(n, ev):
            for i in range(n):
                if ev:
                    ev[i][0].record()
                cq.cqil_stream_read_probe(buf, sink)
                if ev:
                    ev[i][1].record()

        s_wall, s_med, s_min = timed(ctx, stream, 20, 3)
        res["stream_read"] = {"bytes": nbytes, "us_median": round(s_med, 2), "us_min": round(s_min, 2),
                              "gbps": round(nbytes / (s_med * 1e-6) / 1e9, 1),
                              "frac_of_peak": round(nbytes / (s_med * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
        res["step_hbm"]["frac_of_stream"] = round(res["step_hbm"]["gbps"] / res["stream_read"]["gbps"], 4)

    if sequential:
        # the same layers as P groups of one (Eq.1 chain) on the same caches: grouped versus sequential latency
        seq = [rt.Group(dims, [L], b_max=B, device="cuda") for L in layers]
        for l, g in enumerate(seq):
            g.k, g.v = group.k[l:l + 1], group.v[l:l + 1]       # layer l's caches of the group, in place
            g.kv = cq.make_kv(g.k, g.v, g.kv_len, Smax)
        ws1 = seq[0].workspace(B, 1)
        xa, xb = x.clone(), torch.empty_like(x)

        def run_seq(n, ev):
            for i in range(n):
                if i % kv_span == 0:
                    for g in seq:
                        reset(g)
                if ev:
                    ev[i][0].record()
                a, b = xa, xb
                for g in seq:
                    cq.cqil_group_forward(dims, 1, 0, g.packed, g.kv, a, b, B, 1, True, ws1)
                    a, b = b, a
                if ev:
                    ev[i][1].record()

        nseq = max(min(steps, 128) // 2, 10)
        q_wall, q_med, q_min = timed(ctx, run_seq, nseq, min(warmup, 16))
        res["sequential_us_per_step_same_layers"] = round(q_wall, 2)
        res["sequential_event_us"] = {"median": round(q_med, 2), "min": round(q_min, 2)}
        res["grouped_over_sequential"] = round(wall_us / q_wall, 4)
        del seq

    if cpu_steps > 0:
        import oracle as orc
        od = orc.Dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, max_seq, 10000.0, 1e-6, orc.BF16)
        np_layers = [synth.layer_to_numpy(L) for L in layers]
        okc, ovc = orc.new_cache(P, B, od), orc.new_cache(P, B, od)
        for b, S in enumerate(lens0):
            okc[:, b, :, :S] = synth.widen(group.k[:, b, :, :S])
            ovc[:, b, :, :S] = synth.widen(group.v[:, b, :, :S])
        xin = synth.widen(x)
        orc.group_forward(od, np_layers, bypass, okc, ovc, lens0, xin)          # untimed first touch
        t0 = time.perf_counter()
        for i in range(cpu_steps):
            orc.group_forward(od, np_layers, bypass, okc, ovc, [S + 1 + i % kv_span for S in lens0], xin)
        cpu_us = (time.perf_counter() - t0) / cpu_steps * 1e6
        res["cpu_baseline"] = {"value": round(cpu_us / B, 1), "unit": "us/token", "cores": orc.num_threads(),
                               "kind": "oracle",
                               "sample": f"{cpu_steps} decode steps of the same group (same weights, same caches)"}
        if cpu_single_steps > 0:
            nthr = orc.num_threads()
            orc.set_threads(1)
            t0 = time.perf_counter()
            for i in range(cpu_single_steps):
                orc.group_forward(od, np_layers, bypass, okc, ovc, lens0, xin)
            res["cpu_baseline"]["single_thread_us_per_token"] = round(
                (time.perf_counter() - t0) / cpu_single_steps * 1e6 / B, 1)
            orc.set_threads(nthr)
        del okc, ovc, np_layers
    res["_group"] = (group, dims, layers, x, y, lens0, Smax)
    return res


def bypass_sweep(ctx, leg, steps):
    """Latency of the same group step for every bypass distance d = 0 .. P-1 and for the attention-FFN parallel form
    (d = -1): on one GPU the bypass is a window sum in a kernel prologue."""
    torch, cq = ctx.torch, ctx.cq
    group, dims, layers, x, y, lens0, Smax = leg["_group"]
    P, ws = group.P, group.workspace(1, 1)
    out = {}
    for d in list(range(P)) + [cq.CQIL_ATTN_FFN_PARALLEL]:
        def run(n, ev, d=d):
            for i in range(n):
                if ev:
                    ev[i][0].record()
                cq.cqil_group_forward(dims, P, d, group.packed, group.kv, x, y, 1, 1, False, ws)
                if ev:
                    ev[i][1].record()
        group.set_kv_len([Smax + 32])
        w, med, mn = timed(ctx, run, steps, 8)
        out["eq5_three_phases" if d < 0 else f"d{d}"] = {"us_median": round(med, 2), "us_min": round(mn, 2)}
        if d < 0:
            # the same arithmetic on the six-kernel schedule (QKV, attention, O, gate/up, down, merge one after another)
            cq.cqil_set_tuning("eq5_fused", 0)
            w, med, mn = timed(ctx, run, steps, 8)
            cq.cqil_set_tuning("eq5_fused", 1)
            out["eq5_six_kernels"] = {"us_median": round(med, 2), "us_min": round(mn, 2)}
    return out


def batch_sweep(ctx, shape_name, P, kv_start, steps, batches):
    """The paper's latency protocol covers batch sizes 1 to 256: one group of P layers against the same layers run
    as P groups of one, per batch size."""
    rows = {}
    for B in batches:
        # short steps need a longer run-in before the clocks and the caches of translations have settled
        n = steps if B > 32 else 2 * steps
        leg = decode_leg(ctx, shape_name, P, B, kv_start, kv_start, 64, n, 6 if B > 32 else 32, 1, seed=1003,
                         per_kernel=False, sequential=True)
        leg.pop("_group")
        rows[str(B)] = {"grouped_us": leg["event_us"]["median"], "sequential_us": leg["sequential_event_us"]["median"],
                        "grouped_over_sequential": round(leg["event_us"]["median"] / leg["sequential_event_us"]["median"], 4),
                        "tokens_per_s": round(B * 1e6 / leg["event_us"]["median"], 1),
                        "hbm_frac": round(leg["step_hbm"]["bytes"] / (leg["event_us"]["median"] * 1e-6) / 1e9
                                          / HBM_PEAK_GBPS, 4)}
        del leg
        ctx.free()
    return rows


def prefill_leg(ctx, shape_name, P, B, T, bypass, steps, warmup, cpu_positions=0):
    """One token-parallel group step (prefill of B sequences of T tokens onto empty caches), timed as a whole."""
    torch, cq, rt, synth = ctx.torch, ctx.cq, ctx.rt, ctx.synth
    shape = synth.SHAPES[shape_name]
    dtype = torch.bfloat16
    dims = cq.make_dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, T, dtype)
    layers = synth.make_layers(P, shape, dtype, seed=1004, device="cuda")
    group = rt.Group(dims, layers, b_max=B, device="cuda")
    x = synth.normal((B, T, shape.d_model), 1.0, dtype, synth.generator(3004, "cuda"))
    y = torch.empty_like(x)
    group.set_kv_len([0] * B)
    ws = group.workspace(B, T)

    def run(n, ev):
        for i in range(n):
            if ev:
                ev[i][0].record()
            cq.cqil_group_forward(dims, P, bypass, group.packed, group.kv, x, y, B, T, False, ws)
            if ev:
                ev[i][1].record()

    wall_us, med_us, min_us = timed(ctx, run, steps, warmup)
    M, dm, f = B * T, shape.d_model, shape.d_ffn
    # algorithmic flops: every projection once, causal attention without the masked half
    flops = P * (2 * M * (4 * dm * dm + 3 * dm * f) + B * 2 * T * (T + 1) * dm)
    tf = flops / (wall_us * 1e-6) / 1e12
    res = {
        "workload": f"llama{shape_name}_shape_group_P{P}_prefill_B{B}_T{T}",
        "ms_per_step": round(wall_us / 1e3, 3), "event_ms": {"median": round(med_us / 1e3, 3), "min": round(min_us / 1e3, 3)},
        "steps": steps, "warmup": warmup, "tokens_per_s": round(M / (wall_us * 1e-6), 1), "flops_per_step": flops,
        "tflops": round(tf, 1), "bypass_d": bypass,
        "roofline": {"bound": "mfma", "kernel": "whole group step", "achieved": round(tf, 1), "peak": MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(tf / MFMA_PEAK_TFLOPS, 4), "traffic": None},
    }
    if cpu_positions > 0:
        import oracle as orc
        od = orc.Dims(dm, shape.n_heads, shape.head_dim, f, T, 10000.0, 1e-6, orc.BF16)
        np_layers = [synth.layer_to_numpy(L) for L in layers]
        okc, ovc = orc.new_cache(P, 1, od), orc.new_cache(P, 1, od)
        xin = synth.widen(x[:1, :cpu_positions])
        t0 = time.perf_counter()
        orc.group_forward(od, np_layers, bypass, okc, ovc, [0], xin)
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": round(cpu_positions / dt, 2), "unit": "tokens/s", "cores": orc.num_threads(),
                               "kind": "oracle",
                               "sample": f"the first {cpu_positions} positions of one of the {B} sequences "
                                         f"(a causal prefix is independent of the rest)"}
    return res


def model_leg(ctx, steps, bypass):
    """Alg.1 on a LLaMA-33B-shaped decoder: layers 21..60 in groups of four (Sec.4.2), against the plain sequential
    model (every layer a group of one) built from the same weights."""
    torch, cq, rt, synth = ctx.torch, ctx.cq, ctx.rt, ctx.synth
    shape, V, L, Tp = synth.SHAPES["33b"], 32000, 60, 512
    steps = min(steps, 128)
    max_seq = Tp + steps + 8
    dtype = torch.bfloat16
    dims = cq.make_dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, max_seq, dtype)
    sizes = cq.cqil_partition(L, 4, 21, 60)
    gen = synth.generator(1005, "cuda")
    grouped, singles = [], []
    for P in sizes:
        layers = [synth.make_layer(shape, dtype, gen) for _ in range(P)]
        g = rt.Group(dims, layers, b_max=1)
        grouped.append(g)
        singles.extend([g] if P == 1 else [rt.Group(dims, [Ly], b_max=1) for Ly in layers])
        torch.cuda.synchronize()
        del layers
    emb = synth.normal((V, shape.d_model), 1.0, dtype, gen)
    head = synth.normal((V, shape.d_model), 0.02, dtype, gen)
    gfin = torch.ones(shape.d_model, dtype=dtype, device="cuda")
    tokens0 = torch.randint(0, V, (1, Tp), generator=synth.generator(5)).to(torch.int32).cuda()

    def run(groups):
        kv_len = torch.zeros(1, dtype=torch.int32, device="cuda")
        model = cq.Model(dims, [g.P for g in groups], [g.packed for g in groups], [g.k for g in groups],
                         [g.v for g in groups], kv_len, emb, gfin, head)
        nxt = torch.empty(1, dtype=torch.int32, device="cuda")
        ws_p = torch.empty(cq.cqil_model_workspace_bytes(model, 1, Tp), dtype=torch.uint8, device="cuda")
        ws_d = torch.empty(cq.cqil_model_workspace_bytes(model, 1, 1), dtype=torch.uint8, device="cuda")
        out = {}
        for rep in range(2):                     # first pass warms up, second is timed
            kv_len.zero_(); model.c.max_kv_len = 0
            torch.cuda.synchronize(); t0 = time.perf_counter()
            cq.cqil_model_forward(model, tokens0, 1, Tp, bypass, True, None, None, nxt, ws_p)
            torch.cuda.synchronize(); out["prefill_ms"] = (time.perf_counter() - t0) * 1e3
            tok = nxt.reshape(1, 1).clone()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            t0 = time.perf_counter()
            for i in range(steps):
                ev[i][0].record()
                cq.cqil_model_forward(model, tok, 1, 1, bypass, True, None, None, nxt, ws_d)
                tok.copy_(nxt.reshape(1, 1))     # greedy feedback stays on the device
                ev[i][1].record()
            torch.cuda.synchronize(); out["decode_ms"] = (time.perf_counter() - t0) * 1e3 / steps
            per = sorted(a.elapsed_time(b) for a, b in ev)
            out["decode_ms_median"], out["decode_ms_min"] = per[len(per) // 2], per[0]
        return out

    cqil, seq = run(grouped), run(singles)
    dm, f = shape.d_model, shape.d_ffn
    layer_bytes = (4 * dm * dm + 3 * dm * f) * 2
    kv_bytes = L * 2 * (Tp + steps / 2) * dm * 2
    token_bytes = L * layer_bytes + V * dm * 2 + kv_bytes
    gbps = token_bytes / (cqil["decode_ms"] * 1e-3) / 1e9
    return {
        "workload": f"llama33b_shape_model_L60_p4_s21_e60_prefill{Tp}_decode{steps}", "groups": sizes, "vocab": V,
        "bypass_d": bypass, "steps": steps,
        "ms_per_token": round(cqil["decode_ms"], 3),
        "event_ms": {"median": round(cqil["decode_ms_median"], 3), "min": round(cqil["decode_ms_min"], 3)},
        "tokens_per_s": round(1e3 / cqil["decode_ms"], 1), "prefill_ms": round(cqil["prefill_ms"], 2),
        "sequential_ms_per_token": round(seq["decode_ms"], 3), "sequential_prefill_ms": round(seq["prefill_ms"], 2),
        "decode_latency_reduction": round(1.0 - cqil["decode_ms"] / seq["decode_ms"], 4),
        "prefill_latency_reduction": round(1.0 - cqil["prefill_ms"] / seq["prefill_ms"], 4),
        "bytes_per_token": int(token_bytes),
        "roofline": {"bound": "hbm", "kernel": "whole token", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None},
    }


def top_level(leg, metric, value, unit, ms_per_step, hib, extra_config):
    out = {"metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": leg["steps"],
           "warmup": leg.get("warmup", 0), "ms_per_step": ms_per_step, "higher_is_better": hib, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": dict({"workload": leg["workload"]}, **extra_config)}
    for k, v in leg.items():
        if k not in ("workload", "steps", "warmup", "_group") and k not in out:
            out[k] = v
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--only", default="all", choices=["all", "headline"],
                    help="all: headline + the other named configurations and sweeps nested in the same line")
    ap.add_argument("--shape", default="33b", choices=["7b", "13b", "33b"])
    ap.add_argument("--P", type=int, default=4)
    ap.add_argument("--bypass", type=int, default=1)
    ap.add_argument("--kv-start", type=int, default=512)
    ap.add_argument("--kv-span", type=int, default=128)
    ap.add_argument("--batch", type=int, default=1, help="sequences per step (B > 1: token-parallel kernels)")
    ap.add_argument("--kv-hi", type=int, default=0, help="with --batch: lengths uniform in [kv-start, kv-hi]")
    ap.add_argument("--prefill", type=int, default=0, metavar="T",
                    help="time one token-parallel group step over --batch sequences of T new tokens (empty caches) "
                         "instead of decode steps; reports TFLOP/s against the bf16 matrix-core peak")
    ap.add_argument("--model", action="store_true",
                    help="whole LLaMA-33B-shaped model (60 layers, vocabulary 32000): 512-token prefill, then greedy "
                         "decode steps with the partition (p=4, s=21, e=60), against the same layers run one by one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sequential", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=120)  # about 12 s of oracle work at the 33B shape
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="launch-shape knob of the library (cqil_set_tuning), set before anything is sized or run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    ctx = Ctx(args)
    torch, cq, synth = ctx.torch, ctx.cq, ctx.synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    cq.lib()  # fails loudly if libcqil.so has not been built
    for kv in args.tune:
        key, _, value = kv.partition("=")
        cq.cqil_set_tuning(key, int(value))

    if args.prefill > 0:
        leg = prefill_leg(ctx, args.shape, args.P, args.batch, args.prefill, args.bypass, min(args.steps, 20),
                          min(args.warmup, 5))
        shape = synth.SHAPES[args.shape]
        print(json.dumps(top_level(leg, "prefill_tflops_per_P_layer_group", leg["tflops"], "TFLOP/s", leg["ms_per_step"],
                                   True, {"d_model": shape.d_model, "n_heads": shape.n_heads, "d_ffn": shape.d_ffn,
                                          "P": args.P, "bypass_d": args.bypass, "batch": args.batch, "T": args.prefill})))
        return 0
    if args.model:
        leg = model_leg(ctx, args.steps, args.bypass)
        leg["warmup"] = leg["steps"]
        print(json.dumps(top_level(leg, "decode_ms_per_token_whole_model", leg["ms_per_token"], "ms/token",
                                   leg["ms_per_token"], False, {"groups": leg["groups"], "bypass_d": args.bypass,
                                                                "vocab": leg["vocab"]})))
        return 0

    custom = (args.shape, args.P, args.batch) != ("33b", 4, 1) or args.kv_hi or args.kv_start != 512
    cpu = 0 if (args.no_cpu_baseline or args.batch > 1 and custom) else args.cpu_steps
    leg = decode_leg(ctx, args.shape, args.P, args.batch, args.kv_start, args.kv_hi, args.kv_span, args.steps,
                     args.warmup, args.bypass, seed=1005, sequential=not args.no_sequential and args.batch == 1,
                     cpu_steps=cpu, want_stream=True)
    shape = synth.SHAPES[args.shape]
    out = top_level(leg, "decode_us_per_token_per_P_layer_group", leg["us_per_token"], "us/token",
                    round(leg["us_per_step"] / 1e3, 5), False,
                    {"d_model": shape.d_model, "n_heads": shape.n_heads, "d_ffn": shape.d_ffn, "P": args.P,
                     "bypass_d": args.bypass, "batch": args.batch, "kv_len_start": leg["kv_len_start"],
                     "kv_span": args.kv_span})
    if "sequential_us_per_step_same_layers" in out:
        out["sequential_us_per_token_same_layers"] = out["sequential_us_per_step_same_layers"]

    if args.only == "all" and not custom:
        # the other named configurations, the sweeps and the whole model, in the same process and under the same clock
        sweeps = {"bypass_distance_33b_P4_B1": bypass_sweep(ctx, leg, 40)}
        del leg
        ctx.free()
        cfgs = {}
        # the nested legs keep their own step counts whatever --steps says (each reports them): a short headline
        # run must not turn them into cold-start measurements
        n = 200
        l2 = decode_leg(ctx, "7b", 4, 1, 1024, 0, 128, n, 64, 1, seed=1002, cpu_steps=40,
                        cpu_single_steps=3)
        l2.pop("_group")
        cfgs["llama7b_group_P4_B1_kv1024"] = l2
        ctx.free()
        lp1 = decode_leg(ctx, "33b", 1, 1, 512, 0, 128, n, 64, 0, seed=1005, sequential=False)
        lp1.pop("_group")
        cfgs["llama33b_single_layer_P1_B1_kv512"] = lp1
        ctx.free()
        l3 = decode_leg(ctx, "13b", 4, 8, 512, 2048, 64, 128, 32, 1, seed=1003,
                        cpu_steps=3, cpu_single_steps=1)
        l3.pop("_group")
        cfgs["llama13b_group_P4_B8_kv512-2048"] = l3
        ctx.free()
        cfgs["llama13b_prefill_P2_B4_T2048"] = prefill_leg(ctx, "13b", 2, 4, 2048, 1, 10, 3, cpu_positions=12)
        ctx.free()
        sweeps["batch_13b_P4_kv512"] = batch_sweep(ctx, "13b", 4, 512, 30, [1, 2, 4, 8, 16, 32, 64, 128, 256])
        ctx.free()
        cfgs["llama33b_model_L60"] = model_leg(ctx, 128, 1)
        out["configs"] = cfgs
        out["sweeps"] = sweeps
    else:
        out.pop("_group", None)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
