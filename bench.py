#!/usr/bin/env python3
"""Benchmark of the CQIL hot path on one MI355X.

Workload (the one the headline metric is quoted on): ONE LLaMA-33B-shaped group of P=4 input-aligned layers,
bf16, batch 1, single-token decode steps with the KV cache growing from 512 to 640 tokens (the decode phase of
the full-model configuration), bypass distance 1.  A "step" is one whole group step: all six kernels (QKV+rotary+append, attention, O, gate/up, down, merge).

Prints one JSON line: the step latency (the metric), the achieved fraction of the HBM roofline for the dominant
kernel measured live with HIP events, and the CPU oracle timed on a bounded sample of the same workload.
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

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by
# what the same counters read for a plain copy kernel (profiles/decode_step_33b_P4_B1_hbm_traffic.md).  Only valid
# for the workload it was measured on; other workloads report null.
MEASURED_TRAFFIC = {("33b", 4, "gateup"): 1_909_967_600}


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


MFMA_PEAK_TFLOPS = 2500.0


def prefill(args, cq, rt, synth, torch) -> int:
    """One token-parallel group step (prefill of B sequences of T tokens onto empty caches), timed as a whole."""
    shape = synth.SHAPES[args.shape]
    P, B, T = args.P, args.batch, args.prefill
    dtype = torch.bfloat16
    dims = cq.make_dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, T, dtype)
    layers = synth.make_layers(P, shape, dtype, seed=1004, device="cuda")
    group = rt.Group(dims, layers, b_max=B, device="cuda")
    x = synth.normal((B, T, shape.d_model), 1.0, dtype, synth.generator(3004, "cuda"))
    y = torch.empty_like(x)
    steps, warmup = min(args.steps, 20), min(args.warmup, 5)
    group.set_kv_len([0] * B)
    for _ in range(warmup):
        group.forward(x, args.bypass, advance=False, out=y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        group.forward(x, args.bypass, advance=False, out=y)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    M, dm, f = B * T, shape.d_model, shape.d_ffn
    # algorithmic flops: every projection once, causal attention without the masked half
    flops = P * (2 * M * (4 * dm * dm + 3 * dm * f) + B * 2 * T * (T + 1) * dm)
    tf = flops / dt / 1e12
    print(json.dumps({
        "metric": "prefill_tflops_per_P_layer_group", "value": round(tf, 1), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(dt * 1e3, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"llama{args.shape}_shape_group_P{P}_prefill_B{B}_T{T}", "d_model": dm,
                   "n_heads": shape.n_heads, "d_ffn": f, "P": P, "bypass_d": args.bypass, "batch": B, "T": T},
        "tokens_per_s": round(M / dt, 1), "flops_per_step": flops,
        "roofline": {"bound": "mfma", "kernel": "whole group step", "achieved": round(tf, 1),
                     "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / MFMA_PEAK_TFLOPS, 4),
                     "traffic": None},
    }))
    return 0


def whole_model(args, cq, rt, synth, torch) -> int:
    """Alg.1 on a LLaMA-33B-shaped decoder: layers 21..60 in groups of four (Sec.4.2), bypass distance 1, against the
    plain sequential model (every layer a group of one) built from the same weights."""
    shape, V, L, Tp = synth.SHAPES["33b"], 32000, 60, 512
    steps = min(args.steps, 128)
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
            cq.cqil_model_forward(model, tokens0, 1, Tp, args.bypass, True, None, None, nxt, ws_p)
            torch.cuda.synchronize(); out["prefill_ms"] = (time.perf_counter() - t0) * 1e3
            tok = nxt.reshape(1, 1).clone()
            t0 = time.perf_counter()
            for _ in range(steps):
                cq.cqil_model_forward(model, tok, 1, 1, args.bypass, True, None, None, nxt, ws_d)
                tok.copy_(nxt.reshape(1, 1))     # greedy feedback stays on the device
            torch.cuda.synchronize(); out["decode_ms"] = (time.perf_counter() - t0) * 1e3 / steps
        return out

    cqil, seq = run(grouped), run(singles)
    dm, f = shape.d_model, shape.d_ffn
    layer_bytes = (4 * dm * dm + 3 * dm * f) * 2
    kv_bytes = L * 2 * (Tp + steps / 2) * dm * 2
    token_bytes = L * layer_bytes + V * dm * 2 + kv_bytes
    gbps = token_bytes / (cqil["decode_ms"] * 1e-3) / 1e9
    print(json.dumps({
        "metric": "decode_ms_per_token_whole_model", "value": round(cqil["decode_ms"], 3), "unit": "ms/token",
        "n_gpus": 1, "steps": steps, "warmup": steps, "ms_per_step": round(cqil["decode_ms"], 3),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"llama33b_shape_model_L60_p4_s21_e60_prefill{Tp}_decode{steps}", "groups": sizes,
                   "bypass_d": args.bypass, "vocab": V},
        "tokens_per_s": round(1e3 / cqil["decode_ms"], 1), "prefill_ms": round(cqil["prefill_ms"], 2),
        "sequential_ms_per_token": round(seq["decode_ms"], 3), "sequential_prefill_ms": round(seq["prefill_ms"], 2),
        "decode_latency_reduction": round(1.0 - cqil["decode_ms"] / seq["decode_ms"], 4),
        "prefill_latency_reduction": round(1.0 - cqil["prefill_ms"] / seq["prefill_ms"], 4),
        "roofline": {"bound": "hbm", "kernel": "whole token", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None},
    }))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--shape", default="33b", choices=["7b", "13b", "33b"])
    ap.add_argument("--P", type=int, default=4)
    ap.add_argument("--bypass", type=int, default=1)
    ap.add_argument("--kv-start", type=int, default=512)
    ap.add_argument("--kv-span", type=int, default=128)
    ap.add_argument("--batch", type=int, default=1, help="sequences per step (B > 1: token-parallel kernels; per-kernel figures only for B = 1)")
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
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2404_06709_amd import binding as cq
    from paper_2404_06709_amd import runtime as rt
    from paper_2404_06709_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    cq.lib()  # fails loudly if libcqil.so has not been built
    dev = "cuda"
    if args.prefill > 0:
        return prefill(args, cq, rt, synth, torch)
    if args.model:
        return whole_model(args, cq, rt, synth, torch)
    shape = synth.SHAPES[args.shape]
    P, d_byp = args.P, args.bypass
    dtype = torch.bfloat16
    B = args.batch
    if B > 1:
        lens0 = [int(v) for v in synth.kv_lengths(B, args.kv_start, max(args.kv_hi, args.kv_start), seed=1003)]
    else:
        lens0 = [args.kv_start]
    max_seq = max(lens0) + args.kv_span + 8
    dims = cq.make_dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, max_seq, dtype)

    # synthetic inputs: weights N(0, 0.02), gains 1, KV fill and hidden state N(0, 1), all from seed 1005
    layers = synth.make_layers(P, shape, dtype, seed=1005, device=dev)
    group = rt.Group(dims, layers, b_max=B, device=dev)
    gen = synth.generator(2005, dev)
    S0 = args.kv_start
    Smax = max(lens0)
    group.k[:, :, :, :Smax] = synth.normal((P, B, shape.n_heads, Smax, shape.head_dim), 1.0, dtype, gen)
    group.v[:, :, :, :Smax] = synth.normal((P, B, shape.n_heads, Smax, shape.head_dim), 1.0, dtype, gen)
    x = synth.normal((B, 1, shape.d_model), 1.0, dtype, gen)
    y = torch.empty_like(x)
    ws = group.workspace(B, 1)
    torch.cuda.synchronize()

    def run(n):
        # the cache grows by one token per step and wraps every kv_span steps
        for i in range(n):
            if i % args.kv_span == 0:
                group.set_kv_len(lens0)
            cq.cqil_group_forward(dims, P, d_byp, group.packed, group.kv, x, y, B, 1, True, ws)

    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us_step = dt / args.steps * 1e6

    # per-kernel durations, HIP events on the launch stream, at the mean cache length (single-token path only)
    lens_mean = [S + args.kv_span // 2 for S in lens0]
    kb = kernel_bytes(shape, P, lens_mean)
    names = cq.DECODE_KERNELS
    if B == 1:
        group.set_kv_len(lens_mean)
        prof_n = 64
        acc = np.zeros(6)
        for i in range(prof_n + 8):
            ms = cq.cqil_decode_step_profile(dims, P, d_byp, group.packed, group.kv, x, y, ws, B)
            if i >= 8:
                acc += np.array(ms)
        k_us = acc / prof_n * 1e3
        per_kernel = {n: {"us": round(float(k_us[i]), 2), "bytes": int(kb[n]),
                          "gbps": round(kb[n] / (k_us[i] * 1e-6) / 1e9, 1)} for i, n in enumerate(names)}
        dom = max(names, key=lambda n: kb[n])
        achieved = kb[dom] / (k_us[names.index(dom)] * 1e-6) / 1e9
    else:
        # a batch runs the token-parallel kernels: the roofline figure is that of the whole step
        per_kernel = None
        dom = "whole group step"
        achieved = sum(kb.values()) / (us_step * 1e-6) / 1e9
    step_bytes = sum(kb.values())

    out = {
        "metric": "decode_us_per_token_per_P_layer_group",
        "value": round(us_step / B, 2),
        "unit": "us/token",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(us_step / 1e3, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"llama{args.shape}_shape_group_P{P}_decode_B{B}_kv{min(lens0)}-{max(lens0) + args.kv_span}",
                   "d_model": shape.d_model, "n_heads": shape.n_heads, "d_ffn": shape.d_ffn, "P": P,
                   "bypass_d": d_byp, "batch": B, "kv_len_start": lens0, "kv_span": args.kv_span},
        "tokens_per_s": round(B * 1e6 / us_step, 1),
        "step_hbm": {"bytes": int(step_bytes), "gbps": round(step_bytes / (us_step * 1e-6) / 1e9, 1),
                     "frac": round(step_bytes / (us_step * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC.get((args.shape, P, dom)) if B == 1 else None},
        "kernels": per_kernel,
    }

    if not args.no_sequential and B == 1:
        # the same four layers as four groups of one (Eq.1 chain): grouped versus sequential latency
        seq = [rt.Group(dims, [L], b_max=1, device=dev) for L in layers]
        for g in seq:
            g.k[:, :, :, :S0] = group.k[:1, :, :, :S0]
            g.v[:, :, :, :S0] = group.v[:1, :, :, :S0]
        ws1 = seq[0].workspace(1, 1)
        xa, xb = x.clone(), torch.empty_like(x)

        def run_seq(n):
            for i in range(n):
                if i % args.kv_span == 0:
                    for g in seq:
                        g.set_kv_len([S0])
                a, b = xa, xb
                for g in seq:
                    cq.cqil_group_forward(dims, 1, 0, g.packed, g.kv, a, b, 1, 1, True, ws1)
                    a, b = b, a

        nseq = max(args.steps // 4, 32)
        run_seq(16)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_seq(nseq)
        torch.cuda.synchronize()
        us_seq = (time.perf_counter() - t0) / nseq * 1e6
        out["sequential_us_per_token_same_layers"] = round(us_seq, 2)
        out["grouped_over_sequential"] = round(us_step / us_seq, 4)
        del seq

    if not args.no_cpu_baseline and B == 1:
        import oracle as orc
        od = orc.Dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, max_seq, 10000.0, 1e-6, orc.BF16)
        np_layers = [synth.layer_to_numpy(L) for L in layers]
        okc, ovc = orc.new_cache(P, 1, od), orc.new_cache(P, 1, od)
        okc[:, :, :, :S0] = synth.widen(group.k[:, :, :, :S0])
        ovc[:, :, :, :S0] = synth.widen(group.v[:, :, :, :S0])
        xin = synth.widen(x)
        orc.group_forward(od, np_layers, d_byp, okc, ovc, [S0], xin)          # untimed first touch
        t0 = time.perf_counter()
        for i in range(args.cpu_steps):
            orc.group_forward(od, np_layers, d_byp, okc, ovc, [S0 + 1 + i % args.kv_span], xin)
        cpu_us = (time.perf_counter() - t0) / args.cpu_steps * 1e6
        out["cpu_baseline"] = {"value": round(cpu_us, 1), "unit": "us/token", "cores": orc.num_threads(),
                               "kind": "oracle",
                               "sample": f"{args.cpu_steps} decode steps of the same group (same weights, kv {S0}+)"}

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
