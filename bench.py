#!/usr/bin/env python3
"""Benchmark of the W4A16 decode linear on one MI355X.

Workload = the decode GEMV sweep: M = 1, INT4 group-128 weights, the four Linear shapes of a
7B-class decoder layer.  One "step" is one pass over the four shapes through
dmr_qlinear_forward; the same pass through dmr_qlinear_bf16_forward is timed beside it for the
speed-up.  Every launch of a pass reads a different resident copy of its weights (the copies of a
shape add up to >= 1 GiB, four times the 256 MB Infinity Cache), so weights stream from HBM.
Inputs are resident in HBM before the timed region.  The passes are recorded into a HIP graph and
the graph is replayed, so that the Python launch path is not what is measured.

Prints ONE JSON line (last line of stdout).
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

HBM_PEAK_GBS = 8000.0
CACHE_DEFEAT_BYTES = 1 << 30
MS_DEFAULT = "8,16,32,64,128,256,512"


def int4_bytes(K, N, M=1):
    """Algorithmic bytes of one INT4 forward: nibbles + bf16 scale and zero per group + x + y."""
    return N * K // 2 + N * (K // 128) * 4 + M * K * 2 + M * N * 2


def bf16_bytes(K, N, M=1):
    return N * K * 2 + M * K * 2 + M * N * 2


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def full_step(args, dmr, synth, torch, dev):
    """All Linear layers of one decode step of a 32-layer 7B-class decoder: 32 x {qkv, attn_out,
    gate_up, down} in INT4 (or bf16 for the twin) plus the bf16 lm_head, 129 launches on one stream,
    each layer with its own weights and buffers (4.76 GB INT4 step, 15.0 GB bf16 step)."""
    G, M, LAYERS = synth.GROUP, args.m, 32
    gen = torch.Generator(device=dev)
    t0 = time.time()
    int4_layers, bf16_layers, xs, ys = [], [], {}, {}
    for li in range(LAYERS):
        for si, (name, K, N) in enumerate(synth.LAYER_SHAPES):
            gen.manual_seed(synth.seed_for(4, si, 0, layer=li))
            w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
            qw, s, z = dmr.dmr_qlinear_quantize(w, G)
            int4_layers.append((name, dmr.dmr_qlinear_create(qw, s, z, G)))
            bf16_layers.append((name, w.to(torch.bfloat16)))
            del w, qw, s, z
    for si, (name, K, N) in enumerate(synth.LAYER_SHAPES + (synth.LM_HEAD,)):
        gen.manual_seed(synth.seed_for(4, si, 1))
        xs[name] = torch.randn((M, K), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        ys[name] = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    name, K, N = synth.LM_HEAD
    gen.manual_seed(synth.seed_for(4, 4, 0))
    lm_head = (torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)
    torch.cuda.synchronize()
    log(f"[bench] 129 layers resident after {time.time() - t0:.1f}s")
    stream = torch.cuda.Stream()

    def step(low: bool):
        for i in range(len(int4_layers)):
            nm = int4_layers[i][0]
            if low:
                dmr.dmr_qlinear_forward(int4_layers[i][1], xs[nm], out=ys[nm])
            else:
                dmr.dmr_qlinear_bf16_forward(bf16_layers[i][1], xs[nm], out=ys[nm])
        dmr.dmr_qlinear_bf16_forward(lm_head, xs["lm_head"], out=ys["lm_head"])     # lm_head stays bf16

    def timed(low: bool):
        with torch.cuda.stream(stream):
            for _ in range(args.warmup):
                step(low)
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for _ in range(args.steps):
                    step(low)
            for _ in range(2):
                graph.replay()
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t_start = time.perf_counter()
            e0.record(stream)
            graph.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            return (time.perf_counter() - t_start) * 1e3 / args.steps, e0.elapsed_time(e1) / args.steps

    lm_bytes = bf16_bytes(synth.LM_HEAD[1], synth.LM_HEAD[2], M)
    b4 = LAYERS * sum(int4_bytes(K, N, M) for _, K, N in synth.LAYER_SHAPES) + lm_bytes
    b16 = LAYERS * sum(bf16_bytes(K, N, M) for _, K, N in synth.LAYER_SHAPES) + lm_bytes
    w4, e4 = timed(True)
    w16, e16 = timed(False)
    result = {
        "metric": "full decode step over all Linear layers, aggregate HBM GB/s (INT4 copy) and speedup vs bf16 copy",
        "value": round(b4 / (w4 * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(w4, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"full decode step, 32 layers x (qkv, attn_out, gate_up, down) INT4 g128 + bf16 "
                               f"lm_head 4096x128256, M={M}, 129 launches per step, hip-graph replay",
                   "algorithmic_bytes_per_step": b4},
        "us_per_step_int4": round(e4 * 1e3, 1), "us_per_step_bf16": round(e16 * 1e3, 1),
        "bf16_GBps": round(b16 / (w16 * 1e-3) / 1e9, 1), "speedup_vs_bf16": round(w16 / w4, 3),
        "frac_hbm_peak_int4": round(b4 / (w4 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
    }
    print(json.dumps(result), flush=True)


def mixed_step(args, dmr, synth, torch, dev):
    """One decision step of a group of G = 16 parallel rollouts of which the router sends a fraction rho
    to the bf16 copy and the rest to the INT4 copy (Sec. 4.3: group sampling; Eq. 7: budget rho): the two
    copies' Linear layers run concurrently on two streams.  Reports step time against rho and against
    the linear per-token cost model of Eq. 9 fitted to the two pure cases."""
    G_ROLL, LAYERS, G = 16, 32, synth.GROUP
    gen = torch.Generator(device=dev)
    int4_layers, bf16_layers = [], []
    for li in range(LAYERS):
        for si, (name, K, N) in enumerate(synth.LAYER_SHAPES):
            gen.manual_seed(synth.seed_for(4, si, 0, layer=li))
            w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
            qw, s, z = dmr.dmr_qlinear_quantize(w, G)
            int4_layers.append((name, dmr.dmr_qlinear_create(qw, s, z, G)))
            bf16_layers.append((name, w.to(torch.bfloat16)))
            del w, qw, s, z
    xs = {}
    for si, (name, K, N) in enumerate(synth.LAYER_SHAPES):
        gen.manual_seed(synth.seed_for(4, si, 1))
        xs[name] = torch.randn((G_ROLL, K), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    ys = {name: torch.empty((G_ROLL, N), dtype=torch.bfloat16, device=dev) for name, K, N in synth.LAYER_SHAPES}
    torch.cuda.synchronize()
    s_low, s_high = torch.cuda.Stream(), torch.cuda.Stream()      # both at the default priority

    def step(m_high):
        m_low = G_ROLL - m_high
        s_high.wait_stream(s_low)                                  # fork
        if m_low:
            with torch.cuda.stream(s_low):
                for name, layer in int4_layers:
                    dmr.dmr_qlinear_forward(layer, xs[name][:m_low], out=ys[name][:m_low])
        if m_high:
            with torch.cuda.stream(s_high):
                for name, wb in bf16_layers:
                    dmr.dmr_qlinear_bf16_forward(wb, xs[name][m_low:], out=ys[name][m_low:])
        s_low.wait_stream(s_high)                                  # join

    # a step is 256 launches on two streams with a fork and a join: keep the captured graph to a few thousand nodes
    steps = min(args.steps, 20)

    def timed(m_high):
        with torch.cuda.stream(s_low):
            for _ in range(min(args.warmup, 5)):
                step(m_high)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=s_low):
                for _ in range(steps):
                    step(m_high)
            for _ in range(2):
                graph.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s_low)
            graph.replay()
            e1.record(s_low)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / steps
            del graph
            return us

    rows = []
    for rho in (0.0, 0.2, 0.4, 0.7, 1.0):
        m_high = int(round(rho * G_ROLL))
        rows.append({"rho": rho, "m_high": m_high, "m_low": G_ROLL - m_high, "us_per_step": round(timed(m_high), 1)})
        log(f"[bench] {rows[-1]}")
    t_low, t_high = rows[0]["us_per_step"] / G_ROLL, rows[-1]["us_per_step"] / G_ROLL
    for r in rows:
        r["eq9_linear_model_us"] = round(r["m_low"] * t_low + r["m_high"] * t_high, 1)
    result = {
        "metric": "mixed routed decision step of 16 rollouts: us per step vs high-precision budget rho",
        "value": rows[1]["us_per_step"], "unit": "us", "n_gpus": 1, "steps": steps, "warmup": min(args.warmup, 5),
        "ms_per_step": rows[1]["us_per_step"] / 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "32 layers x (qkv, attn_out, gate_up, down), 16 rollouts split by rho between the "
                               "bf16 copy (stream A) and the INT4 copy (stream B); value is rho = 0.2"},
        "by_rho": rows,
    }
    print(json.dumps(result), flush=True)


def chain_step(args, dmr, synth, torch, dev):
    """One decode step (M = 1) of a 32-layer 7B-class decoder as a dependent chain of its Linear layers
    with the glue between them: per layer RMSNorm -> qkv, attn_out + residual, RMSNorm -> gate_up,
    SwiGLU -> down + residual.  Attention itself is not a Linear and is not modelled: the first 4096
    columns of the qkv output stand in for its result, so that the shapes chain.  Timed four ways: the
    glue fused into the Linear launches (4 launches per layer) or as kernels of its own (rmsnorm x 2,
    swiglu, residual add x 2: 9 launches per layer), for the INT4 copy and for the bf16 copy."""
    G, LAYERS, H, I, M = synth.GROUP, 32, 4096, 14336, args.m
    gen = torch.Generator(device=dev)
    t0 = time.time()
    int4, bf16, gammas = [], [], []
    for li in range(LAYERS):
        l4, l16 = {}, {}
        for si, (name, K, N) in enumerate(synth.LAYER_SHAPES):
            gen.manual_seed(synth.seed_for(4, si, 0, layer=li))
            w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
            qw, s, z = dmr.dmr_qlinear_quantize(w, G)
            l4[name] = dmr.dmr_qlinear_create(qw, s, z, G)
            l16[name] = w.to(torch.bfloat16)
            del w, qw, s, z
        int4.append(l4)
        bf16.append(l16)
        gen.manual_seed(synth.seed_for(4, 5, 0, layer=li))
        gammas.append((1.0 + 0.1 * torch.randn((2, H), generator=gen, device=dev)).to(torch.bfloat16))
    gen.manual_seed(synth.seed_for(4, 0, 1))
    h0 = torch.randn((M, H), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    bufs = {"qkv": torch.empty((M, 6144), dtype=torch.bfloat16, device=dev),
            "q": torch.empty((M, H), dtype=torch.bfloat16, device=dev),
            "gu": torch.empty((M, 2 * I), dtype=torch.bfloat16, device=dev),
            "act": torch.empty((M, I), dtype=torch.bfloat16, device=dev),
            "norm": torch.empty((M, H), dtype=torch.bfloat16, device=dev),
            "h": [torch.empty((M, H), dtype=torch.bfloat16, device=dev) for _ in range(3)],
            "ws": torch.empty(64 << 20, dtype=torch.uint8, device=dev)}
    torch.cuda.synchronize()
    log(f"[bench] 128 layers resident after {time.time() - t0:.1f}s")
    stream = torch.cuda.Stream()
    EPS = 1e-6
    R, S, NONE = dmr.DMR_PRO_RMSNORM, dmr.DMR_PRO_SWIGLU, dmr.DMR_PRO_NONE

    def step(low: bool, fused: bool, single_rounding: bool = False, layers: int = LAYERS):
        # single_rounding (check only): the unfused composition with the residual added to the fp32
        # result and rounded once, i.e. the arithmetic the fused epilogue performs
        h = bufs["h"][0]
        h.copy_(h0)
        for li in range(layers):
            g1, g2 = gammas[li][0], gammas[li][1]
            h1, h2 = bufs["h"][1], bufs["h"][2]
            L = int4[li] if low else bf16[li]

            def lin(name, pro, inp, gamma, res, out):
                if fused:
                    if low:
                        dmr.dmr_qlinear_forward_fused(L[name], pro, inp, gamma=gamma, eps=EPS, residual=res, out=out,
                                                      workspace=bufs["ws"])
                    else:
                        dmr.dmr_qlinear_bf16_forward_fused(L[name], pro, inp, gamma=gamma, eps=EPS, residual=res,
                                                           out=out, workspace=bufs["ws"])
                    return
                x = inp
                if pro == R:
                    x = dmr.dmr_glue_rmsnorm(inp, gamma, EPS, out=bufs["norm"])
                if pro == S:
                    x = dmr.dmr_glue_swiglu(inp, out=bufs["act"])
                if single_rounding and res is not None:
                    y32 = (dmr.dmr_qlinear_forward(L[name], x, out_dtype=torch.float32) if low else
                           dmr.dmr_qlinear_bf16_forward(L[name], x, out_dtype=torch.float32))
                    out.copy_((y32 + res.float()).to(torch.bfloat16))
                    return
                if low:
                    dmr.dmr_qlinear_forward(L[name], x, out=out)
                else:
                    dmr.dmr_qlinear_bf16_forward(L[name], x, out=out)
                if res is not None:
                    out.add_(res)

            lin("qkv", R, h, g1, None, bufs["qkv"])
            if M == 1:
                attn = bufs["qkv"][:, :H]                 # attention stand-in: the q slice (a view at M = 1)
            else:
                attn = bufs["q"]
                attn.copy_(bufs["qkv"][:, :H])            # one strided copy per layer, in all four variants
            lin("attn_out", NONE, attn, None, h, h1)
            lin("gate_up", R, h1, g2, None, bufs["gu"])
            lin("down", S, bufs["gu"], None, h1, h2)
            bufs["h"][0], bufs["h"][2] = h2, h
            h = h2
        return h

    def timed(low: bool, fused: bool):
        with torch.cuda.stream(stream):
            for _ in range(args.warmup):
                step(low, fused)
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for _ in range(args.steps):
                    step(low, fused)
            for _ in range(2):
                graph.replay()
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            graph.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps

    with torch.cuda.stream(stream):
        # consistency of the fused kernels with the unfused composition, over the first decoder layer
        # (over all 32 the bf16 residual stream amplifies single-ulp differences: informational only)
        ref1 = step(True, False, single_rounding=True, layers=1).float().clone()
        got1 = step(True, True, layers=1).float().clone()
        ref = step(True, False, single_rounding=True).float().clone()
        got = step(True, True).float().clone()
        stream.synchronize()
    drift1 = float((ref1 - got1).abs().max() / ref1.pow(2).mean().sqrt())
    drift = float((ref - got).abs().max() / ref.pow(2).mean().sqrt())
    times = {(low, fused): timed(low, fused) for low in (True, False) for fused in (True, False)}
    b4 = LAYERS * sum(int4_bytes(K, N, M) for _, K, N in synth.LAYER_SHAPES)
    t = times[(True, True)]
    result = {
        "metric": "dependent decode chain (Linear layers + fused glue) of the INT4 copy: us per step",
        "value": round(t * 1e3, 1), "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"32 layers x (rmsnorm->qkv, attn_out+residual, rmsnorm->gate_up, swiglu->down+residual), "
                               f"M={M}, attention replaced by the q slice, hip-graph replay"},
        "us_per_step": {"int4_fused": round(times[(True, True)] * 1e3, 1),
                        "int4_unfused": round(times[(True, False)] * 1e3, 1),
                        "bf16_fused": round(times[(False, True)] * 1e3, 1),
                        "bf16_unfused": round(times[(False, False)] * 1e3, 1)},
        "speedup_fused_vs_unfused_int4": round(times[(True, False)] / times[(True, True)], 3),
        "speedup_int4_vs_bf16_fused": round(times[(False, True)] / times[(True, True)], 3),
        "int4_GBps_fused": round(b4 / (t * 1e-3) / 1e9, 1),
        "fused_vs_unfused_hidden_max_diff_over_rms": {"after_1_layer": round(drift1, 5),
                                                      "after_32_layers": round(drift, 5)},
    }
    print(json.dumps(result), flush=True)


def layer_sweep(args, dmr, synth, torch, dev):
    """Per-layer times of both copies at the row counts in --ms (rollout batches, prefill) on the four
    decoder shapes: hip-graph replay, weights rotating over >= 1 GiB of resident copies per shape, the
    workspace allocated once outside the timed region."""
    G = synth.GROUP
    Ms = [int(v) for v in args.ms.split(",")]
    which = args.shapes.split(",") if args.shapes else [n for n, _, _ in synth.SWEEP_SHAPES]
    stream = torch.cuda.Stream()

    def timeit(fn, iters):
        torch.cuda.synchronize()          # the inputs were prepared on the default stream
        with torch.cuda.stream(stream):
            for i in range(3):
                fn(i)
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(iters):
                    fn(3 + i)
            for _ in range(2):
                graph.replay()
            stream.synchronize()
            best = float("inf")
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                graph.replay()
                e1.record(stream)
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1) * 1e3 / iters)
        return best

    rows = []
    for si, (name, K, N) in enumerate(synth.SWEEP_SHAPES):
        if name not in which:
            continue
        gen = torch.Generator(device=dev)
        gen.manual_seed(synth.seed_for(2, si, 0))
        w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
        qw, s, z = dmr.dmr_qlinear_quantize(w, G)
        n4 = -(-(1 << 30) // int4_bytes(K, N))
        n16 = -(-(1 << 30) // bf16_bytes(K, N))
        layers = [dmr.dmr_qlinear_create(qw, s, z, G) for _ in range(n4)]
        wbs = [w.to(torch.bfloat16).clone() for _ in range(n16)]
        del w, qw, s, z
        for M in Ms:
            gen.manual_seed(synth.seed_for(2, si, 1) + M)
            x = torch.randn((M, K), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
            y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            ws4 = torch.empty(max(dmr.dmr_qlinear_workspace_bytes(M, K, N), 16), dtype=torch.uint8, device=dev)
            ws16 = torch.empty(max(dmr.dmr_qlinear_bf16_workspace_bytes(M, K, N), 16), dtype=torch.uint8, device=dev)
            iters = 100 if M <= 64 else (20 if M <= 1024 else 5)
            t4 = timeit(lambda i: dmr.dmr_qlinear_forward(layers[i % n4], x, out=y, workspace=ws4), iters)
            t16 = timeit(lambda i: dmr.dmr_qlinear_bf16_forward(wbs[i % n16], x, out=y, workspace=ws16), iters)
            flops = 2.0 * M * K * N
            rows.append({"shape": name, "K": K, "N": N, "M": M, "int4_us": round(t4, 2), "bf16_us": round(t16, 2),
                         "speedup": round(t16 / t4, 3),
                         "int4_GBps": round(int4_bytes(K, N, M) / t4 / 1e3, 1),
                         "bf16_GBps": round(bf16_bytes(K, N, M) / t16 / 1e3, 1),
                         "int4_TFLOPs": round(flops / t4 / 1e6, 1), "bf16_TFLOPs": round(flops / t16 / 1e6, 1)})
            log(f"[bench] {name:9s} M={M:5d} int4 {t4:9.2f} us  bf16 {t16:9.2f} us  x{t16 / t4:5.2f}")
        del layers, wbs
    tot4 = sum(r["int4_us"] for r in rows)
    tot16 = sum(r["bf16_us"] for r in rows)
    result = {
        "metric": "per-layer time of the INT4 copy over the listed shapes and row counts (sum), and speedup vs bf16",
        "value": round(tot4, 1), "unit": "us", "n_gpus": 1, "steps": 1, "warmup": 3, "ms_per_step": round(tot4 * 1e-3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"layer sweep, M in {Ms}, shapes {which}, INT4 g128 vs bf16, hip-graph replay, "
                               "rotating weight copies"},
        "speedup_vs_bf16": round(tot16 / tot4, 3), "rows": rows,
    }
    print(json.dumps(result), flush=True)


def w3_sweep(args, dmr, synth, torch, dev):
    """The W3A16 (group 128) variant next to W4A16 on the four decoder shapes at the row counts in --ms
    (default 1): hip-graph replay, weights rotating over >= 1 GiB of resident copies per shape.  Reports
    the measured W4 / W3 time ratio (the paper projects 1.15 for a native 3-bit kernel, App. A)."""
    G = synth.GROUP
    Ms = [int(v) for v in args.ms.split(",")] if args.ms != MS_DEFAULT else [1]
    stream = torch.cuda.Stream()

    def timeit(fn, iters):
        torch.cuda.synchronize()          # the inputs were prepared on the default stream
        with torch.cuda.stream(stream):
            for i in range(3):
                fn(i)
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(iters):
                    fn(3 + i)
            for _ in range(2):
                graph.replay()
            stream.synchronize()
            best = float("inf")
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                graph.replay()
                e1.record(stream)
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1) * 1e3 / iters)
        return best

    def w3_bytes(K, N, M):
        return N * K * 3 // 8 + N * (K // G) * 4 + M * K * 2 + M * N * 2

    rows = []
    for si, (name, K, N) in enumerate(synth.SWEEP_SHAPES):
        gen = torch.Generator(device=dev)
        gen.manual_seed(synth.seed_for(2, si, 0))
        w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
        q4 = dmr.dmr_qlinear_quantize(w, G)
        q3 = dmr.dmr_qlinear_quantize_w3(w, G)
        n = -(-(1 << 30) // w3_bytes(K, N, 1))
        l4 = [dmr.dmr_qlinear_create(*q4, G) for _ in range(n)]
        l3 = [dmr.dmr_qlinear_w3_create(*q3, G) for _ in range(n)]
        # per-channel symmetric W4 (one scale per row, zero point 8): the codes of the group-wise copy stand in for
        # its codes (timing depends on the bytes only); 0.5 byte per weight + 4 bytes per row
        row_scale = q4[1][:, 0].contiguous()
        lpc = [dmr.dmr_qlinear_create_per_channel(q4[0], row_scale) for _ in range(n)]
        del w, q4, q3
        for M in Ms:
            gen.manual_seed(synth.seed_for(2, si, 1) + M)
            x = torch.randn((M, K), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
            y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            ws4 = torch.empty(max(dmr.dmr_qlinear_workspace_bytes(M, K, N), 16), dtype=torch.uint8, device=dev)
            ws3 = torch.empty(max(dmr.dmr_qlinear_w3_workspace_bytes(M, K, N), 16), dtype=torch.uint8, device=dev)
            t4 = timeit(lambda i: dmr.dmr_qlinear_forward(l4[i % n], x, out=y, workspace=ws4), 100)
            t3 = timeit(lambda i: dmr.dmr_qlinear_forward(l3[i % n], x, out=y, workspace=ws3), 100)
            tpc = timeit(lambda i: dmr.dmr_qlinear_forward(lpc[i % n], x, out=y, workspace=ws4), 100)
            pc_bytes = N * K // 2 + N * 4 + M * K * 2 + M * N * 2
            rows.append({"shape": name, "K": K, "N": N, "M": M, "w4_us": round(t4, 2), "w3_us": round(t3, 2),
                         "w4_over_w3": round(t4 / t3, 3), "w3_GBps": round(w3_bytes(K, N, M) / t3 / 1e3, 1),
                         "w4_GBps": round(int4_bytes(K, N, M) / t4 / 1e3, 1),
                         "w4_per_channel_us": round(tpc, 2), "w4_per_channel_GBps": round(pc_bytes / tpc / 1e3, 1)})
            log(f"[bench] {name:9s} M={M:3d} W4 {t4:7.2f} us  W3 {t3:7.2f} us  W4/W3 {t4 / t3:5.3f}  "
                f"W4 per-channel {tpc:7.2f} us")
        del l4, l3, lpc
    tot4 = sum(r["w4_us"] for r in rows)
    tot3 = sum(r["w3_us"] for r in rows)
    result = {
        "metric": "per-layer time of the W3A16 copy over the four decoder shapes (sum), and W4A16 / W3A16 time ratio",
        "value": round(tot3, 2), "unit": "us", "n_gpus": 1, "steps": 1, "warmup": 3, "ms_per_step": round(tot3 * 1e-3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"W3A16 g128 vs W4A16 g128 sweep, M in {Ms}, hip-graph replay, rotating weight copies"},
        "w4_over_w3": round(tot4 / tot3, 3), "paper_projection_w4_over_w3": 1.15, "rows": rows,
    }
    print(json.dumps(result), flush=True)


def launch_floor(args, dmr, synth, torch, dev):
    """Where the time of a per-layer decode launch goes (M = 1, the four decoder shapes, HIP-graph replay of 200
    launches each, weights rotating over >= 1 GiB): a kernel that does nothing in the launch shape of the real
    one, a plain read of the layer's bytes from 256 and from 1024 workgroups, the real kernel on rotating
    copies and on one hot copy (served by the Infinity Cache: no HBM), against bytes / 8 TB/s."""
    import numpy as np
    G, REPS = synth.GROUP, 200
    stream = torch.cuda.Stream()
    sink = torch.empty(4096 * 256, dtype=torch.int32, device=dev)

    def graph_us(fn):
        torch.cuda.synchronize()          # the inputs were prepared on the default stream
        with torch.cuda.stream(stream):
            for i in range(5):
                fn(i)
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(REPS):
                    fn(i)
            graph.replay()
            stream.synchronize()
            best = []
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                graph.replay()
                e1.record(stream)
                torch.cuda.synchronize()
                best.append(e0.elapsed_time(e1) * 1e3 / REPS)
        return float(np.median(best))

    rows = []
    for idx, (name, K, N) in enumerate(synth.SWEEP_SHAPES):
        w = torch.from_numpy(synth.weights_f32(synth.seed_for(1, idx, 0), N, K)).to(dev)
        qw, s, z = dmr.dmr_qlinear_quantize(w, G)
        copies = -(-CACHE_DEFEAT_BYTES // int4_bytes(K, N))
        layers = [dmr.dmr_qlinear_create(qw, s, z, G) for _ in range(copies)]
        x = torch.from_numpy(synth.activations_bf16(synth.seed_for(1, idx, 1), 1, K).view(np.int16)).to(dev).view(torch.bfloat16)
        y = torch.empty((1, N), dtype=torch.bfloat16, device=dev)
        del w, qw, s, z
        # launch shape of the decode kernel for this layer (the rule of its planner: one 16-wave workgroup per
        # row tile up to 512 tiles, else 512 workgroups of 8 waves looping over tiles)
        groups, tiles = K // G, N // 16
        wgs, threads = (tiles, 1024) if tiles <= 512 else (512, 512)
        lds = groups * 256 + ((groups + 3) & ~3) * 4 + -(-tiles // wgs) * (threads // 64) * 64 + 64
        nbytes = int4_bytes(K, N)
        row = {
            "shape": name, "K": K, "N": N, "bytes": nbytes, "us_at_8TBps": round(nbytes / 8e6, 2),
            "launch_shape": {"workgroups": wgs, "threads": threads, "lds_bytes": lds},
            "empty_same_shape_us": round(graph_us(lambda i: dmr.dmr_probe_empty_launch(wgs, threads, lds)), 3),
            "empty_256x256_us": round(graph_us(lambda i: dmr.dmr_probe_empty_launch(256, 256, 0)), 3),
            "read_256wg_us": round(graph_us(lambda i: dmr.dmr_probe_hbm_read(layers[i % copies].storage, sink, 256)), 3),
            "read_1024wg_us": round(graph_us(lambda i: dmr.dmr_probe_hbm_read(layers[i % copies].storage, sink, 1024)), 3),
            "kernel_us": round(graph_us(lambda i: dmr.dmr_qlinear_forward(layers[i % copies], x, out=y)), 3),
            "kernel_hot_cache_us": round(graph_us(lambda i: dmr.dmr_qlinear_forward(layers[0], x, out=y)), 3),
        }
        row["kernel_frac_of_8TBps"] = round(row["us_at_8TBps"] / row["kernel_us"], 4)
        rows.append(row)
        log(f"[bench] {row}")
        del layers
    total = sum(r["kernel_us"] for r in rows)
    result = {
        "metric": "per-layer decode launch, M = 1: fixed cost vs traffic time (us per launch)",
        "value": round(total, 2), "unit": "us", "n_gpus": 1, "steps": REPS, "warmup": 5,
        "ms_per_step": round(total / 1e3, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "launch floor of the decode GEMV sweep: empty / plain-read / real kernel per shape, "
                               "hip-graph replay of 200 launches, rotating weight copies"},
        "by_shape": rows,
    }
    print(json.dumps(result), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly from Python instead")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the protocol extras (read ceiling, replay spread, hot-cache and single-launch "
                         "times) so that a profiler sees only the launches of the timed passes")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--workload", choices=("decode_sweep", "full_step", "mixed_step", "chain_step", "layer_sweep", "w3_sweep", "launch_floor"), default="decode_sweep",
                    help="decode_sweep (default, the headline metric) or full_step: all 129 Linear layers of "
                         "a 32-layer 7B-class decoder per step")
    ap.add_argument("--m", type=int, default=1, help="rows of activations for --workload full_step / chain_step")
    ap.add_argument("--ms", default=MS_DEFAULT, help="row counts for --workload layer_sweep / w3_sweep (there the default is 1)")
    ap.add_argument("--shapes", default="", help="comma-separated shape names for --workload layer_sweep")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch

    import paper_2602_02711_amd as dmr
    from paper_2602_02711_amd import binding, synth

    binding.lib()                      # fail loudly if the HIP library is not built
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "full_step":
        return full_step(args, dmr, synth, torch, dev)
    if args.workload == "mixed_step":
        return mixed_step(args, dmr, synth, torch, dev)
    if args.workload == "chain_step":
        return chain_step(args, dmr, synth, torch, dev)
    if args.workload == "layer_sweep":
        return layer_sweep(args, dmr, synth, torch, dev)
    if args.workload == "w3_sweep":
        return w3_sweep(args, dmr, synth, torch, dev)
    if args.workload == "launch_floor":
        return launch_floor(args, dmr, synth, torch, dev)
    G = synth.GROUP
    M = 1

    # ---- resident inputs ---------------------------------------------------------------------
    shapes = synth.SWEEP_SHAPES
    layers, bf16_ws, xs, ys, ys_b = [], [], [], [], []
    t0 = time.time()
    for idx, (name, K, N) in enumerate(shapes):
        w = torch.from_numpy(synth.weights_f32(synth.seed_for(1, idx, 0), N, K)).to(dev)
        qw, s, z = dmr.dmr_qlinear_quantize(w, G)
        # the same number of copies for every shape (what the smallest layer needs to reach 1 GiB), so that
        # copy r of a shape is always followed by copy r of the next shape
        r4 = max(-(-CACHE_DEFEAT_BYTES // int4_bytes(Ks, Ns)) for _, Ks, Ns in shapes)
        layers.append([dmr.dmr_qlinear_create(qw, s, z, G) for _ in range(r4)])
        wb = w.to(torch.bfloat16)      # storage conversion (round to nearest even) of the same weights
        rb = -(-CACHE_DEFEAT_BYTES // bf16_bytes(K, N))
        bf16_ws.append([wb.clone() for _ in range(rb)])
        xb = synth.activations_bf16(synth.seed_for(1, idx, 1), M, K)
        xs.append(torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16))
        ys.append(torch.empty((M, N), dtype=torch.bfloat16, device=dev))
        ys_b.append(torch.empty((M, N), dtype=torch.bfloat16, device=dev))
        del w, qw, s, z, wb
    torch.cuda.synchronize()
    log(f"[bench] inputs resident after {time.time() - t0:.1f}s; copies per shape int4 "
        f"{[len(l) for l in layers]} bf16 {[len(l) for l in bf16_ws]}")

    stream = torch.cuda.Stream()       # default priority

    def int4_step(i, only=None):
        for idx in range(len(shapes)):
            if only is None or only == idx:
                dmr.dmr_qlinear_forward(layers[idx][i % len(layers[idx])], xs[idx], out=ys[idx])

    def bf16_step(i, only=None):
        for idx in range(len(shapes)):
            if only is None or only == idx:
                dmr.dmr_qlinear_bf16_forward(bf16_ws[idx][i % len(bf16_ws[idx])], xs[idx], out=ys_b[idx])

    def timed(step_fn, steps, warmup, only=None):
        """Returns (wall ms per step, HIP-event ms per step) for `steps` steps after `warmup`."""
        with torch.cuda.stream(stream):
            for i in range(warmup):
                step_fn(i, only)
            stream.synchronize()
            graph = None
            if not args.no_graph:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    for i in range(steps):
                        step_fn(warmup + i, only)
                for _ in range(3):     # untimed replays: graph upload, instruction caches, clock ramp
                    graph.replay()
                stream.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t_start = time.perf_counter()
            e0.record(stream)
            if graph is not None:
                graph.replay()
            else:
                for i in range(steps):
                    step_fn(warmup + i, only)
            e1.record(stream)
            torch.cuda.synchronize()
            wall = (time.perf_counter() - t_start) * 1e3 / steps
            return wall, e0.elapsed_time(e1) / steps

    # ---- the timed region that defines `value` ------------------------------------------------
    wall_ms, ev_ms = timed(int4_step, args.steps, args.warmup)
    step_bytes = sum(int4_bytes(K, N, M) for _, K, N in shapes)
    value = step_bytes / (wall_ms * 1e-3) / 1e9
    launches = len(shapes)
    achieved = step_bytes / (ev_ms * 1e-3) / 1e9

    # ---- beside it: the bf16 pass, and each shape on its own ----------------------------------
    bwall_ms, bev_ms = timed(bf16_step, args.steps, args.warmup)
    bstep_bytes = sum(bf16_bytes(K, N, M) for _, K, N in shapes)
    per_shape = []
    for idx, (name, K, N) in enumerate(shapes):
        n_inner = max(args.steps, 100)
        _, e4 = timed(int4_step, n_inner, 10, only=idx)
        _, eb = timed(bf16_step, n_inner, 10, only=idx)
        per_shape.append({
            "shape": name, "K": K, "N": N,
            "int4_us": round(e4 * 1e3, 3), "int4_GBps": round(int4_bytes(K, N, M) / e4 / 1e6, 1),
            "int4_frac_hbm_peak": round(int4_bytes(K, N, M) / e4 / 1e6 / HBM_PEAK_GBS, 4),
            "bf16_us": round(eb * 1e3, 3), "bf16_GBps": round(bf16_bytes(K, N, M) / eb / 1e6, 1),
            "speedup": round(eb / e4, 3),
        })
        log(f"[bench] {per_shape[-1]}")

    # ---- protocol extras (outside the timed region that defines `value`) -----------------------
    protocol = None

    def event_us(fn, iters):
        with torch.cuda.stream(stream):
            fn()
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(iters):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    if not args.no_extras:
        # (1) read ceiling: a plain nontemporal read of 1 GiB regions (never the same one twice in a row)
        probe_buf = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        probe_buf.random_(0, 255)
        sink = torch.empty(4096 * 256, dtype=torch.int32, device=dev)
        halves = [probe_buf[: 1 << 30], probe_buf[1 << 30:]]
        flip = [0]

        def probe_once(blocks):
            flip[0] ^= 1
            dmr.dmr_probe_hbm_read(halves[flip[0]], sink, blocks, stream=stream)

        # the read rate depends on how many waves ask at once (fewer is faster here): best of three grids
        ceiling_by_blocks = {b: (1 << 30) / min(event_us(lambda: probe_once(b), 4) for _ in range(2)) / 1e3
                             for b in (256, 512, 2048)}
        ceiling_gbs = max(ceiling_by_blocks.values())
        del probe_buf, halves

        # (2) per-step spread over replays, (3) hot-cache replays of one copy, (4) one eager launch
        spread = []
        with torch.cuda.stream(stream):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(50):
                    int4_step(i)
            graph.replay()
            stream.synchronize()
            for _ in range(20):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                graph.replay()
                e1.record(stream)
                torch.cuda.synchronize()
                spread.append(e0.elapsed_time(e1) * 1e3 / 50)
        spread.sort()
        hot, single = [], []
        for idx, (name, K, N) in enumerate(shapes):
            one = layers[idx][0]
            with torch.cuda.stream(stream):
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    for _ in range(100):
                        dmr.dmr_qlinear_forward(one, xs[idx], out=ys[idx])
                graph.replay()
                stream.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                graph.replay()
                e1.record(stream)
                torch.cuda.synchronize()
            hot.append(round(e0.elapsed_time(e1) * 1e3 / 100, 3))
            cold = layers[idx][len(layers[idx]) // 2]
            single.append(round(event_us(lambda: dmr.dmr_qlinear_forward(cold, xs[idx], out=ys[idx]), 1), 2))
        protocol = {
            "hbm_read_ceiling_GBps": round(ceiling_gbs, 1),
            "hbm_read_GBps_by_workgroups": {str(b): round(v, 1) for b, v in ceiling_by_blocks.items()},
            "value_frac_of_read_ceiling": round(value / ceiling_gbs, 4),
            "us_per_step_over_20_replays_of_50_steps": {"p10": round(spread[2], 3), "median": round(spread[10], 3),
                                                        "p90": round(spread[17], 3)},
            "hot_cache_us_per_launch": dict(zip([n for n, _, _ in shapes], hot)),
            "single_eager_launch_us": dict(zip([n for n, _, _ in shapes], single)),
            "note": "hot cache = the same weight copy 100 times in a row (it stays in the 256 MB Infinity Cache, so "
                    "this is not an HBM rate); single launch = HIP events around one eager launch after a sync",
        }

    # HBM traffic of the dominant kernel, from the committed rocprofv3 counter summary (offline runs
    # of this same command under --pmc FETCH_SIZE / WRITE_SIZE); null when no summary is present.
    traffic = traffic_source = None
    traffic_file = os.path.join(ROOT, "profiles", "decode_sweep_w4_gemv_traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as fh:
            rec = json.load(fh)
        traffic = rec.get("traffic")
        traffic_source = rec.get("source", "profiles/decode_sweep_w4_gemv_traffic.json (offline rocprofv3 --pmc runs)")

    result = {
        "metric": "INT4 W4A16 linear achieved HBM GB/s at M=1 and speedup vs bf16 linear",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "decode GEMV sweep, M=1, INT4 g128 (bf16 scales/zeros), (K,N) in "
                        "{(4096,4096),(4096,6144),(4096,28672),(14336,4096)}; one step = the four "
                        "forwards; weights rotate over >=1 GiB of resident copies per shape",
            "weights": "int4 asymmetric g128, fp32 0.02*N(0,1) quantised by the device RTN quantiser",
            "activations": "bf16 N(0,1)", "accumulate": "fp32", "output": "bf16",
            "launch": "eager" if args.no_graph else "hip-graph replay of all timed steps (after W eager warm-up "
                      "steps and 3 untimed replays)",
            "algorithmic_bytes_per_step": step_bytes,
        },
        "speedup_vs_bf16": round(bwall_ms / wall_ms, 3),
        "bf16_ms_per_step": round(bwall_ms, 6),
        "bf16_GBps": round(bstep_bytes / (bwall_ms * 1e-3) / 1e9, 1),
        "us_per_decode_sweep": round(wall_ms * 1e3, 2),
        "per_shape": per_shape,
        "protocol": protocol,
        "roofline": {
            "kernel": "w4_gemv_kernel (INT4 weight-streaming MFMA GEMV, all four shapes of a step)",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": None if traffic is None else round(traffic),
            "traffic_source": traffic_source,
            "bytes_per_launch": step_bytes // launches,
            "avg_launch_us": round(ev_ms * 1e3 / launches, 3),
        },
    }

    # ---- the oracle on the host cores, same workload, bounded sample --------------------------
    # The oracle as it stands (integer unpack, fp64 dequantise, naive fp64 dot products; rows spread over OpenMP
    # threads): the correctness-only shape and the four shapes of the sweep, once on one core and repeatedly on
    # every thread the host gives this process, within --cpu-seconds in total.
    if not args.no_cpu_baseline:
        from oracle import cpu_oracle as orc
        threads = orc.max_threads()
        table, y_ref0, t_all_sweep, used_all = [], None, 0.0, threads
        cases = [("config0",) + tuple(synth.SMALL_SHAPE[1:])] + [(n, K, N) for n, K, N in shapes]
        budget_each = args.cpu_seconds / (2 * len(cases))
        for ci, (name, K, N) in enumerate(cases):
            seed_w = synth.seed_for(0, 0, 0) if ci == 0 else synth.seed_for(1, ci - 1, 0)
            seed_x = synth.seed_for(0, 0, 1) if ci == 0 else synth.seed_for(1, ci - 1, 1)
            q, s, z = orc.quantize(synth.weights_f32(seed_w, N, K), G)
            words = orc.pack(q)
            xb = synth.activations_bf16(seed_x, M, K)
            t1 = time.perf_counter()
            y_ref, _ = orc.forward(words, s, z, G, xb, threads=1)
            t_one = time.perf_counter() - t1
            passes, t_all = 0, 0.0
            while passes == 0 or (t_all < budget_each and passes < 200):
                t1 = time.perf_counter()
                _, used_all = orc.forward(words, s, z, G, xb, threads=threads)
                t_all += time.perf_counter() - t1
                passes += 1
            nb = int4_bytes(K, N, M)
            table.append({"shape": name, "K": K, "N": N, "one_core_us": round(t_one * 1e6, 1),
                          "one_core_GBps": round(nb / t_one / 1e9, 3), "one_core_GFLOPs": round(2.0 * K * N / t_one / 1e9, 2),
                          "all_threads_us": round(t_all / passes * 1e6, 1), "all_threads_GBps": round(nb / (t_all / passes) / 1e9, 3),
                          "all_threads_GFLOPs": round(2.0 * K * N / (t_all / passes) / 1e9, 2), "passes": passes})
            log(f"[bench] oracle {table[-1]}")
            if ci == 1:
                y_ref0 = y_ref
            if ci >= 1:
                t_all_sweep += t_all / passes
        # parity of the bench's own launch configuration on the first sweep shape (device quantiser == oracle's)
        y_gpu = ys[0].float().cpu().numpy().astype(np.float64)
        err = float(np.max(np.abs(y_gpu - y_ref0)) / np.sqrt(np.mean(y_ref0 ** 2)))
        result["cpu_baseline"] = {
            "value": round(step_bytes / t_all_sweep / 1e9, 3), "unit": "GB/s", "cores": int(used_all), "kind": "oracle",
            "sample": f"one decode sweep (the four shapes, M=1) = {t_all_sweep * 1e3:.1f} ms on {int(used_all)} OpenMP threads "
                      f"(host reports {os.cpu_count()} logical CPUs), mean over the passes listed per shape; same "
                      f"algorithmic-bytes accounting as `value`",
            "by_shape": table,
        }
        result["parity_in_bench_config"] = {"shape": shapes[0][0], "max_err_over_rms_bf16_out": round(err, 5)}

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
