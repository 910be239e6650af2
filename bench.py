#!/usr/bin/env python3
"""Benchmark of the LoCoCo hot path on one MI355X.

A "step" is one call of lococo_sequence_forward -- the whole Alg. 2 scan
(attention, fill / convolution logits, normalisation, fusion for every block)
-- over one synthetic sequence batch of the named workload, with all inputs
already resident in HBM.  value = batch * L / time per step (tokens/s for one
layer's heads).

Prints ONE JSON line with the throughput, a `roofline` object for the dominant
kernel (timed live with HIP events on the library's stream) and a
`cpu_baseline` object (the CPU oracle timed on a bounded sample).
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

PEAK_BF16_MFMA_TFLOPS = 2500.0      # MI355X dense bf16
PEAK_FP32_VALU_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def step_flops(w, m, Bn):
    """Algorithmic flops of one block step for ALL chains, by part (causal-exact attention)."""
    chains = w.batch * w.n_kv_heads
    T = m + Bn
    attn = 4.0 * w.head_dim * Bn * (m + (Bn + 1) / 2.0) * w.group * chains
    if m + Bn <= w.M:
        return {"attn": attn, "conv": 0.0, "mix": 0.0}
    conv = 2.0 * w.M * T * w.C * w.conv_width * chains
    mix = 4.0 * w.M * T * w.head_dim * chains
    return {"attn": attn, "conv": conv, "mix": mix}


def scan_flops(w, plan):
    tot = {"attn": 0.0, "conv": 0.0, "mix": 0.0}
    for (_, ln, _, before, _, _) in plan:
        for k_, f in step_flops(w, before, ln).items():
            tot[k_] += f
    return tot


# which parts of the algorithmic work each kernel of the library carries
KERNEL_PARTS = {
    "attn_generic": ("attn",), "attn_mfma": ("attn",),
    "conv_logits_generic": ("conv",), "mix_generic": ("mix",),
    "conv_logits_mfma": ("conv",), "mix_mfma": ("mix",),
    "compress_mfma": ("conv", "mix"),
}
KERNEL_BOUND = {  # roofline that bounds each kernel, peak, unit
    "attn_generic": ("mfma", PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"),
    "attn_mfma": ("mfma", PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"),
    "conv_logits_generic": ("mfma", PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"),
    "mix_generic": ("mfma", PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"),
    "compress_mfma": ("mfma", PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"),
}


def scan_bytes(w, plan):
    """Algorithmic HBM bytes of the stand-alone passes of the unfused path, summed over the scan: the
    fp32 logits written by Eq. 5 and read (once) by Eq. 6 + Eq. 4, which also reads [K | V] and writes the
    new cache rows."""
    chains = w.batch * w.n_kv_heads
    e = 2 if w.dtype == "bf16" else 4
    tot = {"logits_write": 0.0, "mixnorm": 0.0, "normalise": 0.0}
    for (_, ln, branch, before, _, _) in plan:
        if not branch:
            continue
        T = before + ln
        tot["logits_write"] += 4.0 * w.M * T * chains
        tot["mixnorm"] += (4.0 * w.M * T + 2.0 * T * w.head_dim * e + 2.0 * w.M * w.head_dim * e) * chains
        tot["normalise"] += 8.0 * w.M * T * chains
    return tot


def kernel_rooflines(w, plan, flops, kt, steps):
    """One roofline entry per kernel that ran: the matrix-core fraction of the contractions, the HBM
    fraction of the passes whose arithmetic intensity is left of the ridge (Eq. 6 alone; Eq. 6 + Eq. 4
    from fp32 logits: 4 M T d flops over 4 M T bytes = d flop/B)."""
    by = scan_bytes(w, plan)
    out = {}
    for name, (launches, total_ms) in kt.items():
        if total_ms <= 0:
            continue
        sec = total_ms * 1e-3 / steps
        if name in ("mix_mfma", "normalise_generic"):
            b = by["mixnorm" if name == "mix_mfma" else "normalise"]
            out[name] = {"bound": "hbm", "achieved": b / sec / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": b / sec / 1e9 / PEAK_HBM_GBS, "ms_per_step": sec * 1e3}
        elif name in KERNEL_PARTS:
            f = sum(flops[p_] for p_ in KERNEL_PARTS[name])
            out[name] = {"bound": "mfma", "achieved": f / sec / 1e12, "peak": PEAK_BF16_MFMA_TFLOPS,
                         "unit": "TFLOP/s", "frac": f / sec / 1e12 / PEAK_BF16_MFMA_TFLOPS, "ms_per_step": sec * 1e3}
            if name == "conv_logits_mfma":       # its fp32 logits cross HBM: the achieved write rate beside it
                out[name]["hbm_write_gbs"] = by["logits_write"] / sec / 1e9
        else:
            out[name] = {"ms_per_step": sec * 1e3}
    return out


def measured_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel and
    workload (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known size), or None."""
    import re
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", open(path).read(), re.M)
        return int(m.group(1)) if m else None
    except OSError:
        return None


def graph_replay(torch, call, tokens, steps, warmup=3):
    """The same call captured once into a HIP graph and replayed back to back: what is left when the host's
    launch gaps are gone (kernel nodes only).  Not the headline figure: an extra one beside it."""
    try:
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(stream):
            with torch.cuda.graph(graph, stream=stream):
                call()
        torch.cuda.current_stream().wait_stream(stream)
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        return {"ms_per_step": ms, "value": tokens / (ms * 1e-3), "unit": "tokens/s", "steps": steps}
    except Exception as e:                      # the figure is optional; the headline line is not
        return {"error": str(e)[:200]}


def second_shape(lb, inputs, torch, name="cfg2", steps=50, warmup=5):
    """The other target shape (M = 128, 3.5 K tokens) in the same process, outside the timed region of the
    headline workload: tokens/s of the whole scan and the compression kernel's share of the MFMA peak."""
    w = inputs.CONFIGS[name]
    dev = "cuda"
    cfg = lb.config_for(w)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    qd, kd, vd, cwd, cbd = (t.to(dev) for t in (q, k, v, cw, cb))
    od = torch.empty_like(qd)
    cache = lb.Cache(cfg, dev)
    ws = lb.workspace(cfg, w.L, w.B, 1, dev)
    plan = lb.lococo_plan(w.L, w.B, w.M)
    flops = scan_flops(w, plan)

    def step():
        cache.c.len = 0
        lb.lococo_sequence_forward(cfg, qd, kd, vd, od, cwd, cbd, cache, w.B, ws)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    lb.lococo_timing_begin()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    kt = lb.lococo_timing_end()
    if ws is not None and lb.lococo_scan_status(cfg, ws) != 0:
        return {"workload": w.name, "error": "a chain wait inside the one-launch scan gave up"}
    name_k = max(kt, key=lambda n: kt[n][1])
    part = sum(flops[p] for p in KERNEL_PARTS.get(name_k, ())) * steps
    res = {"workload": w.name, "value": w.batch * w.L / (ms * 1e-3), "unit": "tokens/s", "steps": steps,
           "ms_per_step": ms, "kernel": name_k, "frac": part / (kt[name_k][1] * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
           "kernel_ms_per_step": {n: kt[n][1] / steps for n in kt}, "kernels": lb.lococo_describe_path(cfg, w.B)}
    res["hip_graph"] = graph_replay(torch, step, w.batch * w.L, steps)
    if lb.lococo_scan_status(cfg, ws) != 0:
        res["hip_graph"] = {"error": "a chain wait inside the one-launch scan gave up"}
    return res


def cpu_baseline(w, budget_s=15.0):
    """Oracle (as it stands) on a bounded sample: `threads` chains, the first
    few blocks of the scan, scaled to tokens/s of the whole layer."""
    import numpy as np
    from oracle import lococo_oracle as orc
    from paper_2406_05317_amd import inputs
    threads = min(os.cpu_count() or 1, 16)
    chains_total = w.batch * w.n_kv_heads
    n_chains = min(threads, chains_total)
    cw, cb = inputs.conv_filters(w)
    # size the sample from a one-chain, two-block probe
    def run(nc, nseg):
        L = min(w.L, nseg * w.B)
        qs, ks, vs = [], [], []
        for c in range(nc):
            b, h = divmod(c, w.n_kv_heads)
            q, k, v = inputs.chain_inputs(w, b, h, L)
            qs.append(q); ks.append(k[None]); vs.append(v[None])
        import torch
        q = torch.cat(qs)[None]; k = torch.cat(ks)[None]; v = torch.cat(vs)[None]
        cwx = cw if cw.dim() == 3 else cw[:1].repeat(nc, 1, 1, 1)
        cbx = cb if cb.dim() == 1 else cb[:1].repeat(nc, 1)
        t0 = time.perf_counter()
        orc.sequence_forward(q, k, v, cwx, cbx, B=w.B, M=w.M, conv_in=w.conv_in, norm=w.norm,
                             state_round=w.dtype, nthreads=nc)
        return time.perf_counter() - t0, L
    fills = w.M // w.B
    t_probe, _ = run(1, fills + 1)                       # one compress step on one chain
    nseg = int(max(fills + 1, min(w.L // w.B, fills + budget_s / max(t_probe, 1e-3))))
    t, L = run(n_chains, nseg)
    tokens_equiv = w.batch * L * (n_chains / chains_total)   # whole-layer tokens this work equals
    return {"value": tokens_equiv / t, "unit": "tokens/s", "cores": n_chains, "kind": "oracle",
            "sample": f"{n_chains} of {chains_total} chains x first {nseg} blocks ({L} tokens) of "
                      f"{w.name}, {t:.1f} s, scaled linearly by chain count"}


def decode_bench(args, w, lb, inputs, torch):
    """Generation stage (B = 1): one segment step per token on a full cache, all sequences of the
    batch in one call.  A step here is ONE token of every sequence."""
    dev = "cuda"
    w = w.replace(name=w.name + "-decode", batch=args.decode_batch, L=w.M + args.warmup + args.steps, B=1)
    cfg = lb.config_for(w, impl=args.impl)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    qd, kd, vd, cwd, cbd = (t.to(dev) for t in (q, k, v, cw, cb))
    od = torch.empty_like(qd)
    cache = lb.Cache(cfg, dev)
    # fill the cache with the first M tokens (one block, nothing to compress yet)
    cfg_fill = lb.config_for(w.replace(B=w.M), impl=args.impl)
    lb.lococo_sequence_forward(cfg_fill, qd[:, :, :w.M], kd[:, :, :w.M], vd[:, :, :w.M], od[:, :, :w.M], cwd, cbd,
                               cache, w.M, lb.workspace(cfg_fill, w.M, w.M, False, dev))
    ws = lb.workspace(cfg, 1, 1, False, dev)
    lb.lococo_prepare_filters(cfg, cwd, ws)              # once per generation, not once per token
    cfg.flags |= lb.LOCOCO_FLAG_FILTERS_PREPARED

    def token(t):
        lb.lococo_segment_step(cfg, qd[:, :, t:t + 1], kd[:, :, t:t + 1], vd[:, :, t:t + 1], od[:, :, t:t + 1],
                               cwd, cbd, cache, ws)
    t = w.M
    for _ in range(args.warmup):
        token(t); t += 1
    torch.cuda.synchronize()
    if args.decode_graph:
        # two steps per graph: after two compressions the cache ping-pong is back at its first buffer
        if (args.warmup % 2) or (args.steps % 2):
            raise SystemExit("--decode-graph needs even --warmup and --steps")
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(stream):
            with torch.cuda.graph(graph, stream=stream):
                token(t); token(t + 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps // 2):
            graph.replay()                               # the same two tokens again: timing only
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kt = {"graph": (args.steps // 2, (t1 - t0) * 1e3)}
    else:
        lb.lococo_timing_begin()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            token(t); t += 1
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kt = lb.lococo_timing_end()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flops = step_flops(w, w.M, 1)
    name = max(kt, key=lambda n: kt[n][1])
    launches, total_ms = kt[name]
    part = sum(flops[p] for p in KERNEL_PARTS.get(name, ())) * args.steps
    achieved = part / (total_ms * 1e-3) / 1e12 if total_ms > 0 else 0.0
    out = {"metric": "generation-stage tokens/sec per layer (segment step with B = 1: attention, conv logits, "
                     "normalisation, fusion per token)",
           "value": w.batch / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
           "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                      "head_dim": w.head_dim, "B": 1, "M": w.M, "conv_width": w.conv_width,
                      "conv_channels": w.C, "impl": args.impl, "hip_graph": bool(args.decode_graph)},
           "roofline": {"kernel": name, "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_MFMA_TFLOPS,
                        "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_MFMA_TFLOPS, "traffic": None,
                        "launches": launches, "avg_launch_us": total_ms * 1e3 / max(launches, 1),
                        "kernel_ms_per_step": {n: kt[n][1] / args.steps for n in kt}}}
    print(json.dumps(out))


def backward_scan_bench(args, w, lb, inputs, torch):
    """Backward of the whole scan in one call (lococo_sequence_backward): the cache recurrence recomputed,
    then every block's step backward in reverse."""
    dev = "cuda"
    cfg = lb.config_for(w, impl=args.impl)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    qd, kd, vd, cwd = (t.to(dev) for t in (q, k, v, cw))
    cache = lb.Cache(cfg, dev)
    shape = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    f = lambda *sh: torch.randn(*sh, device=dev, dtype=torch.float32)
    d_o, gk, gv = f(*q.shape), f(*shape), f(*shape)
    dq, dk, dv = torch.empty_like(d_o), f(*k.shape), f(*k.shape)
    dck, dcv = torch.empty_like(gk), torch.empty_like(gv)
    dW = torch.zeros(cw.shape, device=dev, dtype=torch.float32)
    ws_bytes = lb.lococo_sequence_backward_workspace_bytes(cfg, w.L, w.B)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def step():
        lb.lococo_sequence_backward(cfg, qd, kd, vd, w.B, cwd, None, cache, d_o, gk, gv, dq, dk, dv, dck, dcv, dW, None, ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    lb.lococo_timing_begin()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    kt = lb.lococo_timing_end()
    print(json.dumps({"metric": "backward of the whole scan, tokens/sec per layer", "value": w.batch * w.L / (ms * 1e-3),
                      "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                      "dtype": "f32" if args.impl == 1 else "bf16", "data": "synthetic",
                      "config": {"workload": w.name + "-backward-scan", "batch": w.batch, "n_q_heads": w.n_q_heads,
                                 "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "seq_len": w.L, "B": w.B, "M": w.M,
                                 "conv_width": w.conv_width, "conv_channels": w.C, "norm": w.norm,
                                 "workspace_bytes": ws_bytes},
                      "forward_recompute_kernel_ms_per_step": {n: kt[n][1] / args.steps for n in kt}}))


def backward_bench(args, w, lb, inputs, torch):
    """Backward of one compress step (full cache, one block).  --impl 1: every kernel shape-agnostic,
    fp32 vector arithmetic; default: the three Eq. 5 contractions on the matrix cores."""
    dev = "cuda"
    w = w.replace(name=w.name + "-backward-step", L=w.B)
    cfg = lb.config_for(w, impl=args.impl)
    generic = args.impl == 1
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    qd, kd, vd, cwd = (t.to(dev) for t in (q, k, v, cw))
    cache = lb.Cache(cfg, dev)
    shape = (w.batch, w.n_kv_heads, w.M, w.head_dim)
    cache.load(torch.randn(shape, device=dev).to(w.torch_dtype), torch.randn(shape, device=dev).to(w.torch_dtype), w.M)
    f = lambda *sh: torch.randn(*sh, device=dev, dtype=torch.float32)
    d_o, gk, gv = f(*q.shape), f(*shape), f(*shape)
    dq, dk, dv = torch.empty_like(d_o), f(*k.shape), f(*k.shape)
    dck, dcv = torch.empty_like(gk), torch.empty_like(gv)
    dW = torch.zeros(cw.shape, device=dev, dtype=torch.float32)
    ws = torch.empty(lb.lococo_backward_workspace_bytes(cfg, w.B, w.M), dtype=torch.uint8, device=dev)

    def step():
        lb.lococo_segment_step_backward(cfg, qd, kd, vd, cwd, None, cache, d_o, gk, gv, dq, dk, dv, dck, dcv, dW,
                                        None, ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    fl = step_flops(w, w.M, w.B)
    tf = 2.0 * sum(fl.values()) / (ms * 1e-3) / 1e12
    peak = PEAK_FP32_VALU_TFLOPS if generic else PEAK_BF16_MFMA_TFLOPS
    print(json.dumps({"metric": "backward of one compress step, tokens/sec per layer (%s)" %
                                ("shape-agnostic fp32 kernels" if generic else
                                 "contractions on bf16 MFMA with fp32 operands as two bf16 halves, row reductions fp32 vector"),
                      "value": w.batch * w.B / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
                      "vs_baseline": None, "dtype": "f32" if generic else "bf16", "data": "synthetic",
                      "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads,
                                 "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "B": w.B, "M": w.M,
                                 "conv_width": w.conv_width, "conv_channels": w.C, "norm": w.norm},
                      "roofline": {"bound": "alu" if generic else "mfma", "achieved": tf, "peak": peak,
                                   "unit": "TFLOP/s", "frac": tf / peak, "traffic": None}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--impl", type=int, default=0, help="0 auto, 1 generic kernels, 2 MFMA only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-history", action="store_true",
                    help="step-by-step schedule instead of the batched-attention one")
    ap.add_argument("--history-window", type=int, default=0,
                    help="workspace for a window of this many blocks (>= 2) instead of the whole sequence: the "
                         "batched-attention schedule window by window, memory independent of the sequence length")
    ap.add_argument("--conv-width", type=int, default=0, help="override the workload's filter width (e.g. 21)")
    ap.add_argument("--norm", type=int, default=-1, help="override the normalisation (0 softmax, 1 relu-sum)")
    ap.add_argument("--conv-in", type=int, default=0, help="1: the filters read [K | V] (2 d channels) instead of the keys")
    ap.add_argument("--protect-sinks", type=int, default=0,
                    help="protect the first N cache slots (attention sinks kept beside the compressed memory)")
    ap.add_argument("--track-attention", action="store_true",
                    help="accumulate the attention each cache slot receives (lococo_cache.attn_colsum) during the scan")
    ap.add_argument("--backward-scan", action="store_true",
                    help="instead of the forward scan, time lococo_sequence_backward over the whole workload")
    ap.add_argument("--backward", action="store_true",
                    help="instead of the scan, time the backward pass of ONE compress step of the workload's shape "
                         "(--impl 1: shape-agnostic fp32 kernels only)")
    ap.add_argument("--decode-batch", type=int, default=0,
                    help="instead of the prefill scan, time the generation stage: --steps segment steps "
                         "with B = 1 on a full cache, for this many sequences at once (0 = off)")
    ap.add_argument("--decode-graph", action="store_true",
                    help="with --decode-batch: replay pairs of generation steps from a captured HIP graph")
    ap.add_argument("--sustain-seconds", type=float, default=2.0,
                    help="after the timed steps, run sequences back to back for at least this long and report the "
                         "steady-state rate (the chip is power-limited under matrix load; 0 = skip)")
    ap.add_argument("--debug-option", action="append", default=[], metavar="N=V",
                    help="set the library's test / measurement hook number N to V (lococo_debug_option) before the run")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB before the warm-up, so "
                         "that a rocprofv3 --pmc run has a kernel of known HBM traffic to scale "
                         "FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path shards over (batch, kv-head) chains "
              "with no communication, so there is no multi-GPU figure to report. Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2406_05317_amd import binding as lb
    from paper_2406_05317_amd import inputs
    w = inputs.CONFIGS[args.workload]
    for kv in args.debug_option:
        n_, v_ = kv.split("=")
        lb.lococo_debug_option(int(n_), int(v_))
    if args.conv_width:
        w = w.replace(name=f"{w.name}-k{args.conv_width}", conv_width=args.conv_width)
    if args.norm >= 0:
        w = w.replace(name=f"{w.name}-norm{args.norm}", norm=args.norm)
    if args.conv_in:
        w = w.replace(name=f"{w.name}-kv", conv_in=1)
    dev = "cuda"
    torch.cuda.set_device(0)
    if args.decode_batch:
        return decode_bench(args, w, lb, inputs, torch)
    if args.backward_scan:
        return backward_scan_bench(args, w, lb, inputs, torch)
    if args.backward:
        return backward_bench(args, w, lb, inputs, torch)
    cfg = lb.config_for(w, impl=args.impl)
    q, k, v = inputs.qkv(w)
    cw, cb = inputs.conv_filters(w)
    qd, kd, vd, cwd, cbd = (t.to(dev) for t in (q, k, v, cw, cb))
    od = torch.empty_like(qd)
    cache = lb.Cache(cfg, dev)
    if args.protect_sinks:
        import numpy as np
        cache.set_protect(np.arange(w.M) < args.protect_sinks)
    if args.track_attention:
        cache.track_attention()
    ws = lb.workspace(cfg, w.L, w.B, 0 if args.no_history else (args.history_window or 1), dev)
    plan = lb.lococo_plan(w.L, w.B, w.M)
    flops = scan_flops(w, plan)

    def step():
        cache.c.len = 0                                  # fresh sequence (host-side state only)
        lb.lococo_sequence_forward(cfg, qd, kd, vd, od, cwd, cbd, cache, w.B, ws)

    if args.calibration_copy_mib:
        n = args.calibration_copy_mib << 20
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                   # reads n bytes, writes n bytes
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    lb.lococo_timing_begin()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kt = lb.lococo_timing_end()
    # a wait inside the one-launch scan that gave up would end the launch early and look fast
    if ws is not None and lb.lococo_scan_status(cfg, ws) != 0:
        print("bench.py: a chain wait inside the one-launch scan gave up; the run is invalid", file=sys.stderr)
        sys.exit(3)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens = w.batch * w.L
    value = tokens / (ms_per_step * 1e-3)

    # dominant kernel = largest share of device time in the timed region
    name = max(kt, key=lambda n: kt[n][1])
    launches, total_ms = kt[name]
    bound, peak, unit = KERNEL_BOUND.get(name, ("mfma", PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"))
    part_flops = sum(flops[p] for p in KERNEL_PARTS.get(name, ())) * args.steps
    achieved = part_flops / (total_ms * 1e-3) / 1e12 if total_ms > 0 else 0.0
    roofline = {"kernel": name, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": measured_traffic(name, args.workload)
                if w is inputs.CONFIGS[args.workload] and not args.protect_sinks else None,
                "launches": launches,
                "avg_launch_us": total_ms * 1e3 / max(launches, 1),
                "flops_per_launch": part_flops / max(launches, 1),
                "kernel_ms_per_step": {n: kt[n][1] / args.steps for n in kt}}
    path_info = lb.lococo_describe_path(cfg, w.B)
    total_flops = sum(flops.values())
    out = {
        "metric": "segment-step tokens/sec per layer (whole Alg. 2 scan incl. attention, conv "
                  "logits, normalisation, fusion)",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "seq_len": w.L, "B": w.B,
                   "M": w.M, "conv_width": w.conv_width, "conv_channels": w.C,
                   "schedule": "step-by-step" if args.no_history else
                               (f"batched-attention, windows of {args.history_window} blocks" if args.history_window
                                else "batched-attention"),
                   "workspace_bytes": 0 if ws is None else ws.numel(),
                   "protected_slots": args.protect_sinks, "track_attention": bool(args.track_attention),
                   "impl": args.impl, "kernels": path_info},
        "segment_step_tokens_per_s": w.batch * w.B / (ms_per_step * 1e-3 / len(plan)),
        "mfma_util_whole_path": total_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "roofline": roofline,
        "kernel_rooflines": kernel_rooflines(w, plan, flops, kt, args.steps),
    }
    if args.sustain_seconds > 0:
        # steady state: sequences back to back for a couple of seconds, timed as a whole
        n_seq = max(args.steps, int(args.sustain_seconds / (ms_per_step * 1e-3)) + 1)
        lb.lococo_timing_begin()
        t0 = time.perf_counter()
        for _ in range(n_seq):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kts = lb.lococo_timing_end()
        if ws is not None and lb.lococo_scan_status(cfg, ws) != 0:
            print("bench.py: a chain wait inside the one-launch scan gave up; the run is invalid", file=sys.stderr)
            sys.exit(3)
        dom_ms = kts[name][1] / n_seq
        out["sustained"] = {"seconds": t1 - t0, "sequences": n_seq, "value": tokens * n_seq / (t1 - t0), "unit": "tokens/s",
                            "kernel": name, "avg_launch_us": kts[name][1] * 1e3 / max(kts[name][0], 1),
                            "frac": part_flops / args.steps / (dom_ms * 1e-3) / 1e12 / peak if dom_ms > 0 else 0.0}
    if args.sustain_seconds > 0 and not args.track_attention:
        out["hip_graph"] = graph_replay(torch, step, tokens, args.steps)
        if ws is not None and lb.lococo_scan_status(cfg, ws) != 0:
            out["hip_graph"] = {"error": "a chain wait inside the one-launch scan gave up"}
    # what this machine sustains on a bare MFMA loop and a plain copy, after the timed region, so that the
    # fraction can also be read against the measured ceiling (`peak` stays the published figure)
    scratch = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    mfma_tf, copy_gbs = lb.lococo_measure_peaks(scratch)
    del scratch
    out["measured_peaks"] = {"mfma_bf16_tflops": mfma_tf, "copy_gbs": copy_gbs,
                             "how": "bare 32x32x16 bf16 MFMA loop on random operand bits, launches of >= 14 ms; "
                                    "1 GiB -> 1 GiB copy, reads + writes"}
    measured = {"mfma": mfma_tf, "hbm": copy_gbs}.get(bound)
    if measured:
        roofline["frac_of_measured_peak"] = achieved / measured
    if w is inputs.CONFIGS["cfg3"] and args.workload == "cfg3" and not (args.debug_option or args.no_history or
                                                                      args.history_window or args.impl):
        out["second_target_shape"] = second_shape(lb, inputs, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
