#!/usr/bin/env python3
"""Benchmark of the ReAttention per-layer hot path on one MI355X.

A "step" is one decode step of one layer (score -> top-k -> concat -> PE -> attention,
every stage inside libreattn's HIP kernels) over the 1M-token Llama-3.1-8B-shaped
cache of config 3, with all inputs already resident in HBM.  Prints ONE JSON line:
the step latency (ms/layer), the roofline of the dominant kernel (the key scan,
HBM-bound) from HIP events recorded on the launch stream, and the fp64 CPU oracle
timed on this machine's host cores as a baseline.

    python bench.py [--gpus 1] [--steps 20] [--warmup 3] [--config 3] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E bandwidth
# Measured with rocprofv3 --pmc: fetched + written bytes per launch of the scan kernel, per workload.
SCAN_TRAFFIC = {"cfg3_decode_1m_bf16": {"bytes": 2 * 1045784.6 * 1024 + 928.1 * 1024,
                                        "source": "profiles/score_scan_cfg3_pmc.md"}}
# Same for the other dominant kernels (profiles/vote_decode_cfg3_kernel_trace_pmc.md,
# profiles/prefill_chunk_cfg4_kernel_trace_pmc.md, profiles/vote_prefill_cfg4_kernel_trace_pmc.md): fetched bytes per launch.
VOTE_SCAN_TRAFFIC_BYTES = {"cfg3_decode_1m_bf16": 2 * 1044560.7 * 1024 + 32.0 * 1024}
GEMM_FILTER_TRAFFIC_BYTES = 2 * 266407.5 * 1024
VOTE_GEMM_TRAFFIC_BYTES = 2 * 277092.2 * 1024


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 5],
                    help="decode configuration (3 = the 1M-token one the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the decode legs of the configurations other than --config")
    ap.add_argument("--no-prefill", action="store_true",
                    help="skip the config-4 prefill-chunk measurement (MFMA score contraction)")
    ap.add_argument("--only-prefill", action="store_true",
                    help="run the config-4 prefill leg alone and print its object (for profiling runs)")
    ap.add_argument("--no-vote", action="store_true",
                    help="skip the vote-selection decode step (the paper's own way of combining heads)")
    ap.add_argument("--only-vote", action="store_true",
                    help="run the vote-selection leg alone and print its object (for profiling runs)")
    ap.add_argument("--only-vote-prefill", action="store_true",
                    help="run the vote-selection prefill chunk alone (config 4's cache) and print its object")
    ap.add_argument("--chunk", type=int, default=4096, help="query rows of --only-vote-prefill / --only-sequence")
    ap.add_argument("--only-sequence", action="store_true",
                    help="run the streaming prefill of one layer over --seq-len tokens alone (chunk 512 by default)")
    ap.add_argument("--seq-len", type=int, default=65536)
    ap.add_argument("--no-sequence", action="store_true", help="skip the streaming-prefill leg")
    ap.add_argument("--only-batched", action="store_true",
                    help="run the fp16 batched-decode leg alone (context / batch pairs of the paper's throughput table)")
    ap.add_argument("--no-batched", action="store_true", help="skip the fp16 batched-decode leg")
    ap.add_argument("--only-token", action="store_true", help="run the 32-layer decode-token leg alone")
    ap.add_argument("--no-token", action="store_true", help="skip the 32-layer decode-token leg")
    ap.add_argument("--only-paged", action="store_true", help="run the paged-cache decode step alone")
    ap.add_argument("--no-paged", action="store_true", help="skip the paged-cache decode step")
    ap.add_argument("--only-paged-prefill", action="store_true", help="run the paged-cache prefill chunk alone")
    ap.add_argument("--only-unfused", action="store_true",
                    help="run the four separate calls (score, top-k, gather + rotary, attend) alone")
    ap.add_argument("--no-unfused", action="store_true", help="skip the leg of the four separate calls")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy 3 times (a known-size kernel against "
                         "which rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one layer's hot path on one MI355X); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.only_prefill:
        print(json.dumps({"prefill": prefill_leg(min(args.steps, 5))}), flush=True)
        return 0
    if args.only_token:
        print(json.dumps({"decode_token_32_layers": decode_token_leg(min(args.steps, 10))}), flush=True)
        return 0
    if args.only_batched:
        print(json.dumps({"batched_decode_f16": batched_decode_leg(args.steps)}), flush=True)
        return 0
    if args.only_sequence:
        print(json.dumps({"prefill_sequence": sequence_leg(args.seq_len, args.chunk if args.chunk != 4096 else 512)}),
              flush=True)
        return 0
    if args.only_vote_prefill:
        print(json.dumps({"vote_prefill": vote_prefill_leg(min(args.steps, 5), args.chunk)}), flush=True)
        return 0
    if args.only_paged_prefill:
        print(json.dumps({"paged_prefill": paged_prefill_leg(args.steps if args.steps < 5 else 5)}))
        return 0
    if args.only_paged:
        print(json.dumps({"paged_decode": paged_leg(wl.generate(wl.CONFIGS[args.config], "cuda"), args.config,
                                                    args.steps, args.warmup)}), flush=True)
        return 0
    if args.only_unfused:
        print(json.dumps({"unfused_calls": unfused_leg(wl.generate(wl.CONFIGS[args.config], "cuda"), args.config,
                                                       args.steps)}), flush=True)
        return 0
    if args.only_vote:
        print(json.dumps({"vote": vote_leg(wl.generate(wl.CONFIGS[args.config], "cuda"), args.config,
                                           args.steps, args.warmup)}), flush=True)
        return 0
    w = wl.CONFIGS[args.config]
    t = wl.generate(w, "cuda")
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    leg = decode_leg(w, t, args.steps, args.warmup)
    ms_per_step = leg["ms_per_step"]
    result = {
        "metric": "decode-step latency (one layer, 1 query token, ReAttention score+top-k+attend)",
        "value": ms_per_step,
        "unit": "ms/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": leg["config"],
        "kv_scan_GBps": leg["kv_scan_GBps"],
        "warm_workspace": leg["warm_workspace"],
        "stages_ms": leg["stages_ms"],
        "selection_route": leg["selection_route"],
        "step_floor": leg["step_floor"],
        "roofline": leg["roofline"],
    }
    if not args.no_other_configs:
        # the other decode configurations (1: 16K fp32 toy, 2: 128K, 5: 4M tokens), each with its own roofline
        others = {}
        for cfg in (1, 2, 5):
            if cfg == args.config:
                continue
            if cfg == 5:                          # 16 GiB of cache: the main configuration's tensors make room
                t = None
                torch.cuda.empty_cache()
            wc = wl.CONFIGS[cfg]
            tc = wl.generate(wc, "cuda")
            others[wc.name] = decode_leg(wc, tc, args.steps, args.warmup)
            del tc
            torch.cuda.empty_cache()
        result["decode_configs"] = others
        if t is None:
            t = wl.generate(w, "cuda")

    if not args.no_vote:
        result["vote"] = vote_leg(t, args.config, args.steps, args.warmup)
    if not args.no_unfused:
        result["unfused_calls"] = unfused_leg(t, args.config, args.steps)
    if not args.no_paged:
        result["paged_decode"] = paged_leg(t, args.config, args.steps, args.warmup)
        if not args.no_prefill:
            result["paged_prefill"] = paged_prefill_leg(5)
    if not args.no_prefill:
        t = None
        torch.cuda.empty_cache()
        result["prefill"] = prefill_leg(min(args.steps, 5))
        if not args.no_vote:
            torch.cuda.empty_cache()
            result["vote_prefill"] = vote_prefill_leg(min(args.steps, 5))
        if not args.no_sequence:
            torch.cuda.empty_cache()
            result["prefill_sequence"] = sequence_leg(args.seq_len, 512)
        if not args.no_batched:
            torch.cuda.empty_cache()
            result["batched_decode_f16"] = batched_decode_leg(args.steps)
        if not args.no_token:
            torch.cuda.empty_cache()
            result["decode_token_32_layers"] = decode_token_leg(min(args.steps, 10))
        t = None
    if not args.no_cpu_baseline:
        if t is None:
            t = wl.generate(w, "cuda")
        result["cpu_baseline"] = cpu_baseline(w, t)
    print(json.dumps(result), flush=True)
    return 0


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix rate


def wake_device(buf) -> None:
    """About 10 ms of plain reads of `buf` ahead of a leg's warm-up steps.  An idle MI355X needs that long under load
    to reach its clocks (the first twenty decode steps after a pause run 4 % slower, measured, whatever kernel
    runs), and a short warm-up would time the ramp instead of the step."""
    from paper_2407_15176_amd import binding as B
    n = buf.numel() * buf.element_size()
    B.probe_read_bandwidth(buf, iters=max(3, min(2000, int(10e-3 * 6.5e12 / max(n, 1)))))


def decode_leg(w, t: dict, steps: int, warmup: int) -> dict:
    """One decode configuration: wall-clock ms per step over `steps` steps (inputs resident in HBM, sync on
    both sides), the stage times from HIP events on the launch stream (a second set of instrumented steps),
    and the roofline of the key scan.  Caches under 1 GiB of keys are rotated over enough copies that their
    keys sum to 1 GiB (four times the 256 MB last-level cache), so that every step streams from HBM; the
    plain-read ceiling is probed over all the copies for the same reason."""
    import torch
    from paper_2407_15176_amd import binding as B
    p = B.Params.from_workload(w)
    ws = B.alloc_workspace(p)
    out = torch.empty(1, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    idx = torch.empty(1, w.n_kv_heads, w.k_eff, dtype=torch.int32, device="cuda")
    k_bytes = t["k"].numel() * t["k"].element_size()
    n_rot = 1 if k_bytes >= (1 << 30) else min(160, -(-(1 << 30) // k_bytes))
    if n_rot > 1:
        kbig = t["k"].unsqueeze(0).repeat(n_rot, 1, 1, 1)
        vbig = t["v"].unsqueeze(0).repeat(n_rot, 1, 1, 1)
        ks, vs = list(kbig.unbind(0)), list(vbig.unbind(0))
    else:
        kbig, ks, vs = t["k"], [t["k"]], [t["v"]]

    def step(i):
        B.decode_step(p, t["q"], ks[i % n_rot], vs[i % n_rot], ws, idx_out=idx, out=out)

    wake_device(kbig)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    # the same steps with reattn_params.ws_warm: a serving loop that keeps one workspace per shape promises that
    # the previous step left it behind, and the clearing / table launch at the head of a step is not enqueued
    # (measured in alternation with the plain steps, best of two loops each: a loop that runs later in the process
    # is a few microseconds faster whatever it runs, and the pair below is what may be compared)
    from dataclasses import replace
    pw = replace(p, ws_warm=1)

    def loop(pp):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            B.decode_step(pp, t["q"], ks[i % n_rot], vs[i % n_rot], ws, idx_out=idx, out=out)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_warm, ms_cold_again = float("inf"), float("inf")
    for _ in range(2):
        ms_warm = min(ms_warm, loop(pw))
        ms_cold_again = min(ms_cold_again, loop(p))
    stage_sum = {s: 0.0 for s in B.STAGES}
    for i in range(steps):
        _, _, ms = B.decode_step_timed(p, t["q"], ks[i % n_rot], vs[i % n_rot], ws, idx_out=idx, out=out)
        for s in B.STAGES:
            stage_sum[s] += ms[s]
    stages = {s: stage_sum[s] / steps for s in B.STAGES}
    read_ceiling = B.probe_read_bandwidth(kbig, iters=10 if n_rot == 1 else 3)   # plain read of the same keys (all copies)
    scan_ms = stages["scan"]
    scan_gbps = w.scan_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0
    filter_route = B.redo_list(p, ws) is not None
    # the step's algorithmic bytes: the key scan, one fp32 score per key written once and read twice (score
    # route; the filter route moves ~2 % of that), the K and V rows of the attention scope
    gather = 2 * w.scope * w.n_kv_heads * w.head_dim * w.elem_bytes
    floor_bytes = w.scan_bytes + 3 * w.n_kv_heads * w.n_mid * 4 + gather
    floor_ms = floor_bytes / (HBM_PEAK_GBPS * 1e9) * 1e3
    return {
        "workload": w.name, "ms_per_step": round(ms_per_step, 5),
        "warm_workspace": {"ms_per_step": round(ms_warm, 5), "ms_per_step_plain_same_moment": round(ms_cold_again, 5)},
        "steps": steps,
        "config": {
            "workload": w.name, "n_ctx": w.n_ctx, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
            "head_dim": w.head_dim, "n_sink": w.n_sink, "n_local": w.n_local, "top_k": w.top_k,
            "scope": w.scope, "cache_copies_rotated": n_rot,
        },
        "selection_route": "filter (sampled bound, filtering scan, pick)" if filter_route else "scores (scan + radix select)",
        "kv_scan_GBps": round(scan_gbps, 1),
        "stages_ms": {s: round(v, 5) for s, v in stages.items()},
        "step_floor": {"algorithmic_bytes": floor_bytes, "floor_ms_at_peak": round(floor_ms, 5),
                       "floor_over_measured": round(floor_ms / ms_per_step, 4)},
        "roofline": {
            "kernel": "score_scan_kernel", "bound": "hbm",
            "achieved": round(scan_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(scan_gbps / HBM_PEAK_GBPS, 4),
            "algorithmic_bytes": w.scan_bytes,
            # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (KiB per dispatch, each scaled
            # by what the same counter reads for a 1 GiB copy): measured for the workloads listed with the
            # profile they come from, null elsewhere
            "traffic": SCAN_TRAFFIC.get(w.name, {}).get("bytes"),
            "traffic_source": SCAN_TRAFFIC.get(w.name, {}).get("source"),
            "measured_read_ceiling_GBps": round(read_ceiling, 1),
            "frac_of_measured_ceiling": round(scan_gbps / read_ceiling, 4) if read_ceiling > 0 else None,
        },
    }


def prefill_leg(steps: int) -> dict:
    """Config 4: one prefill chunk of 4,096 queries against 262,144 cached keys (one layer).
    Reports the chunk latency and the fused MFMA score contraction's rate from HIP events."""
    import torch
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    w = wl.CONFIGS[4]
    p = B.Params.from_workload(w)
    t = wl.generate(w, "cuda")
    ws = B.alloc_workspace(p)
    out = torch.empty(w.n_query, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    idx = torch.empty(w.n_query, w.n_kv_heads, w.k_eff, dtype=torch.int32, device="cuda")
    B.prefill_chunk(p, t["q"], t["k"], t["v"], ws, idx_out=idx, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.prefill_chunk(p, t["q"], t["k"], t["v"], ws, idx_out=idx, out=out)
    torch.cuda.synchronize()
    ms_chunk = (time.perf_counter() - t0) * 1e3 / steps
    acc = {s: 0.0 for s in B.PREFILL_STAGES}
    for _ in range(steps):
        _, _, ms = B.prefill_chunk_timed(p, t["q"], t["k"], t["v"], ws, idx_out=idx, out=out)
        for s in acc:
            acc[s] += ms[s] / steps
    gemm_ms = acc["score_gemm_filter"]
    alg = w.score_flops                                   # 2*M*Hq*N_mid*D: every head scored (Eq. 2)
    executed = 2 * w.n_query * w.n_kv_heads * w.n_mid * w.head_dim * 2   # hi + lo of the group sum
    alg_tf = alg / (gemm_ms * 1e-3) / 1e12
    visible = w.n_query * w.scope - w.n_query * (w.n_query - 1) // 2      # slots seen, summed over the chunk's rows
    gather = visible * w.n_kv_heads * 2 * w.head_dim * t["k"].element_size()
    return {
        "workload": w.name, "ms_per_chunk": round(ms_chunk, 3), "steps": steps,
        "tokens_per_s": round(w.n_query / (ms_chunk * 1e-3), 1),
        "stages_ms": {s: round(v, 4) for s, v in acc.items()},
        "roofline": {
            "kernel": "score_gemm_kernel (fused threshold filter)", "bound": "mfma",
            "achieved": round(alg_tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(alg_tf / MFMA_BF16_PEAK_TFLOPS, 4),
            "algorithmic_flops": alg,
            "executed_mfma_flops": executed,
            "executed_TFLOPs": round(executed / (gemm_ms * 1e-3) / 1e12, 1),
            "executed_frac": round(executed / (gemm_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "traffic": GEMM_FILTER_TRAFFIC_BYTES,
        },
        # Eq. 3 of the chunk: every query row gathers its own kept K and V rows (causal inside the chunk); the
        # rows requested per second against the HBM peak (part of them is served by L2 and the memory-side cache)
        "attend_gather": {
            "kernel": "attend_prefill_kernel", "requested_bytes": gather,
            # rows asked for, not bytes fetched from HBM: most of them are served by L2 and the memory-side cache
            "requested_not_fetched_GBps": round(gather / (acc["attend"] * 1e-3) / 1e9, 1), "hbm_peak_GBps": HBM_PEAK_GBPS,
        },
    }


def vote_prefill_leg(steps: int, n_query: int = 4096) -> dict:
    """Config 4's cache with the paper's own selection for a chunk of query rows: per-head top-4 lists
    of all rows on the matrix cores (no score written), pooled votes -> 127 centres -> spans of 32,
    then ONE shared set attended by every row (causal inside the local window)."""
    import torch
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    w = wl.CONFIGS[4].scaled(top_k=0, n_query=n_query)
    v = B.Vote(4, 127, 32)
    p = B.Params.from_workload(w)
    t = wl.generate(w, "cuda")
    ws = B.alloc_vote_workspace(p, v)
    out = torch.empty(w.n_query, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    sel = torch.empty(B.vote_cap(p, v), dtype=torch.int32, device="cuda")
    n_sel = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.vote_layer(p, v, t["q"], t["k"], t["v"], ws, sel=sel, n_sel=n_sel, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.vote_layer(p, v, t["q"], t["k"], t["v"], ws, sel=sel, n_sel=n_sel, out=out)
    torch.cuda.synchronize()
    ms_chunk = (time.perf_counter() - t0) * 1e3 / steps
    acc = {s: 0.0 for s in B.VOTE_STAGES}
    for _ in range(steps):
        *_, ms = B.vote_layer_timed(p, v, t["q"], t["k"], t["v"], ws, sel=sel, n_sel=n_sel, out=out)
        for s in acc:
            acc[s] += ms[s] / steps
    flops = w.score_flops                               # 2*M*Hq*N_mid*D, all of it executed (no group-sum shortcut)
    tf = flops / (acc["head_topk_scan"] * 1e-3) / 1e12
    return {
        "workload": w.name, "n_query": n_query, "vote_k": v.vote_k, "n_centres": v.n_centres, "span": v.span,
        "n_selected": int(n_sel.item()), "ms_per_chunk": round(ms_chunk, 3), "steps": steps,
        "tokens_per_s": round(n_query / (ms_chunk * 1e-3), 1),
        "stages_ms": {s: round(x, 4) for s, x in acc.items()},
        "roofline": {
            "kernel": "vote_gemm_kernel (fused per-head running top-k) + list merge", "bound": "mfma",
            "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "algorithmic_flops": flops,
            "traffic": VOTE_GEMM_TRAFFIC_BYTES if n_query == 4096 else None,
        },
    }


def sequence_leg(seq_len: int, chunk: int, steps: int = 2) -> dict:
    """Streaming prefill of ONE layer over a whole sequence (appendix, prefilling phase): first chunk of
    n_sink + n_local tokens, then `chunk` tokens per step, each appended to the cache before it selects
    and attends.  Llama-3.1-8B layer shape, config 2's channel scales; both selections are timed."""
    import torch
    from dataclasses import replace
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    w = wl.CONFIGS[2].scaled(n_ctx=seq_len, n_needles=0, top_k=4096)
    g = torch.Generator(device="cuda").manual_seed(240715000 + 91)
    sig = wl.channel_sigma(w).to("cuda")
    q = torch.randn(seq_len, w.n_q_heads, w.head_dim, generator=g, device="cuda").bfloat16()
    k_new = (torch.randn(seq_len, w.n_kv_heads, w.head_dim, generator=g, device="cuda") * sig[None]).bfloat16()
    v_new = (torch.randn(seq_len, w.n_kv_heads, w.head_dim, generator=g, device="cuda") * sig[None]).bfloat16()
    kc = torch.empty(w.n_kv_heads, seq_len, w.head_dim, dtype=torch.bfloat16, device="cuda")
    vc = torch.empty_like(kc)
    res = {"workload": f"llama3.1-8b layer, {seq_len} tokens, chunk {chunk}, sink {w.n_sink}, local {w.n_local}",
           "seq_len": seq_len, "chunk": chunk}
    for name, vote, top_k in (("vote_4_127_32", B.Vote(4, 127, 32), 0), ("topk_4096_per_query", None, 4096)):
        p = B.Params.from_workload(replace(w, n_query=1, top_k=top_k, max_position=0))
        cp = p.c()
        need = B.lib().reattn_prefill_sequence_workspace_bytes(
            __import__("ctypes").byref(cp), __import__("ctypes").byref(vote.c()) if vote else None, chunk)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        B.prefill_sequence(p, chunk, q, k_new, v_new, kc, vc, vote=vote, ws=ws, want_sets=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            B.prefill_sequence(p, chunk, q, k_new, v_new, kc, vc, vote=vote, ws=ws, want_sets=False)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        res[name] = {"ms_per_layer": round(ms, 2), "tokens_per_s_per_layer": round(seq_len / (ms * 1e-3), 1),
                     "n_chunks": len(B.sequence_chunks(p, chunk)), "workspace_MiB": round(need / 2**20, 1)}
        del ws
        torch.cuda.empty_cache()
    return res


def batched_decode_leg(steps: int) -> dict:
    """Decode steps of one layer at the (context, batch) pairs of the paper's throughput table (Appendix,
    efficiency analysis: LLaMA3-8B, FP16) in fp16 storage.  A batch of equal-length sequences is folded
    into the head axis (cache [B*Hkv][N][D]): one call serves the whole batch (the vote selection pools the
    votes per sequence: reattn_vote.n_seq)."""
    import torch
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    rows = []
    for n_ctx, batch in ((32768, 8), (65536, 5), (98304, 4), (131072, 2), (196608, 1), (262144, 1)):
        w = wl.CONFIGS[2].scaled(dtype="f16", n_ctx=n_ctx, n_q_heads=32 * batch, n_kv_heads=8 * batch, n_needles=0)
        g = torch.Generator(device="cuda").manual_seed(240715000 + n_ctx % 997)
        q = torch.randn(1, w.n_q_heads, 128, generator=g, device="cuda").half()
        n_rot = max(2, min(8, (1 << 30) // (w.n_kv_heads * n_ctx * 128 * 2)))       # keep the caches out of the 256 MB LLC
        ks = [torch.randn(w.n_kv_heads, n_ctx, 128, generator=g, device="cuda").half() for _ in range(n_rot)]
        vs = [torch.randn(w.n_kv_heads, n_ctx, 128, generator=g, device="cuda").half() for _ in range(n_rot)]
        row = {"n_ctx": n_ctx, "batch": batch}
        for name, vote in (("topk_4096", None), ("vote_4_127_32", B.Vote(4, 127, 32))):
            p = B.Params.from_workload(w.scaled(top_k=0) if vote else w)
            ws = None if vote else B.alloc_workspace(p)
            out = torch.empty(1, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
            if vote:
                vb = B.Vote(vote.vote_k, vote.n_centres, vote.span, n_seq=batch)    # votes pooled per sequence
                ws = B.alloc_vote_workspace(p, vb)
                sel = torch.empty(batch * B.vote_cap(p, vb), dtype=torch.int32, device="cuda")
                n_sel = torch.zeros(batch, dtype=torch.int32, device="cuda")

                def step(i):
                    B.vote_layer(p, vb, q, ks[i % n_rot], vs[i % n_rot], ws, sel=sel, n_sel=n_sel, out=out)
            else:
                def step(i):
                    B.decode_step(p, q, ks[i % n_rot], vs[i % n_rot], ws, out=out, want_idx=False)
            wake_device(ks[0])
            for i in range(2):
                step(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                step(i)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
            row[name] = {"ms_per_layer": round(ms, 4), "layer_steps_per_s": round(batch / (ms * 1e-3), 1)}
            if not vote:                                    # the same steps on a workspace declared warm (reattn_params.ws_warm),
                from dataclasses import replace             # in alternation with the plain ones, best of two loops each
                pw = replace(p, ws_warm=1)

                def loop(pp):
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for i in range(steps):
                        B.decode_step(pp, q, ks[i % n_rot], vs[i % n_rot], ws, out=out, want_idx=False)
                    torch.cuda.synchronize()
                    return (time.perf_counter() - t0) * 1e3 / steps

                warm, plain = float("inf"), float("inf")
                for _ in range(2):
                    warm = min(warm, loop(pw))
                    plain = min(plain, loop(p))
                row[name]["warm_workspace"] = {"ms_per_layer": round(warm, 4), "ms_per_layer_plain_same_moment": round(plain, 4)}
        rows.append(row)
        del ks, vs
        torch.cuda.empty_cache()
    return {"workload": "llama3-8b layer shape, fp16 storage, sink 4, local 4096", "pairs": rows}


def paged_leg(t: dict, cfg: int, steps: int, warmup: int, page_size: int = 256) -> dict:
    """The decode step over a paged cache: the same keys and values scattered page by page (a seeded random
    permutation) over pools [Hkv][P * page_size][D] behind a device page table."""
    import torch
    from dataclasses import replace
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    w = wl.CONFIGS[cfg]
    N, Hkv, D = w.n_ctx, w.n_kv_heads, w.head_dim
    n_pages = -(-N // page_size)
    table = torch.randperm(n_pages, generator=torch.Generator().manual_seed(240715000 + 10 * cfg + 9)).to(torch.int32)
    k_pool = torch.empty(Hkv, n_pages * page_size, D, dtype=t["k"].dtype, device="cuda")
    v_pool = torch.empty_like(k_pool)
    tc = table.cuda().long()
    pad = n_pages * page_size - N
    for src, dst in ((t["k"], k_pool), (t["v"], v_pool)):       # page i of the sequence -> page table[i] of the pool
        pages = torch.nn.functional.pad(src, (0, 0, 0, pad)).view(Hkv, n_pages, page_size, D)
        dst.view(Hkv, n_pages, page_size, D)[:, tc] = pages
        del pages
    p = replace(B.Params.from_workload(w), k_stride_head=n_pages * page_size * D, k_stride_tok=D,
                v_stride_head=n_pages * page_size * D, v_stride_tok=D, page_table=table.cuda(), page_size=page_size)
    ws = B.alloc_workspace(p)
    out = torch.empty(1, w.n_q_heads, D, dtype=torch.float32, device="cuda")
    idx = torch.empty(1, Hkv, w.k_eff, dtype=torch.int32, device="cuda")
    wake_device(k_pool)
    for _ in range(warmup):
        B.decode_step(p, t["q"], k_pool, v_pool, ws, idx_out=idx, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.decode_step(p, t["q"], k_pool, v_pool, ws, idx_out=idx, out=out)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    stage_sum = {s: 0.0 for s in B.STAGES}
    for _ in range(steps):
        _, _, st = B.decode_step_timed(p, t["q"], k_pool, v_pool, ws, idx_out=idx, out=out)
        for s in B.STAGES:
            stage_sum[s] += st[s]
    stages = {s: round(v / steps, 5) for s, v in stage_sum.items()}
    gbps = w.scan_bytes / (stages["scan"] * 1e-3) / 1e9
    # the paper's vote selection (k = 4, k' = 127, m = 32) over the same pools
    vote = B.Vote(4, 127, 32)
    pv = replace(p, top_k=0)
    wsv = B.alloc_vote_workspace(pv, vote)
    sel = torch.empty(B.vote_cap(pv, vote), dtype=torch.int32, device="cuda")
    n_sel = torch.zeros(1, dtype=torch.int32, device="cuda")
    wake_device(k_pool)
    for _ in range(warmup):
        B.vote_layer(pv, vote, t["q"], k_pool, v_pool, wsv, sel=sel, n_sel=n_sel, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.vote_layer(pv, vote, t["q"], k_pool, v_pool, wsv, sel=sel, n_sel=n_sel, out=out)
    torch.cuda.synchronize()
    vote_ms = (time.perf_counter() - t0) * 1e3 / steps
    vsum = {s: 0.0 for s in B.VOTE_STAGES}
    for _ in range(steps):
        *_, st = B.vote_layer_timed(pv, vote, t["q"], k_pool, v_pool, wsv, sel=sel, n_sel=n_sel, out=out)
        for s in B.VOTE_STAGES:
            vsum[s] += st[s]
    vstages = {s: round(v / steps, 5) for s, v in vsum.items()}
    del k_pool, v_pool
    return {"workload": w.name, "page_size": page_size, "n_pages": n_pages, "ms_per_step": round(ms, 5),
            "stages_ms": stages, "kv_scan_GBps": round(gbps, 1), "scan_frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "vote_4_127_32": {"ms_per_step": round(vote_ms, 5), "stages_ms": vstages}}


def paged_prefill_leg(steps: int, page_size: int = 256) -> dict:
    """Config 4's chunk (both selections) over a paged cache: the keys and values scattered page by page
    (a seeded random permutation) over pools [Hkv][P * page_size][D] behind a device page table."""
    import torch
    from dataclasses import replace
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    w = wl.CONFIGS[4]
    t = wl.generate(w, "cuda")
    N, Hkv, D = w.n_ctx, w.n_kv_heads, w.head_dim
    n_pages = -(-N // page_size)
    table = torch.randperm(n_pages, generator=torch.Generator().manual_seed(240715000 + 49)).to(torch.int32)
    tc = table.cuda().long()
    k_pool = torch.empty(Hkv, n_pages * page_size, D, dtype=t["k"].dtype, device="cuda")
    v_pool = torch.empty_like(k_pool)
    for src, dst in ((t["k"], k_pool), (t["v"], v_pool)):
        pages = torch.nn.functional.pad(src, (0, 0, 0, n_pages * page_size - N)).view(Hkv, n_pages, page_size, D)
        dst.view(Hkv, n_pages, page_size, D)[:, tc] = pages
        del pages
    del t["k"], t["v"]
    p = replace(B.Params.from_workload(w), k_stride_head=n_pages * page_size * D, k_stride_tok=D,
                v_stride_head=n_pages * page_size * D, v_stride_tok=D, page_table=table.cuda(), page_size=page_size)
    ws = B.alloc_workspace(p)
    acc = {s: 0.0 for s in B.PREFILL_STAGES}
    for i in range(steps + 1):
        _, _, ms = B.prefill_chunk_timed(p, t["q"], k_pool, v_pool, ws)
        if i:
            for s in acc:
                acc[s] += ms[s] / steps
    del ws
    vote = B.Vote(4, 127, 32)
    pv = replace(p, top_k=0)
    wsv = B.alloc_vote_workspace(pv, vote)
    vacc = {s: 0.0 for s in B.VOTE_STAGES}
    for i in range(steps + 1):
        *_, ms = B.vote_layer_timed(pv, vote, t["q"], k_pool, v_pool, wsv)
        if i:
            for s in vacc:
                vacc[s] += ms[s] / steps
    return {"workload": w.name, "page_size": page_size, "n_pages": n_pages,
            "topk_4096_per_query": {"ms_per_chunk": round(sum(acc.values()), 3), "stages_ms": {s: round(x, 4) for s, x in acc.items()}},
            "vote_4_127_32": {"ms_per_chunk": round(sum(vacc.values()), 3), "stages_ms": {s: round(x, 4) for s, x in vacc.items()}}}


def unfused_leg(t: dict, cfg: int, steps: int) -> dict:
    """The same decode step as four separate calls (Eq. 2 scores, Eq. 2 top-k, Eq. 3 concatenation with the
    rotary encoding materialised, Eq. 3 attention on the materialised buffers), each timed with events on the
    launch stream.  The gather writes fp32 rotated keys: D * (4 + b) bytes per slot against 2 * D * b read."""
    import torch
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    w = wl.CONFIGS[cfg]
    p = B.Params.from_workload(w)
    ws = B.alloc_workspace(p)
    eb = t["k"].element_size()
    scores = torch.empty(1, w.n_kv_heads, w.n_mid, dtype=torch.float32, device="cuda")
    idx = torch.empty(1, w.n_kv_heads, w.k_eff, dtype=torch.int32, device="cuda")
    k_sel = torch.empty(1, w.n_kv_heads, w.scope, w.head_dim, dtype=torch.float32, device="cuda")
    v_sel = torch.empty(1, w.n_kv_heads, w.scope, w.head_dim, dtype=t["v"].dtype, device="cuda")
    out = torch.empty(1, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    calls = {
        "score": lambda: B.score(p, t["q"], t["k"], scores=scores, ws=ws),
        "topk": lambda: B.topk(p, scores, ws, idx=idx),
        "gather_rope": lambda: B.gather_rope(p, t["k"], t["v"], idx, k_sel=k_sel, v_sel=v_sel),
        "attend": lambda: B.attend(p, t["q"], k_sel, v_sel, ws, out=out),
    }
    ms = {}
    wake_device(t["k"])
    for name, fn in calls.items():
        fn(); fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        ms[name] = a.elapsed_time(b) / steps
    rows = w.scope * w.n_kv_heads
    gather_read = 2 * rows * w.head_dim * eb + w.k_eff * w.n_kv_heads * 4
    gather_write = rows * w.head_dim * (4 + eb)
    gbps = (gather_read + gather_write) / (ms["gather_rope"] * 1e-3) / 1e9
    return {"workload": w.name, "steps": steps, "ms": {k: round(v, 5) for k, v in ms.items()},
            "ms_total": round(sum(ms.values()), 5),
            "score_GBps": round(w.scan_bytes / (ms["score"] * 1e-3) / 1e9, 1),
            "gather_rope": {"kernel": "gather_rope_kernel", "bound": "hbm", "read_bytes": gather_read,
                            "write_bytes": gather_write, "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
                            "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4)}}


def decode_token_leg(steps: int, n_layers: int = 32) -> dict:
    """One decode token through 32 layers (the layer loop of the appendix's decoding phase without the
    projections and feed-forward blocks): per layer, append the token's key / value rows, then the decode
    step.  Llama-3.1-8B shape, bf16; contexts chosen so that 32 caches fit beside each other."""
    import torch
    from dataclasses import replace
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    rows = []
    for n_ctx in (32768, 131072, 524288):
        w = wl.CONFIGS[2].scaled(n_ctx=n_ctx, n_needles=0, top_k=4096)
        cap = n_ctx + 64
        g = torch.Generator(device="cuda").manual_seed(240715000 + 77)
        kcs = [torch.randn(8, cap, 128, generator=g, device="cuda").bfloat16() for _ in range(n_layers)]
        vcs = [torch.randn(8, cap, 128, generator=g, device="cuda").bfloat16() for _ in range(n_layers)]
        qs = [torch.randn(1, 32, 128, generator=g, device="cuda").bfloat16() for _ in range(n_layers)]
        kn = [torch.randn(1, 8, 128, generator=g, device="cuda").bfloat16() for _ in range(n_layers)]
        vn = [torch.randn(1, 8, 128, generator=g, device="cuda").bfloat16() for _ in range(n_layers)]
        outs = [torch.empty(1, 32, 128, dtype=torch.float32, device="cuda") for _ in range(n_layers)]
        row = {"n_ctx": n_ctx, "n_layers": n_layers}
        for name, vote in (("topk_4096", None), ("vote_4_127_32", B.Vote(4, 127, 32))):
            p = B.Params.from_workload(w.scaled(top_k=0, max_position=0) if vote else w)
            p = replace(p, k_stride_head=cap * 128, k_stride_tok=128, v_stride_head=cap * 128, v_stride_tok=128)
            ws = B.alloc_vote_workspace(p, vote) if vote else B.alloc_workspace(p)
            wake_device(kcs[0])
            for _ in range(2):
                B.decode_token(p, qs, kn, vn, kcs, vcs, ws, outs=outs, vote=vote)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                B.decode_token(p, qs, kn, vn, kcs, vcs, ws, outs=outs, vote=vote)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
            # the same call captured once into a HIP graph and replayed (the library only enqueues kernels)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                B.decode_token(p, qs, kn, vn, kcs, vcs, ws, outs=outs, vote=vote)
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                graph.replay()
            torch.cuda.synchronize()
            gms = (time.perf_counter() - t0) * 1e3 / steps
            del graph
            row[name] = {"ms_per_token": round(ms, 3), "tokens_per_s": round(1e3 / ms, 1),
                         "kv_scan_GBps": round(n_layers * w.scan_bytes / (ms * 1e-3) / 1e9, 1),
                         "graph_replay_ms_per_token": round(gms, 3)}
        rows.append(row)
        del kcs, vcs
        torch.cuda.empty_cache()
    return {"workload": "llama3.1-8b shape, 32 layers' attention path per token, bf16, sink 4, local 4096", "contexts": rows}


def vote_leg(t: dict, cfg: int, steps: int, warmup: int) -> dict:
    """The same decode step with the paper's own selection (Method, last paragraph of the cache
    selection; Setup: every head votes for its top 4, the 127 most voted tokens with spans of
    32): fused score + per-head top-k scan on the matrix cores, vote merge, shared-set attention."""
    import torch
    from paper_2407_15176_amd import binding as B
    from paper_2407_15176_amd import workloads as wl
    w = wl.CONFIGS[cfg].scaled(top_k=0, max_position=0)    # the vote scope is 127 spans of 32, whatever the config's window
    v = B.Vote(4, 127, 32)
    p = B.Params.from_workload(w)
    ws = B.alloc_vote_workspace(p, v)
    out = torch.empty(1, w.n_q_heads, w.head_dim, dtype=torch.float32, device="cuda")
    sel = torch.empty(B.vote_cap(p, v), dtype=torch.int32, device="cuda")
    n_sel = torch.zeros(1, dtype=torch.int32, device="cuda")

    def step():
        B.vote_layer(p, v, t["q"], t["k"], t["v"], ws, sel=sel, n_sel=n_sel, out=out)

    wake_device(t["k"])
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    from dataclasses import replace
    pw = replace(p, ws_warm=1)                               # the same steps without the table launch

    def loop(pp):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            B.vote_layer(pp, v, t["q"], t["k"], t["v"], ws, sel=sel, n_sel=n_sel, out=out)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_warm, ms_cold_again = float("inf"), float("inf")     # in alternation, best of two loops each
    for _ in range(2):
        ms_warm = min(ms_warm, loop(pw))
        ms_cold_again = min(ms_cold_again, loop(p))
    acc = {s: 0.0 for s in B.VOTE_STAGES}
    for _ in range(steps):
        *_, ms = B.vote_layer_timed(p, v, t["q"], t["k"], t["v"], ws, sel=sel, n_sel=n_sel, out=out)
        for s in acc:
            acc[s] += ms[s] / steps
    scan_gbps = w.scan_bytes / (acc["head_topk_scan"] * 1e-3) / 1e9
    return {
        "workload": w.name, "vote_k": v.vote_k, "n_centres": v.n_centres, "span": v.span,
        "n_selected": int(n_sel.item()), "ms_per_step": round(ms_step, 5),
        "warm_workspace": {"ms_per_step": round(ms_warm, 5), "ms_per_step_plain_same_moment": round(ms_cold_again, 5)},
        "steps": steps,
        "stages_ms": {s: round(x, 5) for s, x in acc.items()},
        "roofline": {
            "kernel": "head_topk_mfma_kernel (+ list merge)", "bound": "hbm",
            "achieved": round(scan_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(scan_gbps / HBM_PEAK_GBPS, 4), "algorithmic_bytes": w.scan_bytes,
            "traffic": VOTE_SCAN_TRAFFIC_BYTES.get(wl.CONFIGS[cfg].name),
        },
    }


def cpu_baseline(w, t) -> dict:
    """The fp64 oracle, as it stands, on this machine's host cores: one whole step when that
    is about 10-30 s of CPU work, else the same step on a truncated cache (stated in `sample`)."""
    from oracle import reattn_oracle as ro
    from paper_2407_15176_amd import workloads as wl
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    n_ctx = w.n_ctx
    sample = "whole step, all cached tokens"
    budget_tokens = 2_000_000 * max(1, cores // 8)      # ~20 s of oracle scoring per 8 cores
    if n_ctx > budget_tokens:
        n_ctx = budget_tokens
        sample = f"same step on the first {n_ctx} cached tokens; time scaled by {w.n_ctx / n_ctx:.3f}"
    sh = ro.Shape(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, n_ctx, w.n_sink, w.n_local,
                  w.top_k, w.rope_theta)
    q = wl.to_numpy_store(t["q"])
    k = wl.to_numpy_store(t["k"][:, :n_ctx].contiguous())
    v = wl.to_numpy_store(t["v"][:, :n_ctx].contiguous())
    t0 = time.perf_counter()
    ro.forward(sh, q, k, v)
    secs = (time.perf_counter() - t0) * (w.n_ctx / n_ctx)
    return {"value": round(secs * 1e3, 2), "unit": "ms/layer", "cores": cores, "kind": "oracle",
            "sample": sample}


if __name__ == "__main__":
    sys.exit(main())
