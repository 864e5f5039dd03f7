#!/usr/bin/env python3
"""Benchmark of the PoD attention hot path on one MI355X.

Workload (benchmark configs[1]): LLaMA3-8B-shaped decode, one layer block of G=2 layers,
32 query / 8 KV heads, head_dim 128, batch 1, context 32768 (+1 per step), S=64, W=2048, bf16,
RoPE-rotated keys (base 500000).  A *step* is one pass of the whole path for one new token:
the block's lowest layer takes the token (cache update with window-to-distant demotion +
decode attention), then the upper layer does (shared distant logits).  Each layer's part is
one pod_decode_step launch.

The chip has a 256 MB last-level cache and one block's cache is only 206 MB, so the bench
keeps `--rotate` independent blocks (same shape, different data) and visits them round-robin:
each step streams K/V that left the cache long ago, as a 32-layer model would.

Prints ONE JSON line: whole-step throughput (`value`, algorithmic K/V bytes per second; median
of `--segments` independently captured HIP-graph segments of `--steps` steps each), the roofline
of the dominant kernel (the fused streaming kernel, timed launch by launch with HIP events
through pod_profile_*; lowest-layer launches, whose K/V is all cold, apart from upper-layer ones,
and a plain streaming read of the same size beside them), the CPU oracle timed on the host
cores, the prefill figures (configs[3]) and the large-batch decode configurations (configs[2], [4]).
"""
import argparse
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X datasheet
MFMA_BF16_PEAK_TFLOPS = 2500.0
T_START = time.perf_counter()


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--segments", type=int, default=5, help="independently captured graph segments of --steps steps (median and min reported)")
    ap.add_argument("--rotate", type=int, default=4, help="independent layer blocks visited round-robin")
    ap.add_argument("--context", type=int, default=32768)
    ap.add_argument("--profile-steps", type=int, default=32)
    ap.add_argument("--reuse-steps", type=int, default=64, help="steps timed through the score-reuse entry point (0 = skip)")
    ap.add_argument("--gate-rounds", type=int, default=8, help="rounds over the blocks in the gated-skip section (0 = skip)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of HIP graph replays")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-large", action="store_true", help="skip the large-batch configurations in the default line")
    ap.add_argument("--large-steps", type=int, default=6)
    ap.add_argument("--time-guard", type=float, default=240.0, help="seconds after which optional sections are skipped")
    ap.add_argument("--prefill-n", type=int, default=16384)
    ap.add_argument("--workload", choices=["cfg2", "cfg3", "cfg5"], default="cfg2",
                    help="cfg2 (default): the headline workload; cfg3 / cfg5: only that large-batch decode configuration "
                         "(32 layers, 30-44 GB of cache), one line of the same shape, decode figures only")
    ap.add_argument("--reuse", action="store_true", help="with --workload cfg3|cfg5: the step through the score-reuse entry point")
    ap.add_argument("--separate-calls", action="store_true", help="with --workload cfg3|cfg5: pod_cache_append + pod_decode_attention instead of pod_decode_step")
    ap.add_argument("--chunk", type=int, default=2048, help="chunk length of the chunked-prefill figure (0 = skip)")
    ap.add_argument("--select-keep", type=int, default=1984, help="distant tokens kept per kv head in the token-selection figure (0 = skip)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run plain copy kernels of 1 GiB (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def stats(ms_list):
    return {"median": round(statistics.median(ms_list), 5), "min": round(min(ms_list), 5), "max": round(max(ms_list), 5),
            "n": len(ms_list)}


def run_large(workload, K, Wm, variant):
    """configs[2] (16 ragged sequences of 4K-32K tokens, G=2) or configs[4] (4 sequences of 128K, G=4, 1 % of the
    distant key rows x8): a step = one new token per sequence through all 32 layers.  variant: "step" (one
    pod_decode_step launch per layer), "separate" (pod_cache_append + pod_decode_attention), "reuse" (append +
    pod_decode_attention_reuse)."""
    import torch

    import paper_2412_02252_amd as pod
    from pod_inputs import gen

    dev = "cuda:0"
    Hq, Hkv, d, L = 32, 8, 128, 32
    if workload == "cfg3":
        G, B, S, W, seed = 2, 16, 64, 2048, 20241202 + 3
        lens = gen.ragged_lengths(seed, B, 4096, 32768)
        kgen = {}
        name = "configs[2]: 32 layers G=2, 32q/8kv heads, d=128, 16 sequences of 4096..32768 tokens (seeded), S=64, W=2048"
    else:
        G, B, S, W, seed = 4, 4, 128, 4096, 20241202 + 5
        lens = [131072] * B
        kgen = dict(outlier_rate=0.01, outlier_scale=8.0, outlier_lo=S, outlier_hi=lens[0] - W)
        name = "configs[4]: 32 layers G=4, 32q/8kv heads, d=128, 4 sequences of 131072 tokens, S=128, W=4096, 1 % of distant key rows x8"
    total = K + Wm
    max_ctx = max(lens) + total + 1
    cache = pod.PodCache(pod.make_config(L, G, Hq, Hkv, d, S, W, B, max_ctx), dev)
    scale = 1.0 / math.sqrt(d)
    row = Hkv * d * 2
    for layer in range(L):
        for b in range(B):
            k = gen.keys_bf16(seed, layer, b, lens[b], Hkv, d, device=dev, **kgen)
            v = gen.values_bf16(seed, layer, b, lens[b], Hkv, d, device=dev)
            cache.pod_cache_fill(layer, b, k, v)
            del k, v
    kn = [torch.stack([gen.keys_bf16(seed, l, b, 1, Hkv, d, device=dev, pos0=lens[b] + s)[0] for b in range(B)]) for s in range(total) for l in range(L)]
    vn = [torch.stack([gen.values_bf16(seed, l, b, 1, Hkv, d, device=dev, pos0=lens[b] + s)[0] for b in range(B)]) for s in range(total) for l in range(L)]
    q = [torch.stack([gen.queries_bf16(seed, l, b, 1, Hq, d, device=dev, pos0=lens[b])[0] for b in range(B)]) for l in range(L)]
    out = torch.empty_like(q[0])
    pos = [torch.tensor([n + s for n in lens], dtype=torch.int32, device=dev) for s in range(total)]
    ctx = [torch.tensor([n + s + 1 for n in lens], dtype=torch.int32, device=dev) for s in range(total)]
    scores = cache.new_score_buffer() if variant == "reuse" else None

    def run_step(s):
        bound = max(lens) + s + 1
        for l in range(L):
            if variant == "step":
                cache.pod_decode_step(l, kn[s * L + l], vn[s * L + l], q[l], q[l - l % G] if l % G else None, pos[s], scale,
                                      out=out, max_context_len=bound)
                continue
            if variant == "reuse":  # upper layers of a block take the lowest layer's distant logits instead of its keys
                cache.pod_decode_step_reuse(l, kn[s * L + l], vn[s * L + l], q[l], pos[s], scale, scores, out=out, max_context_len=bound)
                continue
            cache.pod_cache_append(l, kn[s * L + l], vn[s * L + l], pos[s])
            cache.pod_decode_attention(l, q[l], q[l - l % G] if l % G else None, ctx[s], scale, out=out, max_context_len=bound)

    for s in range(Wm):
        run_step(s)
    cache.pod_cache_check()
    cache.pod_profile_enable(K * L)
    per_step = []
    for s in range(Wm, total):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_step(s)
        torch.cuda.synchronize()
        per_step.append((time.perf_counter() - t0) * 1e3)
    each = cache.pod_profile_read_each(K * L)
    cache.pod_profile_disable()
    cache.pod_cache_check()
    dt = sum(per_step) / 1e3
    nbytes = sum(sum(2 * (n + s + 1) * row for n in lens) * L for s in range(Wm, total))
    res = {"workload": name + "; step = one new token per sequence through 32 layers, " +
                       {"step": "one pod_decode_step launch per layer", "separate": "pod_cache_append + pod_decode_attention per layer",
                        "reuse": "one pod_decode_step_reuse launch per layer"}[variant],
           "launch": "eager", "steps": K, "warmup": Wm, "ms_per_step": stats(per_step), "bytes_per_step": nbytes // K}
    if variant == "reuse":
        # its own, smaller byte count: an upper layer reads V rows, proximal K rows and 4 B per (query head, distant
        # token); a lowest layer reads K and V rows and writes those 4 B
        def layer_bytes(n, upper):
            n_prox = min(n, S + W)
            logits = (n - n_prox) * Hq * 4
            return (n * row + n_prox * row + logits) if upper else (2 * n * row + logits)
        reuse_bytes = sum(sum(layer_bytes(n + s + 1, l % G != 0) for n in lens) for l in range(L) for s in range(Wm, total))
        res.update({"bytes_per_step_reuse": reuse_bytes // K, "GBs_of_its_own_bytes": round(reuse_bytes / dt / 1e9, 1),
                    "plain_equivalent_GBs": round(nbytes / dt / 1e9, 1)})
    else:
        per_launch = nbytes / (K * L)
        kus = statistics.median(each) * 1e3 if each else float("nan")
        # a plain read of as many bytes per launch out of the cache's own buffer, a different part every time (the
        # buffer is tens of GB: nothing of it is left in any cache): what a launch of this size can be held to
        part = int(per_launch) // 256 * 256
        span = cache.buf.numel() - part - 4096
        ceil = None
        if variant == "step" and span > 8 * part:
            NCEIL = 12
            cache.pod_profile_enable(NCEIL)
            for i in range(NCEIL):
                pod.pod_profile_stream_read(cache.buf[(i * (span // NCEIL)) // 256 * 256:], part, cache)
            torch.cuda.synchronize()
            cus = [t * 1e3 for t in cache.pod_profile_read_each(NCEIL)][2:]
            cache.pod_profile_disable()
            cmed = statistics.median(cus)
            ceil = {"what": "plain read-only kernel (non-temporal loads) over the same number of bytes of the cache buffer, a different part each launch, same event timing",
                    "us": stats(cus), "GBs": round(part / (cmed * 1e-6) / 1e9, 1), "frac_of_peak": round(part / (cmed * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                    "kernel_vs_ceiling": round(cmed / kus * per_launch / part, 4)}
        res.update({"GBs": round(nbytes / dt / 1e9, 1), "frac_of_hbm_peak": round(nbytes / dt / 1e9 / HBM_PEAK_GBS, 4),
                    "kernel": {"name": ("decode_even_kernel<128, true, 0> (step; one round of workgroups, the batch's rows split evenly over them; decode_combine_kernel merges)"
                                        if variant == "step" else "decode_even_kernel<128, false, 0>"),
                               "bytes_per_launch": int(per_launch), "median_us": round(kus, 3),
                               "GBs": round(per_launch / (kus * 1e-6) / 1e9, 1),
                               "frac_of_hbm_peak": round(per_launch / (kus * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "launches": len(each)}})
        if ceil:
            res["kernel"]["streaming_ceiling"] = ceil
    del cache, kn, vn, q, out, scores
    torch.cuda.empty_cache()
    return res


def main_large(a):
    import torch
    torch.cuda.set_device(0)
    variant = "reuse" if a.reuse else ("separate" if a.separate_calls else "step")
    r = run_large(a.workload, a.steps, a.warmup, variant)
    ms = r["ms_per_step"]["median"]
    line = {"metric": "decode attn HBM GB/s", "value": r.get("GBs", r.get("GBs_of_its_own_bytes")), "unit": "GB/s", "n_gpus": 1,
            "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": r["workload"], "launch": "eager", "bytes_per_step": r["bytes_per_step"]}, "detail": r}
    if "kernel" in r:
        k = r["kernel"]
        line["roofline"] = {"bound": "hbm", "kernel": k["name"], "achieved": k["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": k["frac_of_hbm_peak"], "traffic": None, "bytes_per_launch": k["bytes_per_launch"],
                            "avg_kernel_us": k["median_us"], "launches": k["launches"]}
    print(json.dumps(line))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (nothing here shards across GPUs)", file=sys.stderr)
        sys.exit(2)
    if a.workload != "cfg2":
        return main_large(a)
    import numpy as np
    import torch

    import paper_2412_02252_amd as pod
    from pod_inputs import gen

    dev = "cuda:0"
    torch.cuda.set_device(0)
    G, Hq, Hkv, d, S, W = 2, 32, 8, 128, 64, 2048
    R, n0, K, Wm, P, NSEG = a.rotate, a.context, a.steps, a.warmup, a.profile_steps, max(1, a.segments)
    RU = a.reuse_steps
    GR = K          # replays of the token-reusable step graph (each replay = R steps)
    seed = 20241202 + 2
    TL = 8           # eager steps whose lowest-layer launch leaves per-workgroup device clocks
    total_steps = Wm + NSEG * K + K + P + TL + RU
    per_block = (total_steps + R - 1) // R + GR + 2
    max_ctx = n0 + per_block + 1
    L = G * R
    cfg = pod.make_config(L, G, Hq, Hkv, d, S, W, 1, max_ctx)
    cache = pod.PodCache(cfg, dev)
    scale = 1.0 / math.sqrt(d)
    row = Hkv * d * 2
    rope = dict(rope_base=500000.0, rope_max_pos=max_ctx)

    # ---- fill every block to n0 tokens
    for layer in range(L):
        k = gen.keys_bf16(seed, layer, 0, n0, Hkv, d, device=dev, **rope)
        v = gen.values_bf16(seed, layer, 0, n0, Hkv, d, device=dev)
        cache.pod_cache_fill(layer, 0, k, v)
        del k, v
    # ---- per-step inputs, generated up front
    steps = []
    for s in range(total_steps):
        g, p = s % R, n0 + s // R
        ent = dict(layers=(G * g, G * g + 1), n=p + 1,
                   pos=torch.tensor([p], dtype=torch.int32, device=dev),
                   ctx=torch.tensor([p + 1], dtype=torch.int32, device=dev))
        for j, layer in enumerate(ent["layers"]):
            ent[f"k{j}"] = gen.keys_bf16(seed, layer, 0, 1, Hkv, d, device=dev, pos0=p, **rope)
            ent[f"v{j}"] = gen.values_bf16(seed, layer, 0, 1, Hkv, d, device=dev, pos0=p)
            ent[f"q{j}"] = gen.queries_bf16(seed, layer, 0, 1, Hq, d, device=dev, pos0=p)
            ent[f"o{j}"] = torch.empty((1, Hq, d), dtype=torch.bfloat16, device=dev)
        steps.append(ent)

    def run_step(e):                    # the hot path: one launch per layer
        l0, l1 = e["layers"]
        cache.pod_decode_step(l0, e["k0"], e["v0"], e["q0"], None, e["pos"], scale, out=e["o0"], max_context_len=e["n"])
        cache.pod_decode_step(l1, e["k1"], e["v1"], e["q1"], e["q0"], e["pos"], scale, out=e["o1"], max_context_len=e["n"])

    def run_step_separate(e):           # the same step through the separate calls (two launches per layer)
        l0, l1 = e["layers"]
        cache.pod_cache_append(l0, e["k0"], e["v0"], e["pos"])
        cache.pod_cache_append(l1, e["k1"], e["v1"], e["pos"])
        cache.pod_decode_attention(l0, e["q0"], None, e["ctx"], scale, out=e["o0"], max_context_len=e["n"])
        cache.pod_decode_attention(l1, e["q1"], e["q0"], e["ctx"], scale, out=e["o1"], max_context_len=e["n"])

    def step_bytes(e):
        return 2 * (2 * e["n"] * row)   # two layers, K and V rows of every token once

    scores = cache.new_score_buffer()

    def run_step_reuse_fused(e):        # same step; the upper layer reads the lowest layer's distant logits; one launch per layer
        l0, l1 = e["layers"]
        cache.pod_decode_step_reuse(l0, e["k0"], e["v0"], e["q0"], e["pos"], scale, scores, out=e["o0"], max_context_len=e["n"])
        cache.pod_decode_step_reuse(l1, e["k1"], e["v1"], e["q1"], e["pos"], scale, scores, out=e["o1"], max_context_len=e["n"])

    def run_step_reuse(e):              # ... and through the separate calls
        l0, l1 = e["layers"]
        cache.pod_cache_append(l0, e["k0"], e["v0"], e["pos"])
        cache.pod_cache_append(l1, e["k1"], e["v1"], e["pos"])
        cache.pod_decode_attention_reuse(l0, e["q0"], e["ctx"], scale, scores, out=e["o0"], max_context_len=e["n"])
        cache.pod_decode_attention_reuse(l1, e["q1"], e["ctx"], scale, scores, out=e["o1"], max_context_len=e["n"])

    def step_bytes_reuse(e):            # upper layer: V rows, proximal K rows, 4 B per (query head, distant token)
        n = e["n"]
        n_prox = min(n, S + W)
        return 2 * n * row + (n * row + n_prox * row + (n - n_prox) * Hq * 4) + (n - n_prox) * Hq * 4

    def time_segments(fn, segs):
        """Each segment (a list of consecutive steps) is captured into its own HIP graph, then the graphs are
        replayed in order, each bracketed by a device synchronisation.  Returns seconds per segment."""
        graphs = []
        if not a.no_graph:
            for seg in segs:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for e in seg:
                        fn(e)
                graphs.append(g)
        out = []
        for i, seg in enumerate(segs):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if graphs:
                graphs[i].replay()
            else:
                for e in seg:
                    fn(e)
            torch.cuda.synchronize()
            out.append(time.perf_counter() - t0)
        return out

    if a.pmc_calibration:   # a plain copy kernel of known size: reads 1 GiB, writes 1 GiB per launch
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up
    for e in steps[:Wm]:
        run_step(e)
    torch.cuda.synchronize()
    cache.pod_cache_check()

    # ---- timed region: NSEG segments of exactly K steps each; the headline is the median segment
    mode = "eager" if a.no_graph else "hipgraph"
    segs = [steps[Wm + i * K:Wm + (i + 1) * K] for i in range(NSEG)]
    seg_s = time_segments(run_step, segs)
    cache.pod_cache_check()
    seg_ms_per_step = [t / K * 1e3 for t in seg_s]
    med = statistics.median(seg_s)
    nbytes = sum(step_bytes(e) for e in segs[seg_s.index(med) if med in seg_s else 0])
    value = nbytes / med / 1e9
    cursor = Wm + NSEG * K

    # ---- the same step through the separate calls (append, append, attention, attention), one segment
    sep = steps[cursor:cursor + K]
    cursor += K
    sep_s = time_segments(run_step_separate, [sep])[0]
    cache.pod_cache_check()

    # ---- dominant kernel (the fused streaming kernel of pod_decode_step) with HIP events, eager launches
    prof = steps[cursor:cursor + P]
    cursor += P
    cache.pod_profile_enable(2 * len(prof) + 4)
    for e in prof:
        run_step(e)
    torch.cuda.synchronize()
    each = cache.pod_profile_read_each(2 * len(prof) + 4)
    cache.pod_profile_disable()
    cache.pod_cache_check()
    low_us = [t * 1e3 for t in each[0::2]]      # lowest-layer launches: every K/V byte comes from HBM
    up_us = [t * 1e3 for t in each[1::2]]       # upper-layer launches: the block's distant keys were read a launch earlier
    bytes_per_launch = sum(step_bytes(e) for e in prof) / max(len(each), 1)
    cold_us = statistics.median(low_us)
    achieved = bytes_per_launch / (cold_us * 1e-6) / 1e9
    # where a cold launch's time goes: per-workgroup device clocks (100 MHz) of TL lowest-layer launches
    import numpy as np
    tl = steps[cursor:cursor + TL]
    cursor += TL
    trace = torch.zeros(8 * 4096, dtype=torch.int64, device=dev)
    phases = {"tile_loops_end": [], "partials_stored": [], "arrivals_counted": [], "end": []}
    for e in tl:
        l0, l1 = e["layers"]
        trace.zero_()
        cache.pod_profile_set_trace(trace)
        cache.pod_decode_step(l0, e["k0"], e["v0"], e["q0"], None, e["pos"], scale, out=e["o0"], max_context_len=e["n"])
        torch.cuda.synchronize()
        cache.pod_profile_set_trace(None)
        cache.pod_decode_step(l1, e["k1"], e["v1"], e["q1"], e["q0"], e["pos"], scale, out=e["o1"], max_context_len=e["n"])
        t = trace.cpu().numpy().reshape(-1, 8)
        t = t[t[:, 2] > 0]
        if len(t):
            t0 = t[:, 2].min()
            for name, col in (("tile_loops_end", 3), ("partials_stored", 4), ("arrivals_counted", 5), ("end", 6)):
                phases[name].append(float((t[:, col].max() - t0) / 100.0))
    torch.cuda.synchronize()
    cache.pod_cache_check()
    del trace
    timeline = None
    if phases["end"]:
        tm = {k: round(statistics.median(v), 2) for k, v in phases.items()}
        timeline = {"what": "device clocks of every workgroup of a cold lowest-layer launch, us after the first workgroup's "
                            f"start, last workgroup to reach each point, median of {len(phases['end'])} launches",
                    **tm,
                    "streaming_phase_GBs": round(bytes_per_launch / (tm["tile_loops_end"] * 1e-6) / 1e9, 1),
                    "streaming_phase_frac_of_peak": round(bytes_per_launch / (tm["tile_loops_end"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                    "hand_over_us": round(tm["end"] - tm["tile_loops_end"], 2)}
    # a plain streaming read of the same number of bytes from memory that left the caches long ago
    sweep = torch.empty(8 * int(bytes_per_launch) // 16 * 16 + 4096, dtype=torch.uint8, device=dev).fill_(1)
    part = int(bytes_per_launch) // 256 * 256
    cache.pod_profile_enable(48)
    for i in range(40):
        pod.pod_profile_stream_read(sweep[(i % 8) * part:], part, cache)
    torch.cuda.synchronize()
    ceil_us = [t * 1e3 for t in cache.pod_profile_read_each(48)][8:]
    cache.pod_profile_disable()
    del sweep
    ceil_med = statistics.median(ceil_us)

    out = {
        "metric": "decode attn HBM GB/s @32K ctx",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(med / K * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: LLaMA3-8B-shaped PoD decode, one layer block G=2, 32q/8kv heads, d=128, "
                               f"batch 1, context {n0}+step, S=64, W=2048, RoPE keys; step = pod_decode_step (cache update + "
                               "attention in one launch) on the lowest layer, then on the upper layer",
                   "rotating_blocks": R, "launch": mode, "launch_info": cache.pod_cache_launch_info(), "bytes_per_step": step_bytes(segs[0][0]),
                   "segments": NSEG, "ms_per_step_segments": stats(seg_ms_per_step),
                   "frac_of_hbm_peak_whole_step": round(value / HBM_PEAK_GBS, 4)},
        "roofline": {"bound": "hbm", "kernel": "decode_partial_kernel<128, 0, 2, true, 8> (streams K/V, updates the cache, merges the partials)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": None,
                     "traffic_note": "counters need a rocprofv3 run: profiles/decode_step_kernel_cfg2_pmc.txt holds "
                                     "FETCH_SIZE + WRITE_SIZE of this kernel on this workload, 135.89 MB per launch = 1.011 x algorithmic",
                     "bytes_per_launch": int(bytes_per_launch),
                     "avg_kernel_us": round(cold_us, 3), "launches": len(each),
                     "timed": "HIP event pair per launch (reads 1-2 us more than the kernel's own begin-to-end time); "
                              "achieved/frac are the lowest-layer launches, whose bytes all come from HBM",
                     "lowest_layer_launch_us": stats(low_us), "upper_layer_launch_us": stats(up_us),
                     "upper_layer_frac": round(bytes_per_launch / (statistics.median(up_us) * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                     "timeline": timeline,
                     "streaming_ceiling": {"what": "plain read-only kernel (non-temporal loads) over the same number of cold bytes, same event timing",
                                           "us": stats(ceil_us), "GBs": round(part / (ceil_med * 1e-6) / 1e9, 1),
                                           "frac_of_peak": round(part / (ceil_med * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                           "kernel_vs_ceiling": round(ceil_med / cold_us * bytes_per_launch / part, 4)}},
        "separate_calls": {"what": "the same step as pod_cache_append x2 + pod_decode_attention x2 (4 launches)",
                           "ms_per_step": round(sep_s / K * 1e3, 5), "step_speedup_from_fusing": round((sep_s / K) / (med / K), 3)},
    }

    # ---- the same steps through the score-reuse entry point
    if RU > 0:
        ru = steps[cursor:cursor + RU]
        cursor += RU
        half = max(1, len(ru) // 2)
        ru_f, ru_s = ru[:half], ru[half:]
        el = time_segments(run_step_reuse_fused, [ru_f])[0]
        cache.pod_cache_check()
        el_s = time_segments(run_step_reuse, [ru_s])[0] if ru_s else float("nan")
        cache.pod_cache_check()
        rb = sum(step_bytes_reuse(e) for e in ru_f)
        out["score_reuse"] = {"what": "the same step through pod_decode_step_reuse (one launch per layer; the upper layer reads the "
                                      "lowest layer's distant logits instead of its keys)",
                              "steps": len(ru_f), "ms_per_step": round(el / len(ru_f) * 1e3, 5),
                              "bytes_per_step": step_bytes_reuse(ru_f[0]),
                              "value": round(rb / el / 1e9, 1), "unit": "GB/s (of its own, smaller byte count)",
                              "speedup_vs_plain_step": round((med / K) / (el / len(ru_f)), 3),
                              "ms_per_step_as_separate_calls": round(el_s / max(len(ru_s), 1) * 1e3, 5)}

    # ---- one step graph replayed for successive tokens (lengths taken from device arrays only): every replay is one
    # step on each of the R blocks; the graph advances its own position arrays
    if not a.no_graph and GR > 0:
        lens0 = [cache.pod_cache_seq_len(G * g, 0) for g in range(R)]
        cache.pod_cache_set_length_source(1)
        gpos = [torch.tensor([lens0[g]], dtype=torch.int32, device=dev) for g in range(R)]
        fixed = [dict(steps[g]) for g in range(R)]      # any token's k, v, q: the values do not change the time
        for e in fixed:
            e["o0"], e["o1"] = torch.empty_like(e["o0"]), torch.empty_like(e["o1"])
        bound = max(lens0) + GR + 1
        gg = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gg):
            for g in range(R):
                e = fixed[g]
                cache.pod_decode_step(G * g, e["k0"], e["v0"], e["q0"], None, gpos[g], scale, out=e["o0"], max_context_len=bound)
                cache.pod_decode_step(G * g + 1, e["k1"], e["v1"], e["q1"], e["q0"], gpos[g], scale, out=e["o1"], max_context_len=bound)
                gpos[g].add_(1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(GR):
            gg.replay()
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        cache.pod_cache_check()
        cache.pod_cache_sync_lengths()
        cache.pod_cache_set_length_source(0)
        ok = all(cache.pod_cache_seq_len(G * g + j, 0) == lens0[g] + GR for g in range(R) for j in range(G))
        out["reusable_step_graph"] = {"what": f"one captured graph = one step on each of the {R} blocks, replayed {GR} times for successive "
                                              "tokens; lengths from device arrays, launch sized for the last token",
                                      "ms_per_step": round(el / (GR * R) * 1e3, 5), "lengths_advanced_as_expected": ok}

    # ---- gated skip of distant tokens: decode calls only (no appends), the
    # R blocks round-robin, at the contexts the steps above left behind.  Three timings of the same
    # (lowest layer, upper layer) pair: plain; gated with the generated inputs (no head's gate reaches
    # tau = 0.7, so this is the cost of the two-launch structure); gated after the upper layers'
    # sink and recent keys were scaled x4 (every head's gate reaches 0.7: distant rows are not read).
    if a.gate_rounds > 0:
        tau = 0.7
        lens = [cache.pod_cache_seq_len(G * g, 0) for g in range(R)]
        qs = [[gen.queries_bf16(seed, G * g + j, 0, 1, Hq, d, device=dev, pos0=lens[g] - 1) for j in range(G)] for g in range(R)]
        ctxs = [torch.tensor([lens[g]], dtype=torch.int32, device=dev) for g in range(R)]
        og = torch.empty((1, Hq, d), dtype=torch.bfloat16, device=dev)

        def pair_plain(g):
            cache.pod_decode_attention(G * g, qs[g][0], None, ctxs[g], scale, out=og, max_context_len=lens[g])
            cache.pod_decode_attention(G * g + 1, qs[g][1], qs[g][0], ctxs[g], scale, out=og, max_context_len=lens[g])

        def pair_gated(g):
            cache.pod_decode_attention_gated(G * g, qs[g][0], ctxs[g], scale, tau, scores, out=og, max_context_len=lens[g])
            cache.pod_decode_attention_gated(G * g + 1, qs[g][1], ctxs[g], scale, tau, scores, out=og, max_context_len=lens[g])

        def time_pairs(fn):
            skipped = 0
            for g in range(R):
                fn(g)
            torch.cuda.synchronize()
            gg = None
            if not a.no_graph:
                gg = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gg):
                    for _ in range(a.gate_rounds):
                        for g in range(R):
                            fn(g)
                torch.cuda.synchronize()
            t0 = time.perf_counter()
            if gg is not None:
                gg.replay()
            else:
                for _ in range(a.gate_rounds):
                    for g in range(R):
                        fn(g)
            torch.cuda.synchronize()
            el = (time.perf_counter() - t0) / (a.gate_rounds * R)
            if fn is pair_gated:
                skipped = int(cache.skip_flags(scores)[0].sum().item())
            return el, skipped

        t_plain, _ = time_pairs(pair_plain)
        t_none, sk_none = time_pairs(pair_gated)
        for g in range(R):   # upper layers again, proximal keys x4 (exact in bf16)
            layer = G * g + 1
            n = lens[g]
            k = gen.keys_bf16(seed, layer, 0, n, Hkv, d, device=dev, **rope)
            v = gen.values_bf16(seed, layer, 0, n, Hkv, d, device=dev)
            k[:S] *= 4
            k[n - W:] *= 4
            kl = gen.keys_bf16(seed, G * g, 0, n, Hkv, d, device=dev, **rope)
            vl = gen.values_bf16(seed, G * g, 0, n, Hkv, d, device=dev)
            if g == 0:
                cache.pod_cache_reset()
            cache_fill_pairs = ((G * g, kl, vl), (layer, k, v))
            for (ll, kk, vv) in cache_fill_pairs:
                cache.pod_cache_fill(ll, 0, kk, vv)
            del k, v, kl, vl
        t_all, sk_all = time_pairs(pair_gated)
        cache.pod_cache_check()
        out["tau_gating"] = {"tau": tau, "launch": mode, "unit": "ms per (lowest, upper) decode pair",
                             "plain": round(t_plain * 1e3, 5),
                             "gated_nothing_skips": {"ms": round(t_none * 1e3, 5), "heads_skipped": sk_none, "of": Hq},
                             "gated_all_heads_skip": {"ms": round(t_all * 1e3, 5), "heads_skipped": sk_all, "of": Hq},
                             "speedup_when_all_skip": round(t_plain / t_all, 3)}

    # ---- CPU oracle on the host cores, a bounded sample of the same steps (block 0's)
    if not a.no_cpu:
        from oracle import pod_oracle as po
        oc = po.Cache(G, G, Hkv, d, S, W, 1, max_ctx)
        for layer in range(G):
            k = gen.keys_bf16(seed, layer, 0, n0, Hkv, d, device=dev, **rope)
            v = gen.values_bf16(seed, layer, 0, n0, Hkv, d, device=dev)
            oc.fill(layer, 0, gen.bf16_bits(k), gen.bf16_bits(v))
            del k, v
        mine = [e for i, e in enumerate(steps) if i % R == 0]
        host = [{key: gen.bf16_bits(e[key]) for key in ("k0", "v0", "q0", "k1", "v1", "q1")} for e in mine]
        cpu_t, cpu_bytes, done, worst = 0.0, 0, 0, 0.0
        for e, h in zip(mine, host):
            p = e["n"] - 1
            c0 = time.perf_counter()
            oc.append(0, h["k0"], h["v0"], [p])
            oc.append(1, h["k1"], h["v1"], [p])
            r0 = oc.decode_attention(0, h["q0"], None, [p + 1], scale)
            r1 = oc.decode_attention(1, h["q1"], h["q0"], [p + 1], scale)
            cpu_t += time.perf_counter() - c0
            cpu_bytes += step_bytes(e)
            done += 1
            for r, o in ((r0, e["o0"]), (r1, e["o1"])):
                worst = max(worst, float(np.abs(o.float().cpu().numpy() - r).max()))
            if cpu_t > a.cpu_seconds:
                break
        out["cpu_baseline"] = {"value": round(cpu_bytes / cpu_t / 1e9, 3), "unit": "GB/s", "cores": po.num_threads(),
                               "kind": "oracle", "sample": f"{done} of the same decode steps (one block, both layers)",
                               "ms_per_step": round(cpu_t / done * 1e3, 2), "gpu_vs_oracle_max_abs_err": worst}

    del cache, steps, scores
    torch.cuda.empty_cache()

    # ---- prefill (configs[3]): one block, n tokens, causal, attention + cache construction
    if not a.no_prefill:
        n = a.prefill_n
        pcfg = pod.make_config(G, G, Hq, Hkv, d, S, W, 1, n)
        pc = pod.PodCache(pcfg, dev)
        pseed = 20241202 + 4
        q = [gen.queries_bf16(pseed, l, 0, n, Hq, d, device=dev) for l in range(G)]
        k = [gen.keys_bf16(pseed, l, 0, n, Hkv, d, device=dev) for l in range(G)]
        v = [gen.values_bf16(pseed, l, 0, n, Hkv, d, device=dev) for l in range(G)]
        o = torch.empty_like(q[0])
        flops = 4.0 * d * Hq * n * (n + 1) / 2
        res = {}
        for layer, name in ((0, "lowest_layer"), (1, "upper_layer")):
            times = []
            for it in range(8):
                pc.pod_cache_reset(-1)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                pc.pod_prefill_attention(layer, 0, q[layer], k[layer], v[layer], q[0] if layer else None,
                                         k[0] if layer else None, scale, out=o, write_cache=True)
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            t = statistics.median(times[1:]) / 1e3
            res[name] = {"ms": round(t * 1e3, 4), "ms_min": round(min(times[1:]), 4), "tflops": round(flops / t / 1e12, 2),
                         "frac_of_bf16_mfma_peak": round(flops / t / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
        # the same prompt in chunks (every layer takes a chunk, stores it, then the next chunk)
        if a.chunk > 0:
            ws = torch.empty(pod.pod_prefill_chunk_in_place_bytes(pcfg, n, a.chunk), dtype=torch.uint8, device=dev)
            cuts = list(range(0, n, a.chunk)) + [n]
            # one pass with an event after every chunk (first / last chunk figures), then whole passes between two events
            per, whole = None, []
            for it in range(6):
                pc.pod_cache_reset(-1)
                ev = [torch.cuda.Event(enable_timing=True) for _ in cuts]
                ev[0].record()
                for ci, (c0, c1) in enumerate(zip(cuts[:-1], cuts[1:])):
                    for layer in range(G):
                        pc.pod_prefill_attention_chunk(layer, 0, q[layer][c0:c1], k[layer][c0:c1], v[layer][c0:c1],
                                                       q[0][c0:c1] if layer else None, k[0][c0:c1] if layer else None,
                                                       scale, ws, out=o[c0:c1], write_cache=True)
                    if it == 0 or ci + 2 == len(cuts):
                        ev[ci + 1].record()
                torch.cuda.synchronize()
                if it == 0:
                    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(len(cuts) - 1)]
                else:
                    whole.append(ev[0].elapsed_time(ev[-1]))
            tot = statistics.median(whole) / 1e3
            res["chunked"] = {"chunk": a.chunk, "chunks": len(per), "workspace_bytes": ws.numel(),
                              "ms_both_layers": round(tot * 1e3, 4),
                              "ms_both_layers_min": round(min(whole), 4),
                              "ms_first_chunk": round(per[0], 4), "ms_last_chunk": round(per[-1], 4),
                              "tflops": round(G * flops / tot / 1e12, 2),
                              "vs_one_call": round((res["lowest_layer"]["ms"] + res["upper_layer"]["ms"]) / (tot * 1e3), 3)}
            del ws
        # token selection on the distant store of the same prompt: votes of the last 64 queries at the block's lowest layer,
        # pooled top-k, compaction of both layers down to 4096 stored tokens, then decode steps on the shorter sequence
        if a.select_keep > 0 and n - S - W > a.select_keep:
            obs, keep = 64, a.select_keep
            sws = torch.empty(pod.pod_select_workspace_bytes(pcfg, n, obs, keep), dtype=torch.uint8, device=dev)
            sel = torch.zeros((G, Hkv, keep), dtype=torch.int32, device=dev)
            votes = torch.zeros((Hkv, n - S - W), dtype=torch.float32, device=dev)
            q_obs = q[0][n - obs:].contiguous()
            tv, tt, tc = [], [], []
            for it in range(5):
                pc.pod_cache_reset(-1)
                for layer in range(G):
                    pc.pod_cache_fill(layer, 0, k[layer], v[layer])
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                ev[0].record()
                pc.pod_select_votes(0, q_obs, k[0], scale, sws, votes=votes)
                ev[1].record()
                pc.pod_select_top(0, n, votes, 7, pod.POOL_MAX, keep, sel, sws)
                ev[2].record()
                for layer in range(G):
                    pc.pod_cache_compact(layer, 0, sel, sws)
                ev[3].record()
                torch.cuda.synchronize()
                tv.append(ev[0].elapsed_time(ev[1])); tt.append(ev[1].elapsed_time(ev[2])); tc.append(ev[2].elapsed_time(ev[3]))
            m = S + keep + W
            kn = [gen.keys_bf16(pseed, l, 0, 1, Hkv, d, device=dev, pos0=n) for l in range(G)]
            vn = [gen.values_bf16(pseed, l, 0, 1, Hkv, d, device=dev, pos0=n) for l in range(G)]
            qn = [gen.queries_bf16(pseed, l, 0, 1, Hq, d, device=dev, pos0=n) for l in range(G)]
            od = torch.empty_like(qn[0])
            pos = torch.full((1,), m, dtype=torch.int32, device=dev)
            nst = 24
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(nst + 1)]
            for st in range(nst):
                evs[st].record()
                for layer in range(G):
                    pc.pod_decode_step(layer, kn[layer], vn[layer], qn[layer], qn[0] if layer else None, pos, scale, out=od)
                pos += 1
            evs[nst].record()
            torch.cuda.synchronize()
            steps_us = [evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(4, nst)]
            rows = obs * (Hq // Hkv)
            vflops = 2.0 * d * rows * Hkv * (n + (n - S - W))      # both passes of the votes: all keys, then the distant ones
            tvm = statistics.median(tv[1:])
            res["token_selection"] = {
                "what": f"prompt {n} -> {m} stored tokens per layer: votes of the last {obs} queries (lowest layer), max-pool 7, "
                        f"top {keep} of {n - S - W} distant tokens per kv head, compaction of both layers; then decode steps",
                "ms_votes": round(tvm, 4), "votes_tflops": round(vflops / tvm / 1e9, 2),
                "ms_top": round(statistics.median(tt[1:]), 4), "ms_compact_both_layers": round(statistics.median(tc[1:]), 4),
                "share_of_block_prefill": round((tvm + statistics.median(tt[1:]) + statistics.median(tc[1:]))
                                                / (res["lowest_layer"]["ms"] + res["upper_layer"]["ms"]), 4),
                "decode_step_us_both_layers_after": round(statistics.median(steps_us), 2)}
            del sws, sel, votes
        # what the matrix pipes can do at all when every MFMA takes an operand fragment out of LDS (synthetic loops at the
        # kernel's occupancy; 32 cycles per MFMA and SIMD = never idle)
        feed = {}
        scratch = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
        it_feed = 20000
        for variant, name in ((0, "mfma_only"), (1, "one_lds_fragment_per_mfma"), (2, "one_lds_fragment_per_mfma_plus_softmax_valu"),
                              (3, "one_lds_fragment_per_two_mfma_plus_softmax_valu")):
            pod.pod_profile_mfma_feed(variant, 2000, scratch)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            pod.pod_profile_mfma_feed(variant, it_feed, scratch)
            e1.record()
            torch.cuda.synchronize()
            per_simd = it_feed * 16 * (2 if variant == 3 else 1)
            feed[name] = {"ns_per_mfma_per_simd": round(e0.elapsed_time(e1) * 1e6 / per_simd, 2)}
        base_ns = feed["mfma_only"]["ns_per_mfma_per_simd"]
        for v in feed.values():
            v["pipe_busy"] = round(base_ns / v["ns_per_mfma_per_simd"], 3)
        # the kernel: MFMAs it issues per SIMD (causal pairs, both products: 2 * 2 * d * pairs flops / 32768 flops per MFMA)
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        k_ns = res["lowest_layer"]["ms"] * 1e6 / (flops / 32768.0 / (4 * cus))
        res["mfma_feed"] = {"what": "synthetic loops, two waves per SIMD: what LDS-fed 32x32x16 MFMAs reach on this chip", **feed,
                            "kernel_ns_per_counted_mfma_per_simd": round(k_ns, 2), "kernel_pipe_busy_counted_work": round(base_ns / k_ns, 3),
                            "kernel_vs_lds_fed_loop_with_softmax_valu": round(feed["one_lds_fragment_per_mfma_plus_softmax_valu"]["ns_per_mfma_per_simd"] / k_ns, 3)}
        del scratch
        pc.pod_cache_check()
        out["prefill"] = {"workload": f"configs[3]: one block G=2, 32q/8kv, d=128, prompt {n}, S=64, W=2048, "
                                      "attention + cache construction", "flops_per_layer": flops,
                          "peak_tflops": MFMA_BF16_PEAK_TFLOPS, **res}
        del pc, q, k, v, o
        torch.cuda.empty_cache()

    # ---- the large-batch decode configurations (configs[2] and configs[4]); skipped once the run is past the time guard
    if not a.no_large:
        large = {}
        for wl in ("cfg3", "cfg5"):
            for variant in ("step", "reuse"):
                key = f"{wl}_{variant}"
                if time.perf_counter() - T_START > a.time_guard:
                    large[key] = {"skipped": f"past the time guard of {a.time_guard:.0f} s"}
                    continue
                large[key] = run_large(wl, a.large_steps, 2, variant)
        out["large_batch"] = large
    out["bench_seconds"] = round(time.perf_counter() - T_START, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
