"""GPU: the five workload configurations at full size against the CPU oracle.

Where the whole output is cheap for the oracle (configs 1, 2) every element is compared;
for the large caches (configs 3, 5) and the 16K prefill (config 4) sampled (layer, sequence,
kv-head) slices / query rows are compared, each computed by the oracle from the definition
on regenerated inputs (every output row is independent, so a sampled comparison is exact).

Inputs for these sizes are produced by the seeded generator on the GPU and copied to the
host for the oracle: the generator is integer hashing + a table lookup and gives the same
bits on both devices (test_generator_is_bit_identical_on_cpu_and_gpu checks that).
"""
import math

import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from oracle import pod_oracle as po
from pod_inputs import gen
from podcase import assert_close

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]
DEV = "cuda:0"
SEED0 = 20241202


def host_bits(t):
    return gen.bf16_bits(t)


# ----------------------------------------------------------------------------- config 2
def test_config2_llama_decode_64_steps_with_demotion():
    """One block G=2, 32/8 heads, d=128, B=1, context 32768, S=64, W=2048, RoPE keys (base 5e5);
    64 consecutive decode steps: append both layers, decode both, every output compared."""
    L, G, Hq, Hkv, d, S, W, n0, steps = 2, 2, 32, 8, 128, 64, 2048, 32768, 64
    seed = SEED0 + 2
    max_ctx = n0 + steps
    rope = dict(rope_base=500000.0, rope_max_pos=max_ctx)
    cache = pod.PodCache(pod.make_config(L, G, Hq, Hkv, d, S, W, 1, max_ctx), DEV)
    oc = po.Cache(L, G, Hkv, d, S, W, 1, max_ctx)
    scale = 1.0 / math.sqrt(d)
    K = [gen.keys_bf16(seed, l, 0, max_ctx, Hkv, d, device=DEV, **rope) for l in range(L)]
    V = [gen.values_bf16(seed, l, 0, max_ctx, Hkv, d, device=DEV) for l in range(L)]
    Q = [gen.queries_bf16(seed, l, 0, steps, Hq, d, device=DEV, pos0=n0) for l in range(L)]
    Kh, Vh, Qh = [host_bits(t) for t in K], [host_bits(t) for t in V], [host_bits(t) for t in Q]
    for l in range(L):
        cache.pod_cache_fill(l, 0, K[l][:n0].contiguous(), V[l][:n0].contiguous())
        oc.fill(l, 0, Kh[l][:n0], Vh[l][:n0])
    for s in range(steps):
        p = n0 + s
        pos = torch.tensor([p], dtype=torch.int32, device=DEV)
        ctx = torch.tensor([p + 1], dtype=torch.int32, device=DEV)
        for l in range(L):
            cache.pod_cache_append(l, K[l][p:p + 1].contiguous(), V[l][p:p + 1].contiguous(), pos)
            oc.append(l, Kh[l][p:p + 1], Vh[l][p:p + 1], [p])
        for l in range(L):
            out = cache.pod_decode_attention(l, Q[l][s:s + 1].contiguous(), Q[0][s:s + 1].contiguous() if l else None,
                                             ctx, scale, max_context_len=p + 1)
            ref = oc.decode_attention(l, Qh[l][s:s + 1], Qh[0][s:s + 1] if l else None, [p + 1], scale)
            assert_close(out, ref, f"step {s} layer {l}")
    cache.pod_cache_check()
    for l in range(L):     # 64 demotions happened: the stores must agree bit for bit
        g, c = cache.pod_cache_export_logical(l, 0), oc.export(l, 0)
        assert set(g) == set(c)
        for name in c:
            assert np.array_equal(host_bits(g[name]), c[name]), (l, name)
        assert g["distV"].shape[0] == n0 + steps - S - W


def test_config2_llama_decode_steps_in_one_launch_per_layer():
    """The same workload through pod_decode_step (cache update + attention in one launch per layer), 24 steps, every
    output compared, the stores bit for bit at the end."""
    L, G, Hq, Hkv, d, S, W, n0, steps = 2, 2, 32, 8, 128, 64, 2048, 32768, 24
    seed = SEED0 + 2
    max_ctx = n0 + steps
    rope = dict(rope_base=500000.0, rope_max_pos=max_ctx)
    cache = pod.PodCache(pod.make_config(L, G, Hq, Hkv, d, S, W, 1, max_ctx), DEV)
    oc = po.Cache(L, G, Hkv, d, S, W, 1, max_ctx)
    scale = 1.0 / math.sqrt(d)
    K = [gen.keys_bf16(seed, l, 0, max_ctx, Hkv, d, device=DEV, **rope) for l in range(L)]
    V = [gen.values_bf16(seed, l, 0, max_ctx, Hkv, d, device=DEV) for l in range(L)]
    Q = [gen.queries_bf16(seed, l, 0, steps, Hq, d, device=DEV, pos0=n0) for l in range(L)]
    Kh, Vh, Qh = [host_bits(t) for t in K], [host_bits(t) for t in V], [host_bits(t) for t in Q]
    for l in range(L):
        cache.pod_cache_fill(l, 0, K[l][:n0].contiguous(), V[l][:n0].contiguous())
        oc.fill(l, 0, Kh[l][:n0], Vh[l][:n0])
    assert cache.pod_cache_launch_info()["xcds"] >= 1
    for s in range(steps):
        p = n0 + s
        pos = torch.tensor([p], dtype=torch.int32, device=DEV)
        for l in range(L):
            out = cache.pod_decode_step(l, K[l][p:p + 1].contiguous(), V[l][p:p + 1].contiguous(), Q[l][s:s + 1].contiguous(),
                                        Q[0][s:s + 1].contiguous() if l else None, pos, scale, max_context_len=p + 1)
            oc.append(l, Kh[l][p:p + 1], Vh[l][p:p + 1], [p])
            ref = oc.decode_attention(l, Qh[l][s:s + 1], Qh[0][s:s + 1] if l else None, [p + 1], scale)
            assert_close(out, ref, f"step {s} layer {l}")
    cache.pod_cache_check()
    for l in range(L):
        g, c = cache.pod_cache_export_logical(l, 0), oc.export(l, 0)
        for name in c:
            assert np.array_equal(host_bits(g[name]), c[name]), (l, name)


def test_config2_shape_with_score_reuse():
    """Config-2 shape, 8 decode steps through the score-reuse entry point, every output compared."""
    L, G, Hq, Hkv, d, S, W, n0, steps = 2, 2, 32, 8, 128, 64, 2048, 32768, 8
    seed = SEED0 + 2
    max_ctx = n0 + steps
    rope = dict(rope_base=500000.0, rope_max_pos=max_ctx)
    cache = pod.PodCache(pod.make_config(L, G, Hq, Hkv, d, S, W, 1, max_ctx), DEV)
    oc = po.Cache(L, G, Hkv, d, S, W, 1, max_ctx)
    scale = 1.0 / math.sqrt(d)
    K = [gen.keys_bf16(seed, l, 0, max_ctx, Hkv, d, device=DEV, **rope) for l in range(L)]
    V = [gen.values_bf16(seed, l, 0, max_ctx, Hkv, d, device=DEV) for l in range(L)]
    Q = [gen.queries_bf16(seed, l, 0, steps, Hq, d, device=DEV, pos0=n0) for l in range(L)]
    Kh, Vh, Qh = [host_bits(t) for t in K], [host_bits(t) for t in V], [host_bits(t) for t in Q]
    for l in range(L):
        cache.pod_cache_fill(l, 0, K[l][:n0].contiguous(), V[l][:n0].contiguous())
        oc.fill(l, 0, Kh[l][:n0], Vh[l][:n0])
    scores = cache.new_score_buffer()
    for s in range(steps):
        p = n0 + s
        pos = torch.tensor([p], dtype=torch.int32, device=DEV)
        ctx = torch.tensor([p + 1], dtype=torch.int32, device=DEV)
        for l in range(L):
            cache.pod_cache_append(l, K[l][p:p + 1].contiguous(), V[l][p:p + 1].contiguous(), pos)
            oc.append(l, Kh[l][p:p + 1], Vh[l][p:p + 1], [p])
        for l in range(L):
            out = cache.pod_decode_attention_reuse(l, Q[l][s:s + 1].contiguous(), ctx, scale, scores, max_context_len=p + 1)
            ref = oc.decode_attention(l, Qh[l][s:s + 1], Qh[0][s:s + 1] if l else None, [p + 1], scale)
            assert_close(out, ref, f"step {s} layer {l}")
    cache.pod_cache_check()


# ----------------------------------------------------------------------------- configs 3 and 5
def _big_decode(L, G, B, lens, S, W, seed, samples, outlier_rate=0.0, one_launch=False):
    Hq, Hkv, d = 32, 8, 128
    rep = Hq // Hkv
    max_ctx = max(lens) + 1
    cache = pod.PodCache(pod.make_config(L, G, Hq, Hkv, d, S, W, B, max_ctx), DEV)
    scale = 1.0 / math.sqrt(d)

    def keys(l, b, n, pos0=0, **kw):
        n_tot = lens[b] + 1
        return gen.keys_bf16(seed, l, b, n, Hkv, d, device=DEV, pos0=pos0, outlier_rate=outlier_rate,
                             outlier_lo=S, outlier_hi=n_tot - W, **kw)

    def values(l, b, n, pos0=0, **kw):
        return gen.values_bf16(seed, l, b, n, Hkv, d, device=DEV, pos0=pos0, **kw)

    for l in range(L):
        for b in range(B):
            cache.pod_cache_fill(l, b, keys(l, b, lens[b]), values(l, b, lens[b]))
    pos = torch.tensor(lens, dtype=torch.int32, device=DEV)
    ctx = torch.tensor([n + 1 for n in lens], dtype=torch.int32, device=DEV)
    qs = {}
    outs = {}
    for l in range(L):           # one decode step across all layers
        kn = torch.cat([keys(l, b, 1, pos0=lens[b]) for b in range(B)]).contiguous()
        vn = torch.cat([values(l, b, 1, pos0=lens[b]) for b in range(B)]).contiguous()
        qs[l] = torch.cat([gen.queries_bf16(seed, l, b, 1, Hq, d, device=DEV, pos0=lens[b]) for b in range(B)]).contiguous()
        low = l - l % G
        if one_launch == "reuse":   # ... with score reuse: upper layers read the lowest layer's distant logits
            if l == 0:
                scores = cache.new_score_buffer()
            outs[l] = cache.pod_decode_step_reuse(l, kn, vn, qs[l], pos, scale, scores, max_context_len=max_ctx)
            continue
        if one_launch:           # cache update + attention through pod_decode_step
            outs[l] = cache.pod_decode_step(l, kn, vn, qs[l], qs[low] if low != l else None, pos, scale, max_context_len=max_ctx)
            continue
        cache.pod_cache_append(l, kn, vn, pos)
        outs[l] = cache.pod_decode_attention(l, qs[l], qs[low] if low != l else None, ctx, scale, max_context_len=max_ctx)
    cache.pod_cache_check()
    torch.cuda.synchronize()
    for (l, b, kvh) in samples:
        n = lens[b] + 1
        low = l - l % G
        hs = slice(kvh * rep, (kvh + 1) * rep)
        k = host_bits(keys(l, b, n, head0=kvh, n_heads=1))
        v = host_bits(values(l, b, n, head0=kvh, n_heads=1))
        ka = host_bits(keys(low, b, n, head0=kvh, n_heads=1)) if low != l else None
        q = host_bits(qs[l][b:b + 1, hs].contiguous())
        qa = host_bits(qs[low][b:b + 1, hs].contiguous()) if low != l else None
        ref = po.pod_attention(q, k, v, qa, ka, [n - 1], S, W, scale)
        assert_close(outs[l][b:b + 1, hs], ref, f"layer {l} seq {b} kv head {kvh} n {n}")
    return cache, outs


@pytest.mark.parametrize("one_launch", [False, True, "reuse"], ids=["append+decode", "decode_step", "decode_step_reuse"])
def test_config3_batched_ragged_decode_32_layers(one_launch):
    """32 layers in 16 blocks (G=2), B=16, contexts uniform in [4096, 32768], one decode step over all layers."""
    seed = SEED0 + 3
    lens = [n - 1 for n in gen.ragged_lengths(seed, 16, 4096, 32768)]   # cache holds n-1, the step appends one
    order = np.argsort(lens)
    picks = [int(order[0]), int(order[-1]), int(order[7]), int(order[12])]
    samples = [(l, b, (l * 5 + b * 3) % 8) for l in (0, 1, 14, 15, 30, 31) for b in picks]
    _big_decode(32, 2, 16, lens, 64, 2048, seed, samples, one_launch=one_launch)


@pytest.mark.parametrize("one_launch", [False, True, "reuse"], ids=["append+decode", "decode_step", "decode_step_reuse"])
def test_config5_long_context_g4_with_outlier_keys(one_launch):
    """G=4 (8 blocks over 32 layers), B=4, context 131072, S=128, W=4096, 1 % of distant keys scaled x8."""
    seed = SEED0 + 5
    lens = [131071] * 4
    samples = [(0, 0, 1), (1, 0, 6), (3, 3, 2), (28, 2, 0), (31, 3, 7), (14, 1, 4)]
    cache, _ = _big_decode(32, 4, 4, lens, 128, 4096, seed, samples, outlier_rate=0.01, one_launch=one_launch)
    live, dense = pod.pod_cache_live_bytes(cache.cfg, 131072)
    assert abs((1 - live / dense) - 0.363) < 5e-4       # memory accounting at this configuration


# ----------------------------------------------------------------------------- config 4
def test_config4_prefill_16384_sampled_rows_and_cache():
    """One block G=2, 32/8 heads, d=128, prompt 16384, S=64, W=2048: attention (sampled rows, all heads)
    and the split cache it builds (every element, against the oracle's slice definition)."""
    L, G, Hq, Hkv, d, S, W, n = 2, 2, 32, 8, 128, 64, 2048, 16384
    seed = SEED0 + 4
    cache = pod.PodCache(pod.make_config(L, G, Hq, Hkv, d, S, W, 1, n), DEV)
    oc = po.Cache(L, G, Hkv, d, S, W, 1, n)
    scale = 1.0 / math.sqrt(d)
    Q = [gen.queries_bf16(seed, l, 0, n, Hq, d, device=DEV) for l in range(L)]
    K = [gen.keys_bf16(seed, l, 0, n, Hkv, d, device=DEV) for l in range(L)]
    V = [gen.values_bf16(seed, l, 0, n, Hkv, d, device=DEV) for l in range(L)]
    rng = np.random.default_rng(seed)
    rows = sorted(set(list(range(0, 96)) + list(range(S - 8, S + 8)) + list(range(S + W - 24, S + W + 24)) +
                      list(range(4090, 4102)) + list(range(8188, 8196)) + list(range(n - 64, n)) +
                      [int(x) for x in rng.integers(S + W, n, 64)]))
    rows = np.array(rows)
    Kh, Vh = [host_bits(t) for t in K], [host_bits(t) for t in V]
    for l in range(L):
        out = cache.pod_prefill_attention(l, 0, Q[l], K[l], V[l], Q[0] if l else None, K[0] if l else None, scale,
                                          write_cache=True)
        q = host_bits(Q[l][rows].contiguous())
        qa = host_bits(Q[0][rows].contiguous()) if l else None
        ref = po.pod_attention(q, Kh[l], Vh[l], qa, Kh[0] if l else None, rows, S, W, scale)
        assert_close(out[rows], ref, f"layer {l}")
        oc.fill(l, 0, Kh[l], Vh[l])
        g, c = cache.pod_cache_export_logical(l, 0), oc.export(l, 0)
        assert set(g) == set(c)
        for name in c:
            assert np.array_equal(host_bits(g[name]), c[name]), (l, name)
    cache.pod_cache_check()


def test_config4_prompt_in_chunks_sampled_rows_and_cache():
    """Config 4's prompt processed in chunks (the bench's 2048-token chunks, plus an uneven split): sampled rows
    of every chunk against the whole-sequence definition, and the cache after the last chunk against the
    oracle's slice definition, every element."""
    L, G, Hq, Hkv, d, S, W, n = 2, 2, 32, 8, 128, 64, 2048, 16384
    seed = SEED0 + 4
    cfg = pod.make_config(L, G, Hq, Hkv, d, S, W, 2, n)
    cache = pod.PodCache(cfg, DEV)
    scale = 1.0 / math.sqrt(d)
    Q = [gen.queries_bf16(seed, l, 0, n, Hq, d, device=DEV) for l in range(L)]
    K = [gen.keys_bf16(seed, l, 0, n, Hkv, d, device=DEV) for l in range(L)]
    V = [gen.values_bf16(seed, l, 0, n, Hkv, d, device=DEV) for l in range(L)]
    Kh, Vh = [host_bits(t) for t in K], [host_bits(t) for t in V]
    ws = torch.empty(pod.pod_prefill_chunk_workspace_bytes(cfg, n), dtype=torch.uint8, device=DEV)
    rng = np.random.default_rng(seed + 1)
    for slot, cuts in ((0, list(range(0, n + 1, 2048))), (1, [0, 100, 2211, 2212, 9000, n])):
        out = [torch.empty_like(Q[0]) for _ in range(L)]
        for a, b in zip(cuts[:-1], cuts[1:]):
            for l in range(L):
                cache.pod_prefill_attention_chunk(l, slot, Q[l][a:b], K[l][a:b], V[l][a:b], Q[0][a:b] if l else None,
                                                  K[0][a:b] if l else None, scale, ws, out=out[l][a:b], write_cache=True)
        rows = set()
        for a, b in zip(cuts[:-1], cuts[1:]):   # first and last rows of every chunk, and a few inside
            rows.update(range(a, min(a + 3, b)))
            rows.update(range(max(b - 3, a), b))
            rows.update(int(x) for x in rng.integers(a, b, 6))
        rows = np.array(sorted(rows))
        for l in range(L):
            q = host_bits(Q[l][rows].contiguous())
            qa = host_bits(Q[0][rows].contiguous()) if l else None
            ref = po.pod_attention(q, Kh[l], Vh[l], qa, Kh[0] if l else None, rows, S, W, scale)
            assert_close(out[l][rows], ref, f"slot {slot} layer {l}")
    oc = po.Cache(L, G, Hkv, d, S, W, 1, n)
    for l in range(L):
        oc.fill(l, 0, Kh[l], Vh[l])
        c = oc.export(l, 0)
        for slot in (0, 1):
            g = cache.pod_cache_export_logical(l, slot)
            assert set(g) == set(c)
            for name in c:
                assert np.array_equal(host_bits(g[name]), c[name]), (l, slot, name)
    cache.pod_cache_check()


@pytest.mark.parametrize("cuts", [None, [0, 30000, 30001, 65536, 69700, 100003]], ids=["one-call", "five-chunks"])
def test_long_prompt_100k_sampled_rows(cuts, monkeypatch):
    """A prompt of 100003 tokens (config 5's geometry: S=128, W=4096, 32/8 heads): index arithmetic far beyond the
    benchmark's 16384; sampled rows of the upper layer against the definition, and the distant stores it fills.
    In one call, and in chunks (keys and values read where the cache holds them; the scratch is the small one)."""
    L, G, Hq, Hkv, d, S, W, n = 2, 2, 32, 8, 128, 128, 4096, 100003
    seed = SEED0 + 6
    monkeypatch.delenv("POD_CHUNK_IN_PLACE", raising=False)   # (read when the cache is created: the small scratch needs the usual way)
    cache = pod.PodCache(pod.make_config(L, G, Hq, Hkv, d, S, W, 1, n), DEV)
    scale = 1.0 / math.sqrt(d)
    Q = [gen.queries_bf16(seed, l, 0, n, Hq, d, device=DEV) for l in range(L)]
    K = [gen.keys_bf16(seed, l, 0, n, Hkv, d, device=DEV) for l in range(L)]
    V = [gen.values_bf16(seed, l, 0, n, Hkv, d, device=DEV) for l in range(L)]
    rng = np.random.default_rng(seed)
    rows = np.array(sorted(set([0, 1, S, S + W - 1, S + W, 65535, 65536, 65537, n - 2, n - 1] +
                               [int(x) for x in rng.integers(S + W, n, 12)])))
    Kh, Vh = [host_bits(t) for t in K], [host_bits(t) for t in V]
    if cuts:
        cfg = pod.make_config(L, G, Hq, Hkv, d, S, W, 1, n)
        ws = torch.empty(pod.pod_prefill_chunk_in_place_bytes(cfg, n, max(b - a for a, b in zip(cuts[:-1], cuts[1:]))),
                         dtype=torch.uint8, device=DEV)
        outs = [torch.empty_like(Q[0]) for _ in range(L)]
        for a, b in zip(cuts[:-1], cuts[1:]):
            for l in range(L):
                cache.pod_prefill_attention_chunk(l, 0, Q[l][a:b], K[l][a:b], V[l][a:b], Q[0][a:b] if l else None,
                                                  K[0][a:b] if l else None, scale, ws, out=outs[l][a:b], write_cache=True)
        rows = np.array(sorted(set(rows.tolist() + [c for c in cuts[1:-1]] + [c - 1 for c in cuts[1:-1]])))
    for l in range(L):
        out = outs[l] if cuts else cache.pod_prefill_attention(l, 0, Q[l], K[l], V[l], Q[0] if l else None, K[0] if l else None,
                                                               scale, write_cache=True)
        if l == 1:
            ref = po.pod_attention(host_bits(Q[1][rows].contiguous()), Kh[1], Vh[1], host_bits(Q[0][rows].contiguous()),
                                   Kh[0], rows, S, W, scale)
            assert_close(out[rows], ref, "upper layer")
    g = cache.pod_cache_export_logical(0, 0)
    assert np.array_equal(host_bits(g["distK"]), Kh[0][S:n - W]) and np.array_equal(host_bits(g["distV"]), Vh[0][S:n - W])
    g = cache.pod_cache_export_logical(1, 0)
    assert np.array_equal(host_bits(g["distV"]), Vh[1][S:n - W]) and np.array_equal(host_bits(g["recentK"]), Kh[1][n - W:])
    cache.pod_cache_check()
