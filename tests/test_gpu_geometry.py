"""GPU: degenerate geometries through every entry point against the CPU oracle: no sink tokens, a window of one
token, one query head per kv head and sixteen, a context limit that leaves no room for distant tokens, blocks
of one layer and of three."""
import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from podcase import Case, assert_close
from test_gpu_chunked import append_many_both, run_chunks
from test_gpu_prefill import ref_prefill, run_prefill

pytestmark = pytest.mark.gpu

#            L  G  Hq Hkv  d    S   W  max_ctx  n
GEOMETRIES = [
    pytest.param(2, 2, 2, 2, 64, 0, 16, 200, 150, id="no-sink_rep1"),
    pytest.param(2, 2, 16, 1, 128, 4, 1, 120, 90, id="window1_rep16"),
    pytest.param(2, 2, 4, 2, 128, 5, 20, 25, 25, id="no-room-for-distant"),
    pytest.param(2, 2, 4, 2, 64, 30, 50, 40, 40, id="context-limit-below-sink-plus-window"),
    pytest.param(2, 1, 4, 4, 64, 3, 7, 100, 77, id="blocks-of-one-layer"),
    pytest.param(3, 3, 6, 2, 128, 0, 1, 130, 129, id="block-of-three_no-sink_window1"),
]


@pytest.mark.parametrize("L,G,Hq,Hkv,d,S,W,max_ctx,n", GEOMETRIES)
def test_cache_updates_and_decode(L, G, Hq, Hkv, d, S, W, max_ctx, n):
    c = Case(L, G, Hq, Hkv, d, S, W, 2, max_ctx, seed=1000 + n)
    first = n // 2
    for layer in range(L):
        append_many_both(c, layer, [0, 0], [first, first // 2], first)
    p = [first, first // 2]
    while p[0] < n - 1:                                     # sequence 1 lags behind; then single appends for both
        t = min(7, n - 1 - p[0])
        for layer in range(L):
            append_many_both(c, layer, p, [t, min(t, 3)], t)
        p = [p[0] + t, p[1] + min(t, 3)]
    for layer in range(L):
        c.append(layer, p)
    ctx = [x + 1 for x in p]
    assert ctx[0] == n
    for layer in range(L):
        assert_close(c.decode(layer, ctx), c.decode_ref(layer, ctx), f"decode layer {layer}")
        for b in range(2):
            c.assert_cache_equal(layer, b)
    if G > 1:                                               # the same token through score reuse and the gate at tau = 1
        scores = c.gpu.new_score_buffer()
        ctx_t = torch.tensor(ctx, dtype=torch.int32, device=c.dev)
        for layer in range(L):
            assert_close(c.decode_reuse(layer, ctx, scores), c.decode_ref(layer, ctx), f"reuse layer {layer}")
        for layer in range(L):
            got = c.gpu.pod_decode_attention_gated(layer, c.decode_queries(layer, ctx, c.dev), ctx_t, c.scale, 1.0, scores)
            assert_close(got, c.decode_ref(layer, ctx), f"gated tau=1 layer {layer}")
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("L,G,Hq,Hkv,d,S,W,max_ctx,n", GEOMETRIES)
def test_prefill_in_one_call_and_in_chunks(L, G, Hq, Hkv, d, S, W, max_ctx, n):
    c = Case(L, G, Hq, Hkv, d, S, W, 1, max_ctx, seed=1100 + n, with_oracle_cache=False)
    for layer in range(L):
        assert_close(run_prefill(c, layer, n), ref_prefill(c, layer, n, np.arange(n)), f"prefill layer {layer}")
    c2 = Case(L, G, Hq, Hkv, d, S, W, 1, max_ctx, seed=1100 + n)
    cuts = [n // 3, 1, n - n // 3 - 1]
    run_chunks(c2, [t for t in cuts if t > 0])


@pytest.mark.parametrize("seed", list(range(1, 9)))
def test_random_geometries_and_lengths(seed):
    """Geometry, batch and lengths drawn at random (seeded): cache updates, decode (plain and with score reuse),
    prefill in one call and in chunks, all against the oracle."""
    rng = np.random.default_rng(seed)
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 8]))
    S, W = int(rng.integers(0, 21)), int(rng.integers(1, 71))
    G = int(rng.choice([1, 2, 3]))
    L = G * int(rng.choice([1, 2]))
    B = int(rng.integers(1, 4))
    lens = [int(rng.integers(1, 400)) for _ in range(B)]
    max_ctx = max(lens) + 2
    c = Case(L, G, Hq, Hkv, d, S, W, B, max_ctx, seed=1200 + seed)
    for layer in range(L):
        for b in range(B):
            c.fill(layer, b, lens[b])
        c.append(layer, lens)
    ctx = [n + 1 for n in lens]
    scores = c.gpu.new_score_buffer()
    for layer in range(L):
        ref = c.decode_ref(layer, ctx)
        assert_close(c.decode(layer, ctx), ref, f"decode layer {layer}")
        assert_close(c.decode_reuse(layer, ctx, scores), ref, f"reuse layer {layer}")
        c.assert_cache_equal(layer, int(rng.integers(0, B)))
    c.gpu.pod_cache_check()
    n = int(rng.integers(1, 380))
    p = Case(L, G, Hq, Hkv, d, S, W, 1, n, seed=1300 + seed, with_oracle_cache=False)
    for layer in (0, L - 1):
        assert_close(run_prefill(p, layer, n), ref_prefill(p, layer, n, np.arange(n)), f"prefill layer {layer}")
    cuts = sorted(set(int(x) for x in rng.integers(1, n, size=3)) | {n}) if n > 1 else [n]
    chunks = [b - a for a, b in zip([0] + cuts[:-1], cuts)]
    run_chunks(Case(L, G, Hq, Hkv, d, S, W, 1, n, seed=1300 + seed), chunks)


@pytest.mark.parametrize("scale", [0.01, 1.0, 3.0])
def test_other_scales(scale):
    """scale is an argument: 0.01 gives an almost uniform softmax, 1 and 3 give logits with a standard deviation of
    11 and 34 (a few keys take all the weight, and the running maxima move all the time)."""
    lens = [900, 77]
    c = Case(2, 2, 8, 2, 128, 8, 64, 2, 1000, seed=1400)
    c.scale = scale
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    scores = c.gpu.new_score_buffer()
    for layer in range(2):
        ref = c.decode_ref(layer, lens)
        assert_close(c.decode(layer, lens), ref, f"decode layer {layer}")
        assert_close(c.decode_reuse(layer, lens, scores), ref, f"reuse layer {layer}")
    p = Case(2, 2, 8, 2, 128, 8, 64, 1, 700, seed=1401, with_oracle_cache=False)
    p.scale = scale
    for layer in range(2):
        assert_close(run_prefill(p, layer, 700), ref_prefill(p, layer, 700, np.arange(700)), f"prefill layer {layer}")
    q = Case(2, 2, 8, 2, 128, 8, 64, 1, 700, seed=1401)
    q.scale = scale
    run_chunks(q, [300, 250, 150])
