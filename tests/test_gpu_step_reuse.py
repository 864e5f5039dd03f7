"""GPU: pod_decode_step_reuse = pod_cache_append + pod_decode_attention_reuse of one layer in one streaming launch (two
for a layer with kv heads of both kinds); against the oracle's append + attention, stores bit for bit."""
import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,Hq,Hkv,G", [(128, 8, 2, 2), (64, 4, 2, 4), (128, 16, 1, 2), (64, 6, 6, 3), (128, 32, 8, 4)])
def test_reuse_steps_from_an_empty_cache_across_every_region_edge(d, Hq, Hkv, G):
    """S=4, W=12: positions 0 .. 39 one at a time through every layer of a block of G layers: sink slots, the ring
    filling, the first displaced token at S + W (its logit travels from the lowest layer to the upper ones), and on."""
    S, W = 4, 12
    c = Case(G, G, Hq, Hkv, d, S, W, 1, 64, seed=600 + d + Hq)
    scores = c.gpu.new_score_buffer()
    for p in range(40):
        for layer in range(G):
            assert_close(c.step_reuse(layer, [p], scores), c.decode_ref(layer, [p + 1]), f"position {p} layer {layer}")
        if p in (0, S - 1, S, S + W - 1, S + W, S + W + 1, 39):
            for layer in range(G):
                c.assert_cache_equal(layer, 0)
    c.gpu.pod_cache_check()
    assert c.gpu.pod_cache_seq_len(G - 1, 0) == 40


@pytest.mark.parametrize("env", [{}, {"POD_DECODE_XCD_LOCAL": "0"}, {"POD_DECODE_FUSED": "0"}, {"POD_DECODE_FUSED": "0", "POD_DECODE_EVEN": "0"}],
                         ids=["merge-in-one-xcd", "merge-at-device-scope", "separate-merge-kernel-even-split", "separate-merge-kernel-fixed-pieces"])
def test_reuse_steps_on_long_contexts_ragged_batch(env, monkeypatch):
    """Three sequences of different lengths (one inside S + W, one just past it, one with many split-K pieces), two
    blocks of two layers, 40 steps; merged inside the launch with either hand-off, and by the separate kernel."""
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    S, W = 16, 96
    c = Case(4, 2, 32, 8, 128, S, W, 3, 3000, seed=601)
    lens = [2700, 60, S + W + 1]
    for layer in range(4):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    scores = c.gpu.new_score_buffer()
    for s in range(40):
        pos = [n + s for n in lens]
        for layer in range(4):
            assert_close(c.step_reuse(layer, pos, scores), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for layer in range(4):
        for b in range(3):
            c.assert_cache_equal(layer, b)
    c.gpu.pod_cache_check()


def test_reuse_step_equals_the_separate_calls():
    """The same tokens through pod_decode_step_reuse and through pod_cache_append + pod_decode_attention_reuse:
    identical stores, outputs within bf16 rounding of each other."""
    S, W, n0 = 8, 64, 1000
    a = Case(2, 2, 8, 2, 128, S, W, 2, 1200, seed=602, with_oracle_cache=False)
    b = Case(2, 2, 8, 2, 128, S, W, 2, 1200, seed=602, with_oracle_cache=False)
    lens = [n0, 300]
    for c in (a, b):
        for layer in range(2):
            for s_, n in enumerate(lens):
                c.gpu.pod_cache_fill(layer, s_, c.keys(layer, s_, n, c.dev), c.values(layer, s_, n, c.dev))
    sa, sb = a.gpu.new_score_buffer(), b.gpu.new_score_buffer()
    for s in range(5):
        pos = [n + s for n in lens]
        ctx = torch.tensor([p + 1 for p in pos], dtype=torch.int32, device=a.dev)
        pos_t = torch.tensor(pos, dtype=torch.int32, device=a.dev)
        for layer in range(2):
            oa = a.step_reuse(layer, pos, sa)
            k = torch.cat([b.keys(layer, i, 1, b.dev, pos0=p) for i, p in enumerate(pos)]).contiguous()
            v = torch.cat([b.values(layer, i, 1, b.dev, pos0=p) for i, p in enumerate(pos)]).contiguous()
            b.gpu.pod_cache_append(layer, k, v, pos_t)
            ob = b.gpu.pod_decode_attention_reuse(layer, b.decode_queries(layer, [p + 1 for p in pos], b.dev), ctx, b.scale, sb)
            assert (oa.float() - ob.float()).abs().max() <= 1.6e-2, (s, layer)
    for layer in range(2):
        for s_ in range(2):
            ea, eb = a.gpu.pod_cache_export_logical(layer, s_), b.gpu.pod_cache_export_logical(layer, s_)
            for name in ea:
                assert torch.equal(ea[name], eb[name]), (layer, s_, name)
    a.gpu.pod_cache_check()
    b.gpu.pod_cache_check()


def test_launch_of_several_rounds_merges_the_reuse_step_in_the_second_kernel():
    S, W, B = 8, 56, 40
    c = Case(2, 2, 16, 8, 64, S, W, B, 700, seed=603)
    lens = [30 + (53 * b) % 600 for b in range(B)]
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    scores = c.gpu.new_score_buffer()
    for s in range(2):
        pos = [n + s for n in lens]
        for layer in range(2):
            assert_close(c.step_reuse(layer, pos, scores), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for b in (0, 7, 39):
        c.assert_cache_equal(0, b)
        c.assert_cache_equal(1, b)
    c.gpu.pod_cache_check()


def test_head_wise_blocks_with_layers_that_write_and_read_logits():
    """Layer 1 is the lowest layer of kv head 1's second block and an upper layer for kv head 0: such a layer both
    writes and reads logits (a writing and a reading launch, each performing the cache update of its own kv heads);
    small contexts merge inside the launches, the long one through the separate kernel."""
    S, W = 4, 28
    tab = np.array([[0, 0], [0, 1], [2, 1], [2, 3]], dtype=np.int32)
    c = Case(4, 1, 8, 2, 128, S, W, 2, 400, seed=604, block_lowest=tab)
    lens = [200, 31]
    _mixed_steps(c, lens)


def test_head_wise_blocks_large_batch():
    S, W = 4, 28
    tab = np.array([[0, 0, 0, 0], [0, 1, 0, 1], [2, 1, 0, 1], [2, 3, 0, 3]], dtype=np.int32)
    B = 48
    c = Case(4, 1, 8, 4, 64, S, W, B, 300, seed=607, block_lowest=tab)
    _mixed_steps(c, [20 + (37 * b) % 250 for b in range(B)], steps=2)


def _mixed_steps(c, lens, steps=6):
    S, W = c.S, c.W
    for layer in range(4):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    scores = c.gpu.new_score_buffer()
    for s in range(steps):
        pos = [n + s for n in lens]
        for layer in range(4):
            assert_close(c.step_reuse(layer, pos, scores), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for layer in range(4):
        for b in (0, len(lens) - 1):
            c.assert_cache_equal(layer, b)
    c.gpu.pod_cache_check()


def test_stale_logits_and_wrong_positions_are_refused():
    S, W, n = 8, 32, 500
    c = Case(2, 2, 8, 2, 128, S, W, 1, 600, seed=605)
    for layer in range(2):
        c.fill(layer, 0, n)
    scores = c.gpu.new_score_buffer()
    scores.zero_()
    # the lowest layer takes the token without score reuse: the upper layer finds no logits of this token
    c.step(0, [n])
    out = c.step_reuse(1, [n], scores)
    assert torch.all(out == 0)
    with pytest.raises(pod.PodError):
        c.gpu.pod_cache_check()
    c.gpu.pod_cache_sync_lengths()
    # (the upper layer's cache update itself was valid: both layers hold n + 1 tokens; go on from there)
    assert c.gpu.pod_cache_seq_len(1, 0) == n + 1
    for layer in range(2):
        assert_close(c.step_reuse(layer, [n + 1], scores), c.decode_ref(layer, [n + 2]), f"layer {layer}")
    # a wrong position: nothing stored, zero rows, flag
    k = c.keys(0, 0, 1, c.dev, pos0=n + 2)
    v = c.values(0, 0, 1, c.dev, pos0=n + 2)
    q = c.decode_queries(0, [n + 3], c.dev)
    bad = c.gpu.pod_decode_step_reuse(0, k, v, q, torch.tensor([n + 5], dtype=torch.int32, device=c.dev), c.scale, scores)
    assert torch.all(bad == 0)
    with pytest.raises(pod.PodError):
        c.gpu.pod_cache_check()
    c.gpu.pod_cache_sync_lengths()
    assert c.gpu.pod_cache_seq_len(0, 0) == n + 2
    c.assert_cache_equal(0, 0)


def test_gated_call_refuses_logits_left_by_a_reuse_step():
    """A reuse step leaves the logits but not the heads' distant sums: a gated upper-layer call must not use them."""
    S, W, n = 8, 32, 500
    c = Case(2, 2, 8, 2, 128, S, W, 1, 600, seed=606, with_oracle_cache=False)
    for layer in range(2):
        c.gpu.pod_cache_fill(layer, 0, c.keys(layer, 0, n, c.dev), c.values(layer, 0, n, c.dev))
    scores = c.gpu.new_score_buffer()
    c.step_reuse(0, [n], scores)
    k = c.keys(1, 0, 1, c.dev, pos0=n)
    v = c.values(1, 0, 1, c.dev, pos0=n)
    c.gpu.pod_cache_append(1, k, v, torch.tensor([n], dtype=torch.int32, device=c.dev))
    ctx = torch.tensor([n + 1], dtype=torch.int32, device=c.dev)
    out = c.gpu.pod_decode_attention_gated(1, c.decode_queries(1, [n + 1], c.dev), ctx, c.scale, 0.5, scores)
    assert torch.all(out == 0)
    with pytest.raises(pod.PodError):
        c.gpu.pod_cache_check()
