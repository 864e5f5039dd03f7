"""Decode launches of several rounds of workgroups with the rows split evenly over the workgroups (plain mode,
lengths known to the host): against the oracle on ragged batches, and against the fixed-piece launch of the same call.
The small shapes here would normally merge inside one launch; POD_DECODE_FUSED=0 (read when the cache is created)
sends them down the path that large batches take."""
import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu


def fill_all(c, lens):
    for layer in range(c.L):
        for b, n in enumerate(lens):
            if n:
                c.fill(layer, b, n)


@pytest.mark.parametrize("seed", range(12))
def test_random_ragged_batches_decode_and_steps(seed, monkeypatch):
    """Seeded shapes: head counts, head dim, sink 0, windows, 1..24 sequences of 0..3000 tokens (empty ones, ones
    still inside S + W, long ones): three decode steps, pod_decode_attention, three score-reuse steps, every layer of
    the block."""
    monkeypatch.setenv("POD_DECODE_FUSED", "0")
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3, 8]))
    rep = int(rng.choice([1, 2, 4, 7] if d == 64 else [1, 2, 4, 8]))
    S = int(rng.choice([0, 4, 16, 64]))
    W = int(rng.choice([8, 40, 128, 500]))
    B = int(rng.integers(1, 25))
    G = int(rng.choice([1, 2, 3]))
    lens = [int(x) for x in rng.choice([0, 1, S + W, S + W + 1, 129, 700, 1500, 3000], size=B)]
    lens = [max(0, n - int(rng.integers(0, 3))) for n in lens]
    c = Case(G, G, Hkv * rep, Hkv, d, S, W, B, 3110, seed=9100 + seed)
    fill_all(c, lens)
    for layer in range(G):      # (the oracle has no notion of an empty entry: here only that such rows come out zero)
        out = c.decode(layer, lens)
        for b, n in enumerate(lens):
            if n == 0:
                assert float(out[b].float().abs().max()) == 0.0
    for s in range(3):
        pos = [n + s for n in lens]
        for layer in range(G):
            assert_close(c.step(layer, pos), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer} lens {lens}")
    ctx = [n + 3 for n in lens]
    for layer in range(G):
        assert_close(c.decode(layer, ctx), c.decode_ref(layer, ctx), f"decode layer {layer} ctx {ctx}")
    # ... and three steps with score reuse: the lowest layer writes its distant logits, the upper layers walk units of
    # twice as many distant rows and read them
    scores = c.gpu.new_score_buffer()
    for s in range(3, 6):
        pos = [n + s for n in lens]
        for layer in range(G):
            assert_close(c.step_reuse(layer, pos, scores), c.decode_ref(layer, [p + 1 for p in pos]), f"reuse step {s} layer {layer} lens {lens}")
    for layer in range(G):
        for b in range(B):
            c.assert_cache_equal(layer, b)
    c.gpu.pod_cache_check()


def test_even_split_and_fixed_pieces_agree(monkeypatch):
    """The same calls through both launch shapes: equal up to the order of the merge."""
    lens = [2900, 17, 0, 1300, 1301, 140, 2048, 5]
    outs = {}
    for even in ("1", "0"):
        monkeypatch.setenv("POD_DECODE_FUSED", "0")
        monkeypatch.setenv("POD_DECODE_EVEN", even)
        c = Case(2, 2, 16, 4, 128, 16, 96, len(lens), 3000, seed=9200, with_oracle_cache=False)
        fill_all(c, lens)
        o = [c.decode(layer, lens).float() for layer in range(2)]
        pos = list(lens)
        o += [c.step(layer, pos).float() for layer in range(2)]
        scores = c.gpu.new_score_buffer()
        pos = [n + 1 for n in lens]
        o += [c.step_reuse(layer, pos, scores).float() for layer in range(2)]
        outs[even] = o
        c.gpu.pod_cache_check()
    for a, b in zip(outs["1"], outs["0"]):
        assert (a - b).abs().max() <= 2.0 ** -7 * b.abs().max()


def test_reuse_steps_follow_plain_steps_and_separate_calls_read_their_logits(monkeypatch):
    """Logits written by an even-split reuse step of the lowest layer are read by the upper layer's reuse step and,
    after the next token's lowest-layer call through the separate entry point, by pod_decode_attention_reuse."""
    monkeypatch.setenv("POD_DECODE_FUSED", "0")
    lens = [1900, 300, 41, 2600]
    c = Case(3, 3, 8, 2, 128, 8, 32, len(lens), 2700, seed=9500)
    fill_all(c, lens)
    scores = c.gpu.new_score_buffer()
    for s in range(4):
        pos = [n + s for n in lens]
        for layer in range(3):
            assert_close(c.step_reuse(layer, pos, scores), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    pos = [n + 4 for n in lens]
    ctx = [p + 1 for p in pos]
    for layer in range(3):
        c.append(layer, pos)
    for layer in range(3):
        assert_close(c.decode_reuse(layer, ctx, scores), c.decode_ref(layer, ctx), f"separate calls layer {layer}")
    for layer in range(3):
        for b in range(len(lens)):
            c.assert_cache_equal(layer, b)
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("d,Hkv,rep", [(128, 1, 16), (64, 2, 16), (128, 3, 5), (64, 1, 1)])
def test_sixteen_query_heads_per_kv_head_and_other_group_sizes(d, Hkv, rep, monkeypatch):
    """All 16 MFMA columns hold real heads; odd group sizes; a single head."""
    monkeypatch.setenv("POD_DECODE_FUSED", "0")
    lens = [1500, 0, 333, 64, 2047]
    c = Case(2, 2, Hkv * rep, Hkv, d, 4, 60, len(lens), 2100, seed=9600 + rep)
    fill_all(c, lens)
    scores = c.gpu.new_score_buffer()
    for s in range(2):
        pos = [n + s for n in lens]
        for layer in range(2):
            assert_close(c.step(layer, pos), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for s in range(2, 4):
        pos = [n + s for n in lens]
        for layer in range(2):
            assert_close(c.step_reuse(layer, pos, scores), c.decode_ref(layer, [p + 1 for p in pos]), f"reuse step {s} layer {layer}")
    ctx = [n + 4 for n in lens]
    for layer in range(2):
        assert_close(c.decode(layer, ctx), c.decode_ref(layer, ctx), f"decode layer {layer}")
    c.gpu.pod_cache_check()


def test_one_long_sequence_among_many_short_ones(monkeypatch):
    """The long sequence is cut into many more parts than any other: its partial count per pair is the launch's."""
    monkeypatch.setenv("POD_DECODE_FUSED", "0")
    lens = [40] * 15 + [6000] + [3] * 8
    c = Case(2, 2, 8, 2, 128, 8, 64, len(lens), 6100, seed=9300)
    fill_all(c, lens)
    for layer in range(2):
        assert_close(c.decode(layer, lens), c.decode_ref(layer, lens), f"layer {layer}")
    pos = list(lens)
    for layer in range(2):
        assert_close(c.step(layer, pos), c.decode_ref(layer, [p + 1 for p in pos]), f"step layer {layer}")
    c.gpu.pod_cache_check()


def test_wrong_context_length_is_flagged_in_the_even_split(monkeypatch):
    monkeypatch.setenv("POD_DECODE_FUSED", "0")
    lens = [900, 300, 77]
    c = Case(2, 2, 4, 2, 64, 8, 32, 3, 1000, seed=9400)
    fill_all(c, lens)
    q = c.decode_queries(0, lens, c.dev)
    ctx = torch.tensor([900, 299, 77], dtype=torch.int32, device=c.dev)      # sequence 1 holds 300
    out = c.gpu.pod_decode_attention(0, q, None, ctx, c.scale)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == pod.binding.ERR_STATE
    assert float(out[1].float().abs().max()) == 0.0
    ref = c.decode_ref(0, lens)
    assert_close(out[[0, 2]], ref[[0, 2]], "the other sequences")


@pytest.mark.parametrize("rounds", ["one-round", "several-rounds"])
def test_walk_direction_does_not_change_the_result(rounds, monkeypatch):
    """The layers of a block walk the block's distant keys in alternating directions; with every layer walking forward
    (POD_DECODE_WALK_TURNS=0) the outputs differ only by the order of the sums.  G = 3: forward, backward, forward."""
    outs = {}
    lens = [2500, 700, 90]
    for turns in ("1", "0"):
        monkeypatch.setenv("POD_DECODE_WALK_TURNS", turns)
        if rounds == "several-rounds":
            monkeypatch.setenv("POD_DECODE_FUSED", "0")
        c = Case(3, 3, 8, 2, 128, 8, 64, len(lens), 2600, seed=9700, with_oracle_cache=(turns == "1"))
        fill_all(c, lens)
        o = []
        for s in range(2):
            pos = [n + s for n in lens]
            for layer in range(3):
                out = c.step(layer, pos)
                if turns == "1":
                    assert_close(out, c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
                o.append(out.float())
        ctx = [n + 2 for n in lens]
        o += [c.decode(layer, ctx).float() for layer in range(3)]
        outs[turns] = o
        c.gpu.pod_cache_check()
    for a, b in zip(outs["1"], outs["0"]):
        assert (a - b).abs().max() <= 2.0 ** -7 * b.abs().max()
