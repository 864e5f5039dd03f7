"""GPU: pod_decode_step (one launch = the new token's cache update + decode attention over the tokens including
it) against the CPU oracle's append followed by its decode attention; cache contents bit for bit.  Also the merge
of the split-K partials inside the streaming kernel against the separate merge kernel."""
import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from pod_inputs import gen
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 8, 2), (64, 4, 2), (128, 16, 1), (64, 6, 6), (128, 3, 1), (128, 32, 8), (64, 16, 16)])
def test_steps_from_an_empty_cache_across_every_region_edge(d, Hq, Hkv):
    """S=4, W=12: positions 0 .. 39 one at a time: sink slots, the ring filling, the first displaced token at
    position S + W, and on; after every step both layers' outputs and (at the end) the stores are compared."""
    S, W = 4, 12
    c = Case(2, 2, Hq, Hkv, d, S, W, 1, 64, seed=500 + d + Hq)
    for p in range(40):
        for layer in range(2):
            assert_close(c.step(layer, [p]), c.decode_ref(layer, [p + 1]), f"position {p} layer {layer}")
        if p in (0, S - 1, S, S + W - 1, S + W, S + W + 1, 39):
            for layer in range(2):
                c.assert_cache_equal(layer, 0)
    c.gpu.pod_cache_check()
    assert c.gpu.pod_cache_seq_len(1, 0) == 40


@pytest.mark.parametrize("env", [{}, {"POD_DECODE_XCD_LOCAL": "0"}, {"POD_DECODE_FUSED": "0"}, {"POD_DECODE_FUSED": "0", "POD_DECODE_EVEN": "0"}],
                         ids=["merge-in-one-xcd", "merge-at-device-scope", "separate-merge-kernel-even-split", "separate-merge-kernel-fixed-pieces"])
def test_steps_on_long_contexts_ragged_batch_several_tiles(env, monkeypatch):
    """Three sequences of different lengths (one still inside S + W, one just past it, one with many split-K
    pieces), 70 steps: the short one crosses S + W on the way.  Through the three ways the partials get merged
    (read from the environment when the cache is created)."""
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    S, W = 16, 96
    c = Case(2, 2, 32, 8, 128, S, W, 3, 3000, seed=501)
    lens = [2700, 60, S + W + 1]
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    for s in range(70):
        pos = [n + s for n in lens]
        for layer in range(2):
            assert_close(c.step(layer, pos), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for layer in range(2):
        for b in range(3):
            c.assert_cache_equal(layer, b)
    c.gpu.pod_cache_check()


def test_step_equals_append_then_decode_bit_for_bit_in_the_cache():
    """The same tokens through pod_decode_step and through pod_cache_append + pod_decode_attention: identical stores,
    outputs within bf16 rounding of each other (the order of the merge differs)."""
    S, W, n0 = 8, 64, 1000
    a = Case(2, 2, 8, 2, 128, S, W, 2, 1200, seed=502, with_oracle_cache=False)
    b = Case(2, 2, 8, 2, 128, S, W, 2, 1200, seed=502, with_oracle_cache=False)
    for layer in range(2):
        for seq, n in enumerate((n0, 70)):
            a.fill(layer, seq, n)
            b.fill(layer, seq, n)
    for s in range(5):
        pos = [n0 + s, 70 + s]
        for layer in range(2):
            oa = a.step(layer, pos)
            b.append(layer, pos)
            ob = b.decode(layer, [p + 1 for p in pos])
            assert (oa.float() - ob.float()).abs().max() <= 2.0 ** -7 * ob.float().abs().max()
    for layer in range(2):
        for seq in range(2):
            ga, gb = a.gpu.pod_cache_export_logical(layer, seq), b.gpu.pod_cache_export_logical(layer, seq)
            for name in ga:
                assert torch.equal(ga[name], gb[name]), (layer, seq, name)


@pytest.mark.parametrize("env", [{}, {"POD_DECODE_XCD_LOCAL": "0"}, {"POD_DECODE_FUSED": "0"}, {"POD_DECODE_FUSED": "0", "POD_DECODE_EVEN": "0"}],
                         ids=["merge-in-one-xcd", "merge-at-device-scope", "separate-merge-kernel-even-split", "separate-merge-kernel-fixed-pieces"])
def test_wrong_position_is_flagged_nothing_stored_other_entries_exact(env, monkeypatch):
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    c = Case(2, 2, 4, 2, 64, 8, 32, 3, 512, seed=503)
    lens = [300, 100, 45]
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    k = torch.cat([c.keys(0, b, 1, c.dev, pos0=n) for b, n in enumerate(lens)]).contiguous()
    v = torch.cat([c.values(0, b, 1, c.dev, pos0=n) for b, n in enumerate(lens)]).contiguous()
    q = c.decode_queries(0, [n + 1 for n in lens], c.dev)
    before = c.gpu.pod_cache_export_logical(0, 1)
    pos = torch.tensor([300, 101, 45], dtype=torch.int32, device=c.dev)   # sequence 1 holds 100 tokens, not 101
    out = c.gpu.pod_decode_step(0, k, v, q, None, pos, c.scale)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == pod.binding.ERR_STATE
    assert float(out[1].float().abs().max()) == 0.0
    c.gpu.pod_cache_sync_lengths()                 # the mirror counted the skipped entry
    assert [c.gpu.pod_cache_seq_len(0, b) for b in range(3)] == [301, 100, 46]
    after = c.gpu.pod_cache_export_logical(0, 1)
    for name in before:
        assert torch.equal(before[name], after[name]), name
    c.cpu.append(0, gen.bf16_bits(k.cpu()), gen.bf16_bits(v.cpu()), [300, 100, 45])
    ref = c.decode_ref(0, [301, 101, 46])
    assert_close(out[[0, 2]], ref[[0, 2]], "the other sequences")


def test_upper_layer_before_the_lowest_layer_is_refused():
    c = Case(2, 2, 4, 2, 64, 8, 32, 1, 512, seed=504)
    for layer in range(2):
        c.fill(layer, 0, 100)
    with pytest.raises(pod.PodError) as e:
        c.step(1, [100])
    assert e.value.code == pod.binding.ERR_STATE
    c.gpu.pod_cache_check()
    assert_close(c.step(0, [100]), c.decode_ref(0, [101]), "lowest")


def test_launch_of_several_rounds_uses_the_separate_merge_and_matches():
    """40 sequences x 8 kv heads x several pieces: more workgroups than the chip holds at once, so the step's partials
    are merged by the second kernel; same results."""
    S, W, B = 8, 56, 40
    c = Case(2, 2, 16, 8, 64, S, W, B, 700, seed=509)
    lens = [30 + (53 * b) % 600 for b in range(B)]
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    for s in range(2):
        pos = [n + s for n in lens]
        for layer in range(2):
            assert_close(c.step(layer, pos), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for b in (0, 7, 39):
        c.assert_cache_equal(0, b)
        c.assert_cache_equal(1, b)
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("reuse", [False, True], ids=["plain", "score-reuse"])
def test_more_than_256_sequences_step_with_device_side_lengths(reuse):
    B, S, W = 300, 4, 16
    c = Case(2, 2, 4, 2, 64, S, W, B, 100, seed=505)
    lens = [1 + (37 * b) % 90 for b in range(B)]
    for layer in range(2):
        for b in range(B):
            c.fill(layer, b, lens[b])
    scores = c.gpu.new_score_buffer() if reuse else None
    for s in range(2):
        pos = [n + s for n in lens]
        for layer in range(2):
            out = c.step_reuse(layer, pos, scores) if reuse else c.step(layer, pos)
            assert_close(out, c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for b in (0, 17, 123, 299):
        c.assert_cache_equal(1, b)
        c.assert_cache_equal(0, b)
    c.gpu.pod_cache_check()


def test_headwise_blocks_step():
    """kv head 0: blocks {0,1,2},{3}; kv head 1: {0},{1,2,3}: a layer is the lowest for one head and an upper layer
    for the other; the displaced token's key goes to the store only where the layer is the head's lowest."""
    tab = np.array([[0, 0], [0, 1], [0, 1], [3, 1]], dtype=np.int32)
    S, W = 8, 32
    c = Case(4, 1, 8, 2, 128, S, W, 2, 400, seed=506, block_lowest=tab)
    lens = [300, S + W - 2]
    for layer in range(4):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    for s in range(6):
        pos = [n + s for n in lens]
        for layer in range(4):
            assert_close(c.step(layer, pos), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for layer in range(4):
        for b in range(2):
            c.assert_cache_equal(layer, b)
    c.gpu.pod_cache_check()


def test_outlier_keys_through_the_fused_merge():
    c = Case(4, 4, 8, 2, 128, 8, 64, 1, 3000, seed=507, outlier_rate=0.3, outlier_scale=16.0)
    n = 2900
    for layer in range(4):
        c.fill(layer, 0, n)
    for layer in range(4):
        assert_close(c.step(layer, [n]), c.decode_ref(layer, [n + 1]), f"layer {layer}")
    c.gpu.pod_cache_check()


def test_merge_inside_the_streaming_kernel_equals_the_separate_merge_kernel(monkeypatch):
    """pod_decode_attention with the partials merged by the last workgroup (default) and by the separate kernel
    (POD_DECODE_FUSED=0, read when the cache is created): both within tolerance of the oracle and within rounding
    of each other; a wrong context length is caught by both."""
    lens = [2777, 40, 513]
    fused = Case(2, 2, 8, 2, 128, 16, 300, 3, 3000, seed=508)
    monkeypatch.setenv("POD_DECODE_FUSED", "0")
    split = Case(2, 2, 8, 2, 128, 16, 300, 3, 3000, seed=508, with_oracle_cache=False)
    monkeypatch.delenv("POD_DECODE_FUSED")
    for c in (fused, split):
        for layer in range(2):
            for b, n in enumerate(lens):
                c.fill(layer, b, n)
    for layer in range(2):
        ref = fused.decode_ref(layer, lens)
        of, os_ = fused.decode(layer, lens), split.decode(layer, lens)
        assert_close(of, ref, f"fused layer {layer}")
        assert_close(os_, ref, f"separate layer {layer}")
        assert (of.float() - os_.float()).abs().max() <= 2.0 ** -7 * ref.max()
    for c in (fused, split):
        out = c.decode(1, [2777, 41, 513])
        assert float(out[1].float().abs().max()) == 0.0
        with pytest.raises(pod.PodError):
            c.gpu.pod_cache_check()
        out = c.decode(1, [2777, 0, 513])          # an inactive entry is not an error
        assert float(out[1].float().abs().max()) == 0.0
        c.gpu.pod_cache_check()


@pytest.mark.parametrize("d,Hq,Hkv,n", [(128, 4, 1, 20000), (128, 16, 1, 12000), (64, 8, 1, 20000), (128, 16, 2, 9000),
                                        (128, 64, 8, 12000), (64, 32, 8, 11000)],
                         ids=["rep4-1pair", "rep16-1pair", "d64-rep8-1pair", "rep8-2pairs", "rep8-8pairs", "d64-rep4-8pairs"])
def test_merge_inside_the_launch_with_many_pieces_per_pair(d, Hq, Hkv, n, monkeypatch):
    """One sequence and few kv heads with a long context: the launch is still one resident round, so the last workgroup
    of a pair merges - with one or two pairs more partials than one wave's block of 32, so the merge runs several
    blocks joined by its running maximum, with one wave per head (16 or 8 query heads per kv head) and with two;
    8 pairs take the XCD-local hand-off, fewer the device-scope one.  Decode on the filled cache, then three steps."""
    S, W = 8, 32
    monkeypatch.delenv("POD_DECODE_FUSED", raising=False)   # (read when the cache is created)
    c = Case(2, 2, Hq, Hkv, d, S, W, 1, n + 8, seed=510 + Hq)
    for layer in range(2):
        c.fill(layer, 0, n)
    info = c.gpu.pod_cache_launch_info()
    assert info["fused_merge"]
    for layer in range(2):
        assert_close(c.decode(layer, [n]), c.decode_ref(layer, [n]), f"decode layer {layer}")
    for s in range(3):
        for layer in range(2):
            assert_close(c.step(layer, [n + s]), c.decode_ref(layer, [n + s + 1]), f"step {s} layer {layer}")
    for layer in range(2):
        c.assert_cache_equal(layer, 0)
    c.gpu.pod_cache_check()


def test_pairs_that_do_not_divide_over_the_xcds_evenly():
    """13 sequences x 5 kv heads = 65 (sequence, kv head) pairs on 8 XCDs: the XCD-local hand-off is still used (the
    one-dimensional launch is padded to 72 pair positions, the surplus workgroups leave at once), ragged lengths,
    steps and plain decode."""
    S, W, B = 8, 56, 13
    c = Case(2, 2, 10, 5, 64, S, W, B, 700, seed=511)
    lens = [20 + (97 * b) % 640 for b in range(B)]
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    for layer in range(2):
        assert_close(c.decode(layer, lens), c.decode_ref(layer, lens), f"decode layer {layer}")
    for s in range(2):
        pos = [n + s for n in lens]
        for layer in range(2):
            assert_close(c.step(layer, pos), c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for b in (0, 6, 12):
        c.assert_cache_equal(0, b)
        c.assert_cache_equal(1, b)
    c.gpu.pod_cache_check()


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(count):
        d = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 3, 4, 8]))
        rep = int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
        S = int(rng.integers(0, 40))
        W = int(rng.integers(1, 200))
        B = int(rng.choice([1, 1, 2, 3, 5, 9]))
        lens = [int(x) for x in rng.integers(0, 2500, size=B)]
        shapes.append((d, Hkv * rep, Hkv, S, W, lens))
    return shapes



@pytest.mark.parametrize("shape", _random_shapes(24, 20241205), ids=lambda s: f"d{s[0]}-q{s[1]}-kv{s[2]}-S{s[3]}-W{s[4]}-B{len(s[5])}")
def test_steps_and_reuse_steps_on_seeded_random_shapes(shape):
    """Seeded random head counts, sink and window sizes (sink 0 included), batch sizes and ragged lengths (empty
    sequences included): two steps through pod_decode_step and two through pod_decode_step_reuse, every output against
    the oracle, stores bit for bit."""
    d, Hq, Hkv, S, W, lens = shape
    c = Case(2, 2, Hq, Hkv, d, S, W, len(lens), max(lens) + 8, seed=700 + Hq + W)
    for layer in range(2):
        for b, n in enumerate(lens):
            if n:
                c.fill(layer, b, n)
    scores = c.gpu.new_score_buffer()
    for s in range(4):
        pos = [n + s for n in lens]
        for layer in range(2):
            out = c.step(layer, pos) if s < 2 else c.step_reuse(layer, pos, scores)
            assert_close(out, c.decode_ref(layer, [p + 1 for p in pos]), f"step {s} layer {layer}")
    for layer in range(2):
        for b in range(len(lens)):
            c.assert_cache_equal(layer, b)
    c.gpu.pod_cache_check()
