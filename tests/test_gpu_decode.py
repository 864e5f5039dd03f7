"""GPU: pod_decode_attention against the CPU oracle (max abs <= 2e-2, mean abs <= 2e-3)."""
import math
import os

import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from oracle import pod_oracle as po
from pod_inputs import gen
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu


def test_config1_toy_decode():
    """2 layers in one block, 4/2 heads, d=64, S=16, W=256: cache of 2047 tokens, append, decode at n=2048."""
    c = Case(2, 2, 4, 2, 64, 16, 256, 1, 2048, seed=20241203)
    for layer in range(2):
        c.fill(layer, 0, 2047)
        c.append(layer, [2047])
    for layer in range(2):
        c.assert_cache_equal(layer, 0)
        assert_close(c.decode(layer, [2048]), c.decode_ref(layer, [2048]), f"layer {layer}")
    assert c.gpu.pod_cache_export_logical(0, 0)["distK"].shape[0] == 1776
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 8, 2), (64, 4, 2), (128, 16, 1), (64, 6, 6), (128, 3, 1)])
@pytest.mark.parametrize("n", [1, 2, 7, 40, 41, 42, 73, 200, 457])
def test_small_contexts_all_region_shapes(d, Hq, Hkv, n):
    """S=8, W=32: n below S, inside the window, at S+W, one past it, several tiles with ragged tails."""
    c = Case(2, 2, Hq, Hkv, d, 8, 32, 1, 512, seed=100 + n)
    for layer in range(2):
        c.fill(layer, 0, n)
    for layer in range(2):
        assert_close(c.decode(layer, [n]), c.decode_ref(layer, [n]), f"n={n} layer {layer}")
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("chunk", [128, 256, 1024])
def test_chunk_size_does_not_change_the_result(chunk, monkeypatch):
    monkeypatch.setenv("POD_DECODE_CHUNK", str(chunk))
    c = Case(2, 2, 8, 2, 128, 16, 300, 1, 3000, seed=31)
    n = 2777
    for layer in range(2):
        c.fill(layer, 0, n)
        assert_close(c.decode(layer, [n]), c.decode_ref(layer, [n]), f"chunk {chunk} layer {layer}")


def test_ragged_batch_with_inactive_entry():
    c = Case(4, 2, 8, 2, 128, 8, 64, 5, 1200, seed=33)
    lens = [1100, 5, 0, 72, 73]
    for layer in range(4):
        for b, n in enumerate(lens):
            if n:
                c.fill(layer, b, n)
    for layer in range(4):
        out = c.decode(layer, lens)
        active = [b for b, n in enumerate(lens) if n]
        ref = np.zeros((5, 8, 128))
        # the oracle takes the active sequences one at a time (it has no notion of a skipped entry)
        for b in active:
            q = gen.bf16_bits(c.queries(layer, b, 1, "cpu", pos0=lens[b] - 1))
            qs = gen.bf16_bits(c.queries(layer - layer % 2, b, 1, "cpu", pos0=lens[b] - 1))
            k = gen.bf16_bits(c.keys(layer, b, lens[b], "cpu"))
            ka = gen.bf16_bits(c.keys(layer - layer % 2, b, lens[b], "cpu"))
            v = gen.bf16_bits(c.values(layer, b, lens[b], "cpu"))
            ref[b] = po.pod_attention(q, k, v, qs, ka, [lens[b] - 1], 8, 64, c.scale)[0]
        assert_close(out, ref, f"layer {layer}")
        assert torch.all(out[2] == 0)
    c.gpu.pod_cache_check()


def test_upper_layer_uses_the_lowest_layers_query_and_keys():
    c = Case(2, 2, 4, 2, 128, 8, 32, 1, 512, seed=35)
    n = 300
    for layer in range(2):
        c.fill(layer, 0, n)
    ctx = torch.tensor([n], dtype=torch.int32, device=c.dev)
    q1 = c.decode_queries(1, [n], c.dev)
    q0 = c.decode_queries(0, [n], c.dev)
    paper = c.gpu.pod_decode_attention(1, q1, q0, ctx, c.scale)
    own_q = c.gpu.pod_decode_attention(1, q1, q1, ctx, c.scale)      # "shared keys, own queries" variant
    assert_close(paper, c.decode_ref(1, [n]), "paper rule")
    assert (paper.float() - own_q.float()).abs().max() > 1e-2
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_decode_attention(1, q1, None, ctx, c.scale)
    assert e.value.code == pod.binding.ERR_INVALID_ARG


def test_wrong_context_length_is_flagged_not_faulted():
    c = Case(2, 2, 4, 2, 64, 8, 32, 2, 512, seed=36)
    for layer in range(2):
        c.fill(layer, 0, 100)
        c.fill(layer, 1, 50)
    out = c.decode(0, [100, 51])
    assert torch.all(out[1] == 0)
    assert_close(out[:1], c.decode_ref(0, [100])[:1], "valid entry")
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == pod.binding.ERR_STATE
    # lowest layer out of step with the upper layer: the host mirror knows, the call is refused
    c.append(1, [100, 50])
    with pytest.raises(pod.PodError) as e:
        c.decode(1, [101, 51])
    assert e.value.code == pod.binding.ERR_STATE


def test_decode_steps_with_demotion_match_oracle_every_step():
    """Config-2 pattern on a short context: append to both layers then decode both, 40 steps across S+W."""
    S, W = 16, 96
    c = Case(2, 2, 32, 8, 128, S, W, 1, 400, seed=37)
    n0 = S + W - 5
    for layer in range(2):
        c.fill(layer, 0, n0)
    for step in range(40):
        n = n0 + step + 1
        for layer in range(2):
            c.append(layer, [n - 1])
        for layer in range(2):
            assert_close(c.decode(layer, [n]), c.decode_ref(layer, [n]), f"step {step} layer {layer}")
    for layer in range(2):
        c.assert_cache_equal(layer, 0)
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("rate,scale", [(0.01, 8.0), (0.3, 16.0)])
def test_outlier_keys_do_not_break_the_softmax(rate, scale):
    """Rows of keys scaled by 8 or 16: logits tens of units above the rest, so the running maximum moves inside
    the tiles of a wave, between the waves of a workgroup and between the chunks the combine kernel merges;
    through the plain path, score reuse and the gate at tau = 1."""
    c = Case(4, 4, 8, 2, 128, 8, 64, 1, 3000, seed=38, outlier_rate=rate, outlier_scale=scale)
    n = 2900
    for layer in range(4):
        c.fill(layer, 0, n)
    scores = c.gpu.new_score_buffer()
    ctx_t = torch.tensor([n], dtype=torch.int32, device=c.dev)
    for layer in range(4):
        ref = c.decode_ref(layer, [n])
        assert_close(c.decode(layer, [n]), ref, f"layer {layer}")
        assert_close(c.decode_reuse(layer, [n], scores), ref, f"reuse layer {layer}")
    for layer in range(4):
        got = c.gpu.pod_decode_attention_gated(layer, c.decode_queries(layer, [n], c.dev), ctx_t, c.scale, 1.0, scores)
        assert_close(got, c.decode_ref(layer, [n]), f"gated layer {layer}")
    c.gpu.pod_cache_check()


# ---------------------------------------------------------------- score reuse (distant logits computed once per block)

@pytest.mark.parametrize("d,Hq,Hkv", [(128, 8, 2), (64, 4, 2), (128, 16, 1)])
@pytest.mark.parametrize("n", [7, 40, 41, 73, 457, 1500])
def test_score_reuse_matches_oracle_and_plain_path(d, Hq, Hkv, n):
    """G=4: the lowest layer writes its scaled distant logits, layers 1-3 read them instead of the shared keys."""
    c = Case(4, 4, Hq, Hkv, d, 8, 32, 1, 1600, seed=300 + n)
    for layer in range(4):
        c.fill(layer, 0, n)
    scores = c.gpu.new_score_buffer()
    for layer in range(4):
        out = c.decode_reuse(layer, [n], scores)
        assert_close(out, c.decode_ref(layer, [n]), f"n={n} layer {layer}")
        plain = c.decode(layer, [n])
        assert (out.float() - plain.float()).abs().max() <= 1.6e-2   # two bf16-rounded runs of the same sum
    c.gpu.pod_cache_check()


def test_score_reuse_ragged_batch_and_steps():
    c = Case(2, 2, 32, 8, 128, 16, 96, 3, 700, seed=41)
    lens = [650, 100, 330]
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    scores = c.gpu.new_score_buffer()
    for step in range(6):
        for layer in range(2):
            c.append(layer, [n + step for n in lens])
        ctx = [n + step + 1 for n in lens]
        for layer in range(2):
            assert_close(c.decode_reuse(layer, ctx, scores), c.decode_ref(layer, ctx), f"step {step} layer {layer}")
    c.gpu.pod_cache_check()


def test_score_reuse_detects_stale_scores():
    c = Case(4, 2, 4, 2, 64, 8, 32, 1, 512, seed=42)
    n = 300
    for layer in range(4):
        c.fill(layer, 0, n)
    scores = c.gpu.new_score_buffer()
    scores.zero_()
    out = c.decode_reuse(1, [n], scores)              # upper layer before its lowest layer ran
    assert torch.all(out == 0)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == pod.binding.ERR_STATE
    c.decode_reuse(0, [n], scores)                    # block 0's logits ...
    out = c.decode_reuse(3, [n], scores)              # ... are not block 1's
    assert torch.all(out == 0)
    with pytest.raises(pod.PodError):
        c.gpu.pod_cache_check()
    c.decode_reuse(2, [n], scores)
    assert_close(c.decode_reuse(3, [n], scores), c.decode_ref(3, [n]), "after the right lowest layer")
    c.gpu.pod_cache_check()
    ctx_t = torch.tensor([n], dtype=torch.int32, device=c.dev)
    out = c.gpu.pod_decode_attention_reuse(3, c.decode_queries(3, [n], c.dev), ctx_t, c.scale * 2, scores)
    assert torch.all(out == 0)                        # logits written with another scale are not this call's
    with pytest.raises(pod.PodError):
        c.gpu.pod_cache_check()
    with pytest.raises(pod.PodError) as e:            # undersized buffer
        c.gpu.pod_decode_attention_reuse(0, c.decode_queries(0, [n], c.dev),
                                         torch.tensor([n], dtype=torch.int32, device=c.dev), c.scale, scores[:256])
    assert e.value.code == pod.binding.ERR_CAPACITY


# ---------------------------------------------------------------- gated skip of distant tokens (appendix)

def _gated_setup(d, Hq, Hkv, S, W, lens, boost_heads, seed):
    """One block of two layers; the sink and recent keys of the kv heads in `boost_heads` are scaled x4 at the
    upper layer, so that those heads' gates sit near 1 while the others stay small."""
    B = len(lens)
    c = Case(2, 2, Hq, Hkv, d, S, W, B, max(lens) + 8, seed=seed)
    for layer in range(2):
        for b, n in enumerate(lens):
            k = c.keys(layer, b, n, "cpu").clone()
            v = c.values(layer, b, n, "cpu")
            if layer == 1:
                prox = torch.zeros(n, dtype=torch.bool)
                prox[:S] = True
                prox[max(n - W, 0):] = True
                for h in boost_heads:
                    k[prox, h] = k[prox, h] * 4                       # exact in bf16
            c.gpu.pod_cache_fill(layer, b, k.to(c.dev), v.to(c.dev))
            c.cpu.fill(layer, b, gen.bf16_bits(k), gen.bf16_bits(v))
    return c


def _gated_both(c, ctx, scores, tau):
    q1 = c.decode_queries(1, ctx, c.dev)
    ctx_t = torch.tensor(ctx, dtype=torch.int32, device=c.dev)
    got = c.gpu.pod_decode_attention_gated(1, q1, ctx_t, c.scale, tau, scores)
    flags = c.gpu.skip_flags(scores)[: len(ctx)].cpu().numpy()
    ref, g, skipped = c.cpu.decode_attention_gated(1, gen.bf16_bits(c.decode_queries(1, ctx, "cpu")),
                                                   gen.bf16_bits(c.decode_queries(0, ctx, "cpu")), ctx, c.scale, tau)
    return got, flags, ref, g, skipped


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 8, 2), (64, 4, 2)])
def test_gated_decode_matches_oracle_decisions_and_outputs(d, Hq, Hkv):
    S, W, lens = 8, 64, [700, 333, 150]
    c = _gated_setup(d, Hq, Hkv, S, W, lens, boost_heads=[0], seed=321)
    scores = c.gpu.new_score_buffer()
    ctx_t = torch.tensor(lens, dtype=torch.int32, device=c.dev)
    # lowest layer through the gated entry point: exact, and it leaves the distant sums for the gates
    out0 = c.gpu.pod_decode_attention_gated(0, c.decode_queries(0, lens, c.dev), ctx_t, c.scale, 0.5, scores)
    assert_close(out0, c.decode_ref(0, lens), "lowest layer")
    _, _, _, g, _ = _gated_both(c, lens, scores, 1.0)
    # thresholds: never, always, and one inside the widest gap between the heads' gates
    gs = np.sort(g.ravel())
    gaps = np.diff(gs)
    mid = float(gs[np.argmax(gaps)] + gaps.max() / 2)
    assert gaps.max() > 0.05, "the case must separate the heads"
    for tau in (1.0, 0.0, mid):
        got, flags, ref, g2, skipped = _gated_both(c, lens, scores, tau)
        assert np.abs(g2 - tau).min() > 0.02 or tau in (0.0, 1.0)    # no head near the threshold: the decision is unique
        np.testing.assert_array_equal(flags, skipped, err_msg=f"tau={tau}")
        assert_close(got, ref, f"tau={tau}")
    got, flags, ref, g2, skipped = _gated_both(c, lens, scores, mid)
    assert 0 < skipped.sum() < skipped.size                            # the threshold case really is mixed
    per_group = skipped.reshape(len(lens), Hkv, Hq // Hkv).sum(axis=2)
    assert (per_group == Hq // Hkv).any()                              # a kv head whose distant rows are not read at all
    c.gpu.pod_cache_check()


def test_gated_decode_mixed_decisions_inside_one_kv_head():
    """All query heads share one kv head, no boost: their gates differ by chance; a threshold inside the spread
    makes some heads of the same workgroup skip while the others need the distant rows."""
    S, W, lens = 8, 256, [900]
    c = _gated_setup(128, 8, 1, S, W, lens, boost_heads=[], seed=77)
    scores = c.gpu.new_score_buffer()
    ctx_t = torch.tensor(lens, dtype=torch.int32, device=c.dev)
    c.gpu.pod_decode_attention_gated(0, c.decode_queries(0, lens, c.dev), ctx_t, c.scale, 0.5, scores)
    _, _, _, g, _ = _gated_both(c, lens, scores, 1.0)
    gs = np.sort(g.ravel())
    gaps = np.diff(gs)
    i = int(np.argmax(gaps))
    assert gaps[i] > 0.01
    tau = float(gs[i] + gaps[i] / 2)
    got, flags, ref, g2, skipped = _gated_both(c, lens, scores, tau)
    assert 0 < skipped.sum() < skipped.size
    np.testing.assert_array_equal(flags, skipped)
    assert_close(got, ref, f"tau={tau}")


def test_gated_decode_without_distant_tokens_and_bad_tau():
    c = _gated_setup(64, 4, 2, 8, 64, [50], boost_heads=[], seed=5)     # 50 < S + W: nothing distant
    scores = c.gpu.new_score_buffer()
    ctx_t = torch.tensor([50], dtype=torch.int32, device=c.dev)
    c.gpu.pod_decode_attention_gated(0, c.decode_queries(0, [50], c.dev), ctx_t, c.scale, 0.0, scores)
    got = c.gpu.pod_decode_attention_gated(1, c.decode_queries(1, [50], c.dev), ctx_t, c.scale, 0.0, scores)
    assert_close(got, c.decode_ref(1, [50]), "no distant tokens")
    with pytest.raises(pod.PodError):
        c.gpu.pod_decode_attention_gated(1, c.decode_queries(1, [50], c.dev), ctx_t, c.scale, 1.5, scores)


def test_more_than_256_sequences_use_the_device_side_lengths():
    """Up to 256 sequences the host mirror's lengths travel as kernel arguments; beyond that both kernels read
    and validate the lengths on the device.  300 ragged sequences (some without, some with distant tokens),
    one token appended to all of them, both layers; then one wrong context length is caught on the device."""
    B, S, W = 300, 4, 16
    c = Case(2, 2, 4, 2, 64, S, W, B, 100, seed=61)
    lens = [1 + (37 * b) % 90 for b in range(B)]
    for layer in range(2):
        for b in range(B):
            c.fill(layer, b, lens[b])
        c.append(layer, lens)
    ctx = [n + 1 for n in lens]
    for layer in range(2):
        assert_close(c.decode(layer, ctx), c.decode_ref(layer, ctx), f"layer {layer}")
    for b in (0, 17, 299):
        c.assert_cache_equal(1, b)
    c.gpu.pod_cache_check()
    wrong = list(ctx)
    wrong[123] += 1
    out = c.decode(1, wrong)
    with pytest.raises(pod.PodError):
        c.gpu.pod_cache_check()
    ref = c.decode_ref(1, ctx)
    keep = [b for b in range(B) if b != 123]
    assert_close(out[keep], ref[keep], "the other sequences")
    assert float(out[123].float().abs().max()) == 0.0


def test_launch_bound_below_a_context_is_caught_on_the_device():
    """max_context_len sizes the launch; a sequence longer than it cannot be served by that launch: its row is
    zeroed and the flag raised, the sequences within the bound are exact.  An inactive long sequence is fine."""
    lens = [300, 90, 500]
    c = Case(2, 2, 4, 2, 64, 8, 32, 3, 600, seed=62)
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    ref = c.decode_ref(1, lens)
    out = c.decode(1, lens, max_context_len=320)            # sequence 2 holds 500 tokens
    with pytest.raises(pod.PodError):
        c.gpu.pod_cache_check()
    assert_close(out[:2], ref[:2], "sequences within the bound")
    assert float(out[2].float().abs().max()) == 0.0
    q = c.decode_queries(1, lens, c.dev)
    ctx = torch.tensor([300, 90, 0], dtype=torch.int32, device=c.dev)   # the long one sits this step out
    out = c.gpu.pod_decode_attention(1, q, c.shared_queries(1, lens, c.dev), ctx, c.scale, max_context_len=320)
    c.gpu.pod_cache_check()
    assert_close(out[:2], ref[:2], "with the long sequence inactive")
