"""GPU: pod_prefill_attention against the CPU oracle, and the cache it builds."""
import math

import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from oracle import pod_oracle as po
from pod_inputs import gen
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu


def run_prefill(c, layer, n, write_cache=False, seq=0):
    lowest = layer - layer % c.G
    q, k, v = c.queries(layer, seq, n, c.dev), c.keys(layer, seq, n, c.dev), c.values(layer, seq, n, c.dev)
    qs = c.queries(lowest, seq, n, c.dev) if lowest != layer else None
    ks = c.keys(lowest, seq, n, c.dev) if lowest != layer else None
    return c.gpu.pod_prefill_attention(layer, seq, q, k, v, qs, ks, c.scale, write_cache=write_cache)


def ref_prefill(c, layer, n, rows, seq=0):
    lowest = layer - layer % c.G
    rows = np.asarray(rows)
    q = gen.bf16_bits(c.queries(layer, seq, n, "cpu")[rows])
    k, v = gen.bf16_bits(c.keys(layer, seq, n, "cpu")), gen.bf16_bits(c.values(layer, seq, n, "cpu"))
    qs = gen.bf16_bits(c.queries(lowest, seq, n, "cpu")[rows]) if lowest != layer else None
    ks = gen.bf16_bits(c.keys(lowest, seq, n, "cpu")) if lowest != layer else None
    return po.pod_attention(q, k, v, qs, ks, rows, c.S, c.W, c.scale)


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 4, 2), (64, 4, 1)])
@pytest.mark.parametrize("n", [1, 5, 63, 64, 65, 127, 128, 129, 300, 517])
def test_small_prompts_every_tile_kind(d, Hq, Hkv, n):
    """S=8, W=40 with 64-key tiles: sink-only, band, distant and mixed tiles all occur; ragged tails."""
    c = Case(2, 2, Hq, Hkv, d, 8, 40, 1, 600, seed=200 + n, with_oracle_cache=False)
    for layer in range(2):
        out = run_prefill(c, layer, n)
        assert_close(out, ref_prefill(c, layer, n, np.arange(n)), f"n={n} layer {layer}")


def test_window_larger_than_tile_and_prompt_shorter_than_window():
    c = Case(2, 2, 8, 2, 128, 64, 512, 1, 1500, seed=41, with_oracle_cache=False)
    for n in (400, 1500):
        out = run_prefill(c, 1, n)
        assert_close(out, ref_prefill(c, 1, n, np.arange(n)), f"n={n}")


def test_prefill_2048_llama_heads_full_compare():
    c = Case(2, 2, 32, 8, 128, 64, 512, 1, 2048, seed=42, with_oracle_cache=False)
    for layer in range(2):
        out = run_prefill(c, layer, 2048)
        assert_close(out, ref_prefill(c, layer, 2048, np.arange(2048)), f"layer {layer}")


def test_prefill_builds_the_same_cache_as_fill():
    c = Case(2, 2, 8, 2, 128, 8, 40, 2, 600, seed=43)
    n = 333
    for layer in range(2):
        run_prefill(c, layer, n, write_cache=True, seq=1)
        c.cpu.fill(layer, 1, gen.bf16_bits(c.keys(layer, 1, n, "cpu")), gen.bf16_bits(c.values(layer, 1, n, "cpu")))
        c.assert_cache_equal(layer, 1)
    with pytest.raises(pod.PodError) as e:
        run_prefill(c, 0, n, write_cache=True, seq=1)
    assert e.value.code == pod.binding.ERR_STATE
    c.gpu.pod_cache_check()


def test_prefill_then_decode_continues():
    c = Case(2, 2, 8, 2, 128, 8, 40, 1, 600, seed=44)
    n = 200
    for layer in range(2):
        run_prefill(c, layer, n, write_cache=True)
        c.cpu.fill(layer, 0, gen.bf16_bits(c.keys(layer, 0, n, "cpu")), gen.bf16_bits(c.values(layer, 0, n, "cpu")))
    for step in range(3):
        for layer in range(2):
            c.append(layer, [n + step])
        for layer in range(2):
            assert_close(c.decode(layer, [n + step + 1]), c.decode_ref(layer, [n + step + 1]), f"step {step} layer {layer}")
    c.gpu.pod_cache_check()


def test_prefill_argument_errors():
    c = Case(2, 2, 4, 2, 64, 4, 8, 1, 64, seed=45, with_oracle_cache=False)
    q, k, v = c.queries(1, 0, 32, c.dev), c.keys(1, 0, 32, c.dev), c.values(1, 0, 32, c.dev)
    with pytest.raises(pod.PodError) as e:      # upper layer with distant tokens needs the shared tensors
        c.gpu.pod_prefill_attention(1, 0, q, k, v, None, None, c.scale)
    assert e.value.code == pod.binding.ERR_INVALID_ARG
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_prefill_attention(1, 0, q, k, v, q, None, c.scale)
    assert e.value.code == pod.binding.ERR_INVALID_ARG
    big = c.queries(0, 0, 65, c.dev)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_prefill_attention(0, 0, big, c.keys(0, 0, 65, c.dev), c.values(0, 0, 65, c.dev), None, None, c.scale,
                                    write_cache=True)
    assert e.value.code == pod.binding.ERR_CAPACITY


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 8, 2), (64, 4, 2)])
@pytest.mark.parametrize("rate,scale", [(0.02, 8.0), (0.3, 16.0)])
def test_outlier_keys_move_the_reference_maximum(d, Hq, Hkv, rate, scale):
    """Rows of keys scaled by 8 or 16 give logits tens of units above the rest, arriving at random tiles: the
    running reference of the softmax has to move (and the accumulated sums to be rescaled) many times per row,
    which unit-variance inputs never ask for.  With 30 % outliers at x16 most probabilities underflow to zero."""
    n = 700
    c = Case(2, 2, Hq, Hkv, d, 8, 40, 1, n, seed=260, with_oracle_cache=False, outlier_rate=rate, outlier_scale=scale)
    for layer in range(2):
        assert_close(run_prefill(c, layer, n), ref_prefill(c, layer, n, np.arange(n)), f"layer {layer}")


def test_logits_growing_along_the_prompt():
    """Keys whose norm grows with the position: every tile raises the maximum of the rows that see it."""
    n, Hq, Hkv, d = 600, 4, 2, 128
    c = Case(2, 2, Hq, Hkv, d, 8, 40, 1, n, seed=261, with_oracle_cache=False)
    ramp = (1.0 + torch.arange(n, dtype=torch.float32) / 20.0).view(n, 1, 1)
    for layer in range(2):
        q = c.queries(layer, 0, n, c.dev)
        k = (c.keys(layer, 0, n, c.dev).float() * ramp.to(c.dev)).to(torch.bfloat16)
        v = c.values(layer, 0, n, c.dev)
        qs = c.queries(0, 0, n, c.dev) if layer else None
        ks = (c.keys(0, 0, n, c.dev).float() * ramp.to(c.dev)).to(torch.bfloat16) if layer else None
        out = c.gpu.pod_prefill_attention(layer, 0, q, k, v, qs, ks, c.scale)
        rows = np.arange(n)
        kc = (c.keys(layer, 0, n, "cpu").float() * ramp).to(torch.bfloat16)
        ksc = (c.keys(0, 0, n, "cpu").float() * ramp).to(torch.bfloat16) if layer else None
        ref = po.pod_attention(gen.bf16_bits(c.queries(layer, 0, n, "cpu")), gen.bf16_bits(kc),
                               gen.bf16_bits(c.values(layer, 0, n, "cpu")),
                               gen.bf16_bits(c.queries(0, 0, n, "cpu")) if layer else None,
                               gen.bf16_bits(ksc) if layer else None, rows, c.S, c.W, c.scale)
        assert_close(out, ref, f"layer {layer}")
