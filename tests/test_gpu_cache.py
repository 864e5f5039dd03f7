"""GPU: cache update / construction kernels against the oracle's cache model, bit for bit."""
import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from pod_inputs import gen
from podcase import Case

pytestmark = pytest.mark.gpu


def test_generator_is_bit_identical_on_cpu_and_gpu():
    for fn in (gen.keys_bf16, gen.values_bf16, gen.queries_bf16):
        a = fn(3, 1, 2, 700, 4, 64, device="cpu", pos0=5)
        b = fn(3, 1, 2, 700, 4, 64, device="cuda:0", pos0=5)
        assert torch.equal(a, b.cpu())
    a = gen.keys_bf16(3, 0, 0, 300, 2, 128, device="cpu", rope_base=500000.0, rope_max_pos=512, outlier_rate=0.05)
    b = gen.keys_bf16(3, 0, 0, 300, 2, 128, device="cuda:0", rope_base=500000.0, rope_max_pos=512, outlier_rate=0.05)
    assert torch.equal(a, b.cpu())


@pytest.mark.parametrize("n", [1, 3, 4, 5, 11, 12, 13, 40, 97])
@pytest.mark.parametrize("d", [64, 128])
def test_fill_matches_oracle(n, d):
    c = Case(2, 2, 4, 2, d, 4, 8, 2, 128, seed=n)
    for layer in range(2):
        c.fill(layer, 1, n)
        c.assert_cache_equal(layer, 1)
        assert c.gpu.pod_cache_seq_len(layer, 1) == n
        assert c.gpu.pod_cache_seq_len(layer, 0) == 0
    c.gpu.pod_cache_check()


def test_appends_from_empty_equal_fill_and_oracle():
    n = 45   # S + W = 12: the ring wraps several times
    a = Case(4, 2, 4, 2, 64, 4, 8, 1, 64, seed=5)
    b = Case(4, 2, 4, 2, 64, 4, 8, 1, 64, seed=5)
    for layer in range(4):
        for p in range(n):
            a.append(layer, [p])
            if p in (0, 3, 4, 11, 12, 13, 20, 44):
                a.assert_cache_equal(layer, 0)
        b.fill(layer, 0, n)
        ea, eb = a.gpu.pod_cache_export_logical(layer, 0), b.gpu.pod_cache_export_logical(layer, 0)
        for name in ea:
            assert torch.equal(ea[name], eb[name]), name
    a.gpu.pod_cache_check()


def test_batched_appends_at_ragged_positions():
    c = Case(2, 2, 8, 2, 128, 3, 5, 3, 64, seed=9)
    lens = [2, 8, 30]
    for layer in range(2):
        for b, n in enumerate(lens):
            c.fill(layer, b, n)
    for step in range(12):
        for layer in range(2):
            c.append(layer, [n + step for n in lens])
    for layer in range(2):
        for b in range(3):
            c.assert_cache_equal(layer, b)
            assert c.gpu.pod_cache_seq_len(layer, b) == lens[b] + 12
    c.gpu.pod_cache_check()


def test_llama_shaped_demotion_sequence():
    """Config-2 shape on a short context: fill to S+W-2, then 70 appends crossing into demotion."""
    S, W = 64, 2048
    c = Case(2, 2, 32, 8, 128, S, W, 1, S + W + 100, seed=2)
    n0 = S + W - 2
    for layer in range(2):
        c.fill(layer, 0, n0)
    for step in range(70):
        for layer in range(2):
            c.append(layer, [n0 + step])
    for layer in range(2):
        c.assert_cache_equal(layer, 0)
    c.gpu.pod_cache_check()


def test_other_slots_and_layers_stay_untouched():
    c = Case(4, 2, 4, 2, 64, 4, 8, 3, 64, seed=4)
    c.gpu.buf.fill_(0x5A)
    c.gpu.pod_cache_reset(-1)
    before = c.gpu.buf.clone()
    c.fill(2, 1, 40)
    torch.cuda.synchronize()
    after = c.gpu.buf
    changed = (before != after).nonzero().flatten()
    # bytes written = header + (2*12 + 28 + 28) rows of 2 heads * 128 B  (layer 2 is a lowest layer)
    assert 0 < changed.numel() <= 16 + (2 * 12 + 28 + 28) * 2 * 128
    exp = c.gpu.pod_cache_export_logical(2, 1)
    assert exp["distK"].shape[0] == 28


def test_error_paths():
    c = Case(2, 2, 4, 2, 64, 4, 8, 2, 16, seed=6)
    E = pod.binding
    k = c.keys(0, 0, 1, c.dev)
    pos = torch.zeros(1, dtype=torch.int32, device=c.dev)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_append(2, k, k, pos)
    assert e.value.code == E.ERR_INVALID_ARG
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_fill(0, 0, c.keys(0, 0, 17, c.dev), c.values(0, 0, 17, c.dev))
    assert e.value.code == E.ERR_CAPACITY
    c.fill(0, 0, 16)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_fill(0, 0, c.keys(0, 0, 4, c.dev), c.values(0, 0, 4, c.dev))
    assert e.value.code == E.ERR_STATE
    with pytest.raises(pod.PodError) as e:    # slot 0 is full
        c.gpu.pod_cache_append(0, k, k, pos + 16)
    assert e.value.code == E.ERR_CAPACITY
    # wrong position inside the device array: kernel skips the entry and raises the flag
    c.gpu.pod_cache_check()
    c.gpu.pod_cache_append(1, k, k, pos + 3)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == E.ERR_STATE
    c.gpu.pod_cache_check()                    # flag was cleared
    # distant keys of an upper layer do not exist
    rc = pod.load().pod_cache_export_logical(c.gpu.handle, 1, 0, None, None, None, None, c.gpu.buf.data_ptr(), None, None)
    assert rc == E.ERR_INVALID_ARG
    c.gpu.pod_cache_reset(0)
    assert c.gpu.pod_cache_seq_len(0, 0) == 0
    c.gpu.pod_cache_fill(0, 0, c.keys(0, 0, 4, c.dev), c.values(0, 0, 4, c.dev))
    c.gpu.pod_cache_check()
