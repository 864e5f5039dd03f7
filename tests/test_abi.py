"""The C-ABI library: loads without a GPU, exports what include/pod.h declares, and its
host-only calls (sizes, memory accounting, argument checks) behave."""
import ctypes as C
import os
import re

import pytest

import paper_2412_02252_amd as pod
from oracle import pod_oracle as po

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pod.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pod_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = pod.load()
    names = declared_functions()
    assert len(names) >= 13
    for name in names:
        assert hasattr(L, name), name
    assert sorted(pod.EXPORTS) == names


def test_cache_bytes_cover_all_regions():
    cfg = pod.make_config(4, 2, 8, 2, 128, 4, 12, 3, 100)
    row = 128 * 2
    heads = 4 * 3 * 2
    payload = heads * 16 * row * 2 + heads * 84 * row + (heads // 2) * 84 * row
    total = pod.pod_cache_bytes(cfg)
    assert payload <= total <= payload + 4096


@pytest.mark.parametrize("L,G,S,W,n", [(32, 2, 64, 2048, 32768), (32, 4, 128, 4096, 131072), (2, 2, 16, 256, 2048),
                                       (2, 1, 16, 256, 2048), (4, 2, 16, 256, 100)])
def test_live_bytes_match_the_oracles_accounting(L, G, S, W, n):
    cfg = pod.make_config(L, G, 32, 8, 128, S, W, 1, max(n, 1))
    got = pod.pod_cache_live_bytes(cfg, n)
    want = po.cache_bytes_formula(L, G, 8, 128, S, W, n)
    assert got == (int(want[0]), int(want[1]))


@pytest.mark.parametrize("kw", [dict(num_layers=3), dict(num_q_heads=7), dict(head_dim=96), dict(window=0),
                                dict(max_context=0), dict(num_q_heads=64, num_kv_heads=2), dict(group_size=0)])
def test_bad_configs_are_rejected(kw):
    base = dict(num_layers=4, group_size=2, num_q_heads=8, num_kv_heads=2, head_dim=128, sink=4, window=8,
                max_batch=1, max_context=64)
    base.update(kw)
    with pytest.raises(pod.PodError) as e:
        pod.pod_cache_bytes(pod.make_config(**base))
    assert e.value.code == pod.binding.ERR_INVALID_ARG
    assert pod.load().pod_last_error()


def test_init_rejects_null_and_small_buffers():
    L = pod.load()
    cfg = pod.make_config(2, 2, 4, 2, 64, 4, 8, 1, 64)
    h = C.c_void_p()
    assert L.pod_cache_init(C.byref(cfg), None, 1 << 20, None, C.byref(h)) == pod.binding.ERR_INVALID_ARG
    assert L.pod_cache_init(C.byref(cfg), 256, 16, None, C.byref(h)) == pod.binding.ERR_CAPACITY
    assert L.pod_cache_init(C.byref(cfg), 257, 1 << 30, None, C.byref(h)) == pod.binding.ERR_INVALID_ARG


def test_selection_workspace_sizes_and_shape_checks():
    cfg = pod.make_config(2, 2, 32, 8, 128, 64, 2048, 1, 40000)
    n, obs, keep = 32768, 64, 1984
    b = pod.pod_select_workspace_bytes(cfg, n, obs, keep)
    rows = 2 * 8 * (keep + 2048) * 128 * 2                   # keys and values on their way during a compaction
    pooled = 8 * (n - 64 - 2048) * 4                         # one pooled vote per kv head and distant token
    assert b >= max(rows, pooled) and b % 256 == 0 and b < 2 * max(rows, pooled)
    assert pod.pod_select_workspace_bytes(cfg, n, obs, 1) >= pooled
    for bad in ((64 + 2048, obs, 1),                         # no distant token
                (n, 0, keep), (n, 2049, keep),               # observation window outside [1, W]
                (n, obs, 0), (n, obs, n - 64 - 2048 + 1),    # keep outside [1, n - S - W]
                (n, 1025, keep)):                            # more than 4096 query rows per kv head
        with pytest.raises(pod.PodError) as e:
            pod.pod_select_workspace_bytes(cfg, *bad)
        assert e.value.code == pod.binding.ERR_INVALID_ARG
    with pytest.raises(pod.PodError) as e:
        pod.pod_select_workspace_bytes(cfg, 40001, obs, keep)
    assert e.value.code == pod.binding.ERR_CAPACITY
