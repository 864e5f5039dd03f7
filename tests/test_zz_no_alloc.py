"""GPU: pod_decode_attention_static (split-K partials in the library's own fixed array, nothing allocated)
against pod_decode_attention with a caller's workspace: same kernels, so the outputs must be equal bit for bit;
both are also held to the oracle.  Two calls in a row, the second on a smaller input, so that what the first
call left in the shared array must not leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from pod_inputs import gen
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu


def _static(c, layer, ctx):
    q = c.decode_queries(layer, ctx, c.dev)
    qs = c.shared_queries(layer, ctx, c.dev)
    ctx_t = torch.tensor(ctx, dtype=torch.int32, device=c.dev)
    out = torch.full_like(q, float("nan"))
    L = pod.load()
    rc = L.pod_decode_attention_static(c.gpu.handle, layer, q.data_ptr(), qs.data_ptr() if qs is not None else None,
                                       ctx_t.data_ptr(), len(ctx), 0, c.scale, out.data_ptr(),
                                       torch.cuda.current_stream().cuda_stream)
    assert rc == 0, L.pod_last_error().decode()
    return out


def test_static_scratch_matches_the_workspace_entry_point_twice_in_a_row():
    big = Case(2, 2, 8, 2, 128, 16, 300, 2, 6000, seed=71)
    small = Case(2, 2, 4, 2, 64, 8, 32, 1, 512, seed=72)
    for layer in range(2):
        big.fill(layer, 0, 5555)
        big.fill(layer, 1, 1234)
        small.fill(layer, 0, 200)
    for case, ctx in ((big, [5555, 1234]), (small, [200])):   # the second call is the smaller one
        for layer in range(2):
            got = _static(case, layer, ctx)
            want = case.decode(layer, ctx)
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int16), want.view(torch.int16)), f"layer {layer} ctx {ctx}"
            assert_close(got, case.decode_ref(layer, ctx), f"static, layer {layer} ctx {ctx}")
        case.gpu.pod_cache_check()


def test_static_scratch_rejects_what_does_not_fit():
    # 64 sequences x 32 query heads x 128 at up to 40000 tokens: 40 split-K pieces each -> 42.6 MB of partials
    cfg = pod.make_config(1, 1, 32, 8, 128, 4, 60, 64, 40000)
    cache = pod.PodCache(cfg, "cuda:0")
    q = torch.zeros((64, 32, 128), dtype=torch.bfloat16, device="cuda:0")
    out = torch.zeros_like(q)
    ctx = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    with pytest.raises(pod.PodError) as e:
        cache.pod_decode_attention_static(0, q, None, ctx, 0.1, out, max_context_len=40000)
    assert e.value.code == pod.binding.ERR_CAPACITY and "scratch too small" in str(e.value)
