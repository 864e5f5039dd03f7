"""GPU: the entry points captured into a HIP graph (no allocation, no synchronisation, no host-dependent
state inside the kernels beyond what a capture fixes) give the eager results on every replay.

A captured call freezes its host-side arguments, among them the host mirror's sequence lengths, so a graph is
valid for the cache state it was captured at: between replays the test brings the cache back to that state
with ordinary eager calls, and every replay is compared with the eager run."""
import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from pod_inputs import gen
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu


def _prepare(c, n0):
    c.gpu.pod_cache_reset(-1)
    for layer in range(c.L):
        for b in range(c.B):
            c.gpu.pod_cache_fill(layer, b, c.keys(layer, b, n0[b], c.dev), c.values(layer, b, n0[b], c.dev))


def _step_inputs(c, n0, steps):
    ins = []
    for s in range(steps):
        pos = [n + s for n in n0]
        e = dict(pos=torch.tensor(pos, dtype=torch.int32, device=c.dev),
                 ctx=torch.tensor([p + 1 for p in pos], dtype=torch.int32, device=c.dev), n=max(pos) + 1)
        for layer in range(c.L):
            e[f"k{layer}"] = torch.cat([c.keys(layer, b, 1, c.dev, pos0=p) for b, p in enumerate(pos)]).contiguous()
            e[f"v{layer}"] = torch.cat([c.values(layer, b, 1, c.dev, pos0=p) for b, p in enumerate(pos)]).contiguous()
            e[f"q{layer}"] = c.decode_queries(layer, [p + 1 for p in pos], c.dev)
            e[f"o{layer}"] = torch.zeros_like(e[f"q{layer}"])
        ins.append(e)
    return ins


@pytest.mark.parametrize("rounds", ["one-round", "several-rounds"])
@pytest.mark.parametrize("variant", ["plain", "step", "reuse", "gated", "step_reuse"])
def test_decode_steps_in_a_graph_equal_eager_steps_on_every_replay(variant, rounds, monkeypatch):
    """several-rounds: the launch shapes of large batches (a second kernel merges the partials; plain calls and the upper
    layers' reuse steps split the rows evenly over the workgroups), forced on this small shape through the environment."""
    if rounds == "several-rounds":
        monkeypatch.setenv("POD_DECODE_FUSED", "0")
    n0, steps = [700, 150], 3
    c = Case(2, 2, 8, 2, 128, 8, 64, 2, 800, seed=900)
    ins = _step_inputs(c, n0, steps)
    scores = c.gpu.new_score_buffer()

    def run(e):
        if variant == "step_reuse":
            for layer in range(2):
                c.gpu.pod_decode_step_reuse(layer, e[f"k{layer}"], e[f"v{layer}"], e[f"q{layer}"], e["pos"], c.scale, scores,
                                            out=e[f"o{layer}"], max_context_len=e["n"])
            return
        if variant == "step":
            for layer in range(2):
                c.gpu.pod_decode_step(layer, e[f"k{layer}"], e[f"v{layer}"], e[f"q{layer}"], e["q0"] if layer else None, e["pos"],
                                      c.scale, out=e[f"o{layer}"], max_context_len=e["n"])
            return
        for layer in range(2):
            c.gpu.pod_cache_append(layer, e[f"k{layer}"], e[f"v{layer}"], e["pos"])
        for layer in range(2):
            q, o = e[f"q{layer}"], e[f"o{layer}"]
            if variant == "plain":
                c.gpu.pod_decode_attention(layer, q, e["q0"] if layer else None, e["ctx"], c.scale, out=o, max_context_len=e["n"])
            elif variant == "reuse":
                c.gpu.pod_decode_attention_reuse(layer, q, e["ctx"], c.scale, scores, out=o, max_context_len=e["n"])
            else:
                c.gpu.pod_decode_attention_gated(layer, q, e["ctx"], c.scale, 0.6, scores, out=o, max_context_len=e["n"])

    _prepare(c, n0)
    for e in ins:
        run(e)
    torch.cuda.synchronize()
    eager = [[e[f"o{layer}"].clone() for layer in range(2)] for e in ins]
    final = {(layer, b): c.gpu.pod_cache_export_logical(layer, b) for layer in range(2) for b in range(2)}
    c.gpu.pod_cache_check()

    _prepare(c, n0)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for e in ins:
            run(e)
    for replay in range(3):
        for e in ins:
            for layer in range(2):
                e[f"o{layer}"].zero_()
        g.replay()
        c.gpu.pod_cache_sync_lengths()       # a replay does not advance the host mirror
        for s, e in enumerate(ins):
            for layer in range(2):
                assert torch.equal(e[f"o{layer}"], eager[s][layer]), (variant, replay, s, layer)
        for (layer, b), want in final.items():
            got = c.gpu.pod_cache_export_logical(layer, b)
            for name in want:
                assert torch.equal(got[name], want[name]), (variant, replay, layer, b, name)
        c.gpu.pod_cache_check()
        # eager work between the replays: back to the state the graph was captured at (the host mirror too)
        _prepare(c, n0)
        torch.cuda.synchronize()


def test_chunked_prefill_in_a_graph_equals_eager_on_every_replay():
    c = Case(2, 2, 8, 2, 128, 8, 64, 1, 700, seed=901, with_oracle_cache=False)
    cuts = [0, 200, 329, 600]
    n = cuts[-1]
    q = [c.queries(l, 0, n, c.dev) for l in range(2)]
    k = [c.keys(l, 0, n, c.dev) for l in range(2)]
    v = [c.values(l, 0, n, c.dev) for l in range(2)]
    out = [torch.zeros_like(q[0]) for _ in range(2)]
    ws = c.gpu.new_chunk_workspace(n)

    def run():
        for a, b in zip(cuts[:-1], cuts[1:]):
            for l in range(2):
                c.gpu.pod_prefill_attention_chunk(l, 0, q[l][a:b], k[l][a:b], v[l][a:b], q[0][a:b] if l else None,
                                                  k[0][a:b] if l else None, c.scale, ws, out=out[l][a:b], write_cache=True)

    run()
    torch.cuda.synchronize()
    eager = [o.clone() for o in out]
    final = {l: c.gpu.pod_cache_export_logical(l, 0) for l in range(2)}
    c.gpu.pod_cache_reset(-1)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for replay in range(3):
        for o in out:
            o.zero_()
        ws.zero_()
        g.replay()
        c.gpu.pod_cache_sync_lengths()
        assert c.gpu.pod_cache_seq_len(1, 0) == n
        for l in range(2):
            assert torch.equal(out[l], eager[l]), (replay, l)
            got = c.gpu.pod_cache_export_logical(l, 0)
            for name in final[l]:
                assert torch.equal(got[name], final[l][name]), (replay, l, name)
        c.gpu.pod_cache_check()
        c.gpu.pod_cache_reset(-1)          # eager work between replays: empty again, as at capture
        torch.cuda.synchronize()


@pytest.mark.parametrize("variant", ["step", "append+decode", "step_reuse"])
def test_one_captured_step_graph_serves_successive_tokens(variant):
    """Lengths from device arrays only (pod_cache_set_length_source(1)): ONE captured step (both layers of a block, two
    ragged sequences) is replayed for 8 successive tokens; between replays only device memory changes (positions,
    context lengths, the new token's k, v and the queries are copied into the buffers the graph reads).  Every replay is
    compared with the oracle's append + attention, the stores at the end bit for bit."""
    S, W = 8, 64
    n0 = [S + W - 3, 700]            # the first sequence crosses S + W during the replays
    c = Case(2, 2, 8, 2, 128, S, W, 2, 900, seed=902)
    for layer in range(2):
        for b, n in enumerate(n0):
            c.fill(layer, b, n)
    c.gpu.pod_cache_set_length_source(1)
    pos = torch.tensor(n0, dtype=torch.int32, device=c.dev)
    ctx = torch.tensor([n + 1 for n in n0], dtype=torch.int32, device=c.dev)
    k = [torch.zeros((2, 2, 128), dtype=torch.bfloat16, device=c.dev) for _ in range(2)]
    v = [torch.zeros_like(k[0]) for _ in range(2)]
    q = [torch.zeros((2, 8, 128), dtype=torch.bfloat16, device=c.dev) for _ in range(2)]
    out = [torch.zeros_like(q[0]) for _ in range(2)]
    bound = max(n0) + 8              # the launch is sized for the longest context any replay will see

    def load_inputs(s):
        p = [n + s for n in n0]
        pos.copy_(torch.tensor(p, dtype=torch.int32, device=c.dev))
        ctx.copy_(torch.tensor([x + 1 for x in p], dtype=torch.int32, device=c.dev))
        for layer in range(2):
            k[layer].copy_(torch.cat([c.keys(layer, b, 1, c.dev, pos0=x) for b, x in enumerate(p)]))
            v[layer].copy_(torch.cat([c.values(layer, b, 1, c.dev, pos0=x) for b, x in enumerate(p)]))
            q[layer].copy_(c.decode_queries(layer, [x + 1 for x in p], c.dev))
        return p

    scores = c.gpu.new_score_buffer()

    def one_step():
        for layer in range(2):
            if variant == "step_reuse":
                c.gpu.pod_decode_step_reuse(layer, k[layer], v[layer], q[layer], pos, c.scale, scores, out=out[layer],
                                            max_context_len=bound)
                continue
            if variant == "step":
                c.gpu.pod_decode_step(layer, k[layer], v[layer], q[layer], q[0] if layer else None, pos, c.scale,
                                      out=out[layer], max_context_len=bound)
            else:
                c.gpu.pod_cache_append(layer, k[layer], v[layer], pos)
        if variant == "append+decode":
            for layer in range(2):
                c.gpu.pod_decode_attention(layer, q[layer], q[0] if layer else None, ctx, c.scale, out=out[layer],
                                           max_context_len=bound)

    load_inputs(0)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        one_step()
    for s in range(8):
        p = load_inputs(s)
        for o in out:
            o.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for layer in range(2):
            kc = torch.cat([c.keys(layer, b, 1, "cpu", pos0=x) for b, x in enumerate(p)])
            vc = torch.cat([c.values(layer, b, 1, "cpu", pos0=x) for b, x in enumerate(p)])
            c.cpu.append(layer, gen.bf16_bits(kc), gen.bf16_bits(vc), p)
        for layer in range(2):
            assert_close(out[layer], c.decode_ref(layer, [x + 1 for x in p]), f"{variant} replay {s} layer {layer}")
    c.gpu.pod_cache_check()
    c.gpu.pod_cache_sync_lengths()
    c.gpu.pod_cache_set_length_source(0)
    for layer in range(2):
        for b in range(2):
            assert c.gpu.pod_cache_seq_len(layer, b) == n0[b] + 8
            c.assert_cache_equal(layer, b)
