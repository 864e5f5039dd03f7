"""GPU: several tokens per cache update (pod_cache_append_many) and a prompt processed in chunks
(pod_prefill_attention_chunk), against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from oracle import pod_oracle as po
from pod_inputs import gen
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu


def kv_rows(c, layer, seq, p0, t, device):
    return c.keys(layer, seq, t, device, pos0=p0), c.values(layer, seq, t, device, pos0=p0)


def append_many_both(c, layer, starts, counts, T):
    """Sequences 0..B-1 take counts[b] tokens from position starts[b]; rows beyond counts[b] are filler."""
    B = len(starts)
    kd = torch.stack([kv_rows(c, layer, b, starts[b], T, c.dev)[0] for b in range(B)]).contiguous()
    vd = torch.stack([kv_rows(c, layer, b, starts[b], T, c.dev)[1] for b in range(B)]).contiguous()
    pos = torch.tensor(starts, dtype=torch.int32, device=c.dev)
    c.gpu.pod_cache_append_many(layer, kd, vd, pos, counts)
    kc = torch.stack([kv_rows(c, layer, b, starts[b], T, "cpu")[0] for b in range(B)])
    vc = torch.stack([kv_rows(c, layer, b, starts[b], T, "cpu")[1] for b in range(B)])
    c.cpu.append_many(layer, gen.bf16_bits(kc), gen.bf16_bits(vc), starts, counts)


@pytest.mark.parametrize("d,Hkv", [(128, 2), (64, 3)])
@pytest.mark.parametrize("chunks", [[1, 1, 1], [7, 40, 9], [48], [49, 1], [3, 120, 2, 60], [100, 100, 100], [8, 40, 40, 40]])
def test_append_many_matches_the_oracle_bit_for_bit(d, Hkv, chunks):
    """S = 8, W = 40: chunks shorter than, equal to and longer than the sink, the window and both; after every
    call all regions of every layer equal the oracle's lists, and lengths agree."""
    c = Case(2, 2, 2 * Hkv, Hkv, d, 8, 40, 2, 400, seed=300 + len(chunks))
    p = [0, 0]
    for t in chunks:
        counts = [t, max(t - 3, 0)]            # the second sequence lags: ragged counts
        for layer in range(2):
            append_many_both(c, layer, p, counts, t)
        p = [p[0] + counts[0], p[1] + counts[1]]
        for layer in range(2):
            for b in range(2):
                assert c.gpu.pod_cache_seq_len(layer, b) == p[b] == c.cpu.length(layer, b)
                if p[b]:
                    c.assert_cache_equal(layer, b)
    c.gpu.pod_cache_check()


def test_append_many_then_single_appends_and_decode():
    """Mixed use: chunk, single tokens, chunk; then decode attention on both layers agrees with the oracle."""
    c = Case(2, 2, 8, 2, 128, 8, 40, 1, 400, seed=311)
    p = 0
    for step in ([57], 1, 1, [44], 1, [130], 1):
        for layer in range(2):
            if isinstance(step, list):
                append_many_both(c, layer, [p], [step[0]], step[0])
            else:
                c.append(layer, [p])
        p += step[0] if isinstance(step, list) else 1
    for layer in range(2):
        c.assert_cache_equal(layer, 0)
        assert_close(c.decode(layer, [p]), c.decode_ref(layer, [p]), f"layer {layer}")


def test_append_many_head_wise_blocks():
    """Keys of demoted and directly stored distant tokens go to the store of each head's own block."""
    table = [[0, 0], [0, 1], [0, 1], [3, 1]]
    c = Case(4, 1, 4, 2, 128, 8, 40, 1, 300, seed=312, block_lowest=table)
    p = 0
    for t in (30, 100, 5, 77):
        for layer in range(4):
            append_many_both(c, layer, [p], [t], t)
        p += t
    for layer in range(4):
        c.assert_cache_equal(layer, 0)
    for layer in range(4):
        assert_close(c.decode(layer, [p]), c.decode_ref(layer, [p]), f"layer {layer}")


def test_append_many_contract_violations():
    c = Case(1, 1, 2, 1, 64, 4, 8, 2, 32, seed=313)
    k = torch.zeros(2, 6, 1, 64, dtype=torch.bfloat16, device=c.dev)
    pos = torch.zeros(2, dtype=torch.int32, device=c.dev)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_append_many(0, k, k, pos, [7, 0])             # more rows than the call carries
    assert e.value.code == pod.binding.ERR_INVALID_ARG
    c.gpu.pod_cache_append_many(0, k, k, pos, [6, 2])
    with pytest.raises(pod.PodError) as e:
        big = torch.zeros(2, 30, 1, 64, dtype=torch.bfloat16, device=c.dev)
        c.gpu.pod_cache_append_many(0, big, big, pos, [27, 0])        # 6 + 27 > 32
    assert e.value.code == pod.binding.ERR_CAPACITY
    # wrong start position for sequence 0: the kernel skips it and raises the flag; sequence 1 is stored
    c.gpu.pod_cache_append_many(0, k, k, torch.tensor([5, 2], dtype=torch.int32, device=c.dev), [3, 1])
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == pod.binding.ERR_STATE


# ---------------------------------------------------------------------------------------------- chunked prefill

def chunk_inputs(c, layer, seq, p0, t, device):
    src = c.lowest[layer]
    q, (k, v) = c.queries(layer, seq, t, device, pos0=p0), kv_rows(c, layer, seq, p0, t, device)
    if (src == layer).all():
        return q, k, v, None, None
    rep = c.Hq // c.Hkv
    qs = torch.stack([c.queries(int(src[h // rep]), seq, t, device, pos0=p0)[:, h] for h in range(c.Hq)], dim=1).contiguous()
    ks = torch.stack([c.keys(int(src[h]), seq, t, device, pos0=p0)[:, h] for h in range(c.Hkv)], dim=1).contiguous()
    return q, k, v, qs, ks


def run_chunks(c, chunks, seq=0, check_rows=None, small_workspace=False):
    """Every layer processes the prompt chunk by chunk (attention, then the chunk enters the cache) on the GPU
    and in the oracle's cache model; outputs are compared chunk by chunk.  small_workspace: the scratch sized for
    calls that store the chunk themselves (guard bands around it: the fixture checks them after the test)."""
    n_total = sum(chunks)
    ws = c.gpu.new_chunk_workspace(n_total, in_place_chunk=max(chunks) if small_workspace else 0)
    p = 0
    for t in chunks:
        for layer in range(c.L):
            q, k, v, qs, ks = chunk_inputs(c, layer, seq, p, t, c.dev)
            out = c.gpu.pod_prefill_attention_chunk(layer, seq, q, k, v, qs, ks, c.scale, ws, write_cache=True)
            qc, kc, vc, qsc, ksc = [gen.bf16_bits(x) if x is not None else None for x in chunk_inputs(c, layer, seq, p, t, "cpu")]
            ref = c.cpu.chunk_attention(layer, seq, qc, kc, vc, qsc, ksc, c.scale)
            assert_close(out, ref, f"chunk at {p} (+{t}) layer {layer}")
            counts = [0] * c.B
            counts[seq] = t
            c.cpu.append_many(layer, np.broadcast_to(kc, (c.B, *kc.shape)).copy(), np.broadcast_to(vc, (c.B, *vc.shape)).copy(),
                              [c.cpu.length(layer, b) for b in range(c.B)], counts)
        p += t
    for layer in range(c.L):
        c.assert_cache_equal(layer, seq)
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("in_place", [True, False], ids=["from_the_cache", "from_a_copy"])
@pytest.mark.parametrize("d,Hq,Hkv", [(128, 4, 2), (64, 4, 1)])
@pytest.mark.parametrize("chunks", [[300], [1, 1, 1], [5, 59, 1, 63], [64, 64, 64], [127, 2, 128, 43], [40, 200, 17], [129, 300]])
def test_chunked_prefill_matches_the_oracle(d, Hq, Hkv, chunks, in_place, monkeypatch):
    """S = 8, W = 40, 64-key tiles and 128-row query tiles: chunk starts inside tiles, chunks shorter and longer
    than the window, a first chunk that is the whole prompt.  Both ways the library has of finding the keys and
    values below the chunk: where the cache holds them (the chunk is stored first), or in a contiguous copy."""
    if not in_place:
        monkeypatch.setenv("POD_CHUNK_IN_PLACE", "0")   # read when the cache is created
    c = Case(2, 2, Hq, Hkv, d, 8, 40, 2, 600, seed=320 + len(chunks))
    run_chunks(c, chunks, seq=1)


@pytest.mark.parametrize("S,W,chunks", [
    (64, 128, [256, 256, 128, 64]),          # every region edge on a 64-key tile edge: no tile is staged
    (64, 128, [64, 64, 64, 64, 64, 64]),     # chunks shorter than the window, the ring wraps on a tile edge
    (64, 192, [100, 156, 64, 192, 1]),       # edges inside tiles after an odd first chunk
    (0, 64, [64, 128, 70]),                  # no sink tokens
    (128, 64, [32, 96, 64, 200]),            # sink longer than the window
    (8, 40, [700]),                          # one chunk far longer than the window: most of it goes straight to the distant stores
    (8, 300, [50, 100, 100]),                # everything still inside the window (no distant token)
])
def test_chunked_prefill_region_edges_and_key_tiles(S, W, chunks, monkeypatch):
    """Where the sink, the distant stores, the rows kept for this call and the two parts of the ring meet, relative to
    the 64-key tiles the kernel requests by one address each."""
    monkeypatch.delenv("POD_CHUNK_IN_PLACE", raising=False)   # (read when the cache is created: this is about the usual way)
    c = Case(2, 2, 4, 2, 128, S, W, 1, 1024, seed=340 + len(chunks))
    run_chunks(c, chunks, small_workspace=True)


def test_chunked_prefill_g4_block_three_upper_layers():
    c = Case(4, 4, 8, 2, 128, 16, 100, 1, 700, seed=347)
    run_chunks(c, [130, 64, 300, 77])


def test_chunked_prefill_equals_one_shot_prefill_rows():
    """Same prompt in one call and in chunks: the oracle's rows are the same by definition; the two GPU paths
    agree with each other to bf16 rounding of the same sums taken in a different tile order."""
    c = Case(2, 2, 8, 2, 128, 64, 512, 2, 1600, seed=331, with_oracle_cache=False)
    n, cuts = 1500, [0, 700, 701, 1100, 1500]
    ws = c.gpu.new_chunk_workspace(n)
    t = {}
    for layer in range(2):
        t[layer] = (c.queries(layer, 0, n, c.dev), c.keys(layer, 0, n, c.dev), c.values(layer, 0, n, c.dev))
    whole = {}
    for layer in range(2):
        q, k, v = t[layer]
        whole[layer] = c.gpu.pod_prefill_attention(layer, 0, q, k, v, t[0][0] if layer else None, t[0][1] if layer else None, c.scale)
    for a, b in zip(cuts[:-1], cuts[1:]):
        for layer in range(2):
            q, k, v = (x[a:b].contiguous() for x in t[layer])
            qs = t[0][0][a:b].contiguous() if layer else None
            ks = t[0][1][a:b].contiguous() if layer else None
            part = c.gpu.pod_prefill_attention_chunk(layer, 1, q, k, v, qs, ks, c.scale, ws, write_cache=True)
            diff = (part.float() - whole[layer][a:b].float()).abs()
            assert diff.max().item() <= 2e-2 and diff.mean().item() <= 1e-3, (layer, a, b, diff.max().item())
    c.gpu.pod_cache_check()


def test_chunked_prefill_head_wise_blocks_and_deferred_cache_writes():
    """Head-wise table; the lowest layers store the chunk before (write_cache) or after the upper layers run."""
    table = [[0, 0], [0, 1], [0, 1], [3, 1]]
    for defer in (False, True):
        c = Case(4, 1, 4, 2, 128, 8, 40, 1, 400, seed=332, block_lowest=table)
        ws = c.gpu.new_chunk_workspace(330)
        p = 0
        for t in (100, 30, 200):
            held = []
            for layer in range(4):
                q, k, v, qs, ks = chunk_inputs(c, layer, 0, p, t, c.dev)
                out = c.gpu.pod_prefill_attention_chunk(layer, 0, q, k, v, qs, ks, c.scale, ws, write_cache=not defer)
                qc, kc, vc, qsc, ksc = [gen.bf16_bits(x) if x is not None else None for x in chunk_inputs(c, layer, 0, p, t, "cpu")]
                assert_close(out, c.cpu.chunk_attention(layer, 0, qc, kc, vc, qsc, ksc, c.scale), f"defer={defer} p={p} layer {layer}")
                if defer:
                    held.append((layer, k, v, kc, vc))
                else:
                    c.cpu.append_many(layer, kc[None], vc[None], [p])
            for layer, k, v, kc, vc in held:
                c.gpu.pod_cache_append_many(layer, k[None].contiguous(), v[None].contiguous(),
                                            torch.tensor([p], dtype=torch.int32, device=c.dev))
                c.cpu.append_many(layer, kc[None], vc[None], [p])
            p += t
        for layer in range(4):
            c.assert_cache_equal(layer, 0)
        c.gpu.pod_cache_check()


def test_chunked_prefill_then_decode():
    c = Case(2, 2, 8, 2, 128, 8, 40, 1, 600, seed=333)
    run_chunks(c, [150, 90, 61])
    n = 302   # one more token after the 301 of the prompt
    for layer in range(2):
        c.append(layer, [n - 1])
    for layer in range(2):
        assert_close(c.decode(layer, [n]), c.decode_ref(layer, [n]), f"layer {layer}")


def test_chunked_prefill_contract_violations():
    c = Case(2, 2, 4, 2, 128, 8, 40, 1, 200, seed=334, with_oracle_cache=False)
    ws = c.gpu.new_chunk_workspace(200)
    q, k, v, qs, ks = chunk_inputs(c, 1, 0, 0, 100, c.dev)
    with pytest.raises(pod.PodError) as e:        # upper layer, distant tokens, no shared tensors
        c.gpu.pod_prefill_attention_chunk(1, 0, q, k, v, None, None, c.scale, ws)
    assert e.value.code == pod.binding.ERR_INVALID_ARG
    with pytest.raises(pod.PodError) as e:        # workspace too small
        c.gpu.pod_prefill_attention_chunk(1, 0, q, k, v, qs, ks, c.scale, ws[:1024])
    assert e.value.code == pod.binding.ERR_CAPACITY
    c.gpu.pod_cache_fill(0, 0, c.keys(0, 0, 50, c.dev), c.values(0, 0, 50, c.dev))
    with pytest.raises(pod.PodError) as e:        # lowest layer holds 50 tokens, this layer 0, chunk 100: out of step
        c.gpu.pod_prefill_attention_chunk(1, 0, q, k, v, qs, ks, c.scale, ws)
    assert e.value.code == pod.binding.ERR_STATE
    q2, k2, v2, _, _ = chunk_inputs(c, 0, 0, 50, 160, c.dev)
    with pytest.raises(pod.PodError) as e:        # 50 + 160 > max_context
        c.gpu.pod_prefill_attention_chunk(0, 0, q2, k2, v2, None, None, c.scale, ws)
    assert e.value.code == pod.binding.ERR_CAPACITY
    with pytest.raises(pod.PodError):
        pod.pod_prefill_chunk_workspace_bytes(c.cfg, 201)
    with pytest.raises(pod.PodError):
        pod.pod_prefill_chunk_in_place_bytes(c.cfg, 100, 101)
    assert pod.pod_prefill_chunk_in_place_bytes(c.cfg, 200, 50) < pod.pod_prefill_chunk_workspace_bytes(c.cfg, 200)


def test_chunk_on_a_mirror_that_is_ahead_of_the_device_stores_nothing_and_raises_the_flag(monkeypatch):
    """A rejected append leaves the host mirror one token ahead of the stored length.  The next chunk call then starts
    from the wrong position: both of its launches see that, the cache keeps its content, the flag goes up."""
    monkeypatch.delenv("POD_CHUNK_IN_PLACE", raising=False)   # (read when the cache is created: this is about the usual way)
    c = Case(1, 1, 4, 2, 128, 8, 40, 1, 400, seed=335)
    run_chunks(c, [100])
    k1 = c.keys(0, 0, 1, c.dev, pos0=100).contiguous()
    c.gpu.pod_cache_append(0, k1, k1, torch.tensor([7], dtype=torch.int32, device=c.dev))   # wrong position: rejected on the device
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == pod.binding.ERR_STATE                    # (the check clears the flag; the mirror says 101)
    ws = c.gpu.new_chunk_workspace(400)
    q, k, v, _, _ = chunk_inputs(c, 0, 0, 101, 150, c.dev)
    c.gpu.pod_prefill_attention_chunk(0, 0, q, k, v, None, None, c.scale, ws, write_cache=True)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == pod.binding.ERR_STATE
    c.gpu.pod_cache_sync_lengths()
    c.assert_cache_equal(0, 0)                                      # still the 100 tokens of the first chunk


def test_append_many_more_sequences_than_one_launch_covers():
    """Counts travel as kernel arguments, 256 sequences per launch: 300 sequences take two launches."""
    B, T = 300, 5
    c = Case(1, 1, 2, 1, 64, 4, 8, B, 40, seed=340)
    starts = [0] * B
    for rnd in range(3):
        counts = [(b + rnd) % (T + 1) for b in range(B)]
        append_many_both(c, 0, starts, counts, T)
        starts = [s + k for s, k in zip(starts, counts)]
    for b in (0, 1, 255, 256, 257, 299):
        assert c.gpu.pod_cache_seq_len(0, b) == starts[b] == c.cpu.length(0, b)
        if starts[b]:
            c.assert_cache_equal(0, b)
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_sequences_of_cache_updates(seed):
    """Random mixes of single appends, ragged multi-token appends, resets of one slot and prompt fills, every
    layer kept in step: after each operation lengths agree, and at intervals every region of every slot is
    compared bit for bit and decode attention is compared on all sequences."""
    rng = np.random.default_rng(seed)
    L, G, Hq, Hkv, d, S, W, B, cap = 2, 2, 4, 2, 64, 6, 24, 3, 160
    c = Case(L, G, Hq, Hkv, d, S, W, B, cap, seed=350 + seed)
    n = [0] * B
    for step in range(60):
        op = rng.choice(["append", "many", "many", "reset", "fill"], p=[0.3, 0.25, 0.2, 0.1, 0.15])
        if op == "append" and max(n) < cap:
            for layer in range(L):
                c.append(layer, list(n))
            n = [x + 1 for x in n]
        elif op == "many":
            T = int(rng.integers(1, 40))
            counts = [int(min(rng.integers(0, T + 1), cap - n[b])) for b in range(B)]
            for layer in range(L):
                append_many_both(c, layer, list(n), counts, T)
            n = [x + k for x, k in zip(n, counts)]
        elif op == "reset":
            b = int(rng.integers(0, B))
            c.gpu.pod_cache_reset(b)
            c.cpu.reset(b)
            n[b] = 0
        elif op == "fill":
            empty = [b for b in range(B) if n[b] == 0]
            if empty:
                b, m = empty[0], int(rng.integers(1, 100))
                for layer in range(L):
                    c.fill(layer, b, m)
                n[b] = m
        for layer in range(L):
            for b in range(B):
                assert c.gpu.pod_cache_seq_len(layer, b) == n[b] == c.cpu.length(layer, b), (step, op)
        if step % 6 == 5 or step == 59:
            for layer in range(L):
                for b in range(B):
                    if n[b]:
                        c.assert_cache_equal(layer, b)
            if min(n) >= 1:
                for layer in range(L):
                    assert_close(c.decode(layer, list(n)), c.decode_ref(layer, list(n)), f"step {step} layer {layer}")
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 8, 2), (64, 4, 2)])
def test_chunked_prefill_with_outlier_keys(d, Hq, Hkv):
    """Outlier keys (x16, 30 % of the rows) in the cache and in the chunks: the softmax reference moves inside
    chunk calls whose keys come from the gathered copies."""
    c = Case(2, 2, Hq, Hkv, d, 8, 40, 1, 700, seed=360, outlier_rate=0.3, outlier_scale=16.0)
    run_chunks(c, [130, 257, 1, 200])
