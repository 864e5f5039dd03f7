"""GPU: token selection on the distant store (pod_select_votes, pod_select_top, pod_cache_compact) against the CPU
oracle (oracle/pod_select.py for the selection, oracle/pod_oracle.c for the cache and the attention after it).

What is compared how:
  votes       element by element.  Inputs are bf16 (exact on both sides); the GPU accumulates the d-term dot products
              in fp32 (relative error of a logit's terms ~ d 2^-24, i.e. <= 1e-5 absolute at |q.k| scale ~ 1 after
              scaling), takes exp2 in fp32 (2^-22 relative) and sums <= 4096 weights in fp32: a vote is within 1e-4
              of its value; the bound used is |got - ref| <= 2e-4 ref + 1e-9.
  selection   an integer decided by floating point.  On votes that both sides hold in the same precision (float32
              arrays made by the test) the result must be identical, ties included.  On the GPU's own votes the
              selection must be VALID for the oracle's float64 pooled votes within the vote tolerance: nothing
              selected is below the keep-th largest minus eps, nothing left out is above it plus eps; where no vote
              lies within eps of the threshold that means equality, which is asserted too.
  compaction  bit-exact, from the oracle's selection (uploaded), against the oracle's cache of the shorter sequence;
              decode steps after it against the oracle's attention to the usual bounds.
"""
import math

import numpy as np
import pytest
import torch

import paper_2412_02252_amd as pod
from oracle import pod_oracle as po
from oracle import pod_select as ps
from pod_inputs import gen
from podcase import Case, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def assert_votes_close(got, ref, what=""):
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    bad = np.abs(got - ref) > 2e-4 * ref + 1e-9
    assert not bad.any(), f"{what}: {int(bad.sum())} votes off, worst {np.abs(got - ref).max():.3e} at ref {ref[bad][0]:.3e}"


def assert_valid_selection(sel, pooled_ref, keep, eps_rel, what=""):
    """sel: int [keep] from the GPU; pooled_ref: float64 [m].  Returns True if the selection is forced (no near-tie)."""
    m = pooled_ref.shape[0]
    s = sel.tolist()
    assert s == sorted(set(s)) and len(s) == keep and 0 <= s[0] and s[-1] < m, f"{what}: not an ascending set of {keep}"
    thr = np.sort(pooled_ref)[::-1][keep - 1]
    eps = eps_rel * max(thr, pooled_ref.max() * 1e-3)
    inside = np.zeros(m, dtype=bool)
    inside[s] = True
    assert (pooled_ref[inside] >= thr - eps).all(), f"{what}: a selected token is below the threshold"
    assert (pooled_ref[~inside] <= thr + eps).all(), f"{what}: a token above the threshold was left out"
    return not (np.abs(pooled_ref - thr) <= eps).sum() > 1


@pytest.mark.parametrize("d,Hq,Hkv,S,W,n,obs", [
    (128, 8, 2, 4, 40, 700, 32),       # rep 4, several key pieces, ragged tail
    (64, 6, 3, 3, 33, 431, 5),         # rep 2, 10 query rows: one padded row block
    (128, 16, 1, 8, 64, 1000, 64),     # rep 16: 1024 query rows, 32 row blocks
    (128, 5, 5, 0, 16, 300, 16),       # no sink, rep 1
    (128, 5, 1, 2, 70, 900, 60),       # rep 5: 300 query rows = one full chunk of 256 and a second of 44 (two row blocks, the last ragged)
    (64, 12, 2, 1, 64, 520, 64),       # rep 6: 384 rows, d 64
    (64, 4, 4, 16, 100, 117, 1),       # a single distant token, a single query
])
def test_votes_match_the_oracle(d, Hq, Hkv, S, W, n, obs):
    cfg = pod.make_config(1, 1, Hq, Hkv, d, S, W, 1, n + 8)
    cache = pod.PodCache(cfg, DEV, guard_bytes=4096)
    scale = 1.0 / math.sqrt(d)
    q = gen.queries_bf16(41, 0, 0, n, Hq, d, device=DEV)[n - obs:].contiguous()
    k = gen.keys_bf16(41, 0, 0, n, Hkv, d, device=DEV)
    ws = cache.new_select_workspace(n, obs, 1)
    votes = cache.pod_select_votes(0, q, k, scale, ws)
    torch.cuda.synchronize()
    ref = ps.distant_votes(gen.bf16_bits(gen.queries_bf16(41, 0, 0, n, Hq, d)[n - obs:]),
                           gen.bf16_bits(gen.keys_bf16(41, 0, 0, n, Hkv, d)), S, W, scale)
    assert_votes_close(votes.cpu().numpy().astype(np.float64), ref, f"d={d} n={n}")
    again = cache.pod_select_votes(0, q, k, scale, ws)          # fixed summation order: the same bits every time
    assert torch.equal(votes, again)


def test_votes_of_a_peaked_prompt_with_large_logits():
    # one key per head draws nearly all attention (logit ~ +60 above the rest): maxima move, weights span 26 decades
    d, Hq, Hkv, S, W, n, obs = 128, 4, 2, 2, 20, 500, 8
    cfg = pod.make_config(1, 1, Hq, Hkv, d, S, W, 1, n)
    cache = pod.PodCache(cfg, DEV, guard_bytes=4096)
    q = gen.queries_bf16(43, 0, 0, n, Hq, d)[n - obs:].clone()
    k = gen.keys_bf16(43, 0, 0, n, Hkv, d).clone()
    k[311, 0] = (q[3, 0].float() * 6).to(torch.bfloat16)
    k[37, 1] = (q[0, 3].float() * 6).to(torch.bfloat16)
    scale = 1.0 / math.sqrt(d)
    votes = cache.pod_select_votes(0, q.to(DEV).contiguous(), k.to(DEV).contiguous(), scale, cache.new_select_workspace(n, obs, 1))
    ref = ps.distant_votes(gen.bf16_bits(q), gen.bf16_bits(k), S, W, scale)
    assert ref[0].argmax() == 311 - S and ref[1].argmax() == 37 - S
    assert_votes_close(votes.cpu().numpy().astype(np.float64), ref, "peaked")


@pytest.mark.parametrize("m,keep", [(40000, 3000), (32769, 1), (5000, 1), (5000, 700), (5000, 5000), (1024, 1000), (1025, 3), (37, 36), (1, 1)])
@pytest.mark.parametrize("width,kind", [(1, "avg"), (7, "max"), (5, "avg")])
def test_selection_is_identical_on_the_same_float32_votes(m, keep, width, kind):
    Hkv, S, W = 3, 2, 6
    n = m + S + W
    cfg = pod.make_config(1, 1, Hkv, Hkv, 64, S, W, 1, n)
    cache = pod.PodCache(cfg, DEV, guard_bytes=4096)
    rng = np.random.default_rng(m * 31 + keep)
    votes = np.stack([rng.random(m).astype(np.float32) * np.float32(3),                 # spread, no ties
                      rng.integers(0, 5, m).astype(np.float32) / np.float32(8),          # five levels: ties everywhere
                      np.where(rng.random(m) < 0.3, np.where(rng.random(m) < 0.5, 0.0, -0.0), rng.standard_normal(m)).astype(np.float32)])   # signs, +0 and -0
    want = ps.select_top(ps.pool_votes(votes, width, kind), keep)
    sel = torch.full((1, Hkv, keep), -1, dtype=torch.int32, device=DEV)
    cache.pod_select_top(0, n, torch.from_numpy(votes).to(DEV), width, pod.POOL_MAX if kind == "max" else pod.POOL_AVG,
                         keep, sel, cache.new_select_workspace(n, 1, keep))
    assert np.array_equal(sel.cpu().numpy()[0], want)


def _prefill(c, n, seq, obs, lowest_sel_inputs):
    """Stores a prompt of n tokens at every layer (through the prefill call); keeps, per lowest layer, (q_obs, k)."""
    for layer in range(c.L):
        q, k, v = c.queries(layer, seq, n, c.dev), c.keys(layer, seq, n, c.dev), c.values(layer, seq, n, c.dev)
        src = c.lowest[layer]
        rep = c.Hq // c.Hkv
        if (src == layer).all():
            qs = ks = None
        else:
            perq = {int(l): c.queries(int(l), seq, n, c.dev) for l in set(src.tolist())}
            perk = {int(l): c.keys(int(l), seq, n, c.dev) for l in set(src.tolist())}
            qs = torch.stack([perq[int(src[h // rep])][:, h] for h in range(c.Hq)], dim=1).contiguous()
            ks = torch.stack([perk[int(src[h])][:, h] for h in range(c.Hkv)], dim=1).contiguous()
        c.gpu.pod_prefill_attention(layer, seq, q, k, v, qs, ks, c.scale, write_cache=True)
        if (src == layer).any():
            lowest_sel_inputs[layer] = (q[n - obs:].contiguous(), k)


def _oracle_selection(c, n, seq, obs, width, kind, keep):
    """int32 [L][Hkv][keep] (rows of layers that start no block for a head stay -1) and the float64 pooled votes."""
    sel = np.full((c.L, c.Hkv, keep), -1, dtype=np.int32)
    pooled = {}
    for layer in range(c.L):
        heads = [h for h in range(c.Hkv) if c.lowest[layer][h] == layer]
        if not heads:
            continue
        v = ps.distant_votes(gen.bf16_bits(c.queries(layer, seq, n, "cpu")[n - obs:]),
                             gen.bf16_bits(c.keys(layer, seq, n, "cpu")), c.S, c.W, c.scale)
        p = ps.pool_votes(v, width, kind)
        s = ps.select_top(p, keep)
        for h in heads:
            sel[layer, h] = s[h]
            pooled[(layer, h)] = p[h]
    return sel, pooled


def _oracle_compacted_cache(c, n, seq, sel, B):
    cpu = po.Cache(c.L, c.G, c.Hkv, c.d, c.S, c.W, B, c.max_ctx, block_lowest=c.lowest)
    for layer in range(c.L):
        mine = np.stack([sel[c.lowest[layer][h], h] for h in range(c.Hkv)])
        cpu.fill(layer, seq, ps.compact_sequence(gen.bf16_bits(c.keys(layer, seq, n, "cpu")), mine, c.S, c.W),
                 ps.compact_sequence(gen.bf16_bits(c.values(layer, seq, n, "cpu")), mine, c.S, c.W))
    return cpu


MAP4 = np.array([[0, 0, 0], [0, 0, 1], [0, 2, 2], [0, 2, 3]], dtype=np.int32)   # head-wise blocks


@pytest.mark.parametrize("name,L,G,Hq,Hkv,d,S,W,n,obs,keep,width,kind,table", [
    ("uniform", 4, 2, 8, 2, 128, 4, 24, 400, 16, 61, 5, "avg", None),
    ("turned ring", 2, 2, 4, 2, 64, 3, 16, 270, 8, 13, 7, "max", None),      # the ring turns by (n - S - keep) % W = 14
    ("head-wise", 4, 1, 6, 3, 128, 8, 32, 333, 32, 100, 3, "max", MAP4),
    ("keep all", 2, 2, 4, 4, 128, 2, 20, 150, 4, 128, 1, "avg", None),
])
def test_select_compact_and_decode_on(name, L, G, Hq, Hkv, d, S, W, n, obs, keep, width, kind, table):
    steps = 2 * W + 3                                         # the ring wraps twice: every kept recent token is demoted
    c = Case(L, G, Hq, Hkv, d, S, W, 2, n + steps + 8, seed=900 + n, with_oracle_cache=False, block_lowest=table)
    inputs = {}
    _prefill(c, n, 1, obs, inputs)
    c.gpu.pod_cache_fill(0, 0, c.keys(0, 0, 50, c.dev), c.values(0, 0, 50, c.dev))      # a neighbour that must not change
    before = {k: v.clone() for k, v in c.gpu.pod_cache_export_logical(0, 0).items()}
    ws = c.gpu.new_select_workspace(n, obs, keep)
    sel_gpu = torch.full((L, Hkv, keep), -1, dtype=torch.int32, device=c.dev)
    want, pooled = _oracle_selection(c, n, 1, obs, width, kind, keep)
    for layer, (q_obs, k) in inputs.items():
        votes = c.gpu.pod_select_votes(layer, q_obs, k, c.scale, ws)
        c.gpu.pod_select_top(layer, n, votes, width, pod.POOL_MAX if kind == "max" else pod.POOL_AVG, keep, sel_gpu, ws)
    got = sel_gpu.cpu().numpy()
    for (layer, h), p in pooled.items():
        forced = assert_valid_selection(got[layer, h], p, keep, 4e-4, f"{name} layer {layer} head {h}")
        if forced:
            assert np.array_equal(got[layer, h], want[layer, h]), f"{name} layer {layer} head {h}"
    assert (got[want < 0] == -1).all()                        # rows of layers that start no block for a head: untouched
    # compaction from the oracle's selection
    sel_dev = torch.from_numpy(want).to(c.dev)
    for layer in range(L):
        c.gpu.pod_cache_compact(layer, 1, sel_dev, ws)
        assert c.gpu.pod_cache_seq_len(layer, 1) == S + keep + W
    c.gpu.pod_cache_check()
    c.gpu.pod_cache_sync_lengths()
    assert c.gpu.pod_cache_seq_len(L - 1, 1) == S + keep + W and c.gpu.pod_cache_seq_len(0, 0) == 50
    c.cpu = _oracle_compacted_cache(c, n, 1, want, 2)
    for layer in range(L):
        g, r = c.gpu.pod_cache_export_logical(layer, 1), c.cpu.export(layer, 1)
        assert set(g) == set(r)
        for key in r:
            assert np.array_equal(gen.bf16_bits(g[key]), r[key]), f"{name} layer {layer} {key}"
    after = c.gpu.pod_cache_export_logical(0, 0)
    assert all(torch.equal(before[k], after[k]) for k in before)
    # the shorter sequence goes on: steps with demotion out of the turned ring, against the oracle's attention
    c.cpu.fill(0, 0, gen.bf16_bits(c.keys(0, 0, 50, "cpu")), gen.bf16_bits(c.values(0, 0, 50, "cpu")))
    for layer in range(1, L):
        c.fill(layer, 0, 50)
    m = S + keep + W
    for step in range(steps):
        pos = [50 + step, m + step]
        outs = [c.step(layer, pos) for layer in range(L)]
        if step % 7 == 0 or step >= steps - 2:
            ctx = [p + 1 for p in pos]
            for layer in range(L):
                assert_close(outs[layer], c.decode_ref(layer, ctx), f"{name} step {step} layer {layer}")
    for layer in range(L):
        c.assert_cache_equal(layer, 1)
    c.gpu.pod_cache_check()


@pytest.mark.parametrize("d,S,W,n,chunk", [(128, 8, 48, 1000, 300), (64, 0, 32, 555, 555), (128, 5, 100, 106, 50)])
def test_votes_from_the_cached_keys_are_the_same_bits(d, S, W, n, chunk):
    # the prompt goes in through the chunk call (sink slots, distant rows and a wrapped ring), then the votes are taken
    # from where the cache holds the keys; and once more from a cache that pod_cache_fill wrote
    L, G, Hq, Hkv, obs = 2, 2, 8, 2, min(16, W)
    c = Case(L, G, Hq, Hkv, d, S, W, 2, n + 8, seed=1234 + n, with_oracle_cache=False)
    q = [c.queries(l, 1, n, c.dev) for l in range(L)]
    k = [c.keys(l, 1, n, c.dev) for l in range(L)]
    v = [c.values(l, 1, n, c.dev) for l in range(L)]
    cws = c.gpu.new_chunk_workspace(n)
    for c0 in range(0, n, chunk):
        c1 = min(n, c0 + chunk)
        for l in range(L):
            c.gpu.pod_prefill_attention_chunk(l, 1, q[l][c0:c1], k[l][c0:c1], v[l][c0:c1], q[0][c0:c1] if l else None,
                                              k[0][c0:c1] if l else None, c.scale, cws, write_cache=True)
    ws = c.gpu.new_select_workspace(n, obs, 1)
    q_obs = q[0][n - obs:].contiguous()
    given = c.gpu.pod_select_votes(0, q_obs, k[0], c.scale, ws)
    cached = c.gpu.pod_select_votes(0, q_obs, None, c.scale, ws, seq_slot=1, n=n)
    assert torch.equal(given, cached)
    c.gpu.pod_cache_fill(0, 0, k[0], v[0])
    assert torch.equal(given, c.gpu.pod_select_votes(0, q_obs, None, c.scale, ws, seq_slot=0, n=n))
    ref = ps.distant_votes(gen.bf16_bits(c.queries(0, 1, n, "cpu")[n - obs:]), gen.bf16_bits(c.keys(0, 1, n, "cpu")), S, W, c.scale)
    assert_votes_close(cached.cpu().numpy().astype(np.float64), ref, "from the cache")
    with pytest.raises(pod.PodError) as e:                    # the slot does not hold n + 1 tokens
        c.gpu.pod_select_votes(0, q_obs, None, c.scale, c.gpu.new_select_workspace(n + 1, obs, 1), seq_slot=1, n=n + 1)
    assert e.value.code == pod.binding.ERR_STATE
    c.gpu.pod_cache_check()


def test_bad_arguments_and_bad_selections_are_reported():
    L, G, Hq, Hkv, d, S, W, n, obs, keep = 2, 2, 4, 2, 64, 2, 16, 100, 8, 10
    c = Case(L, G, Hq, Hkv, d, S, W, 1, 200, seed=77, with_oracle_cache=False)
    inputs = {}
    _prefill(c, n, 0, obs, inputs)
    q_obs, k = inputs[0]
    ws = c.gpu.new_select_workspace(n, obs, keep)
    sel = torch.zeros((L, Hkv, keep), dtype=torch.int32, device=c.dev)
    votes = c.gpu.pod_select_votes(0, q_obs, k, c.scale, ws)
    for call in (lambda: c.gpu.pod_select_votes(1, q_obs, k, c.scale, ws),                          # layer 1 starts no block
                 lambda: c.gpu.pod_select_votes(0, c.queries(0, 0, W + 1, c.dev), k, c.scale, ws),  # obs > W
                 lambda: c.gpu.pod_select_votes(0, q_obs, k[:S + W].contiguous(), c.scale, ws),     # no distant token
                 lambda: c.gpu.pod_select_top(0, n, votes, 4, pod.POOL_AVG, keep, sel, ws),         # even width
                 lambda: c.gpu.pod_select_top(0, n, votes, 3, 2, keep, sel, ws),                    # unknown pooling
                 lambda: c.gpu.pod_cache_compact(0, 0, torch.zeros((L, Hkv, n), dtype=torch.int32, device=c.dev), ws)):
        with pytest.raises(pod.PodError) as e:
            call()
        assert e.value.code == pod.binding.ERR_INVALID_ARG
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_select_votes(0, q_obs, k, c.scale, ws[:256])
    assert e.value.code == pod.binding.ERR_CAPACITY
    assert pod.pod_select_workspace_bytes(c.cfg, n, obs, keep) >= 2 * Hkv * (keep + W) * d * 2
    # an entry outside the distant range: replaced by row 0, reported by the sticky flag
    sel[:] = torch.arange(keep, dtype=torch.int32, device=c.dev)
    sel[0, 1, 3] = n - S - W
    c.gpu.pod_cache_compact(0, 0, sel, ws)
    with pytest.raises(pod.PodError) as e:
        c.gpu.pod_cache_check()
    assert e.value.code == pod.binding.ERR_STATE
    assert c.gpu.pod_cache_seq_len(0, 0) == S + keep + W
    c.gpu.pod_cache_check()                                   # the flag was cleared by the failed check


def test_selection_at_the_benchmark_shape():
    # 32K-token prompt, 8 kv heads x 4, d 128, S 64, W 2048, observation window 64, 1984 of 30656 distant tokens kept
    # (the cache then holds 4096 tokens, the budget the paper's comparison uses)
    L, G, Hq, Hkv, d, S, W, n, obs, keep = 2, 2, 32, 8, 128, 64, 2048, 32768, 64, 1984
    c = Case(L, G, Hq, Hkv, d, S, W, 1, n + 16, seed=4242, with_oracle_cache=False)
    for layer in range(L):
        c.gpu.pod_cache_fill(layer, 0, c.keys(layer, 0, n, c.dev), c.values(layer, 0, n, c.dev))
    ws = c.gpu.new_select_workspace(n, obs, keep)
    q_obs = c.queries(0, 0, obs, c.dev, pos0=n - obs).contiguous()
    votes = c.gpu.pod_select_votes(0, q_obs, c.keys(0, 0, n, c.dev), c.scale, ws)
    sel_gpu = torch.full((L, Hkv, keep), -1, dtype=torch.int32, device=c.dev)
    c.gpu.pod_select_top(0, n, votes, 7, pod.POOL_MAX, keep, sel_gpu, ws)
    ref = ps.distant_votes(gen.bf16_bits(c.queries(0, 0, obs, "cpu", pos0=n - obs)), gen.bf16_bits(c.keys(0, 0, n, "cpu")),
                           S, W, c.scale)
    assert_votes_close(votes.cpu().numpy().astype(np.float64), ref, "32K prompt")
    pooled = ps.pool_votes(ref, 7, "max")
    got = sel_gpu.cpu().numpy()
    for h in range(Hkv):
        assert_valid_selection(got[0, h], pooled[h], keep, 4e-4, f"head {h}")
    want = np.full((L, Hkv, keep), -1, dtype=np.int32)
    want[0] = ps.select_top(pooled, keep)
    sel_dev = torch.from_numpy(want).to(c.dev)
    for layer in range(L):
        c.gpu.pod_cache_compact(layer, 0, sel_dev, ws)
    c.cpu = _oracle_compacted_cache(c, n, 0, want, 1)
    for layer in range(L):
        c.assert_cache_equal(layer, 0)
    m = S + keep + W
    for step in range(2):
        outs = [c.step(layer, [m + step]) for layer in range(L)]
        for layer in range(L):
            assert_close(outs[layer], c.decode_ref(layer, [m + step + 1]), f"step {step} layer {layer}")
    c.gpu.pod_cache_check()


def test_selection_on_a_128k_prompt_with_blocks_of_four_layers():
    # the long-context shape (131072 tokens, S 128, W 4096, one block of 4 layers), 2 kv heads x 4 query heads:
    # 126848 distant tokens per head (more than the selection kernel keeps in registers), 3968 kept -> 8192 stored
    L, G, Hq, Hkv, d, S, W, n, obs, keep = 4, 4, 8, 2, 128, 128, 4096, 131072, 64, 3968
    c = Case(L, G, Hq, Hkv, d, S, W, 1, n + 16, seed=5151, with_oracle_cache=False)
    for layer in range(L):
        c.gpu.pod_cache_fill(layer, 0, c.keys(layer, 0, n, c.dev), c.values(layer, 0, n, c.dev))
    ws = c.gpu.new_select_workspace(n, obs, keep)
    q_obs = c.queries(0, 0, obs, c.dev, pos0=n - obs).contiguous()
    votes = c.gpu.pod_select_votes(0, q_obs, None, c.scale, ws, seq_slot=0, n=n)       # keys from the cache
    sel_gpu = torch.full((L, Hkv, keep), -1, dtype=torch.int32, device=c.dev)
    c.gpu.pod_select_top(0, n, votes, 5, pod.POOL_AVG, keep, sel_gpu, ws)
    ref = ps.distant_votes(gen.bf16_bits(c.queries(0, 0, obs, "cpu", pos0=n - obs)), gen.bf16_bits(c.keys(0, 0, n, "cpu")),
                           S, W, c.scale)
    assert_votes_close(votes.cpu().numpy().astype(np.float64), ref, "128K prompt")
    # pooled in float64 by a cumulative sum (the plain loop takes minutes at this length; same definition)
    pad = np.pad(ref, ((0, 0), (3, 2)))
    cs = np.cumsum(pad, axis=1)
    pooled = (cs[:, 5:] - cs[:, :-5]) / 5.0
    assert np.allclose(pooled[:, 1000:1004], ps.pool_votes(ref[:, 990:1014], 5, "avg")[:, 10:14], rtol=1e-12)
    got = sel_gpu.cpu().numpy()
    for h in range(Hkv):
        assert_valid_selection(got[0, h], pooled[h], keep, 4e-4, f"head {h}")
    assert (got[1:] == -1).all()
    # compaction from a selection made here from the oracle's votes (top by sorting)
    want = np.full((L, Hkv, keep), -1, dtype=np.int32)
    for h in range(Hkv):
        order = np.lexsort((np.arange(pooled.shape[1]), -pooled[h]))
        want[0, h] = np.sort(order[:keep])
    sel_dev = torch.from_numpy(want).to(c.dev)
    for layer in range(L):
        c.gpu.pod_cache_compact(layer, 0, sel_dev, ws)
    c.cpu = _oracle_compacted_cache(c, n, 0, want, 1)
    for layer in range(L):
        c.assert_cache_equal(layer, 0)
    m = S + keep + W
    outs = [c.step(layer, [m]) for layer in range(L)]
    for layer in range(L):
        assert_close(outs[layer], c.decode_ref(layer, [m + 1]), f"layer {layer}")
    c.gpu.pod_cache_check()
