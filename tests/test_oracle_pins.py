"""Pins for the CPU oracle (no GPU): what the paper and the mathematics fix.

Each test is chosen so that one plausible mistake in oracle/pod_oracle.c (wrong
window edge, own keys used for distant tokens, a shared value, a dropped region,
a transposed head mapping ...) fails it.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import pod_oracle as po
from pod_inputs import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_facts.txt")


def paper_facts():
    facts = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            facts[k.strip()] = float(v)
    return facts


def rand_qkv(seed, n, Hq, Hkv, d, layer=0):
    q = gen.queries_bf16(seed, layer, 0, n, Hq, d)
    k = gen.keys_bf16(seed, layer, 0, n, Hkv, d)
    v = gen.values_bf16(seed, layer, 0, n, Hkv, d)
    return q, k, v


def bits(x):
    return gen.bf16_bits(x)


def sdpa_causal(q, k, v, scale):
    """Library routine: torch's scaled_dot_product_attention, float64, causal, GQA by repetition."""
    Hq, Hkv = q.shape[1], k.shape[1]
    qq = q.double().permute(1, 0, 2)[None]
    kk = k.double().repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
    vv = v.double().repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
    o = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


# ---------------------------------------------------------------- textbook reductions

@pytest.mark.parametrize("Hq,Hkv,d", [(4, 2, 16), (6, 1, 8), (3, 3, 32)])
def test_lowest_layer_is_textbook_causal_attention(Hq, Hkv, d):
    """Eq. 3 with l = l_a: every logit is q_l . k_l, so the joint softmax is plain attention."""
    n, S, W = 96, 4, 16
    q, k, v = rand_qkv(11, n, Hq, Hkv, d)
    scale = 1.0 / math.sqrt(d)
    got = po.pod_attention(bits(q), bits(k), bits(v), None, None, np.arange(n), S, W, scale)
    np.testing.assert_allclose(got, sdpa_causal(q, k, v, scale), rtol=0, atol=1e-12)


def test_no_distant_tokens_is_textbook_even_for_upper_layer():
    """Footnote to Eq. 3: without distant tokens the distant term is omitted -> plain attention
    with the layer's own q and k, whatever the shared tensors hold."""
    n, S, W, Hq, Hkv, d = 40, 8, 32, 4, 2, 16   # n <= S + W
    q, k, v = rand_qkv(12, n, Hq, Hkv, d, layer=1)
    qa, ka, _ = rand_qkv(12, n, Hq, Hkv, d, layer=0)
    scale = 0.3
    got = po.pod_attention(bits(q), bits(k), bits(v), bits(qa), bits(ka), np.arange(n), S, W, scale)
    np.testing.assert_allclose(got, sdpa_causal(q, k, v, scale), rtol=0, atol=1e-12)


def test_identical_shared_tensors_give_textbook_attention():
    n, S, W, Hq, Hkv, d = 80, 3, 9, 4, 2, 8
    q, k, v = rand_qkv(13, n, Hq, Hkv, d)
    scale = 1.0 / math.sqrt(d)
    got = po.pod_attention(bits(q), bits(k), bits(v), bits(q), bits(k), np.arange(n), S, W, scale)
    np.testing.assert_allclose(got, sdpa_causal(q, k, v, scale), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- brute force on a tiny case

# Which (query i, key j) pairs are proximal for S = 1, W = 2, written out by hand:
# 'P' proximal (sink j=0, or j in {i-1, i}), 'D' distant, '.' not visible (j > i).
TINY_TABLE = [
    "P.......",
    "PP......",
    "PPP.....",
    "PDPP....",
    "PDDPP...",
    "PDDDPP..",
    "PDDDDPP.",
    "PDDDDDPP",
]


def test_brute_force_tiny_against_handwritten_region_table():
    n, S, W, Hq, Hkv, d = 8, 1, 2, 2, 1, 4
    q, k, v = rand_qkv(21, n, Hq, Hkv, d, layer=1)
    qa, ka, _ = rand_qkv(21, n, Hq, Hkv, d, layer=0)
    scale = 0.5
    got = po.pod_attention(bits(q), bits(k), bits(v), bits(qa), bits(ka), np.arange(n), S, W, scale)
    Q, K, V, QA, KA = (t.double().numpy() for t in (q, k, v, qa, ka))
    for i in range(n):
        for h in range(Hq):
            logits, vals = [], []
            for j in range(n):
                c = TINY_TABLE[i][j]
                if c == "P":
                    logits.append(scale * float(Q[i, h] @ K[j, 0]))
                elif c == "D":
                    logits.append(scale * float(QA[i, h] @ KA[j, 0]))
                else:
                    continue
                vals.append(V[j, 0])
            w = np.exp(np.array(logits))
            ref = (w[:, None] * np.array(vals)).sum(0) / w.sum()
            np.testing.assert_allclose(got[i, h], ref, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- gate form == joint form

def test_gate_form_equals_joint_softmax():
    """Appendix derivation: g*o^P + (1-g)*o^D is the softmax over the union."""
    n, S, W, Hq, Hkv, d = 70, 4, 8, 4, 2, 16
    q, k, v = rand_qkv(31, n, Hq, Hkv, d, layer=1)
    qa, ka, _ = rand_qkv(31, n, Hq, Hkv, d, layer=0)
    rows = np.arange(n)
    joint = po.pod_attention(bits(q), bits(k), bits(v), bits(qa), bits(ka), rows, S, W, 0.25)
    gated, g = po.pod_attention(bits(q), bits(k), bits(v), bits(qa), bits(ka), rows, S, W, 0.25, gate=True)
    np.testing.assert_allclose(gated, joint, rtol=0, atol=1e-12)
    assert np.all(g[: S + W] == 1.0)                # no distant tokens yet: term omitted
    assert np.all((g[S + W:] > 0) & (g[S + W:] < 1))


def test_gate_value_matches_eq4_by_hand():
    """g = sum exp(a^P) / (sum exp(a^P) + sum exp(a^D)) for one row, from raw exponentials."""
    n, S, W, d = 12, 2, 3, 4
    q, k, v = rand_qkv(32, n, 1, 1, d, layer=1)
    qa, ka, _ = rand_qkv(32, n, 1, 1, d, layer=0)
    i = n - 1
    _, g = po.pod_attention(bits(q[i:i + 1]), bits(k), bits(v), bits(qa[i:i + 1]), bits(ka), [i], S, W, 0.5, gate=True)
    Q, K, QA, KA = (t.double().numpy() for t in (q, k, qa, ka))
    prox = [0, 1, 9, 10, 11]
    dist = [2, 3, 4, 5, 6, 7, 8]
    eP = sum(math.exp(0.5 * float(Q[i, 0] @ K[j, 0])) for j in prox)
    eD = sum(math.exp(0.5 * float(QA[i, 0] @ KA[j, 0])) for j in dist)
    assert abs(g[0, 0] - eP / (eP + eD)) < 1e-12


# ---------------------------------------------------------------- the sharing rule

def _upper_layer_case(seed=41, n=64, S=4, W=8, Hq=4, Hkv=2, d=16):
    q, k, v = rand_qkv(seed, n, Hq, Hkv, d, layer=1)
    qa, ka, _ = rand_qkv(seed, n, Hq, Hkv, d, layer=0)
    return n, S, W, q, k, v, qa, ka


def test_upper_layer_ignores_its_own_distant_keys():
    n, S, W, q, k, v, qa, ka = _upper_layer_case()
    i = n - 1
    row = lambda t: bits(t[i:i + 1])
    base = po.pod_attention(row(q), bits(k), bits(v), row(qa), bits(ka), [i], S, W, 0.25)
    k2 = k.clone()
    k2[S:i - W + 1] = k2[S:i - W + 1] * 3 + 1          # own keys at distant positions
    same = po.pod_attention(row(q), bits(k2), bits(v), row(qa), bits(ka), [i], S, W, 0.25)
    assert np.array_equal(base, same)
    ka2 = ka.clone()
    ka2[S:i - W + 1] = ka2[S:i - W + 1] * 3 + 1        # lowest layer's keys there
    diff = po.pod_attention(row(q), bits(k), bits(v), row(qa), bits(ka2), [i], S, W, 0.25)
    assert np.abs(diff - base).max() > 1e-3
    qa2 = qa.clone()
    qa2[i] = -qa2[i]                                   # lowest layer's query
    diff = po.pod_attention(row(q), bits(k), bits(v), bits(qa2[i:i + 1]), bits(ka), [i], S, W, 0.25)
    assert np.abs(diff - base).max() > 1e-3


def test_upper_layer_ignores_shared_keys_at_proximal_positions():
    n, S, W, q, k, v, qa, ka = _upper_layer_case(seed=42)
    i = n - 1
    row = lambda t: bits(t[i:i + 1])
    base = po.pod_attention(row(q), bits(k), bits(v), row(qa), bits(ka), [i], S, W, 0.25)
    ka2 = ka.clone()
    ka2[:S] = 7.0
    ka2[i - W + 1:] = -7.0
    same = po.pod_attention(row(q), bits(k), bits(v), row(qa), bits(ka2), [i], S, W, 0.25)
    assert np.array_equal(base, same)
    # the edge tokens: i-W is the newest distant token, i-W+1 the oldest recent one
    ka3 = ka.clone(); ka3[i - W] += 1.0
    assert np.abs(po.pod_attention(row(q), bits(k), bits(v), row(qa), bits(ka3), [i], S, W, 0.25) - base).max() > 1e-6
    k3 = k.clone(); k3[i - W + 1] += 1.0
    assert np.abs(po.pod_attention(row(q), bits(k3), bits(v), row(qa), bits(ka), [i], S, W, 0.25) - base).max() > 1e-6
    k4 = k.clone(); k4[S - 1] += 1.0
    assert np.abs(po.pod_attention(row(q), bits(k4), bits(v), row(qa), bits(ka), [i], S, W, 0.25) - base).max() > 1e-6
    ka4 = ka.clone(); ka4[S] += 1.0
    assert np.abs(po.pod_attention(row(q), bits(k), bits(v), row(qa), bits(ka4), [i], S, W, 0.25) - base).max() > 1e-6


def test_values_always_come_from_the_layer_itself():
    n, S, W, q, k, v, qa, ka = _upper_layer_case(seed=43)
    ones = torch.ones_like(v)
    out = po.pod_attention(bits(q), bits(k), bits(ones), bits(qa), bits(ka), np.arange(n), S, W, 0.25)
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=1e-12)   # softmax weights sum to one


def test_gqa_head_mapping():
    """Query head h reads KV head h // (Hq/Hkv): make KV head 1 the only one that matters."""
    n, S, W, Hq, Hkv, d = 32, 2, 4, 4, 2, 8
    q, k, v = rand_qkv(44, n, Hq, Hkv, d)
    v2 = v.clone(); v2[:, 0] = 0.0
    out = po.pod_attention(bits(q), bits(k), bits(v2), None, None, np.arange(n), S, W, 0.3)
    assert np.all(out[:, :2] == 0.0) and np.abs(out[:, 2:]).max() > 0.1


# ---------------------------------------------------------------- closed forms

def test_zero_keys_give_running_mean_of_values():
    n, S, W, Hq, Hkv, d = 50, 3, 5, 2, 1, 8
    q, k, v = rand_qkv(51, n, Hq, Hkv, d)
    z = torch.zeros_like(k)
    out = po.pod_attention(bits(q), bits(z), bits(v), bits(q), bits(z), np.arange(n), S, W, 1.0)
    V = v.double().numpy()[:, 0]
    ref = np.cumsum(V, 0) / np.arange(1, n + 1)[:, None]
    np.testing.assert_allclose(out[:, 0], ref, rtol=0, atol=1e-12)


def test_zero_shared_query_weights_each_distant_token_by_one():
    n, S, W, Hq, Hkv, d = 40, 2, 6, 1, 1, 8
    q, k, v = rand_qkv(52, n, Hq, Hkv, d, layer=1)
    _, ka, _ = rand_qkv(52, n, Hq, Hkv, d, layer=0)
    i = n - 1
    qa0 = torch.zeros_like(q[i:i + 1])
    out = po.pod_attention(bits(q[i:i + 1]), bits(k), bits(v), bits(qa0), bits(ka), [i], S, W, 0.4)
    Q, K, V = (t.double().numpy() for t in (q, k, v))
    prox = [j for j in range(n) if j < S or j > i - W]
    dist = [j for j in range(n) if j not in prox]
    e = np.array([math.exp(0.4 * float(Q[i, 0] @ K[j, 0])) for j in prox])
    ref = ((e[:, None] * V[prox, 0]).sum(0) + V[dist, 0].sum(0)) / (e.sum() + len(dist))
    assert len(dist) == n - S - W
    np.testing.assert_allclose(out[0, 0], ref, rtol=0, atol=1e-12)


def test_dominant_key_returns_its_value():
    n, S, W, Hq, Hkv, d = 48, 2, 6, 1, 1, 8
    q, k, v = rand_qkv(53, n, Hq, Hkv, d, layer=1)
    qa, ka, _ = rand_qkv(53, n, Hq, Hkv, d, layer=0)
    i, t = n - 1, 20                                   # t is a distant position
    ka = ka.clone(); ka[t, 0] = qa[i, 0] * 64.0
    out = po.pod_attention(bits(q[i:i + 1]), bits(k), bits(v), bits(qa[i:i + 1]), bits(ka), [i], S, W, 1.0)
    np.testing.assert_allclose(out[0, 0], v[t, 0].double().numpy(), rtol=0, atol=1e-9)


def test_permuting_distant_tokens_changes_nothing():
    n, S, W, q, k, v, qa, ka = _upper_layer_case(seed=54)
    i = n - 1
    perm = torch.arange(n)
    perm[S:i - W + 1] = torch.flip(perm[S:i - W + 1], dims=[0])
    a = po.pod_attention(bits(q[i:i + 1]), bits(k), bits(v), bits(qa[i:i + 1]), bits(ka), [i], S, W, 0.25)
    v2 = v.clone(); v2[S:i - W + 1] = v[perm[S:i - W + 1]]
    ka2 = ka.clone(); ka2[S:i - W + 1] = ka[perm[S:i - W + 1]]
    b = po.pod_attention(bits(q[i:i + 1]), bits(k), bits(v2), bits(qa[i:i + 1]), bits(ka2), [i], S, W, 0.25)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- region arithmetic, cache model

def test_region_sizes_match_the_papers_window_column():
    f = paper_facts()
    n, S, W = int(f["context_32k"]), int(f["n_s"]), int(f["n_r"])
    c = po.Cache(1, 1, 1, 1, S, W, 1, n)
    z = np.zeros((n, 1, 1), dtype=np.uint16)
    c.fill(0, 0, z, z)
    e = c.export(0, 0)
    assert (len(e["sinkK"]), len(e["recentK"]), len(e["distV"])) == (S, W, int(f["distant_at_32k"]))


def test_toy_config_has_1776_distant_tokens():
    c = po.Cache(2, 2, 1, 1, 16, 256, 1, 2048)
    z = np.zeros((2047, 1, 1), dtype=np.uint16)
    c.fill(0, 0, z, z)
    c.append(0, z[:1], z[:1], [2047])
    assert len(c.export(0, 0)["distV"]) == 1776


def _tagged_kv(n, Hkv, d, layer):
    """K/V whose every element encodes (layer, kind, position, head, dim) so misplaced rows show."""
    pos = np.arange(n, dtype=np.uint32)[:, None, None]
    head = np.arange(Hkv, dtype=np.uint32)[None, :, None]
    dim = np.arange(d, dtype=np.uint32)[None, None, :]
    base = (pos * 31 + head * 7 + dim * 3 + layer * 1009) % 60000
    k = (base * 2).astype(np.uint16) % np.uint16(0x7F00)      # finite bf16 patterns
    v = (base * 2 + 1).astype(np.uint16) % np.uint16(0x7F00)
    return np.ascontiguousarray(k), np.ascontiguousarray(v)


@pytest.mark.parametrize("n", [1, 3, 4, 5, 11, 12, 13, 40])
def test_appends_equal_fill_and_views_are_slices(n):
    L, G, Hkv, d, S, W = 2, 2, 2, 4, 4, 8
    a = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    b = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    for layer in range(L):
        k, v = _tagged_kv(n, Hkv, d, layer)
        for p in range(n):
            a.append(layer, k[p:p + 1], v[p:p + 1], [p])
        b.fill(layer, 0, k, v)
        ea, eb = a.export(layer, 0), b.export(layer, 0)
        lo = max(S, n - W)
        want = dict(sinkK=k[:min(n, S)], sinkV=v[:min(n, S)], recentK=k[lo:n], recentV=v[lo:n],
                    distV=v[S:max(S, n - W)])
        if layer % G == 0:
            want["distK"] = k[S:max(S, n - W)]
        assert set(ea) == set(eb) == set(want)
        for name in want:
            assert np.array_equal(ea[name], want[name]), name
            assert np.array_equal(eb[name], want[name]), name
        assert len(ea["distV"]) == max(0, n - S - W)
    assert a.stored_elems() == b.stored_elems()


def test_upper_layer_keeps_no_distant_keys():
    c = po.Cache(2, 2, 1, 2, 1, 2, 1, 16)
    k, v = _tagged_kv(10, 1, 2, 1)
    c.fill(1, 0, k, v)
    assert "distK" not in c.export(1, 0)
    per_row = 1 * 2
    assert c.stored_elems() == per_row * (2 * 1 + 2 * 2 + 7)      # sink K,V + recent K,V + distant V only


def test_append_rejects_wrong_position_and_overflow():
    c = po.Cache(1, 1, 1, 2, 1, 2, 1, 4)
    k, v = _tagged_kv(5, 1, 2, 0)
    with pytest.raises(po.OracleError):
        c.append(0, k[:1], v[:1], [1])
    for p in range(4):
        c.append(0, k[p:p + 1], v[p:p + 1], [p])
    with pytest.raises(po.OracleError):
        c.append(0, k[4:5], v[4:5], [4])


# ---------------------------------------------------------------- memory accounting

@pytest.mark.parametrize("L,G,n", [(4, 2, 100), (4, 1, 100), (4, 4, 9), (6, 3, 57), (2, 2, 12)])
def test_counted_entries_match_closed_form(L, G, n):
    Hkv, d, S, W = 2, 4, 4, 8
    c = po.Cache(L, G, Hkv, d, S, W, 1, 128)
    for layer in range(L):
        k, v = _tagged_kv(n, Hkv, d, layer)
        c.fill(layer, 0, k, v)
    pod, dense = po.cache_bytes_formula(L, G, Hkv, d, S, W, n)
    assert c.stored_elems() * 2 == pod
    assert dense == 2 * 2 * Hkv * d * L * n
    n_dist = max(0, n - S - W)
    assert abs((1 - pod / dense) - (1 - 1 / G) * n_dist / (2 * n)) < 1e-12


def test_saving_limits_and_config_values():
    f = paper_facts()
    sav = lambda L, G, S, W, n: 1 - np.divide(*po.cache_bytes_formula(L, G, 8, 128, S, W, n))
    assert sav(32, 1, 64, 2048, 32768) == 0.0                       # no sharing
    assert sav(32, 2, 64, 2048, 2000) == 0.0                        # nothing distant yet
    assert abs(sav(2, 2, 64, 2048, 32768) - 0.234) < 5e-4           # (1-1/2)*30656/65536
    assert abs(sav(32, 4, 128, 4096, 131072) - 0.363) < 5e-4        # (1-1/4)*126848/262144
    # sharing K only (not V) between 2 layers saves half of what sharing both saves
    assert abs(sav(2, 2, 0, 1, 10 ** 7) - f["cla_factor2_saving"] / 2) < 1e-6
    assert sav(64, 64, 0, 1, 10 ** 7) < 0.5 and sav(64, 64, 0, 1, 10 ** 7) > 0.49


# ---------------------------------------------------------------- decode from the cache model

@pytest.mark.parametrize("layer", [0, 1])
@pytest.mark.parametrize("n", [5, 12, 13, 37])
def test_decode_from_cache_equals_definition(layer, n):
    L, G, Hq, Hkv, d, S, W = 2, 2, 4, 2, 8, 4, 8
    c = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    ks, vs, qs = {}, {}, {}
    for l in range(L):
        qs[l], ks[l], vs[l] = rand_qkv(61, n, Hq, Hkv, d, layer=l)
        c.fill(l, 0, bits(ks[l][: n - 1]), bits(vs[l][: n - 1]))
        c.append(l, bits(ks[l][n - 1:]), bits(vs[l][n - 1:]), [n - 1])
    i = n - 1
    q, qa = bits(qs[layer][i:i + 1]), bits(qs[0][i:i + 1])
    got = c.decode_attention(layer, q, qa if layer else None, [n], 0.35)
    ref = po.pod_attention(q, bits(ks[layer]), bits(vs[layer]), qa if layer else None,
                           bits(ks[0]) if layer else None, [i], S, W, 0.35)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- gated skip of distant tokens (appendix)

def _gated_case(n, scale=0.35, boost=None):
    """Two-layer block filled to n tokens; returns the cache model and the per-layer tensors."""
    L, G, Hq, Hkv, d, S, W = 2, 2, 4, 2, 8, 4, 8
    c = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    ks, vs, qs = {}, {}, {}
    for l in range(L):
        qs[l], ks[l], vs[l] = rand_qkv(71, n, Hq, Hkv, d, layer=l)
        if boost is not None:  # make the proximal keys of the upper layer dominate for head pairs of kv head 0
            ks[l] = ks[l].clone()
            ks[l][:, 0] *= boost
        c.fill(l, 0, bits(ks[l]), bits(vs[l]))
    return c, qs, ks, vs, (L, G, Hq, Hkv, d, S, W)


def test_gated_tau_one_is_exact_and_gate_matches_definition_form():
    n = 37
    c, qs, ks, vs, (L, G, Hq, Hkv, d, S, W) = _gated_case(n)
    i = n - 1
    q, qa = bits(qs[1][i:i + 1]), bits(qs[0][i:i + 1])
    out, g, skipped = c.decode_attention_gated(1, q, qa, [n], 0.35, 1.0)
    ref, g_ref = po.pod_attention(q, bits(ks[1]), bits(vs[1]), qa, bits(ks[0]), [i], S, W, 0.35, gate=True)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)     # tau = 1 never skips (g < 1 with distant tokens)
    np.testing.assert_allclose(g, g_ref, rtol=1e-12)              # the gate of Eq. 4, from the full-tensor form
    assert not skipped.any()


def test_gated_tau_zero_is_attention_over_proximal_tokens_only():
    """g >= 0 always: every upper-layer head leaves the distant part out, and what remains is textbook
    softmax attention over the sink and recent tokens (checked with the library routine on those rows)."""
    n = 37
    c, qs, ks, vs, (L, G, Hq, Hkv, d, S, W) = _gated_case(n)
    i = n - 1
    q, qa = bits(qs[1][i:i + 1]), bits(qs[0][i:i + 1])
    out, g, skipped = c.decode_attention_gated(1, q, qa, [n], 0.35, 0.0)
    assert skipped.all()
    prox = list(range(S)) + list(range(n - W, n))
    kp, vp = ks[1][prox], vs[1][prox]
    qq = qs[1][i:i + 1].double().permute(1, 0, 2)[None]
    kk = kp.double().repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
    vv = vp.double().repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, scale=0.35)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


def test_gated_lowest_layer_and_short_contexts_never_skip():
    n = 37
    c, qs, ks, vs, (L, G, Hq, Hkv, d, S, W) = _gated_case(n)
    q0 = bits(qs[0][n - 1:n])
    out, g, skipped = c.decode_attention_gated(0, q0, None, [n], 0.35, 0.0)
    np.testing.assert_allclose(out, c.decode_attention(0, q0, None, [n], 0.35), rtol=0, atol=1e-13)
    assert not skipped.any()
    n2 = 10                                                       # S + W = 12 > n: no distant tokens
    c2, qs2, ks2, vs2, _ = _gated_case(n2)
    q, qa = bits(qs2[1][n2 - 1:n2]), bits(qs2[0][n2 - 1:n2])
    out2, g2, skipped2 = c2.decode_attention_gated(1, q, qa, [n2], 0.35, 0.0)
    assert (g2 == 1.0).all() and not skipped2.any()
    np.testing.assert_allclose(out2, c2.decode_attention(1, q, qa, [n2], 0.35), rtol=0, atol=1e-13)


def test_gated_threshold_splits_heads_by_their_gate():
    """With a threshold between the heads' gates exactly the heads at or above it skip; a skipped head
    returns o^P, the others the exact output; the error of a skipped head is (1 - g) |o^P - o^D|."""
    n = 37
    c, qs, ks, vs, (L, G, Hq, Hkv, d, S, W) = _gated_case(n, boost=3.0)
    i = n - 1
    q, qa = bits(qs[1][i:i + 1]), bits(qs[0][i:i + 1])
    exact, g, _ = c.decode_attention_gated(1, q, qa, [n], 0.35, 1.0)
    gs = np.sort(g.ravel())
    assert gs[-1] - gs[0] > 0.05                                  # the case has spread
    tau = float((gs[1] + gs[2]) / 2)
    out, g2, skipped = c.decode_attention_gated(1, q, qa, [n], 0.35, tau)
    np.testing.assert_array_equal(g2, g)
    np.testing.assert_array_equal(skipped.astype(bool), g >= tau)
    assert skipped.sum() == 2
    prox_only, _, _ = c.decode_attention_gated(1, q, qa, [n], 0.35, 0.0)
    for h in range(Hq):
        want = prox_only[0, h] if skipped[0, h] else exact[0, h]
        np.testing.assert_allclose(out[0, h], want, rtol=0, atol=1e-13)
        if skipped[0, h]:                                         # o = g oP + (1-g) oD  =>  oP - o = (1-g)(oP - oD)
            oD = (exact[0, h] - g[0, h] * prox_only[0, h]) / (1 - g[0, h])
            np.testing.assert_allclose(out[0, h] - exact[0, h], (1 - g[0, h]) * (prox_only[0, h] - oD), atol=1e-12)


# ---------------------------------------------------------------- head-wise blocks and offline grouping

from oracle import pod_grouping as pg

MAP4 = np.array([[0, 0, 0],     # kv head 0: one block {0,1,2,3}; head 1: {0,1},{2,3}; head 2: every layer alone
                 [0, 0, 1],
                 [0, 2, 2],
                 [0, 2, 3]], dtype=np.int32)


def _filled_map_cache(n, block_lowest, L=4, Hq=6, Hkv=3, d=8, S=4, W=8, seed=83):
    c = po.Cache(L, 1, Hkv, d, S, W, 1, 64, block_lowest=block_lowest)
    qs, ks, vs = {}, {}, {}
    for l in range(L):
        qs[l], ks[l], vs[l] = rand_qkv(seed, n, Hq, Hkv, d, layer=l)
        c.fill(l, 0, bits(ks[l]), bits(vs[l]))
    return c, qs, ks, vs


def test_explicit_uniform_map_equals_group_size():
    n, L, G, Hq, Hkv, d, S, W = 37, 4, 2, 4, 2, 8, 4, 8
    uni = np.array([[l - l % G] * Hkv for l in range(L)], dtype=np.int32)
    a = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    b = po.Cache(L, 1, Hkv, d, S, W, 1, 64, block_lowest=uni)
    for l in range(L):
        q, k, v = rand_qkv(91, n, Hq, Hkv, d, layer=l)
        for c in (a, b):
            c.fill(l, 0, bits(k), bits(v))
    assert a.stored_elems() == b.stored_elems()
    for l in range(L):
        q = bits(rand_qkv(91, n, Hq, Hkv, d, layer=l)[0][n - 1:])
        qa = bits(rand_qkv(91, n, Hq, Hkv, d, layer=l - l % G)[0][n - 1:])
        np.testing.assert_array_equal(a.decode_attention(l, q, qa, [n], 0.3), b.decode_attention(l, q, qa, [n], 0.3))
        ea, eb = a.export(l, 0), b.export(l, 0)
        assert set(ea) == set(eb)
        for key in ea:
            np.testing.assert_array_equal(ea[key], eb[key])


def test_headwise_map_decode_equals_definition_with_per_head_sources():
    """Each kv head takes its distant logits from the lowest layer of ITS block: the definition, fed with
    k_shared / q_shared gathered head by head from those layers, must give the cache model's result."""
    n, L, Hq, Hkv, d, S, W = 37, 4, 6, 3, 8, 4, 8
    c, qs, ks, vs = _filled_map_cache(n, MAP4)
    rep, i = Hq // Hkv, n - 1
    for layer in range(L):
        k_sh = torch.stack([ks[int(MAP4[layer, h])][:, h] for h in range(Hkv)], dim=1)          # [n][Hkv][d]
        q_sh = torch.stack([qs[int(MAP4[layer, h // rep])][i, h] for h in range(Hq)], dim=0)[None]  # [1][Hq][d]
        q = bits(qs[layer][i:i + 1])
        got = c.decode_attention(layer, q, bits(q_sh), [n], 0.35)
        ref = po.pod_attention(q, bits(ks[layer]), bits(vs[layer]), bits(q_sh), bits(k_sh), [i], S, W, 0.35)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)
    # kv head 2 is alone in every block: textbook attention for its query heads at every layer
    for layer in range(L):
        q_sh = torch.stack([qs[int(MAP4[layer, h // rep])][i, h] for h in range(Hq)], dim=0)[None]
        got = c.decode_attention(layer, bits(qs[layer][i:i + 1]), bits(q_sh), [n], 0.35)
        ref = sdpa_causal(qs[layer], ks[layer], vs[layer], 0.35)[i]
        np.testing.assert_allclose(got[0, 2 * rep:], ref[2 * rep:], rtol=0, atol=1e-12)


def test_headwise_map_keeps_distant_keys_only_where_lowest_and_counts_match_closed_form():
    n, L, Hq, Hkv, d, S, W = 37, 4, 6, 3, 8, 4, 8
    c, qs, ks, vs = _filled_map_cache(n, MAP4)
    n_dist = n - S - W
    for layer in range(L):
        e = c.export(layer, 0)
        assert e["distV"].shape[0] == n_dist
        for h in range(Hkv):
            want = bits(ks[layer][S:n - W, h]) if MAP4[layer, h] == layer else np.zeros((n_dist, d), np.uint16)
            np.testing.assert_array_equal(e["distK"][:, h], want)
    pod_b, dense_b = po.cache_bytes_formula_map(MAP4, d, S, W, n)
    assert c.stored_elems() * 2 == pod_b
    blocks = [1, 2, 4]                                    # per kv head
    by_hand = sum(d * 2 * (L * (2 * (S + W) + n_dist) + nb * n_dist) for nb in blocks)
    assert pod_b == by_hand and dense_b == 2 * L * n * Hkv * d * 2
    uni = np.array([[l - l % 2] * Hkv for l in range(L)], dtype=np.int32)
    assert po.cache_bytes_formula_map(uni, d, S, W, n) == po.cache_bytes_formula(L, 2, Hkv, d, S, W, n)


def test_headwise_map_must_describe_consecutive_blocks():
    bad = MAP4.copy()
    bad[3, 1] = 1                                         # layer 3 cannot join block {0,1} across block {2}
    with pytest.raises(po.OracleError):
        po.Cache(4, 1, 3, 8, 4, 8, 1, 64, block_lowest=bad)


def test_greedy_grouping_by_hand():
    L = 5
    sim = np.zeros((2, L, L))
    # head 0: 0~1, 1~2 but 0 and 2 dissimilar -> layer 2 must be similar to ALL of {0,1}: new block; 2~3~4 all similar
    for a, b, v in [(0, 1, .9), (1, 2, .9), (0, 2, .2), (2, 3, .6), (2, 4, .5), (3, 4, .7), (1, 3, .9), (0, 3, .9)]:
        sim[0, a, b] = sim[0, b, a] = v
    # head 1: nothing similar
    lowest = pg.group_layers(sim, 0.5)
    assert lowest[:, 0].tolist() == [0, 0, 2, 2, 2]       # 0.5 counts as similar (>=)
    assert lowest[:, 1].tolist() == [0, 1, 2, 3, 4]
    assert pg.group_layers(np.ones((3, L, L)), 0.5).tolist() == [[0, 0, 0]] * L


def test_gqa_grouping_is_a_strict_majority_vote():
    L, Hq, Hkv = 3, 4, 1
    sim = np.zeros((Hq, L, L))
    sim[:3, 0, 1] = sim[:3, 1, 0] = 0.8                   # 3 of 4 heads: similar
    sim[:2, 1, 2] = sim[:2, 2, 1] = 0.8                   # 2 of 4 heads: a tie, not a majority
    sim[:, 0, 2] = sim[:, 2, 0] = 0.9
    assert pg.group_layers_gqa(sim, Hkv, 0.5)[:, 0].tolist() == [0, 0, 2]
    sim[2, 1, 2] = sim[2, 2, 1] = 0.8                     # now 3 of 4
    assert pg.group_layers_gqa(sim, Hkv, 0.5)[:, 0].tolist() == [0, 0, 0]


def test_js_similarity_special_cases():
    assert pg.js_divergence_base2([1, 0], [0, 1]) == pytest.approx(1.0)           # disjoint support
    assert pg.js_divergence_base2([.2, .3, .5], [.2, .3, .5]) == 0.0
    p, q = np.array([.7, .2, .1]), np.array([.1, .1, .8])
    assert pg.js_divergence_base2(p, q) == pytest.approx(pg.js_divergence_base2(q, p))
    # closed form for p = (1, 0), q = (1/2, 1/2): 1/2 log2(4/3) + 1/2 (1/2 log2(2/3) + 1/2 log2 2)
    want = 0.5 * math.log2(4 / 3) + 0.5 * (0.5 * math.log2(2 / 3) + 0.5)
    assert pg.js_divergence_base2([1, 0], [.5, .5]) == pytest.approx(want)
    from scipy.spatial.distance import jensenshannon                                # library routine: sqrt of JS
    assert pg.js_divergence_base2(p, q) == pytest.approx(jensenshannon(p, q, base=2) ** 2)
    a = np.random.default_rng(0).dirichlet(np.ones(16), size=(2, 3))
    assert pg.layer_similarity(a, a) == pytest.approx(1.0)
    b = np.roll(a, 5, axis=2)
    manual = 1 - np.mean([pg.js_divergence_base2(a[i, j], b[i, j]) for i in range(2) for j in range(3)])
    assert pg.layer_similarity(a, b) == pytest.approx(manual) and 0 < manual < 1


# ---------------------------------------------------------------- several tokens at once; a prompt in chunks

@pytest.mark.parametrize("chunks", [[40], [1, 39], [3, 1, 8, 9, 19], [12, 12, 16], [5, 30, 5], [13, 27]])
def test_append_many_equals_single_appends_and_the_slice_rule(chunks):
    """A chunk of tokens is by definition the tokens one at a time; the end state is again the slice
    rule of Eq. 3's index ranges, whatever the chunk boundaries (shorter, equal, longer than S, W, S + W)."""
    L, G, Hkv, d, S, W = 2, 2, 2, 4, 4, 8
    n = sum(chunks)
    a = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    b = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    for layer in range(L):
        k, v = _tagged_kv(n, Hkv, d, layer)
        p = 0
        for t in chunks:
            a.append_many(layer, k[None, p:p + t], v[None, p:p + t], [p])
            p += t
        for p in range(n):
            b.append(layer, k[p:p + 1], v[p:p + 1], [p])
        ea, eb = a.export(layer, 0), b.export(layer, 0)
        lo = max(S, n - W)
        want = dict(sinkK=k[:min(n, S)], sinkV=v[:min(n, S)], recentK=k[lo:n], recentV=v[lo:n], distV=v[S:lo])
        if layer % G == 0:
            want["distK"] = k[S:lo]
        assert set(ea) == set(eb) == set(want)
        for name in want:
            assert np.array_equal(ea[name], want[name]), name
            assert np.array_equal(eb[name], want[name]), name


def test_append_many_ragged_counts_and_checks():
    L, G, Hkv, d, S, W, B, T = 1, 1, 1, 2, 2, 3, 3, 6
    c = po.Cache(L, G, Hkv, d, S, W, B, 16)
    k, v = _tagged_kv(B * T, Hkv, d, 0)
    k, v = k.reshape(B, T, Hkv, d), v.reshape(B, T, Hkv, d)
    c.append_many(0, k, v, [0, 0, 0], counts=[6, 0, 2])
    assert [c.length(0, b) for b in range(B)] == [6, 0, 2]
    e0, e2 = c.export(0, 0), c.export(0, 2)
    assert np.array_equal(e0["recentK"], k[0, 3:6]) and np.array_equal(e0["distV"], v[0, 2:3])
    assert np.array_equal(e2["sinkK"], k[2, :2]) and len(e2["recentK"]) == 0
    with pytest.raises(po.OracleError):                      # wrong start position: nothing is stored, for any sequence
        c.append_many(0, k, v, [6, 0, 3], counts=[1, 1, 1])
    assert [c.length(0, b) for b in range(B)] == [6, 0, 2]
    with pytest.raises(po.OracleError):                      # over the capacity of 16
        c.append_many(0, np.concatenate([k, k], axis=1), np.concatenate([v, v], axis=1), [6, 0, 2], counts=[11, 0, 0])
    with pytest.raises(po.OracleError):
        c.append_many(0, k, v, [6, 0, 2], counts=[7, 0, 0])  # more rows than the call carries


@pytest.mark.parametrize("layer", [0, 1])
@pytest.mark.parametrize("chunks,lowest_first", [([37], True), ([5, 32], True), ([12, 1, 24], True), ([13, 9, 15], False),
                                                 ([3, 20, 14], True), ([30, 7], False)])
def test_chunk_attention_from_cache_equals_rows_of_the_definition(layer, chunks, lowest_first):
    """Rows p0 .. p0+T-1 of Eq. 3 on the whole sequence, computed from what the cache model holds plus the
    chunk: fails if the model drops a key some later query still needs (e.g. the lowest layer's key of a
    token that is in the window for early rows of the chunk and distant for late ones), or takes a key
    from the wrong layer.  lowest_first: the lowest layer has stored the chunk already when the upper layer runs."""
    L, G, Hq, Hkv, d, S, W = 2, 2, 4, 2, 8, 4, 8
    n = sum(chunks)
    c = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    qs, ks, vs = {}, {}, {}
    for l in range(L):
        qs[l], ks[l], vs[l] = rand_qkv(81, n, Hq, Hkv, d, layer=l)
    full = po.pod_attention(bits(qs[layer]), bits(ks[layer]), bits(vs[layer]), bits(qs[0]) if layer else None,
                            bits(ks[0]) if layer else None, np.arange(n), S, W, 0.35)
    p = 0
    for t in chunks:
        sl = slice(p, p + t)
        if lowest_first:
            c.append_many(0, bits(ks[0][sl])[None], bits(vs[0][sl])[None], [p])
        if layer == 1 or not lowest_first:
            got = c.chunk_attention(layer, 0, bits(qs[layer][sl]), bits(ks[layer][sl]), bits(vs[layer][sl]),
                                    bits(qs[0][sl]) if layer else None, bits(ks[0][sl]) if layer else None, 0.35)
            np.testing.assert_allclose(got, full[sl], rtol=0, atol=1e-13)
        if not lowest_first:
            c.append_many(0, bits(ks[0][sl])[None], bits(vs[0][sl])[None], [p])
        c.append_many(1, bits(ks[1][sl])[None], bits(vs[1][sl])[None], [p])
        p += t


def test_chunk_attention_rejects_a_lowest_layer_out_of_step():
    L, G, Hq, Hkv, d, S, W = 2, 2, 2, 1, 4, 2, 4
    c = po.Cache(L, G, Hkv, d, S, W, 1, 64)
    q, k, v = rand_qkv(82, 12, Hq, Hkv, d)
    c.append_many(0, bits(k[:7])[None], bits(v[:7])[None], [0])
    c.append_many(1, bits(k[:6])[None], bits(v[:6])[None], [0])
    with pytest.raises(po.OracleError):   # chunk of 3 at p0 = 6: the lowest layer must hold 6 or 9 tokens, not 7
        c.chunk_attention(1, 0, bits(q[6:9]), bits(k[6:9]), bits(v[6:9]), bits(q[6:9]), bits(k[6:9]), 0.5)


def test_reset_forgets_one_slot_or_all():
    c = po.Cache(2, 2, 1, 2, 1, 2, 2, 16)
    k, v = _tagged_kv(6, 1, 2, 0)
    for layer in range(2):
        for b in range(2):
            c.fill(layer, b, k, v)
    c.reset(1)
    assert [c.length(l, b) for l in range(2) for b in range(2)] == [6, 0, 6, 0]
    c.fill(0, 1, k[:3], v[:3])                               # an emptied slot takes a new prompt
    assert np.array_equal(c.export(0, 1)["recentK"], k[1:3])
    c.reset()
    assert [c.length(l, b) for l in range(2) for b in range(2)] == [0, 0, 0, 0]
