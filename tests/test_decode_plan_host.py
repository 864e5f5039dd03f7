"""The split-K plan of a decode launch (host logic, no GPU): pod_decode_plan.  Whatever the shape, the pieces are whole
tiles, cover both regions, fit the workspace bound, and the partials are merged inside the launch only where the
launch is about one resident round of workgroups."""
import itertools

import numpy as np

import pytest

import paper_2412_02252_amd as pod

TILE = 32


def _slots(rows, chunk):
    return (rows + chunk - 1) // chunk


@pytest.mark.parametrize("cus", [256, 304, 64])
def test_plan_invariants_over_a_sweep_of_shapes(cus):
    lens = [1, 31, 40, 41, 129, 2111, 2112, 2113, 4096, 32768, 32769, 32832, 131072, 500000]
    for B, Hkv, P, n in itertools.product([1, 2, 3, 4, 16, 64, 300], [1, 2, 8, 16], [40, 2112, 4224], lens):
        pl = pod.pod_decode_plan(cus, B, Hkv, P, n)
        prox, dist = min(n, P), n - min(n, P)
        what = (cus, B, Hkv, P, n, pl)
        assert pl["waves"] in (4, 8), what
        assert pl["chunk"] % TILE == 0 and pl["chunk_prox"] % TILE == 0, what
        assert pl["chunk"] >= TILE * pl["waves"] and pl["chunk_prox"] >= TILE * pl["waves"], what   # a tile per wave at least
        assert pl["chunk"] <= 8192 and pl["chunk_prox"] <= 8192, what                                 # 16-bit fields in the kernel
        assert pl["distant_pieces"] == _slots(dist, pl["chunk"]), what                               # the pieces cover the regions
        assert pl["pieces"] == pl["distant_pieces"] + _slots(prox, pl["chunk_prox"]), what
        assert pl["pieces"] <= _slots(dist, 128) + _slots(prox, 128), what                           # what the workspace provides for
        assert (pl["waves"] == 8) == pl["merge_inside"], what
        if pl["merge_inside"]:
            assert pl["pieces"] * B * Hkv <= cus * 5 // 4, what                                      # about one resident round


def test_plan_of_the_benchmark_shapes():
    # one sequence of 32K tokens, 8 kv heads, S + W = 2112, on 256 CUs: one workgroup of 8 waves per CU, no more
    for n in (32768, 32769, 32800, 32832):
        pl = pod.pod_decode_plan(256, 1, 8, 2112, n)
        assert pl["merge_inside"] and pl["waves"] == 8, (n, pl)
        assert pl["pieces"] * 8 <= 256, (n, pl)
        assert pl["pieces"] * 8 >= 240, (n, pl)
    # 16 sequences of up to 32K tokens / 4 of 128K: many rounds of 1024-token pieces, merged by the second kernel
    for B, P, n in ((16, 2112, 32777), (4, 4224, 131081)):
        pl = pod.pod_decode_plan(256, B, 8, P, n)
        assert not pl["merge_inside"] and pl["waves"] == 4 and pl["chunk"] == 1024 and pl["chunk_prox"] == 1024, pl


def test_plan_rejects_bad_arguments():
    for args in ((0, 1, 8, 2112, 100), (256, 0, 8, 2112, 100), (256, 1, 0, 2112, 100), (256, 1, 8, 0, 100), (256, 1, 8, 2112, 0)):
        with pytest.raises(pod.PodError) as e:
            pod.pod_decode_plan(*args)
        assert e.value.code == pod.binding.ERR_INVALID_ARG


# ---------------------------------------------------------------------------------------------- the even split

def walk_even_split(plan, Hkv, P, lens):
    """The walk decode_even_kernel makes, in Python: for every workgroup the (sequence, kv head, first unit, units)
    parts it takes, and the slot (workgroup - first workgroup of the pair) its partial goes to."""
    q, nwg, total, cum = plan["units_per_workgroup"], plan["workgroups"], plan["units"], plan["unit_cum"]
    parts = []
    for w in range(nwg):
        g, g_end = w * q, min((w + 1) * q, total)
        b = max(i for i in range(len(lens)) if cum[i] * Hkv <= g)      # (the kernel's binary search finds the same one)
        while g < g_end:
            U = cum[b + 1] - cum[b]
            rel = g - cum[b] * Hkv
            if U <= 0 or rel >= U * Hkv:
                b += 1
                continue
            h, u0 = divmod(rel, U)
            cnt = min(U - u0, g_end - g)
            w_lo = (cum[b] * Hkv + h * U) // q
            parts.append((w, b, h, u0, cnt, w - w_lo))
            g += cnt
    return parts


@pytest.mark.parametrize("seed", range(40))
def test_even_split_covers_every_unit_once_and_the_merge_counts_agree(seed):
    rng = np.random.default_rng(7000 + seed)
    cus = int(rng.choice([4, 64, 256, 304]))
    Hkv = int(rng.choice([1, 2, 8, 11]))
    P = int(rng.choice([40, 136, 2112, 4224]))
    B = int(rng.integers(1, 40))
    lens = [int(x) for x in rng.choice([0, 0, 1, 127, 128, 129, P, P + 1, 5000, 40000, 131072], size=B)]
    ud = int(rng.choice([128, 256]))      # 256: a score-reuse step of an upper layer (distant rows cost about half)
    plan = pod.pod_decode_even_plan(cus, Hkv, P, lens, distant_unit_tokens=ud)
    units = [(max(n - P, 0) + ud - 1) // ud + (min(n, P) + 127) // 128 for n in lens]
    assert plan["unit_cum"] == [sum(units[:b]) for b in range(B + 1)]
    total = Hkv * sum(units)
    if total == 0:
        assert plan["workgroups"] == 0
        return
    q, nwg = plan["units_per_workgroup"], plan["workgroups"]
    assert plan["units"] == total and nwg <= 2 * cus and (nwg - 1) * q < total <= nwg * q
    parts = walk_even_split(plan, Hkv, P, lens)
    seen = {}
    for w, b, h, u0, cnt, slot in parts:
        assert 0 <= slot < plan["partials_per_pair"]
        for u in range(u0, u0 + cnt):
            assert (b, h, u) not in seen
            seen[(b, h, u)] = w
    assert len(seen) == total
    # what decode_combine_kernel derives from a pair's length alone: as many partials as workgroups touch the pair,
    # in slots 0 .. count - 1, each written by exactly one workgroup
    most = 0
    for b in range(B):
        for h in range(Hkv):
            U = units[b]
            g0 = plan["unit_cum"][b] * Hkv + h * U
            count = (g0 + U - 1) // q - g0 // q + 1 if U else 0
            slots = sorted(s for w, bb, hh, u0, cnt, s in parts if (bb, hh) == (b, h))
            assert slots == list(range(count)), (b, h)
            most = max(most, count)
    assert most == plan["partials_per_pair"]


def test_even_split_rejects_bad_arguments():
    with pytest.raises(pod.PodError):
        pod.pod_decode_even_plan(0, 8, 2112, [100])
    with pytest.raises(pod.PodError):
        pod.pod_decode_even_plan(256, 8, 2112, [100] * 257)
    with pytest.raises(pod.PodError):
        pod.pod_decode_even_plan(256, 8, 2112, [100], distant_unit_tokens=64)
