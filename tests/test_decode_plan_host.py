"""The split-K plan of a decode launch (host logic, no GPU): pod_decode_plan.  Whatever the shape, the pieces are whole
tiles, cover both regions, fit the workspace bound, and the partials are merged inside the launch only where the
launch is about one resident round of workgroups."""
import itertools

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
