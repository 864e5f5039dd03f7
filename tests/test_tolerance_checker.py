"""The parity checker itself (tests/podcase.py): at the headline shape (32768 tokens of unit-variance values, where
an output element is about 0.01) it must reject a 5 % error and accept the rounding a correct bf16 result carries.
CPU only: both inputs come from the oracle."""
import math

import numpy as np
import torch

from oracle import pod_oracle as po
from pod_inputs import gen
from podcase import MAX_ABS, MEAN_ABS, closeness_failures


def _config2_shaped_reference():
    G, Hq, Hkv, d, S, W, n, seed = 2, 32, 8, 128, 64, 2048, 32768, 20241202 + 2
    oc = po.Cache(G, G, Hkv, d, S, W, 1, n)
    rope = dict(rope_base=500000.0, rope_max_pos=n)
    for layer in range(G):
        oc.fill(layer, 0, gen.bf16_bits(gen.keys_bf16(seed, layer, 0, n, Hkv, d, device="cpu", **rope)),
                gen.bf16_bits(gen.values_bf16(seed, layer, 0, n, Hkv, d, device="cpu")))
    q = [gen.bf16_bits(gen.queries_bf16(seed, layer, 0, 1, Hq, d, device="cpu", pos0=n - 1)) for layer in range(G)]
    scale = 1.0 / math.sqrt(d)
    return np.stack([oc.decode_attention(0, q[0], None, [n], scale), oc.decode_attention(1, q[1], q[0], [n], scale)])


def test_checker_rejects_five_percent_and_accepts_bf16_rounding():
    ref = _config2_shaped_reference()
    assert 5e-3 < np.sqrt(np.mean(ref ** 2)) < 2e-2          # the regime the relative bounds are for
    # the absolute bounds alone would accept a 20 % error here
    off = ref * 1.2
    assert np.abs(off - ref).max() <= MAX_ABS and np.abs(off - ref).mean() <= MEAN_ABS
    assert closeness_failures(off, ref)
    assert closeness_failures(ref * 1.05, ref)
    assert closeness_failures(ref * 0.95, ref)
    rounded = torch.from_numpy(ref).to(torch.bfloat16).double().numpy()
    assert closeness_failures(rounded, ref) == []
    # one element off by 3 % of the largest value, everything else exact: the max bound notices
    one = ref.copy()
    one.flat[1234] += 0.03 * np.abs(ref).max()
    assert closeness_failures(one, ref)


def test_checker_handles_zero_rows_and_empty_results():
    z = np.zeros((2, 4, 8))
    assert closeness_failures(z, z) == []
    assert closeness_failures(np.zeros((0, 4)), np.zeros((0, 4))) == []
    assert closeness_failures(z + 1e-3, z)
