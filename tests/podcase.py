"""Shared set-up for the GPU parity tests: the same seeded inputs go into libpod's cache on
the GPU and into the CPU oracle's cache model.  Inputs are generated separately on each side
(the generator is counter-based and bit-identical across devices)."""
import math

import numpy as np
import torch

import paper_2412_02252_amd as pod
from oracle import pod_oracle as po
from pod_inputs import gen

MAX_ABS, MEAN_ABS = 2e-2, 2e-3   # bf16 inputs, fp32 accumulation, bf16 output: the stated bounds, absolute
# Relative bounds, which keep their meaning where the outputs are small (at 32K tokens of unit-variance values an
# output element is ~0.01, so the absolute bounds alone would let a 20 % error through).  Per element the GPU result
# differs from the exact one by (a) the round-to-nearest of the output to bf16, at most 2^-8 of the element (half an
# ulp of an 8-bit significand), about 2^-9.5 of it on average; (b) the bf16 rounding of the probabilities that enter
# the PV product: sum_j p_j e_j v_j with independent |e_j| <= 2^-8, whose standard deviation is at most
# 2^-8 / sqrt(3) of sqrt(sum_j p_j^2 v_j^2), i.e. of the size of the output itself when the weights are spread over
# many tokens; (c) fp32 summation order, 2^-24 per operation, negligible.  Together about 2^-9 of the output's rms
# per element on average.  The bounds below leave a factor of about two to four over that and over the largest
# error measured on the GPU at the large configurations:
#   max |err| <= 2^-7 max |ref|        mean |err| <= 2^-8 rms(ref)
REL_MAX, REL_MEAN = 2.0 ** -7, 2.0 ** -8


def closeness_failures(got: np.ndarray, ref: np.ndarray):
    """The bounds a result must keep against the oracle's: a list of the violated ones (empty = close enough)."""
    err = np.abs(got - ref)
    peak, rms = float(np.abs(ref).max(initial=0.0)), float(np.sqrt(np.mean(np.square(ref)))) if ref.size else 0.0
    bad = []
    if err.size == 0:
        return bad
    if err.max() > MAX_ABS:
        bad.append(f"max abs err {err.max():.3e} > {MAX_ABS:g}")
    if err.mean() > MEAN_ABS:
        bad.append(f"mean abs err {err.mean():.3e} > {MEAN_ABS:g}")
    if err.max() > REL_MAX * peak:
        bad.append(f"max abs err {err.max():.3e} > 2^-7 of the largest reference value {peak:.3e}")
    if err.mean() > REL_MEAN * rms:
        bad.append(f"mean abs err {err.mean():.3e} > 2^-8 of the reference rms {rms:.3e}")
    return bad


def assert_close(got_bf16: torch.Tensor, ref_f64: np.ndarray, what=""):
    got = got_bf16.float().cpu().numpy().astype(np.float64)
    assert got.shape == ref_f64.shape, (got.shape, ref_f64.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    bad = closeness_failures(got, ref_f64)
    assert not bad, f"{what}: " + "; ".join(bad)


class Case:
    def __init__(self, L, G, Hq, Hkv, d, S, W, B, max_ctx, seed=1, device="cuda:0", with_oracle_cache=True,
                 block_lowest=None, **kgen):
        self.L, self.G, self.Hq, self.Hkv, self.d, self.S, self.W, self.B = L, G, Hq, Hkv, d, S, W, B
        self.max_ctx, self.seed, self.dev, self.kgen = max_ctx, seed, device, kgen
        # lowest[l][h]: lowest layer of the block of (layer l, kv head h); uniform blocks of G layers by default
        self.lowest = (np.array([[l - l % G] * Hkv for l in range(L)], dtype=np.int32) if block_lowest is None
                       else np.ascontiguousarray(block_lowest, dtype=np.int32))
        self.cfg = pod.make_config(L, G, Hq, Hkv, d, S, W, B, max_ctx, block_lowest=block_lowest)
        self.gpu = pod.PodCache(self.cfg, device, guard_bytes=4096)   # guard bands around every caller buffer (conftest checks them)
        self.cpu = po.Cache(L, G, Hkv, d, S, W, B, max_ctx, block_lowest=block_lowest) if with_oracle_cache else None
        self.scale = 1.0 / math.sqrt(d)

    # ---- inputs (device = "cpu" or the GPU) -------------------------------------------
    def keys(self, layer, seq, n, device, pos0=0, **kw):
        return gen.keys_bf16(self.seed, layer, seq, n, self.Hkv, self.d, device=device, pos0=pos0, **self.kgen, **kw)

    def values(self, layer, seq, n, device, pos0=0, **kw):
        return gen.values_bf16(self.seed, layer, seq, n, self.Hkv, self.d, device=device, pos0=pos0, **kw)

    def queries(self, layer, seq, n, device, pos0=0):
        return gen.queries_bf16(self.seed, layer, seq, n, self.Hq, self.d, device=device, pos0=pos0)

    # ---- both sides ---------------------------------------------------------------------
    def fill(self, layer, seq, n):
        self.gpu.pod_cache_fill(layer, seq, self.keys(layer, seq, n, self.dev), self.values(layer, seq, n, self.dev))
        if self.cpu is not None:
            self.cpu.fill(layer, seq, gen.bf16_bits(self.keys(layer, seq, n, "cpu")),
                          gen.bf16_bits(self.values(layer, seq, n, "cpu")))

    def append(self, layer, positions):
        """positions: list with one entry per sequence 0..len-1."""
        B = len(positions)
        k = torch.cat([self.keys(layer, b, 1, self.dev, pos0=p) for b, p in enumerate(positions)])
        v = torch.cat([self.values(layer, b, 1, self.dev, pos0=p) for b, p in enumerate(positions)])
        pos = torch.tensor(positions, dtype=torch.int32, device=self.dev)
        self.gpu.pod_cache_append(layer, k.contiguous(), v.contiguous(), pos)
        if self.cpu is not None:
            kc = torch.cat([self.keys(layer, b, 1, "cpu", pos0=p) for b, p in enumerate(positions)])
            vc = torch.cat([self.values(layer, b, 1, "cpu", pos0=p) for b, p in enumerate(positions)])
            self.cpu.append(layer, gen.bf16_bits(kc), gen.bf16_bits(vc), positions)
        assert B <= self.B

    def step(self, layer, positions, max_context_len=0):
        """pod_decode_step on the GPU (append + attention in one launch) and the plain append on the oracle's model;
        returns the GPU output for contexts positions + 1."""
        k = torch.cat([self.keys(layer, b, 1, self.dev, pos0=p) for b, p in enumerate(positions)]).contiguous()
        v = torch.cat([self.values(layer, b, 1, self.dev, pos0=p) for b, p in enumerate(positions)]).contiguous()
        ctx = [p + 1 for p in positions]
        q = self.decode_queries(layer, ctx, self.dev)
        qs = self.shared_queries(layer, ctx, self.dev)
        pos = torch.tensor(positions, dtype=torch.int32, device=self.dev)
        out = self.gpu.pod_decode_step(layer, k, v, q, qs, pos, self.scale, max_context_len=max_context_len)
        if self.cpu is not None:
            kc = torch.cat([self.keys(layer, b, 1, "cpu", pos0=p) for b, p in enumerate(positions)])
            vc = torch.cat([self.values(layer, b, 1, "cpu", pos0=p) for b, p in enumerate(positions)])
            self.cpu.append(layer, gen.bf16_bits(kc), gen.bf16_bits(vc), positions)
        return out

    def step_reuse(self, layer, positions, scores, max_context_len=0):
        """pod_decode_step_reuse on the GPU (the block's lowest layer must take the token first) and the plain append on
        the oracle's model; returns the GPU output for contexts positions + 1."""
        k = torch.cat([self.keys(layer, b, 1, self.dev, pos0=p) for b, p in enumerate(positions)]).contiguous()
        v = torch.cat([self.values(layer, b, 1, self.dev, pos0=p) for b, p in enumerate(positions)]).contiguous()
        q = self.decode_queries(layer, [p + 1 for p in positions], self.dev)
        pos = torch.tensor(positions, dtype=torch.int32, device=self.dev)
        out = self.gpu.pod_decode_step_reuse(layer, k, v, q, pos, self.scale, scores, max_context_len=max_context_len)
        if self.cpu is not None:
            kc = torch.cat([self.keys(layer, b, 1, "cpu", pos0=p) for b, p in enumerate(positions)])
            vc = torch.cat([self.values(layer, b, 1, "cpu", pos0=p) for b, p in enumerate(positions)])
            self.cpu.append(layer, gen.bf16_bits(kc), gen.bf16_bits(vc), positions)
        return out

    def decode_queries(self, layer, ctx, device):
        """Query of the token at position ctx[b]-1 of each sequence: [B][Hq][d]."""
        return torch.cat([self.queries(layer, b, 1, device, pos0=max(n, 1) - 1) for b, n in enumerate(ctx)]).contiguous()

    def shared_queries(self, layer, ctx, device):
        """q_shared for `layer`: head by head the query of the lowest layer of that head's block; None if the
        layer is the lowest for every head."""
        src = self.lowest[layer]
        if (src == layer).all():
            return None
        rep = self.Hq // self.Hkv
        per_layer = {int(l): self.decode_queries(int(l), ctx, device) for l in set(src.tolist())}
        return torch.stack([per_layer[int(src[h // rep])][:, h] for h in range(self.Hq)], dim=1).contiguous()

    def decode(self, layer, ctx, max_context_len=0):
        q = self.decode_queries(layer, ctx, self.dev)
        qs = self.shared_queries(layer, ctx, self.dev)
        ctx_t = torch.tensor(ctx, dtype=torch.int32, device=self.dev)
        return self.gpu.pod_decode_attention(layer, q, qs, ctx_t, self.scale, max_context_len=max_context_len)

    def decode_reuse(self, layer, ctx, scores, max_context_len=0):
        """Score-reuse entry point: the block's lowest layer must be called first for this token."""
        q = self.decode_queries(layer, ctx, self.dev)
        ctx_t = torch.tensor(ctx, dtype=torch.int32, device=self.dev)
        return self.gpu.pod_decode_attention_reuse(layer, q, ctx_t, self.scale, scores, max_context_len=max_context_len)

    def decode_ref(self, layer, ctx):
        q = gen.bf16_bits(self.decode_queries(layer, ctx, "cpu"))
        qs = self.shared_queries(layer, ctx, "cpu")
        qs = gen.bf16_bits(qs) if qs is not None else None
        return self.cpu.decode_attention(layer, q, qs, ctx, self.scale)

    def assert_cache_equal(self, layer, seq):
        g = self.gpu.pod_cache_export_logical(layer, seq)
        c = self.cpu.export(layer, seq)
        assert set(g) == set(c)
        for name in c:
            assert np.array_equal(gen.bf16_bits(g[name]), c[name]), f"layer {layer} seq {seq} {name}"
