"""Seeded synthetic inputs for the PoD attention path (test / bench plumbing only).

Everything here is a *counter-based* generator: the value of element
(pos, head, dim) of a tensor depends only on (seed, tensor id, layer, seq, pos,
head, dim), so the GPU side can build a 40 GB cache on the device while the CPU
side regenerates only the few (layer, seq, head) slices it wants to check, and
both get the same bits.  The arithmetic is integer hashing followed by a lookup
in a host-built table of N(0,1) quantiles, run through torch integer ops, which
give identical results on CPU and GPU tensors.  Nothing of the attention method
itself lives in this module.

Shapes follow LLaMA3-8B style workloads: K/V are [n_pos][n_kv_heads][d],
Q is [n_pos][n_q_heads][d], all bf16.
"""
from __future__ import annotations

import functools
import math

import numpy as np
import torch

M32 = 0xFFFFFFFF

# tensor ids (one stream of random numbers per kind of tensor)
T_K, T_V, T_Q, T_OUTLIER = 1, 2, 3, 4


def _mix_scalar(*words: int) -> int:
    """Fold python ints into one 32-bit stream key (host only)."""
    h = 0x9E3779B1
    for w in words:
        w &= M32
        h ^= w
        h = (h * 0x2545F491) & M32
        h ^= h >> 15
        h = (h * 0x1B873593) & M32
        h ^= h >> 13
    return h


def _mix_tensor(x: torch.Tensor, key: int) -> torch.Tensor:
    """32-bit avalanche of an int64 tensor whose values lie in [0, 2^32).

    Multipliers are below 2^31 so no product leaves the int64 range: the result
    never depends on overflow behaviour and is identical on any device.
    """
    x = (x + (key & M32)) & M32
    x = x ^ (x >> 16)
    x = (x * 0x45D9F3B) & M32
    x = x ^ (x >> 15)
    x = (x * 0x2C1B3C6D) & M32
    x = x ^ (key >> 7)
    x = x ^ (x >> 13)
    x = (x * 0x297A2D39) & M32
    x = x ^ (x >> 16)
    return x


@functools.lru_cache(maxsize=None)
def _normal_table_host() -> torch.Tensor:
    """65536 N(0,1) quantiles at the bin centres, float32 (built in float64)."""
    from scipy.special import ndtri

    u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return torch.from_numpy(ndtri(u).astype(np.float32))


_table_cache: dict = {}


def normal_table(device) -> torch.Tensor:
    device = torch.device(device)
    if device not in _table_cache:
        _table_cache[device] = _normal_table_host().to(device)
    return _table_cache[device]


def _counters(pos0, n_pos, head0, n_heads, n_heads_total, d, device):
    pos = torch.arange(pos0, pos0 + n_pos, dtype=torch.int64, device=device)
    head = torch.arange(head0, head0 + n_heads, dtype=torch.int64, device=device)
    dim = torch.arange(d, dtype=torch.int64, device=device)
    c = (pos[:, None, None] * n_heads_total + head[None, :, None]) * d + dim[None, None, :]
    return c  # < 2^32 for every workload here (checked by the caller)


def normal_f32(seed, tensor_id, layer, seq, n_pos, n_heads_total, d, *, device="cpu",
               pos0=0, head0=0, n_heads=None) -> torch.Tensor:
    """float32 [n_pos][n_heads][d] of N(0,1) draws for positions pos0.. and heads head0.."""
    if n_heads is None:
        n_heads = n_heads_total - head0
    assert (pos0 + n_pos) * n_heads_total * d < (1 << 32), "slice too large for 32-bit counters"
    key = _mix_scalar(seed, tensor_id, layer, seq)
    out = torch.empty((n_pos, n_heads, d), dtype=torch.float32, device=device)
    table = normal_table(device)
    step = max(1, (1 << 24) // max(1, n_heads * d))  # bound the int64 temporaries
    for a in range(0, n_pos, step):
        b = min(n_pos, a + step)
        c = _counters(pos0 + a, b - a, head0, n_heads, n_heads_total, d, device)
        idx = _mix_tensor(c, key) >> 16
        out[a:b] = table[idx]
    return out


def to_bf16(x: torch.Tensor) -> torch.Tensor:
    return x.to(torch.bfloat16)  # round-to-nearest-even on every device


def normal_bf16(seed, tensor_id, layer, seq, n_pos, n_heads_total, d, **kw) -> torch.Tensor:
    return to_bf16(normal_f32(seed, tensor_id, layer, seq, n_pos, n_heads_total, d, **kw))


@functools.lru_cache(maxsize=8)
def _rope_tables_host(max_pos: int, d: int, base: float):
    half = d // 2
    inv = base ** (-np.arange(half, dtype=np.float64) / half)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * inv[None, :]
    return (torch.from_numpy(np.cos(ang).astype(np.float32)),
            torch.from_numpy(np.sin(ang).astype(np.float32)))


def rope_rotate(x: torch.Tensor, pos0: int, base: float, max_pos: int) -> torch.Tensor:
    """Rotary embedding (half-split pairing) of float32 x [n_pos][H][d] at positions pos0..

    cos/sin come from a host float64 table so CPU and GPU see the same float32
    factors; products and sums are separate float32 ops (no fused multiply-add).
    """
    n, _, d = x.shape
    half = d // 2
    cos, sin = _rope_tables_host(max_pos, d, float(base))
    cos = cos[pos0:pos0 + n].to(x.device)[:, None, :]
    sin = sin[pos0:pos0 + n].to(x.device)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    a = x1 * cos
    b = x2 * sin
    c = x2 * cos
    e = x1 * sin
    return torch.cat([a - b, c + e], dim=-1)


def outlier_rows(seed, layer, seq, n_pos, n_heads_total, *, device="cpu", pos0=0,
                 head0=0, n_heads=None, rate=0.01) -> torch.Tensor:
    """bool [n_pos][n_heads]: rows Bernoulli(rate)-selected to carry outlier keys."""
    if n_heads is None:
        n_heads = n_heads_total - head0
    key = _mix_scalar(seed, T_OUTLIER, layer, seq)
    c = _counters(pos0, n_pos, head0, n_heads, n_heads_total, 1, device)[..., 0]
    u = _mix_tensor(c, key) >> 8  # 24 bits
    return u < int(rate * (1 << 24))


def keys_bf16(seed, layer, seq, n_pos, n_kv_heads, d, *, device="cpu", pos0=0, head0=0,
              n_heads=None, rope_base=None, rope_max_pos=None, outlier_rate=0.0,
              outlier_scale=8.0, outlier_lo=0, outlier_hi=None) -> torch.Tensor:
    """Keys [n_pos][n_heads][d] bf16: N(0,1), optionally RoPE-rotated, optionally with
    a fraction of rows in positions [outlier_lo, outlier_hi) scaled before rounding."""
    x = normal_f32(seed, T_K, layer, seq, n_pos, n_kv_heads, d, device=device, pos0=pos0,
                   head0=head0, n_heads=n_heads)
    if rope_base is not None:
        x = rope_rotate(x, pos0, rope_base, rope_max_pos)
    if outlier_rate > 0.0:
        sel = outlier_rows(seed, layer, seq, n_pos, n_kv_heads, device=device, pos0=pos0,
                           head0=head0, n_heads=n_heads, rate=outlier_rate)
        p = torch.arange(pos0, pos0 + n_pos, device=device)
        hi = outlier_hi if outlier_hi is not None else (1 << 62)
        sel = sel & ((p >= outlier_lo) & (p < hi))[:, None]
        x = torch.where(sel[..., None], x * outlier_scale, x)
    return to_bf16(x)


def values_bf16(seed, layer, seq, n_pos, n_kv_heads, d, **kw) -> torch.Tensor:
    return normal_bf16(seed, T_V, layer, seq, n_pos, n_kv_heads, d, **kw)


def queries_bf16(seed, layer, seq, n_pos, n_q_heads, d, **kw) -> torch.Tensor:
    return normal_bf16(seed, T_Q, layer, seq, n_pos, n_q_heads, d, **kw)


def ragged_lengths(seed, batch, lo, hi) -> list:
    """Per-sequence context lengths, uniform integers in [lo, hi]."""
    key = _mix_scalar(seed, 99)
    c = torch.arange(batch, dtype=torch.int64)
    u = _mix_tensor(c, key)
    return [int(lo + (int(v) % (hi - lo + 1))) for v in u]


# ---- bf16 <-> raw 16-bit helpers (the CPU checker takes bf16 as uint16 bit patterns) ----

def bf16_bits(x: torch.Tensor) -> np.ndarray:
    assert x.dtype == torch.bfloat16
    return x.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def bits_to_bf16(b: np.ndarray, device="cpu") -> torch.Tensor:
    return torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).to(device)
