"""CPU oracle of token selection on the distant store (test infrastructure only: the product never imports it).

The paper combines its cache with a token-selection method (the rows "PoD+SnapKV" of its result tables and the
appendix section on SnapKV: an observation window of 64 prompt positions, extended to grouped-query attention) and
gives no rule of its own.  This module restates the published selection rule on the part of the cache that the
combination can shrink, the distant tokens (the proximal ones are kept in full by definition, Section 3):

  1. vote:   every query of the last `obs` prompt positions, in every query head of a kv head's group, spreads its
             attention over the keys up to its own position (the joint softmax of Eq. 4; at a block's lowest layer
             every logit is that layer's own q.k, Eq. 3, and these logits are the ones the whole block uses for its
             distant tokens).  vote[h][t] = the attention that distant token t receives, summed over those queries.
  2. pool:   each vote is replaced by the mean (zeros outside the distant range) or the maximum of the 2r+1 votes
             around it, so that neighbours of an important token survive with it.
  3. select: the `keep` largest pooled votes per kv head; of equal votes the earlier token wins; ascending order.
  4. compact: the cache then holds, per (block, kv head), the sink tokens, the selected distant tokens and the recent
             tokens, i.e. it is the cache of that shorter sequence.

Plain numpy in float64 (steps 2-3 also in the precision they are handed, since they decide integers); loops over
heads and queries, no blocking.  Pins: tests/test_oracle_select_pins.py (library softmax, convolution and rank-filter
routines, closed forms for constant queries, brute force, conservation of the attention mass, the memory figures of
the paper's efficiency table).  Each function is pinned to the mathematics stated above; that this rule is the one the
paper's authors ran is a reading (the paper names the method and two settings, prints no rule and no worked example):
against the paper's own combination, parity unpinned.
"""
from __future__ import annotations

import numpy as np


def bf16_to_f64(u16):
    """float64 values of raw bf16 bit patterns (numpy uint16)."""
    u = np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def distant_votes(q_obs, k, S, W, scale):
    """q_obs: uint16 [obs][Hq][d], the queries of prompt positions n-obs .. n-1; k: uint16 [n][Hkv][d], the prompt's
    keys at the same layer.  Returns float64 [Hkv][n - S - W]: the attention distant token S + t receives (step 1)."""
    obs, Hq, d = q_obs.shape
    n, Hkv, _ = k.shape
    assert Hq % Hkv == 0 and 1 <= obs <= W and n - S - W >= 1
    rep = Hq // Hkv
    qf, kf = bf16_to_f64(q_obs), bf16_to_f64(k)
    votes = np.zeros((Hkv, n - S - W))
    for hq in range(Hq):
        h = hq // rep
        for i in range(obs):
            pos = n - obs + i                       # the query's own position: it sees keys 0 .. pos
            logits = scale * (kf[:pos + 1, h, :] @ qf[i, hq, :])
            w = np.exp(logits - logits.max())
            w /= w.sum()
            votes[h] += w[S:n - W]
    return votes


def pool_votes(votes, width, kind):
    """Step 2 over the last axis.  width odd; kind 'avg' (window sum / width, zeros outside) or 'max' (over the
    positions that exist).  Computed in the dtype of `votes`, left to right."""
    assert width >= 1 and width % 2 == 1 and kind in ("avg", "max")
    r = width // 2
    H, m = votes.shape
    out = np.empty_like(votes)
    for h in range(H):
        for t in range(m):
            lo, hi = max(0, t - r), min(m, t + r + 1)
            if kind == "max":
                out[h, t] = votes[h, lo:hi].max()
            else:
                acc = votes.dtype.type(0)
                for u in range(lo, hi):
                    acc = acc + votes[h, u]
                out[h, t] = acc / votes.dtype.type(width)
    return out


def select_top(pooled, keep):
    """Step 3: int32 [H][keep], ascending token indices of the `keep` largest entries of each row (ties: lower index)."""
    H, m = pooled.shape
    assert 1 <= keep <= m
    sel = np.empty((H, keep), dtype=np.int32)
    for h in range(H):
        order = sorted(range(m), key=lambda t: (-pooled[h, t], t))
        sel[h] = sorted(order[:keep])
    return sel


def compact_sequence(x, sel_of_head, S, W):
    """Step 4 for one layer: x uint16 [n][Hkv][d] (keys or values of the whole prompt), sel_of_head int [Hkv][keep]
    (the selection of the block each kv head belongs to at this layer).  Returns uint16 [S + keep + W][Hkv][d]."""
    n, Hkv, d = x.shape
    keep = sel_of_head.shape[1]
    out = np.empty((S + keep + W, Hkv, d), dtype=np.uint16)
    for h in range(Hkv):
        tokens = list(range(S)) + [S + int(t) for t in sel_of_head[h]] + list(range(n - W, n))
        out[:, h, :] = x[tokens, h, :]
    return out
