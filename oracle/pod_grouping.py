"""TEST INFRASTRUCTURE ONLY (CPU oracle): offline grouping of layers into head-wise blocks.

Written from the paper's "Offline Inter-Layer Attention Sharing Exploration": the similarity of two
layers for one head is computed from the Jensen-Shannon divergence of their attention rows
(the equation defining sim_h), and consecutive layers are merged bottom-up into blocks (Greedy Layer
Grouping Algorithm).  Plain Python / numpy; nothing here is used by the product.

Readings taken where the text leaves a choice:
  * sim_h is said to be 1 for identical and 0 for completely dissimilar rows while being built from
    the JS divergence, which is 0 for identical rows: sim = 1 - mean JS with logarithms to base 2
    (base-2 JS lies in [0, 1]).
  * GQA: the similarity test for a kv head is a majority vote of its query heads (appendix); a tie is
    not a majority.
"""
import numpy as np


def js_divergence_base2(p, q):
    """Jensen-Shannon divergence of two probability vectors, logarithms to base 2 (in [0, 1])."""
    p = np.asarray(p, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    m = 0.5 * (p + q)

    def kl(a, b):
        nz = a > 0
        return float(np.sum(a[nz] * np.log2(a[nz] / b[nz])))

    return 0.5 * kl(p, m) + 0.5 * kl(q, m)


def layer_similarity(att_a, att_b):
    """sim_h(l_a, l_b) for one head: att_*: [N samples][q rows][n] attention rows of the two layers."""
    att_a = np.asarray(att_a, dtype=np.float64)
    att_b = np.asarray(att_b, dtype=np.float64)
    N, q, _ = att_a.shape
    total = 0.0
    for i in range(N):
        for j in range(q):
            total += js_divergence_base2(att_a[i, j], att_b[i, j])
    return 1.0 - total / (N * q)


def _lowest_layers(L, similar):
    """What the greedy bottom-up grouping (Greedy Layer Grouping Algorithm) arrives at, stated as a recurrence on the
    result rather than as the construction: blocks are runs of consecutive layers, layer 0 starts the first one, and
    layer l stays in the block of layer l - 1 exactly when it is similar to EVERY layer that block holds so far,
    i.e. to all of lowest[l-1] .. l-1; otherwise it is the lowest layer of a new block.
    similar(a, b) -> bool.  Returns the list lowest[0..L-1]."""
    lowest = [0] * L
    for l in range(1, L):
        start = lowest[l - 1]
        lowest[l] = start if all(similar(l, m) for m in range(start, l)) else l
    return lowest


def group_layers(sim, threshold=0.5):
    """sim: [H][L][L] with sim[h][a][b] the similarity of layers a, b for head h; two layers are similar for a head if
    sim >= threshold.  Returns lowest: int32 [L][H], the lowest layer of the block each layer belongs to."""
    sim = np.asarray(sim, dtype=np.float64)
    H, L, _ = sim.shape
    cols = [_lowest_layers(L, lambda a, b, h=h: sim[h, a, b] >= threshold) for h in range(H)]
    return np.array(cols, dtype=np.int32).T.reshape(L, H).copy()


def group_layers_gqa(sim, num_kv_heads, threshold=0.5):
    """The same per kv head: two layers count as similar for a kv head if more than half of its query heads say so
    (the appendix's majority vote; a tie is not a majority).  sim: [Hq][L][L].  Returns lowest: int32 [L][Hkv]."""
    sim = np.asarray(sim, dtype=np.float64)
    Hq, L, _ = sim.shape
    rep = Hq // num_kv_heads
    assert rep * num_kv_heads == Hq

    def majority(g):
        votes = (sim[g * rep:(g + 1) * rep] >= threshold).sum(axis=0)   # [L][L] query heads in favour
        return lambda a, b: 2 * int(votes[a, b]) > rep

    cols = [_lowest_layers(L, majority(g)) for g in range(num_kv_heads)]
    return np.array(cols, dtype=np.int32).T.reshape(L, num_kv_heads).copy()
