"""TEST INFRASTRUCTURE ONLY (CPU oracle): offline grouping of layers into head-wise blocks.

Written from the paper's "Offline Inter-Layer Attention Sharing Exploration": the similarity of two
layers for one head is computed from the Jensen-Shannon divergence of their attention rows
(the equation defining sim_h), and consecutive layers are merged bottom-up into blocks (Greedy Layer
Grouping Algorithm).  Plain Python / numpy, loops as in the text; nothing here is used by the product.

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


def group_layers(sim, threshold=0.5):
    """Greedy Layer Grouping Algorithm.  sim: [H][L][L] with sim[h][a][b] the similarity of layers a, b for head h.
    Returns lowest: int32 [L][H], the lowest layer of the block each layer was put in."""
    sim = np.asarray(sim, dtype=np.float64)
    H, L, _ = sim.shape
    lowest = np.zeros((L, H), dtype=np.int32)
    for h in range(H):
        blocks = [[0]]
        for l in range(1, L):
            current = blocks[-1]
            if all(sim[h, l, lh] >= threshold for lh in current):
                current.append(l)
            else:
                blocks.append([l])
        for blk in blocks:
            for l in blk:
                lowest[l, h] = blk[0]
    return lowest


def group_layers_gqa(sim, num_kv_heads, threshold=0.5):
    """The same per kv head: two layers count as similar for a kv head if more than half of its query heads say so.
    sim: [Hq][L][L].  Returns lowest: int32 [L][Hkv]."""
    sim = np.asarray(sim, dtype=np.float64)
    Hq, L, _ = sim.shape
    rep = Hq // num_kv_heads
    assert rep * num_kv_heads == Hq
    lowest = np.zeros((L, num_kv_heads), dtype=np.int32)
    for g in range(num_kv_heads):
        heads = range(g * rep, (g + 1) * rep)

        def similar(a, b):
            votes = sum(1 for h in heads if sim[h, a, b] >= threshold)
            return 2 * votes > rep

        blocks = [[0]]
        for l in range(1, L):
            current = blocks[-1]
            if all(similar(l, lh) for lh in current):
                current.append(l)
            else:
                blocks.append([l])
        for blk in blocks:
            for l in blk:
                lowest[l, g] = blk[0]
    return lowest
