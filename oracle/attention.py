"""Forest attention, written out from its definition (Section 3.3).

Each input beam keeps its own key-value cache; each tree of the draft forest is
decoded against the cache of the beam it grows from, with a mask that follows the
tree's topology.  So node n of tree b, head h, attends to
  * every prefix position of beam b, and
  * the tree rows of n's ancestors and of n itself,
with ordinary scaled dot-product attention (scale 1/sqrt(D) by default).
Grouped-query attention: query head h reads KV head h // (Hq // Hkv).
"""
import numpy as np

from .forest import ancestors_or_self, tree_of_node


def forest_attention(parent, tree_off, q, k_tree, v_tree, prefix_k, prefix_v, scale=None):
    """
    q        [N,Hq,D]   float64
    k_tree   [N,Hkv,D]  float64 (row n = key of forest node n), v_tree likewise
    prefix_k list over trees of [L_b,Hkv,D] float64 (the beam's whole prefix), prefix_v likewise
    returns  out [N,Hq,D] float64, lse [N,Hq] float64
    """
    q = np.asarray(q, dtype=np.float64)
    k_tree = np.asarray(k_tree, dtype=np.float64)
    v_tree = np.asarray(v_tree, dtype=np.float64)
    N, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    group = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    tree = tree_of_node(tree_off, N)
    out = np.zeros((N, Hq, D))
    lse = np.zeros((N, Hq))
    for n in range(N):
        b = int(tree[n])
        anc = sorted(ancestors_or_self(parent, n))
        for h in range(Hq):
            g = h // group
            keys = np.concatenate([np.asarray(prefix_k[b], dtype=np.float64)[:, g, :], k_tree[anc, g, :]], axis=0)
            vals = np.concatenate([np.asarray(prefix_v[b], dtype=np.float64)[:, g, :], v_tree[anc, g, :]], axis=0)
            s = (keys @ q[n, h]) * scale
            m = s.max()
            e = np.exp(s - m)
            z = e.sum()
            out[n, h] = (e / z) @ vals
            lse[n, h] = m + np.log(z)
    return out, lse


def forest_attention_at(parent, tree_off, q, k_tree, v_tree, prefix_k_b, prefix_v_b, n, h, scale=None):
    """The same definition for a single (node n, head h); prefix_*_b is the prefix of n's own beam."""
    N, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    g = h // (Hq // Hkv)
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    anc = sorted(ancestors_or_self(parent, n))
    keys = np.concatenate([np.asarray(prefix_k_b[:, g, :], dtype=np.float64),
                           np.asarray(k_tree[anc, g, :], dtype=np.float64)], axis=0)
    vals = np.concatenate([np.asarray(prefix_v_b[:, g, :], dtype=np.float64),
                           np.asarray(v_tree[anc, g, :], dtype=np.float64)], axis=0)
    s = (keys @ np.asarray(q[n, h], dtype=np.float64)) * scale
    m = s.max()
    e = np.exp(s - m)
    z = e.sum()
    return (e / z) @ vals, m + np.log(z)
