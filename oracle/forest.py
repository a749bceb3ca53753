"""Forest topology: depths, layers and ancestor sets by walking parent pointers.

The draft forest has one tree per input beam (Section 3.1, Overview); the
attention mask of a tree is its topology: a node sees its ancestors and itself
(Section 3.3 and the caption of the forest-attention figure).
"""
import numpy as np


def check_forest(parent, tree_off):
    """Raise ValueError unless trees are contiguous, rooted at their first node, parent < child."""
    parent = np.asarray(parent)
    T = len(tree_off) - 1
    if tree_off[0] != 0 or tree_off[-1] != len(parent):
        raise ValueError("tree_off must cover all nodes")
    for t in range(T):
        a, b = int(tree_off[t]), int(tree_off[t + 1])
        if b <= a:
            raise ValueError("empty tree")
        if parent[a] != -1:
            raise ValueError("first node of a tree must be its root")
        for n in range(a + 1, b):
            if not (a <= parent[n] < n):
                raise ValueError("parent outside the tree or not before the child")


def depths(parent):
    """depth[root] = 0, depth[n] = depth[parent[n]] + 1."""
    parent = np.asarray(parent)
    d = np.zeros(len(parent), dtype=np.int32)
    for n in range(len(parent)):
        d[n] = 0 if parent[n] < 0 else d[parent[n]] + 1
    return d


def ancestors_or_self(parent, n):
    """Node ids on the path from n up to its root (n first)."""
    out = []
    while n >= 0:
        out.append(int(n))
        n = int(parent[n])
    return out


def tree_of_node(tree_off, n_nodes):
    t = np.zeros(n_nodes, dtype=np.int32)
    for i in range(len(tree_off) - 1):
        t[tree_off[i]:tree_off[i + 1]] = i
    return t


def ancestor_masks(parent, tree_off):
    """anc_mask[n]: bit j set iff the j-th node of n's tree is an ancestor of n or n itself."""
    parent = np.asarray(parent)
    tree = tree_of_node(tree_off, len(parent))
    out = np.zeros(len(parent), dtype=np.uint64)
    for n in range(len(parent)):
        base = int(tree_off[tree[n]])
        m = 0
        for a in ancestors_or_self(parent, n):
            m |= 1 << (a - base)
        out[n] = np.uint64(m)
    return out
