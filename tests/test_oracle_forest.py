"""Pins for the oracle's forest topology: ancestor masks must equal the reflexive-transitive closure
of the parent relation, computed here a different way (boolean matrix powers)."""
import numpy as np
import pytest

from dsbd_synth import make_workload
from oracle import forest


def closure_by_matrix_powers(parent):
    n = len(parent)
    A = np.eye(n, dtype=bool)
    step = np.zeros((n, n), dtype=bool)
    for c, p in enumerate(parent):
        if p >= 0:
            step[c, p] = True
    reach = A.copy()
    cur = A.copy()
    stepf = step.astype(np.float32)
    for _ in range(n):
        cur = (cur.astype(np.float32) @ stepf) > 0
        if not cur.any():
            break
        reach |= cur
    return reach        # reach[c, a] = a is an ancestor of c or c itself


@pytest.mark.parametrize("cfg", ["c1", "c2", "c3", "c4", "c5"])
def test_ancestor_masks_equal_closure(cfg):
    w = make_workload(cfg, L=4, V=8, Hq=2, Hkv=1, D=64) if cfg != "c4" else make_workload(cfg, L=(2, 4), V=8, Hq=2, Hkv=1, D=64)
    forest.check_forest(w.parent, w.tree_off)
    masks = forest.ancestor_masks(w.parent, w.tree_off)
    reach = closure_by_matrix_powers(w.parent)
    tree = forest.tree_of_node(w.tree_off, w.n_nodes)
    for n in range(w.n_nodes):
        base = int(w.tree_off[tree[n]])
        size = int(w.tree_off[tree[n] + 1]) - base
        bits = [(int(masks[n]) >> j) & 1 for j in range(size)]
        assert bits == [int(reach[n, base + j]) for j in range(size)]
        # nothing outside the node's own tree is reachable
        assert reach[n].sum() == sum(bits)
        assert int(masks[n]) >> size == 0


def test_depths_and_known_tree():
    # root with children 1, 2; 3 under 1; 4 under 3
    parent = [-1, 0, 0, 1, 3]
    assert forest.depths(parent).tolist() == [0, 1, 1, 2, 3]
    m = forest.ancestor_masks(parent, [0, 5])
    assert [int(x) for x in m] == [0b00001, 0b00011, 0b00101, 0b01011, 0b11011]
    assert forest.ancestors_or_self(parent, 4) == [4, 3, 1, 0]


def test_check_forest_rejects_bad_topologies():
    forest.check_forest([-1, 0, -1, 2], [0, 2, 4])
    for parent, off in [([-1, 0, 0, 2], [0, 2, 4]),      # second tree's first node is not a root
                        ([-1, 0, -1, 1], [0, 2, 4]),     # parent in another tree
                        ([-1, 1], [0, 2]),               # parent not before child
                        ([0, -1], [0, 2])]:
        with pytest.raises(ValueError):
            forest.check_forest(parent, off)
