"""Physical key/value cache update after an iteration (test infrastructure: CPU oracle, not the product path).

After verification the caches are updated to follow the output beams (Section 3.3, last paragraph): the
cache of a next-iteration beam is the cache of the input beam it descends from, extended by the key/value
rows of the forest nodes between that beam's root and the node the output beam hangs from (the root's row
is produced by this iteration's forward pass, so it is appended too; the output beam's own last token is the
root of the next iteration's tree and gets its row in the next pass).  In the memory-reduced variant a single
output beam survives, hence a single cache (Section 3.4).  Rows are copied bit for bit.
"""
import numpy as np


def commit_kv(k_own, v_own, k_tree, v_tree, n_next, src_tree, path_len, path):
    """
    k_own, v_own : per tree b, array [len_b, Hkv, D] (any dtype; uint16 bf16 bit patterns in the tests):
                   the input beam's own cache segment (a segment shared by the beams of a prompt is not copied:
                   it stays shared)
    k_tree, v_tree : [N, Hkv, D] rows of the forest nodes
    n_next [P], src_tree [P, W_cap], path_len [P, W_cap], path [P, W_cap, Lmax+1] : the plan of select_beams
    Returns (dst_k, dst_v, dst_len): dict (p, slot) -> array [dst_len, Hkv, D] for slot < n_next[p], and
    dst_len [P, W_cap] (0 in unused slots).
    """
    P, W_cap = src_tree.shape
    dst_k, dst_v = {}, {}
    dst_len = np.zeros((P, W_cap), dtype=np.int32)
    for p in range(P):
        for s in range(int(n_next[p])):
            b = int(src_tree[p, s])
            nodes = [int(n) for n in path[p, s, :int(path_len[p, s])]]
            rows_k = [k_own[b]] + [k_tree[n][None] for n in nodes]
            rows_v = [v_own[b]] + [v_tree[n][None] for n in nodes]
            dst_k[(p, s)] = np.concatenate(rows_k, axis=0)
            dst_v[(p, s)] = np.concatenate(rows_v, axis=0)
            dst_len[p, s] = dst_k[(p, s)].shape[0]
    return dst_k, dst_v, dst_len
