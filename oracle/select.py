"""Selection of the next beam set from the verification outputs.

The output beams of an iteration are the beams accepted at layer l_last plus the
sampled ones (Algorithm 1, return statement); the key-value caches kept for the
next iteration are those of the trees the output beams descend from (Section 3.3,
last paragraph).  The memory-reduced variant keeps only the output beam with the
lowest perplexity, so a single cache survives (Section 3.4); all output beams have
the same length, so lowest perplexity = highest cumulative target log-likelihood
(ties: lowest output index).
"""
import numpy as np

from .forest import ancestors_or_self, tree_of_node


def select_beams(tree_off, parent, n_out, out_parent, out_token, out_logp_p, out_logp_q, path_cap, keep_one=False):
    """
    For every prompt p and output beam j < n_out[p]:
      src_tree  = tree (input beam) the beam descends from,
      path      = forest nodes root..out_parent (the tree rows whose K/V extend that beam's cache),
      token     = the beam's new last token, logp_* = its cumulative log-likelihoods.
    keep_one: keep only the arg-max of out_logp_p.
    Returns dict of arrays [P, W_cap] (+ path [P, W_cap, path_cap], padded with -1).
    """
    P, W_cap = out_parent.shape
    tree = tree_of_node(tree_off, len(parent))
    res = {
        "n_next": np.zeros(P, dtype=np.int32),
        "src_tree": np.full((P, W_cap), -1, dtype=np.int32),
        "src_out": np.full((P, W_cap), -1, dtype=np.int32),
        "path_len": np.zeros((P, W_cap), dtype=np.int32),
        "path": np.full((P, W_cap, path_cap), -1, dtype=np.int32),
        "token": np.full((P, W_cap), -1, dtype=np.int32),
        "logp_p": np.zeros((P, W_cap)), "logp_q": np.zeros((P, W_cap)),
    }
    for p in range(P):
        keep = list(range(int(n_out[p])))
        if keep_one and keep:
            best = keep[0]
            for j in keep[1:]:
                if out_logp_p[p, j] > out_logp_p[p, best]:
                    best = j
            keep = [best]
        res["n_next"][p] = len(keep)
        for slot, j in enumerate(keep):
            a = int(out_parent[p, j])
            path = ancestors_or_self(parent, a)[::-1]
            res["src_tree"][p, slot] = tree[a]
            res["src_out"][p, slot] = j
            res["path_len"][p, slot] = len(path)
            res["path"][p, slot, :len(path)] = path
            res["token"][p, slot] = out_token[p, j]
            res["logp_p"][p, slot] = out_logp_p[p, j]
            res["logp_q"][p, slot] = out_logp_q[p, j]
    return res
