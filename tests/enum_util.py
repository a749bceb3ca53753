"""Exhaustive-enumeration helpers for the oracle's verification (test code only).

The oracle is a deterministic function of the draft forest and the uniforms.  To get the exact
distribution of what one verification layer outputs, the helpers
  * enumerate every tuple of drafts, each draft drawn jointly (parent beam, token) ~ q_beam iid,
    which is how the paper's draft stage works (Section 3.1),
  * force every accept / reject pattern through the accept uniforms (0 forces an accept,
    1 - 2^-24 forces a reject whenever the accept probability is below 1), and weight the pattern
    with the accept probabilities min(1, ratio) the oracle itself reports in its trace,
  * push sampling steps through as the distributions the oracle sampled from.
Everything that is weighed comes out of the oracle's own run, so a mistake in the oracle's
arithmetic shows up as a wrong output distribution.
"""
import itertools

import numpy as np

from oracle import verify

U_ACC = np.float32(0.0)
U_REJ = np.float32(1.0 - 2.0 ** -24)


def build_forest(W_in, layer1, layer2=()):
    """layer1: [(root slot, token)] in draw order; layer2: [(index into layer1, token)] in draw order.
    Trees are contiguous: root, its layer-1 drafts, then the layer-2 drafts below them.
    Returns dict(tree_off, parent, token, rank, node1, node2) with node1/node2 the node ids of the drafts."""
    parent, token, rank, tree_off = [], [], [], [0]
    node1 = [None] * len(layer1)
    node2 = [None] * len(layer2)
    for b in range(W_in):
        root = len(parent)
        parent.append(-1); token.append(0); rank.append(0)
        for j, (slot, x) in enumerate(layer1):
            if slot == b:
                node1[j] = len(parent)
                parent.append(root); token.append(x); rank.append(j)
        for j, (pj, x) in enumerate(layer2):
            if layer1[pj][0] == b:
                node2[j] = len(parent)
                parent.append(node1[pj]); token.append(x); rank.append(j)
        tree_off.append(len(parent))
    return dict(tree_off=np.array(tree_off, dtype=np.int32), parent=np.array(parent, dtype=np.int32),
                token=np.array(token, dtype=np.int32), rank=np.array(rank, dtype=np.int32),
                node1=node1, node2=node2)


def run(fr, z_p, z_q, blp, blq, u_accept, W_L, t, W_min=1, W_cap=8, top_k=0, top_p=1.0):
    """One oracle call on forest `fr`; z_p/z_q are per-node logit rows. Returns (result, trace)."""
    N = len(fr["parent"])
    T = len(fr["tree_off"]) - 1
    Lmax = 2
    traces = []
    res = verify.verify_forest(np.zeros(T, dtype=np.int32), fr["tree_off"], fr["parent"], fr["token"], z_p, z_q,
                               blp, blq, u_accept, np.full((1, Lmax + 2), 0.5, dtype=np.float32),
                               np.full((1, Lmax + 2, W_cap), 0.5, dtype=np.float32), W_L, W_min, W_cap, t,
                               rank=fr["rank"], traces=traces, top_k=top_k, top_p=top_p)
    assert N == len(u_accept)
    return res, traces[0]


def layer_outcome_distribution(fr, z_p, z_q, blp, blq, W_L, t, layer, free_nodes, fixed_u, W_cap=8, top_k=0, top_p=1.0):
    """Exact distribution of the beams that layer `layer` hands on (accepted drafts, then the
    residual sample, then fills), over flat indices slot*V + token of I^(layer) x V.

    free_nodes: nodes whose accept/reject is enumerated (the layer's drafts);
    fixed_u: dict node -> forced uniform for all other nodes.
    Returns (tensor of shape [K]*width, accept-count histogram, I of that layer, p_beam of that layer)."""
    N = len(fr["parent"])
    V = z_p.shape[1]
    total = None
    acc_hist = np.zeros(len(free_nodes) + 1)
    info = None
    for pattern in itertools.product([True, False], repeat=len(free_nodes)):
        u = np.zeros(N, dtype=np.float32)
        for n, val in fixed_u.items():
            u[n] = val
        for n, a in zip(free_nodes, pattern):
            u[n] = U_ACC if a else U_REJ
        res, trace = run(fr, z_p, z_q, blp, blq, u, W_L, t, W_cap=W_cap, top_k=top_k, top_p=top_p)
        rec = [r for r in trace if r["l"] == layer]
        if not rec:
            return None, None, None, None
        rec = rec[0]
        tested = {tst["node"]: tst for tst in rec["tests"]}
        forced = dict(zip(free_nodes, pattern))
        prob = 1.0
        canonical = True
        for n in free_nodes:
            if n in tested:
                a = min(1.0, tested[n]["ratio"])
                if tested[n]["accepted"] != forced[n]:
                    canonical = False       # a reject could not be forced (accept probability 1)
                prob *= a if forced[n] else (1.0 - a)
            elif not forced[n]:
                canonical = False           # untested nodes are represented by the all-accept pattern
        if not canonical or prob == 0.0:
            continue
        I = rec["I"]
        K = len(I) * V
        dists = []
        n_acc = 0
        for tst in rec["tests"]:
            if tst["accepted"]:
                n_acc += 1
                d = np.zeros(K)
                d[I.index(int(fr["parent"][tst["node"]])) * V + int(fr["token"][tst["node"]])] = 1.0
                dists.append(d)
        for s in rec["samples"]:
            dists.append(np.asarray(s["dist"]).ravel())
        acc_hist[n_acc] += prob
        width = rec["W_L"]
        assert len(dists) == width
        joint = np.array(prob)
        for d in dists:
            joint = np.multiply.outer(joint, d)
        total = joint if total is None else total + joint
        info = (I, rec["p_beam"])
    return total, acc_hist, info[0], info[1]
