"""Draft stage of one iteration: beam sampling with the small model, and the draft forest it leaves behind.

TEST INFRASTRUCTURE: a plain, slow CPU statement of what the library's draft-side calls compute.  Only the
tests, the smoke check and the benchmark's CPU baseline may use it; the product never does.

Section 3.1 "Overview": in every iteration the small model runs beam sampling of width W_S for gamma steps;
the trajectory is a forest with one tree per input beam, whose layers from the second on hold W_S nodes each
(the intermediate beams of the beam-sampling run).  Section 3.1 "Details": a draft beam of the next layer is a
sample of q_beam = T o q / Q over (beams of the current layer) x V, with Q the sum over that set and T the
warping operation (Section 2.1); the W_S draft beams of a layer are drawn independently.

Readings:
  * the beams a layer is drawn from are ALL the beams of the layer before (W_S of them from the second
    layer on, the input beams for the first), as in beam sampling of width W_S;
  * a draw is the inverse-CDF sample of verify.sample (flat order beam-major / token-minor), one uniform each;
  * the likelihood stored with a new beam is that of the unwarped small model (Section 2.1 keeps sequence
    likelihoods): cum_q[parent] + log q(token | parent);
  * forest layout: trees contiguous, a tree's nodes ordered by (layer, draw index), so a parent precedes its
    children; draft_rank of a node is its draw index within its layer, which is the order the verification
    must test a layer's candidates in.
"""
import numpy as np

from .verify import beam_joint, warp_joint, sample, log_sum_exp_rows


def draft_layer(z_q, cum_q, u, top_k=0, top_p=1.0):
    """One step of the small model's beam sampling.

    z_q [n_beams, V]: the small model's logits at the current layer's beams; cum_q [n_beams]: their stored
    log-likelihoods; u [W_S]: one uniform per draw.  Returns (parent [W_S] index of the beam continued,
    token [W_S], logp [W_S] log-likelihood of the new beam)."""
    z = np.asarray(z_q, dtype=np.float64)
    cum = [float(c) for c in cum_q]
    V = z.shape[1]
    q_beam = warp_joint(beam_joint(cum, z), top_k, top_p)
    lse = log_sum_exp_rows(z)
    parent, token, logp = [], [], []
    for uj in u:
        e = sample(q_beam, uj)
        i, x = divmod(e, V)
        parent.append(i)
        token.append(x)
        logp.append(cum[i] + z[i, x] - lse[i])
    return np.asarray(parent, dtype=np.int32), np.asarray(token, dtype=np.int32), np.asarray(logp, dtype=np.float64)


def build_forest(root_off, layer_parent, layer_token, root_token=None):
    """Lay the sampled layers out as a draft forest.

    root_off [P+1]: input beams of prompt p are rows root_off[p] .. root_off[p+1]-1 of layer 0.
    layer_parent[l-1] [P*W_S], layer_token[l-1] [P*W_S] for l = 1..gamma: draw j of prompt p in layer l is row
    p*W_S + j; its parent is a row of layer l-1 (of the same prompt).
    root_token [T] (optional): last tokens of the input beams, stored at the roots (nothing reads them).
    Returns dict(tree_prompt, tree_off, parent, token, draft_rank, node_of) where node_of[l][row] is the forest
    node of a layer's row."""
    root_off = [int(v) for v in root_off]
    P = len(root_off) - 1
    gamma = len(layer_parent)
    T = root_off[-1]
    W_S = len(layer_parent[0]) // P if gamma else 0
    # root (layer-0 row) of every row of every layer
    root_of = [list(range(T))]
    for l in range(1, gamma + 1):
        root_of.append([root_of[l - 1][int(a)] for a in layer_parent[l - 1]])
    tree_prompt = []
    for p in range(P):
        tree_prompt += [p] * (root_off[p + 1] - root_off[p])
    tree_off, parent, token, rank = [0], [], [], []
    node_of = [[-1] * len(r) for r in root_of]
    for b in range(T):
        p = tree_prompt[b]
        node_of[0][b] = len(parent)
        parent.append(-1); token.append(0 if root_token is None else int(root_token[b])); rank.append(0)
        for l in range(1, gamma + 1):
            for j in range(W_S):
                row = p * W_S + j
                if root_of[l][row] != b:
                    continue
                node_of[l][row] = len(parent)
                parent.append(node_of[l - 1][int(layer_parent[l - 1][row])])
                token.append(int(layer_token[l - 1][row]))
                rank.append(j)
        tree_off.append(len(parent))
    return {
        "tree_prompt": np.asarray(tree_prompt, dtype=np.int32), "tree_off": np.asarray(tree_off, dtype=np.int32),
        "parent": np.asarray(parent, dtype=np.int32), "token": np.asarray(token, dtype=np.int32),
        "draft_rank": np.asarray(rank, dtype=np.int32),
        "node_of": [np.asarray(n, dtype=np.int32) for n in node_of],
    }
