"""Layer-wise verification of a draft forest (Section 3.1 "Details", Algorithm 1) with the
dynamic layer width of Section 3.2 (Eq. 1-6), step by step in numpy fp64.

Notation follows the paper: p / q are the large / small model's next-token
distributions, I^(l) the input beams of layer l, S^(l) its draft beams,
p_beam / q_beam the beam-sampling joints over I^(l) x V (Section 2.1), p' the
running residual, W_L^(l) the layer's target width, gamma the number of draft layers.

Readings taken where the text is ambiguous (each is restated in the design notes):
  * accept iff r <= p'(x)/q_beam(x)  (the appendix proof, Eq. 3 and Section 2.2 use p/q; the
    ratio printed in Section 3.1 / Algorithm 1 is the inverse and contradicts them);
  * p_beam^(l), q_beam^(l) are normalised over I^(l) x V with I^(l) the accepted beams of layer l-1;
  * candidates of a layer are tested in ascending (draft rank, node index);
  * warping T acts on the joint over I x V, as the formulas of Section 3.1 are written (T applied to p/P and
    q/Q): top-k keeps the k largest joint entries (ties: lower flat index first), top-p then keeps the smallest
    leading part of those, in descending order, whose share of the kept mass exceeds p; the result is
    renormalised.  top_k = 0 and top_p >= 1 switch the respective step off (both off: T is the identity);
  * the bonus layer samples W_L beams with W_L the call's input width;
  * P(m,0) = prod_{j<=m}(1 - alpha_j); the "at least K" tail sums k = 0..K-1 (Eq. 6);
  * W_L^(l) is additionally capped by the output capacity W_cap.
"""
import numpy as np

from .forest import depths

NOT_REACHED, ACCEPTED, REJECTED, PRUNED, ROOT = 0, 1, 2, 3, 4
NEAR_TIE = 1e-6

FAULT_ZERO_RESIDUAL = 8   # bit raised when a residual had no mass (cannot happen in exact arithmetic)


# ----------------------------------------------------------------------------- per-node softmax
def log_sum_exp_rows(z):
    """lse[n] = log sum_x exp(z[n,x]) for every row."""
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=1)
    return m + np.log(np.exp(z - m[:, None]).sum(axis=1))


def node_log_probs(parent, token, z, lse):
    """lp[n] = log-probability of node n's own token under its parent's distribution (0 at roots)."""
    N = len(parent)
    lp = np.zeros(N)
    for n in range(N):
        if parent[n] >= 0:
            lp[n] = float(z[parent[n], token[n]]) - lse[parent[n]]
    return lp


def cumulative_log_probs(parent, lp, beam_logp, tree_off):
    """cum[root of tree b] = stored likelihood of beam b (Section 2.1); cum[n] = cum[parent] + lp[n]."""
    N = len(parent)
    cum = np.zeros(N)
    for b in range(len(tree_off) - 1):
        cum[tree_off[b]] = beam_logp[b]
    for n in range(N):
        if parent[n] >= 0:
            cum[n] = cum[parent[n]] + lp[n]
    return cum


# ----------------------------------------------------------------------------- joint distributions
def softmax(v):
    v = np.asarray(v, dtype=np.float64)
    e = np.exp(v - v.max())
    return e / e.sum()


def beam_joint(cum_I, z_I):
    """Beam-sampling distribution over I x V (Section 2.1): likelihood of beam i times the
    next-token distribution at beam i, normalised over all of I x V."""
    w = softmax(cum_I)
    z_I = np.asarray(z_I, dtype=np.float64)
    rows = np.exp(z_I - z_I.max(axis=1, keepdims=True))
    rows = rows / rows.sum(axis=1, keepdims=True)
    return w[:, None] * rows


def warp_joint(d, top_k=0, top_p=1.0):
    """T o d for a joint d over I x V (Section 2.1 "warping operation"; Section 3.1 "Details": p_beam = T o p/P,
    q_beam = T o q/Q; the experiments use top-k then top-p, appendix "Experiment Configuration").
    Entries are ranked by descending value, equal values by ascending flat index (beam-major, token-minor)."""
    d = np.asarray(d, dtype=np.float64)
    if top_k <= 0 and top_p >= 1.0:
        return d
    flat = d.ravel()
    order = sorted(range(len(flat)), key=lambda j: (-flat[j], j))
    if top_k > 0:
        order = order[:top_k]
    if top_p < 1.0:
        mass = 0.0
        for j in order:
            mass += flat[j]
        cum, keep = 0.0, []
        for j in order:
            keep.append(j)
            cum += flat[j]
            if cum / mass > top_p:
                break
        order = keep
    out = np.zeros_like(flat)
    z = 0.0
    for j in order:
        z += flat[j]
    for j in order:
        out[j] = flat[j] / z
    return out.reshape(d.shape)


def residual(p_prime, q_beam):
    """norm(max(0, p' - q_beam)); returns (distribution, mass before normalisation)."""
    r = np.maximum(0.0, p_prime - q_beam)
    s = r.sum()
    if s <= 0.0:
        return None, s
    return r / s, s


def sample(d, u):
    """Inverse-CDF draw: flatten beam-major / token-minor, return the smallest flat index whose
    inclusive prefix sum exceeds u * total."""
    flat = np.asarray(d, dtype=np.float64).ravel()
    C = np.cumsum(flat)
    Z = C[-1]
    j = int(np.searchsorted(C, float(u) * Z, side="right"))
    if j >= len(flat):
        nz = np.nonzero(flat)[0]
        j = int(nz[-1]) if len(nz) else len(flat) - 1
    return j


# ----------------------------------------------------------------------------- dynamic width (Eq. 1-6)
def acceptance_chain(p_beam, q_beam, M):
    """alpha_j, j = 1..M (Eq. 3): probability that the j-th draft is accepted given that the
    first j-1 were rejected, along p_1 = p_beam, p_{k} = norm(max(p_{k-1} - q_beam, 0))."""
    alpha = np.ones(M + 1)          # alpha[0] unused
    p_j = p_beam
    for j in range(1, M + 1):
        alpha[j] = np.minimum(p_j, q_beam).sum()
        p_j, s = residual(p_j, q_beam)
        if p_j is None:
            # no residual mass: the j-th draft is accepted with certainty, later terms carry weight 0
            alpha[j:] = 1.0
            break
    return alpha


def accept_count_table(alpha, M):
    """P[m,k] = probability that k of m drafts are accepted (Eq. 1-2).

    P[0,0] = 1, P[m,k] = 0 for k > m, P[m,0] = prod_{j<=m}(1-alpha_j) and, conditioning on which
    draft i is the first accepted one (after it the residual resets, so the remaining m-i drafts
    start again from alpha_1):  P[m,k] = sum_i alpha_i prod_{j<i}(1-alpha_j) P[m-i,k-1]."""
    first = np.zeros(M + 1)         # first[i] = P~(m,i): draft i is the first accepted one (Eq. 2)
    for i in range(1, M + 1):
        f = alpha[i]
        for j in range(1, i):
            f *= (1.0 - alpha[j])
        first[i] = f
    P = np.zeros((M + 1, M + 1))
    P[0, 0] = 1.0
    for m in range(1, M + 1):
        none = 1.0
        for j in range(1, m + 1):
            none *= (1.0 - alpha[j])
        P[m, 0] = none
        for k in range(1, m + 1):
            tot = 0.0
            for i in range(1, m + 1):
                tot += first[i] * P[m - i, k - 1]
            P[m, k] = tot
    return P


def dynamic_width(p_beam, q_beam, M, t, W_min, W_cap):
    """W_L^(l) = max(W_min, W~(t)), W~(t) = max{K : P(at least K of the M drafts accepted) >= t},
    capped by W_cap.  Returns (W_L, W~, alpha, P)."""
    alpha = acceptance_chain(p_beam, q_beam, M)
    P = accept_count_table(alpha, M)
    W_tilde = 0
    for K in range(0, M + 1):
        tail = 1.0 - P[M, :K].sum()
        if tail >= t:
            W_tilde = K
    return min(W_cap, max(W_min, W_tilde)), W_tilde, alpha, P


# ----------------------------------------------------------------------------- Algorithm 1
def verify_prompt(nodes, roots, parent, token, depth, rank, z_p, z_q, lse_p, lse_q, cum_p, cum_q,
                  u_accept, u_resid, u_fill, W_L, W_min, W_cap, t, status, trace=None, top_k=0, top_p=1.0):
    """Verify the draft layers of one prompt.

    nodes: node ids of the prompt (ascending); roots: its input beams.
    u_resid [gamma+2], u_fill [gamma+2, W_cap]: the prompt's rows of the role-indexed uniforms.
    W_L <= 0 means "the number of input beams".  t < 0 selects the fixed width.
    Writes status[] in place and returns a dict with l_last, layer_width, the output beams,
    near-tie count and fault bits.
    """
    V = z_p.shape[1]
    gamma = max(int(depth[n]) for n in nodes)
    W_in = int(W_L) if W_L > 0 else len(roots)
    I = list(roots)
    for r in roots:
        status[r] = ROOT
    layer_width = {0: len(roots)}
    near_tie = 0
    fault = 0
    out = []                       # (parent node, token, node id or -1)
    l_last = gamma + 1

    for l in range(1, gamma + 1):
        layer = [n for n in nodes if depth[n] == l]
        S = [n for n in layer if parent[n] in I]
        for n in layer:
            if parent[n] not in I:
                status[n] = PRUNED
        S.sort(key=lambda n: (int(rank[n]) if rank is not None else 0, n))
        M = len(S)
        p_beam = warp_joint(beam_joint([cum_p[i] for i in I], z_p[I]), top_k, top_p)
        q_beam = warp_joint(beam_joint([cum_q[i] for i in I], z_q[I]), top_k, top_p)
        if t < 0:
            WL = W_in
        else:
            WL = dynamic_width(p_beam, q_beam, M, float(t), W_min, W_cap)[0]
        layer_width[l] = WL
        p_prime = p_beam
        acc = []
        rec = {"l": l, "I": list(I), "S": list(S), "p_beam": p_beam, "q_beam": q_beam, "W_L": WL,
               "tests": [], "samples": []}
        for pos, c in enumerate(S):
            i = I.index(parent[c])
            x = int(token[c])
            num, den = p_prime[i, x], q_beam[i, x]
            ratio = np.inf if den == 0.0 else num / den
            u = float(u_accept[c])
            if abs(ratio - u) <= NEAR_TIE:
                near_tie += 1
            ok = u <= ratio
            rec["tests"].append({"node": c, "ratio": float(ratio), "u": u, "accepted": bool(ok)})
            if ok:
                status[c] = ACCEPTED
                acc.append(c)
                p_prime = p_beam
            else:
                status[c] = REJECTED
                nxt, _ = residual(p_prime, q_beam)
                if nxt is None:
                    fault |= FAULT_ZERO_RESIDUAL
                    nxt = p_beam
                p_prime = nxt
            if len(acc) == WL:
                for c2 in S[pos + 1:]:
                    status[c2] = REJECTED
                break
        if len(acc) < WL:
            out = [(int(parent[c]), int(token[c]), int(c)) for c in acc]
            e = sample(p_prime, u_resid[l])
            rec["samples"].append({"dist": p_prime, "u": float(u_resid[l]), "flat": e})
            out.append((I[e // V], e % V, -1))
            for j in range(WL - len(acc) - 1):
                e = sample(p_beam, u_fill[l, j])
                rec["samples"].append({"dist": p_beam, "u": float(u_fill[l, j]), "flat": e})
                out.append((I[e // V], e % V, -1))
            l_last = l
            if trace is not None:
                trace.append(rec)
            break
        if trace is not None:
            trace.append(rec)
        I = acc

    if l_last == gamma + 1:
        p_beam = warp_joint(beam_joint([cum_p[i] for i in I], z_p[I]), top_k, top_p)
        layer_width[gamma + 1] = W_in
        rec = {"l": gamma + 1, "I": list(I), "S": [], "p_beam": p_beam, "q_beam": None, "W_L": W_in,
               "tests": [], "samples": []}
        for j in range(W_in):
            e = sample(p_beam, u_fill[gamma + 1, j])
            rec["samples"].append({"dist": p_beam, "u": float(u_fill[gamma + 1, j]), "flat": e})
            out.append((I[e // V], e % V, -1))
        if trace is not None:
            trace.append(rec)

    out_lp_p = [cum_p[a] + float(z_p[a, x]) - lse_p[a] for (a, x, _) in out]
    out_lp_q = [cum_q[a] + float(z_q[a, x]) - lse_q[a] for (a, x, _) in out]
    return {"l_last": l_last, "gamma": gamma, "layer_width": layer_width, "out": out,
            "out_logp_p": out_lp_p, "out_logp_q": out_lp_q, "near_tie": near_tie, "fault": fault}


def verify_forest(tree_prompt, tree_off, parent, token, logits_p, logits_q, beam_logp_p, beam_logp_q,
                  u_accept, u_resid, u_fill, W_L, W_min, W_cap, t, rank=None, traces=None, top_k=0, top_p=1.0):
    """Whole-forest verification: per-node softmax statistics, cumulative beam likelihoods, then
    Algorithm 1 independently for every prompt.  Returns a dict of arrays shaped like the
    library's outputs (output slots beyond n_out hold -1 / 0)."""
    parent = np.asarray(parent)
    token = np.asarray(token)
    N = len(parent)
    T = len(tree_off) - 1
    P = int(tree_prompt[-1]) + 1
    z_p = np.asarray(logits_p, dtype=np.float64)
    z_q = np.asarray(logits_q, dtype=np.float64)
    depth = depths(parent)
    Lmax = int(depth.max())
    lse_p = log_sum_exp_rows(z_p)
    lse_q = log_sum_exp_rows(z_q)
    lp_p = node_log_probs(parent, token, z_p, lse_p)
    lp_q = node_log_probs(parent, token, z_q, lse_q)
    cum_p = cumulative_log_probs(parent, lp_p, beam_logp_p, tree_off)
    cum_q = cumulative_log_probs(parent, lp_q, beam_logp_q, tree_off)

    status = np.zeros(N, dtype=np.uint8)
    res = {
        "node_status": status, "lse_p": lse_p, "lse_q": lse_q, "node_logp_p": lp_p, "node_logp_q": lp_q,
        "cum_p": cum_p, "cum_q": cum_q,
        "l_last": np.zeros(P, dtype=np.int32), "layer_width": np.zeros((P, Lmax + 2), dtype=np.int32),
        "n_out": np.zeros(P, dtype=np.int32),
        "out_parent": np.full((P, W_cap), -1, dtype=np.int32), "out_token": np.full((P, W_cap), -1, dtype=np.int32),
        "out_node": np.full((P, W_cap), -1, dtype=np.int32),
        "out_logp_p": np.zeros((P, W_cap)), "out_logp_q": np.zeros((P, W_cap)),
        "near_tie": np.zeros(P, dtype=np.int32), "fault": 0,
    }
    for p in range(P):
        trees = [b for b in range(T) if tree_prompt[b] == p]
        roots = [int(tree_off[b]) for b in trees]
        nodes = list(range(int(tree_off[trees[0]]), int(tree_off[trees[-1] + 1])))
        tr = [] if traces is not None else None
        r = verify_prompt(nodes, roots, parent, token, depth, rank, z_p, z_q, lse_p, lse_q, cum_p, cum_q,
                          u_accept, u_resid[p], u_fill[p], W_L, W_min, W_cap, t, status, trace=tr,
                          top_k=top_k, top_p=top_p)
        if traces is not None:
            traces.append(tr)
        res["l_last"][p] = r["l_last"]
        for l, wdt in r["layer_width"].items():
            res["layer_width"][p, l] = wdt
        n_out = len(r["out"])
        if n_out > W_cap:
            raise ValueError("W_cap too small for the requested width")
        res["n_out"][p] = n_out
        for j, (a, x, c) in enumerate(r["out"]):
            res["out_parent"][p, j] = a
            res["out_token"][p, j] = x
            res["out_node"][p, j] = c
            res["out_logp_p"][p, j] = r["out_logp_p"][j]
            res["out_logp_q"][p, j] = r["out_logp_q"][j]
        res["near_tie"][p] = r["near_tie"]
        res["fault"] |= r["fault"]
    return res
