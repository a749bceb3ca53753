"""Pins for the oracle's verification arithmetic that do not need enumeration.

* log-sum-exp / cumulative likelihoods against library routines;
* W = 1 on a chain must be standard speculative sampling (Section 2.2, step 3), written here
  independently with python loops;
* appendix identities of the residual chain and the closed form of the chain;
* Eq. 1-2 invariants of the accept-count table, monotonicity of the width in t;
* the worked scenario of the method figure (words only in the paper);
* the inverse-CDF convention by brute force and a frequency test (a convention of this build).
"""
import json
import os

import numpy as np
import pytest
import scipy.special
import torch

from dsbd_synth import make_workload
from oracle import forest, select, verify

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_oracle(w, W_L=0, t=-1.0, W_min=1, rank=None, traces=None):
    return verify.verify_forest(w.tree_prompt, w.tree_off, w.parent, w.token, w.logits_p, w.logits_q,
                                w.beam_logp_p, w.beam_logp_q, w.u_accept, w.u_resid, w.u_fill,
                                W_L, W_min, w.W_cap, t, rank=rank, traces=traces)


# ------------------------------------------------------------------ library pins
def test_log_sum_exp_and_node_log_probs_against_libraries():
    w = make_workload("c2", L=2, V=997, Hq=1, Hkv=1, D=64)
    r = run_oracle(w)
    zp = w.logits_p.astype(np.float64)
    assert np.max(np.abs(r["lse_p"] - scipy.special.logsumexp(zp, axis=1))) < 1e-12
    lsm = torch.log_softmax(torch.from_numpy(w.logits_q.astype(np.float64)), dim=1).numpy()
    for n in range(w.n_nodes):
        a = w.parent[n]
        expect = 0.0 if a < 0 else lsm[a, w.token[n]]
        assert abs(r["node_logp_q"][n] - expect) < 1e-12
    # cumulative = stored beam likelihood + sum of the log-probabilities along the path
    tree = forest.tree_of_node(w.tree_off, w.n_nodes)
    for n in range(w.n_nodes):
        path = forest.ancestors_or_self(w.parent, n)
        tot = w.beam_logp_q[tree[n]] + sum(0.0 if w.parent[m] < 0 else lsm[w.parent[m], w.token[m]] for m in path)
        assert abs(r["cum_q"][n] - tot) < 1e-12


def test_beam_joint_is_the_normalised_product():
    rng = np.random.default_rng(1)
    cum = rng.normal(0, 2, 3)
    z = rng.normal(0, 3, (3, 50))
    pb = verify.beam_joint(cum, z)
    # definition of Section 2.1: p(beam_i, x) / sum over I x V, with p(beam_i, x) = p(beam_i) p(x | beam_i)
    unnorm = np.exp(cum)[:, None] * torch.softmax(torch.from_numpy(z), 1).numpy()
    assert np.max(np.abs(pb - unnorm / unnorm.sum())) < 1e-15
    assert abs(pb.sum() - 1) < 1e-14


# ------------------------------------------------------------------ W = 1 is speculative sampling
def inverse_cdf_loop(d, u):
    tot = 0.0
    for v in d:
        tot += v
    c = 0.0
    for j, v in enumerate(d):
        c += v
        if c > u * tot:
            return j
    return max(j for j, v in enumerate(d) if v > 0)


def speculative_sampling(P, Q, drafts, u_acc, u_corr, u_bonus):
    """Section 2.2 step 3: accept draft t with probability min(1, p/q); the drafts before the first
    rejection are kept; a correction token comes from the residual; if all pass, a bonus token from p."""
    for t, x in enumerate(drafts):
        if not (u_acc[t] <= P[t][x] / Q[t][x]):
            res = [max(0.0, a - b) for a, b in zip(P[t], Q[t])]
            return t, inverse_cdf_loop(res, u_corr[t])
    return len(drafts), inverse_cdf_loop(P[len(drafts)], u_bonus)


@pytest.mark.parametrize("noise", [0.5, 2.0])
def test_single_chain_width_one_is_speculative_sampling(noise):
    n_acc = []
    for seed in range(40):
        w = make_workload("c1", W=1, tree_nodes=6, L=1, V=64, Hq=1, Hkv=1, D=64, seed=seed,
                          draft="noise", noise_std=noise)
        r = run_oracle(w, W_L=1)
        sm = lambda z: torch.softmax(torch.from_numpy(z.astype(np.float64)), 1).numpy().tolist()
        P, Q = sm(w.logits_p), sm(w.logits_q)
        gamma = 5
        k, tok = speculative_sampling(P, Q, w.token[1:].tolist(), w.u_accept[1:].tolist(),
                                      [float(w.u_resid[0, l]) for l in range(1, gamma + 1)],
                                      float(w.u_fill[0, gamma + 1, 0]))
        assert r["l_last"][0] - 1 == k
        assert r["n_out"][0] == 1 and r["out_token"][0, 0] == tok and r["out_parent"][0, 0] == k
        assert r["out_node"][0, 0] == -1
        expect = [verify.ROOT] + [verify.ACCEPTED] * k + ([verify.REJECTED] if k < gamma else []) \
            + [verify.NOT_REACHED] * max(0, gamma - k - 1)
        assert r["node_status"].tolist() == expect
        n_acc.append(k)
    assert min(n_acc) < max(n_acc)      # the seeds exercise both early and late rejections


# ------------------------------------------------------------------ residual chain
def test_residual_chain_identities():
    rng = np.random.default_rng(3)
    p = verify.beam_joint(rng.normal(0, 1, 3), rng.normal(0, 2, (3, 40)))
    q = verify.beam_joint(rng.normal(0, 1, 3), rng.normal(0, 2, (3, 40)))
    M = 6
    alpha = verify.acceptance_chain(p, q, M)
    p_j = p
    c, F = 0.0, 1.0                      # closed form: p_j = max(p - c_j q, 0) / F(c_j)
    for j in range(1, M + 1):
        # appendix: alpha_j = sum q min(1, p_j/q) = 1 - sum max(p_j - q, 0)
        assert abs(alpha[j] - (q * np.minimum(1.0, p_j / q)).sum()) < 1e-14
        assert abs(alpha[j] - (1.0 - np.maximum(p_j - q, 0).sum())) < 1e-14
        # appendix: p_{j+1} = (p_j - min(q, p_j)) / (1 - alpha_j)
        nxt, mass = verify.residual(p_j, q)
        assert np.max(np.abs(nxt - (p_j - np.minimum(q, p_j)) / (1.0 - alpha[j]))) < 1e-13
        assert abs(mass - (1.0 - alpha[j])) < 1e-14
        # appendix: P_{1,j} + P_{2,j} = p_j with P_{1,j} = q min(1, p_j/q), P_{2,j} = (1 - alpha_j) p_{j+1}
        assert np.max(np.abs(q * np.minimum(1.0, p_j / q) + (1.0 - alpha[j]) * nxt - p_j)) < 1e-14
        # closed form of the chain
        assert np.max(np.abs(p_j - np.maximum(p - c * q, 0) / F)) < 1e-13
        c = c + F
        F_next = np.maximum(p - c * q, 0).sum()
        assert abs(alpha[j] - (1.0 - F_next / F)) < 1e-13
        F = F_next
        p_j = nxt
    assert abs(p_j.sum() - 1.0) < 1e-13 and (p_j >= 0).all()


def test_acceptance_chain_with_identical_models_and_exhausted_residual():
    p = verify.beam_joint([0.0, 0.3], np.array([[0.1, 0.5, -1.0], [0.0, 0.2, 0.4]]))
    alpha = verify.acceptance_chain(p, p.copy(), 4)
    assert alpha[1:].tolist() == [1.0, 1.0, 1.0, 1.0]
    P = verify.accept_count_table(alpha, 4)
    assert P[4].tolist() == [0, 0, 0, 0, 1.0]
    assert verify.dynamic_width(p, p.copy(), 4, 0.9, 1, 8)[0] == 4
    assert verify.dynamic_width(p, p.copy(), 4, 0.9, 1, 3)[0] == 3      # capacity cap


# ------------------------------------------------------------------ Eq. 1-6
def test_accept_count_table_invariants_and_width_monotone_in_t():
    rng = np.random.default_rng(11)
    for M in [1, 2, 5, 9]:
        alpha = np.concatenate([[1.0], rng.uniform(0.05, 0.95, M)])
        P = verify.accept_count_table(alpha, M)
        assert P[0, 0] == 1.0
        for m in range(M + 1):
            assert abs(P[m, :m + 1].sum() - 1.0) < 1e-13
            assert np.all(P[m, m + 1:] == 0.0)
        assert abs(P[1, 1] - alpha[1]) < 1e-15
        if M >= 2:
            # two drafts: both accepted = a1 * a1 (residual resets after an accept)
            assert abs(P[2, 2] - alpha[1] * alpha[1]) < 1e-15
            assert abs(P[2, 0] - (1 - alpha[1]) * (1 - alpha[2])) < 1e-15
    p = verify.beam_joint(rng.normal(0, 1, 4), rng.normal(0, 2, (4, 30)))
    q = verify.beam_joint(rng.normal(0, 1, 4), rng.normal(0, 2, (4, 30)))
    widths = [verify.dynamic_width(p, q, 8, t, 1, 16)[1] for t in (0.0, 0.1, 0.3, 0.5, 0.7, 0.9, 1.0)]
    assert widths[0] == 8 and all(a >= b for a, b in zip(widths, widths[1:]))
    assert verify.dynamic_width(p, q, 8, 0.999999, 3, 16)[0] == 3      # floor W_min


def test_dynamic_mode_widths_are_reported_and_respected():
    w = make_workload("c3", L=1, V=400, Hq=1, Hkv=1, D=64)
    tr = []
    r = run_oracle(w, t=0.7, traces=tr)
    for rec in tr[0]:
        if rec["q_beam"] is None:
            continue
        WL = verify.dynamic_width(rec["p_beam"], rec["q_beam"], len(rec["S"]), np.float32(0.7), 1, w.W_cap)[0]
        assert rec["W_L"] == WL == r["layer_width"][0, rec["l"]]
        assert sum(t["accepted"] for t in rec["tests"]) <= WL


# ------------------------------------------------------------------ the figure's scenario
def test_method_figure_scenario():
    g = json.load(open(os.path.join(GOLDEN, "fig2_scenario.json")))
    vocab = g["vocab"]
    V = len(vocab)
    tok = {wd: i for i, wd in enumerate(vocab)}
    names, parent, token, tree_off = [], [], [], [0]
    for tr in g["trees"]:
        base = len(parent)
        names.append(tr["root"]); parent.append(-1); token.append(tok[tr["root"]])
        for wd, pi in tr["nodes"]:
            par = base if pi < 0 else base + 1 + pi
            names.append(names[par] + " " + wd); parent.append(par); token.append(tok[wd])
        tree_off.append(len(parent))
    N = len(parent)
    idx = {nm: i for i, nm in enumerate(names)}
    rank = np.zeros(N, dtype=np.int32)
    for order in (g["draft_order_layer1"], g["draft_order_layer2"]):
        for j, nm in enumerate(order):
            rank[idx[nm]] = j
    # logits: uniform everywhere except at "who are", where the target prefers "you" and "they" and the
    # draft prefers "it", so that "it" can be rejected and the residual concentrates on "you"
    z_p = np.zeros((N, V)); z_q = np.zeros((N, V))
    z_p[idx["who are"], tok["you"]] = 6.0
    z_p[idx["who are"], tok["they"]] = 3.0
    z_q[idx["who are"], tok["it"]] = 4.0
    z_q[idx["who are"], tok["they"]] = 3.0
    u = np.zeros(N, dtype=np.float32)                     # accept whatever can be accepted ...
    u[idx["who are it"]] = 0.9                            # ... except the draft the figure rejects
    u[idx["why is"]] = 0.9                                # never tested: two beams are accepted before it
    u_res = np.full((1, 4), 0.5, dtype=np.float32)
    u_fill = np.full((1, 4, 4), 0.5, dtype=np.float32)
    r = verify.verify_forest(np.zeros(2, dtype=np.int32), np.array(tree_off), np.array(parent), np.array(token),
                             z_p, z_q, np.zeros(2), np.zeros(2), u, u_res, u_fill, g["W_L"], 1, 4, -1.0, rank=rank)
    code = {"accepted": verify.ACCEPTED, "rejected": verify.REJECTED, "pruned": verify.PRUNED}
    for nm, st in g["expected_status"].items():
        assert r["node_status"][idx[nm]] == code[st], nm
    assert r["l_last"][0] == g["expected_l_last"]
    outs = [[names[r["out_parent"][0, j]], vocab[r["out_token"][0, j]]] for j in range(r["n_out"][0])]
    assert outs == g["expected_outputs"]
    assert r["out_node"][0, 0] == idx["who are they"] and r["out_node"][0, 1] == -1
    # Section 3.3: both output beams descend from the tree of "who", so only that cache is kept
    s = select.select_beams(np.array(tree_off), np.array(parent), r["n_out"], r["out_parent"], r["out_token"],
                            r["out_logp_p"], r["out_logp_q"], 3)
    assert s["src_tree"][0, :2].tolist() == [0, 0]
    assert s["path"][0, 0, :2].tolist() == [idx["who"], idx["who are"]] and s["path_len"][0, 0] == 2
    one = select.select_beams(np.array(tree_off), np.array(parent), r["n_out"], r["out_parent"], r["out_token"],
                              r["out_logp_p"], r["out_logp_q"], 3, keep_one=True)
    assert one["n_next"][0] == 1 and vocab[one["token"][0, 0]] == "you"      # "you" is the likelier beam under p


# ------------------------------------------------------------------ sampling convention (unpinned by the paper)
def test_inverse_cdf_convention_brute_force_and_frequencies():
    d = np.array([[0.0, 0.2, 0.0], [0.5, 0.0, 0.3]])
    assert verify.sample(d, 0.0) == 1                      # zero-mass cells are never returned
    assert verify.sample(d, 0.19) == 1 and verify.sample(d, 0.2) == 3
    assert verify.sample(d, 0.6999) == 3 and verify.sample(d, 0.7001) == 5
    assert verify.sample(d, np.float32(1 - 2.0 ** -24)) == 5
    rng = np.random.default_rng(0)
    for _ in range(200):
        dd = rng.random(17) * (rng.random(17) > 0.3)
        dd[3] = 0.7
        u = rng.random()
        assert verify.sample(dd, u) == inverse_cdf_loop(dd.tolist(), u)
    # frequencies over the 24-bit grid of uniforms follow the distribution (chi-square, 5 cells)
    from dsbd_synth import uniform01_f32
    us = uniform01_f32(20000, 3, 9)
    dist = np.array([0.1, 0.0, 0.4, 0.25, 0.2, 0.05])
    cnt = np.bincount([verify.sample(dist, u) for u in us], minlength=6)
    assert cnt[1] == 0
    nz = dist > 0
    chi2 = (((cnt[nz] - 20000 * dist[nz]) ** 2) / (20000 * dist[nz])).sum()
    assert chi2 < 20.5          # 99.9 % quantile of chi-square with 4 degrees of freedom is 18.5


def test_near_tie_counter_and_role_indexed_uniforms():
    w = make_workload("c2", L=1, V=300, Hq=1, Hkv=1, D=64)
    tr = []
    r0 = run_oracle(w, traces=tr)
    first = tr[0][0]["tests"][0]
    w.u_accept[first["node"]] = np.float32(first["ratio"]) if first["ratio"] < 1 else np.float32(0.5)
    r1 = run_oracle(w)
    if first["ratio"] < 1:
        assert r1["near_tie"][0] == r0["near_tie"][0] + 1
    # changing a uniform whose role is never reached changes nothing
    w2 = make_workload("c2", L=1, V=300, Hq=1, Hkv=1, D=64)
    l_last = int(r0["l_last"][0])
    for l in range(w2.u_resid.shape[1]):
        if l != l_last:
            w2.u_resid[0, l] = 0.123
    r2 = run_oracle(w2)
    for k in ("node_status", "out_parent", "out_token", "out_node", "l_last"):
        assert np.array_equal(r0[k], r2[k])


# ------------------------------------------------------------------ masked tokens
@pytest.mark.parametrize("top_k,top_p,t", [(0, 1.0, -1.0), (0, 1.0, 0.6), (5, 0.8, -1.0), (8, 1.0, 0.5)])
def test_masked_tokens_are_tokens_that_are_not_there(top_k, top_p, t):
    """A logit of -Inf gives its token the probability 0 in every distribution of the method, so verifying with some
    vocabulary entries masked in both models must be the same as verifying over the vocabulary without them (tokens
    renumbered in order): same decisions, widths and draws, same likelihoods."""
    for seed in range(6):
        w = make_workload("c2", L=2, V=60, Hq=1, Hkv=1, D=64, seed=seed, noise_std=1.0)
        rng = np.random.default_rng(seed)
        keep = rng.random(w.V) < 0.6
        keep[w.token[w.token >= 0]] = True                     # drafted tokens exist in both vocabularies
        new_id = np.cumsum(keep) - 1
        old_id = np.flatnonzero(keep)
        zp, zq = w.logits_p.copy(), w.logits_q.copy()
        zp[:, ~keep] = -np.inf
        zq[:, ~keep] = -np.inf
        tok_small = np.where(w.token >= 0, new_id[np.maximum(w.token, 0)], w.token).astype(np.int32)
        args = (w.beam_logp_p, w.beam_logp_q, w.u_accept, w.u_resid, w.u_fill, 0, 1, w.W_cap, t)
        with np.errstate(all="ignore"):
            big = verify.verify_forest(w.tree_prompt, w.tree_off, w.parent, w.token, zp, zq, *args,
                                       top_k=top_k, top_p=top_p)
        small = verify.verify_forest(w.tree_prompt, w.tree_off, w.parent, tok_small,
                                     np.ascontiguousarray(w.logits_p[:, keep]), np.ascontiguousarray(w.logits_q[:, keep]),
                                     *args, top_k=top_k, top_p=top_p)
        assert big["fault"] == small["fault"] == 0
        for key in ("node_status", "l_last", "layer_width", "n_out", "out_parent", "out_node", "near_tie"):
            assert np.array_equal(big[key], small[key]), (seed, key)
        used = big["out_token"] >= 0
        assert np.array_equal(used, small["out_token"] >= 0)
        assert np.array_equal(big["out_token"][used], old_id[small["out_token"][used]]), seed
        for key in ("lse_p", "lse_q", "node_logp_p", "node_logp_q", "out_logp_p", "out_logp_q"):
            assert np.allclose(big[key], small[key], rtol=0, atol=1e-12), (seed, key)
