"""Pins of the draft stage (Section 3.1 "Overview": beam sampling of width W_S with the small model, gamma steps,
the trajectory laid out as a forest; "Details": draft beams are iid samples of q_beam = T o q/Q over I x V).

Independent references: the joint written with scipy's softmax, the logits warpers of the transformers library,
counting draws on a grid of uniforms, sequences rebuilt from the layers' own parent pointers, a forest written
out by hand, and a Monte-Carlo run of draft + verification against the correctness theorem."""
import numpy as np
import pytest
from scipy.special import log_softmax, softmax

from oracle import draft, forest, verify


def joint_ref(cum, z):
    """q_beam over I x V: softmax over the beams' stored likelihoods times each beam's next-token softmax."""
    return softmax(np.asarray(cum, dtype=np.float64))[:, None] * softmax(np.asarray(z, dtype=np.float64), axis=1)


@pytest.mark.parametrize("seed,W,V", [(0, 1, 7), (1, 3, 5), (2, 4, 11)])
def test_draws_on_a_grid_of_uniforms_fill_the_joint_in_proportion(seed, W, V):
    """With N equally spaced uniforms the number of draws landing on an entry is N q_beam(entry) up to one."""
    rng = np.random.default_rng(seed)
    z, cum = rng.normal(0, 1.5, (W, V)), rng.normal(0, 1, W)
    N = 20000
    u = (np.arange(N) + 0.5) / N
    par, tok, _ = draft.draft_layer(z, cum, u)
    counts = np.bincount(par.astype(np.int64) * V + tok, minlength=W * V).reshape(W, V)
    assert np.max(np.abs(counts - N * joint_ref(cum, z))) <= 1.0 + 1e-9
    # inverse CDF in flat order: the draws are non-decreasing in the flat index as u grows
    flat = par.astype(np.int64) * V + tok
    assert np.all(np.diff(flat) >= 0)


def test_one_beam_is_plain_multinomial_sampling_of_the_softmax():
    rng = np.random.default_rng(5)
    z = rng.normal(0, 2, (1, 9))
    N = 9000
    par, tok, _ = draft.draft_layer(z, [-3.7], (np.arange(N) + 0.5) / N)
    assert np.all(par == 0)
    assert np.max(np.abs(np.bincount(tok, minlength=9) - N * softmax(z[0]))) <= 1.0 + 1e-9


def test_new_beam_likelihood_is_the_parents_plus_the_tokens_log_probability():
    rng = np.random.default_rng(6)
    z, cum = rng.normal(0, 2, (3, 8)), rng.normal(-4, 1, 3)
    par, tok, lp = draft.draft_layer(z, cum, rng.random(50), top_k=5, top_p=0.9)
    want = cum[par] + log_softmax(z, axis=1)[par, tok]          # the unwarped model's likelihood
    assert np.max(np.abs(lp - want)) < 1e-12


def test_each_draw_uses_its_own_uniform_only():
    rng = np.random.default_rng(7)
    z, cum, u = rng.normal(0, 2, (3, 8)), rng.normal(0, 1, 3), rng.random(12)
    a = draft.draft_layer(z, cum, u)
    perm = rng.permutation(12)
    b = draft.draft_layer(z, cum, u[perm])
    for x, y in zip(a, b):
        assert np.array_equal(x[perm], y)


@pytest.mark.parametrize("top_k,top_p", [(10, 0.8), (4, 1.0), (6, 0.5)])
def test_warped_draws_follow_the_library_warpers(top_k, top_p):
    import torch
    from transformers import TopKLogitsWarper, TopPLogitsWarper
    rng = np.random.default_rng(8)
    W, V = 3, 13
    z, cum = rng.normal(0, 2, (W, V)), rng.normal(0, 1, W)
    x = torch.log(torch.tensor(joint_ref(cum, z)).reshape(1, -1))
    x = TopKLogitsWarper(top_k)(None, x)
    if top_p < 1.0:
        x = TopPLogitsWarper(top_p)(None, x)
    want = torch.softmax(x, dim=-1).numpy().reshape(W, V)
    N = 20000
    par, tok, _ = draft.draft_layer(z, cum, (np.arange(N) + 0.5) / N, top_k=top_k, top_p=top_p)
    counts = np.bincount(par.astype(np.int64) * V + tok, minlength=W * V).reshape(W, V)
    assert np.all(counts[want == 0] == 0)
    assert np.max(np.abs(counts - N * want)) <= 1.0 + 1e-9


# ------------------------------------------------------------------------------------------- forest layout
def random_layers(rng, root_off, gamma, W_S, V):
    P = len(root_off) - 1
    lp, lt = [], []
    for l in range(1, gamma + 1):
        par = np.zeros(P * W_S, dtype=np.int32)
        for p in range(P):
            lo, hi = (root_off[p], root_off[p + 1]) if l == 1 else (p * W_S, (p + 1) * W_S)
            par[p * W_S:(p + 1) * W_S] = rng.integers(lo, hi, W_S)
        lp.append(par)
        lt.append(rng.integers(0, V, P * W_S).astype(np.int32))
    return lp, lt


def sequence_by_layers(l, row, lp, lt):
    """(root row, tokens) of a layer's row, following the layers' own parent pointers."""
    toks = []
    while l > 0:
        toks.append(int(lt[l - 1][row]))
        row = int(lp[l - 1][row])
        l -= 1
    return row, toks[::-1]


@pytest.mark.parametrize("seed,root_off,gamma,W_S", [(0, [0, 2], 3, 4), (1, [0, 1, 4, 6], 2, 5), (2, [0, 3], 1, 2),
                                                     (3, [0, 4, 5], 4, 3)])
def test_forest_layout_keeps_every_sequence_and_the_layout_rules(seed, root_off, gamma, W_S):
    rng = np.random.default_rng(seed)
    lp, lt = random_layers(rng, root_off, gamma, W_S, 50)
    f = draft.build_forest(root_off, lp, lt)
    forest.check_forest(f["parent"], f["tree_off"])               # contiguous trees, root first, parent < child
    P = len(root_off) - 1
    assert len(f["parent"]) == root_off[-1] + gamma * P * W_S
    depth = forest.depths(f["parent"])
    tree = forest.tree_of_node(f["tree_off"], len(f["parent"]))
    seen = set()
    for l in range(gamma + 1):
        for row, n in enumerate(f["node_of"][l]):
            seen.add(int(n))
            assert depth[n] == l
            root_row, toks = sequence_by_layers(l, row, lp, lt)
            path = forest.ancestors_or_self(f["parent"], int(n))[::-1]
            assert path[0] == f["tree_off"][root_row] and tree[n] == root_row
            assert [int(f["token"][m]) for m in path[1:]] == toks
            if l > 0:
                assert f["draft_rank"][n] == row % W_S and f["tree_prompt"][tree[n]] == row // W_S
    assert seen == set(range(len(f["parent"])))
    # inside a tree: layer by layer, draw order inside a layer
    for b in range(root_off[-1]):
        nodes = range(int(f["tree_off"][b]), int(f["tree_off"][b + 1]))
        keys = [(int(depth[n]), int(f["draft_rank"][n])) for n in nodes]
        assert keys == sorted(keys)


def test_forest_layout_of_a_hand_written_run():
    """Two input beams, W_S = 3, two steps.  Step 1 continues beam 1, beam 0, beam 1; step 2 continues draws 2, 2, 0."""
    f = draft.build_forest([0, 2], [np.array([1, 0, 1]), np.array([2, 2, 0])], [np.array([7, 8, 9]), np.array([4, 5, 6])],
                           root_token=[11, 12])
    # tree 0: root, draw 1 of step 1 (token 8);  tree 1: root, draws 0 and 2 of step 1, then the three draws of step 2
    assert f["tree_off"].tolist() == [0, 2, 8]
    # (step 2's draws 0 and 1 hang under step 1's draw 2 = node 4, its draw 2 under step 1's draw 0 = node 3)
    assert f["parent"].tolist() == [-1, 0, -1, 2, 2, 4, 4, 3]
    assert f["token"].tolist() == [11, 8, 12, 7, 9, 4, 5, 6]
    assert f["draft_rank"].tolist() == [0, 1, 0, 0, 2, 0, 1, 2]
    assert f["tree_prompt"].tolist() == [0, 0]
    assert [n.tolist() for n in f["node_of"]] == [[0, 2], [3, 1, 4], [5, 6, 7]]


# ------------------------------------------------------------------------------------------- draft + verify
def test_draft_then_verify_returns_beams_distributed_as_p_beam():
    """Monte-Carlo form of Theorem 3.1 through the draft call itself: one draft layer of W_S draws from q_beam,
    verified with width W_L; the beams the layer ends up with (its accepted drafts if it passes, the call's output
    beams if it falls short) must be iid p_beam over I x V."""
    rng = np.random.default_rng(11)
    W, W_S, V, trials = 2, 3, 3, 6000
    z_p, z_q = rng.normal(0, 1.2, (W, V)), rng.normal(0, 1.2, (W, V))
    cum_p, cum_q = rng.normal(0, 0.7, W), rng.normal(0, 0.7, W)
    want = joint_ref(cum_p, z_p)
    counts = np.zeros((W, V))
    pair_counts = np.zeros((W * V, W * V))
    for _ in range(trials):
        par, tok, _ = draft.draft_layer(z_q, cum_q, rng.random(W_S))
        f = draft.build_forest([0, W], [par], [tok])
        N = len(f["parent"])
        logits_p, logits_q = np.zeros((N, V)), np.zeros((N, V))
        for b in range(W):
            logits_p[f["tree_off"][b]], logits_q[f["tree_off"][b]] = z_p[b], z_q[b]
        res = verify.verify_forest(f["tree_prompt"], f["tree_off"], f["parent"], f["token"], logits_p, logits_q,
                                   cum_p, cum_q, rng.random(N), rng.random((1, 3)), rng.random((1, 3, 4)),
                                   W, 1, 4, -1.0, rank=f["draft_rank"])
        assert res["n_out"][0] == W
        tree = forest.tree_of_node(f["tree_off"], N)
        if res["l_last"][0] == 1:      # the layer fell short: its beams are the call's output beams
            e = [int(tree[res["out_parent"][0, j]]) * V + int(res["out_token"][0, j]) for j in range(W)]
        else:                          # the layer passed (the output then is the bonus layer): its accepted drafts, in draw order
            acc = [n for n in f["node_of"][1] if res["node_status"][n] == verify.ACCEPTED]
            assert len(acc) == W
            e = [int(tree[n]) * V + int(f["token"][n]) for n in acc]
        counts[e[0] // V, e[0] % V] += 1
        pair_counts[e[0], e[1]] += 1
    # six-sigma bands of the binomial counts
    sd = np.sqrt(trials * want * (1 - want))
    assert np.all(np.abs(counts - trials * want) <= 6 * sd + 1)
    pw = np.outer(want.ravel(), want.ravel())                      # the two output beams are independent
    assert np.all(np.abs(pair_counts - trials * pw) <= 6 * np.sqrt(trials * pw * (1 - pw)) + 1)
