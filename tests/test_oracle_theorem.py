"""Pin: the correctness theorem of the draft-and-verify scheme (Theorem 3.1 and its appendix proof).

On tiny vocabularies every draft tuple and every accept/reject pattern is enumerated through the
oracle itself; the beams a verified layer hands on must be iid draws from p_beam over I x V: every
marginal equals p_beam and the joint is the product.  Reference distributions are computed with
torch's softmax, not with the oracle.
"""
import itertools

import numpy as np
import pytest
import torch

from enum_util import U_ACC, U_REJ, build_forest, layer_outcome_distribution, run
from oracle import verify


def ref_joint(beam_logp, rows):
    w = torch.softmax(torch.tensor(beam_logp, dtype=torch.float64), 0)
    r = torch.softmax(torch.tensor(rows, dtype=torch.float64), 1)
    return (w[:, None] * r).numpy()


def iid_product(p, width):
    out = np.array(1.0)
    for _ in range(width):
        out = np.multiply.outer(out, p.ravel())
    return out


def z_for(fr, rows_root, rows_l1, rows_l2, V):
    N = len(fr["parent"])
    z = np.zeros((N, V))
    for b in range(len(fr["tree_off"]) - 1):
        z[fr["tree_off"][b]] = rows_root[b]
    for j, n in enumerate(fr["node1"]):
        z[n] = rows_l1[j]
    for j, n in enumerate(fr["node2"]):
        z[n] = rows_l2[j]
    return z


CASES = [  # W_in, W_S, W_L, V, t
    (1, 1, 1, 3, -1.0),      # vanilla speculative sampling
    (2, 2, 1, 3, -1.0),
    (2, 3, 2, 2, -1.0),
    (2, 2, 2, 3, -1.0),
    (1, 3, 2, 3, -1.0),      # one input beam, two output beams (memory-reduced variant, Section 3.4)
    (2, 3, 3, 2, -1.0),      # W_L = W_S: every draft must be accepted for the layer to pass
    (2, 3, 0, 2, 0.5),       # dynamic width: the layer's width depends on (p_beam, q_beam) only
    (2, 4, 0, 2, 0.3),
]


@pytest.mark.parametrize("W_in,W_S,W_L,V,t", CASES)
def test_one_layer_outputs_are_iid_p_beam(W_in, W_S, W_L, V, t):
    rng = np.random.default_rng(100 * W_in + 10 * W_S + V)
    rows_p = rng.normal(0, 1.0, (W_in, V))
    rows_q = rows_p + rng.normal(0, 0.8, (W_in, V))
    blp = rng.normal(0, 1, W_in)
    blq = blp + rng.normal(0, 0.5, W_in)
    rows1_p = rng.normal(0, 1, (W_S, V))
    rows1_q = rng.normal(0, 1, (W_S, V))
    p_ref = ref_joint(blp, rows_p)
    q_ref = ref_joint(blq, rows_q)
    K = W_in * V
    total = None
    widths = set()
    for tup in itertools.product(range(K), repeat=W_S):
        wgt = float(np.prod([q_ref.ravel()[d] for d in tup]))
        fr = build_forest(W_in, [(d // V, d % V) for d in tup])
        z_p = z_for(fr, rows_p, rows1_p, [], V)
        z_q = z_for(fr, rows_q, rows1_q, [], V)
        dist, _, I, pb = layer_outcome_distribution(fr, z_p, z_q, blp, blq, W_L, t, 1, fr["node1"], {})
        assert np.allclose(pb, p_ref, atol=1e-14)
        widths.add(dist.ndim)
        total = wgt * dist if total is None else total + wgt * dist
    assert len(widths) == 1
    width = widths.pop()
    if t < 0:
        assert width == (W_L if W_L > 0 else W_in)
    assert abs(total.sum() - 1.0) < 1e-12
    assert np.max(np.abs(total - iid_product(p_ref, width))) < 1e-12
    # each marginal on its own
    for ax in range(width):
        other = tuple(a for a in range(width) if a != ax)
        assert np.max(np.abs(total.sum(axis=other) - p_ref.ravel())) < 1e-12


def test_testing_drafts_in_tree_order_instead_of_draw_order_breaks_the_theorem():
    """Why the forest carries a draft rank: a tree-contiguous layout sorts a layer's drafts by parent,
    and testing them in that order (instead of the order they were drawn in) is no longer a test of
    iid drafts - the first output stops being distributed as p_beam."""
    W_in, W_S, W_L, V = 2, 3, 2, 2
    rng = np.random.default_rng(100 * W_in + 10 * W_S + V)
    rows_p = rng.normal(0, 1.0, (W_in, V)); rows_q = rows_p + rng.normal(0, 0.8, (W_in, V))
    blp = rng.normal(0, 1, W_in); blq = blp + rng.normal(0, 0.5, W_in)
    p_ref = ref_joint(blp, rows_p); q_ref = ref_joint(blq, rows_q)
    total = None
    for tup in itertools.product(range(W_in * V), repeat=W_S):
        wgt = float(np.prod([q_ref.ravel()[d] for d in tup]))
        fr = build_forest(W_in, [(d // V, d % V) for d in tup])
        fr["rank"] = np.zeros_like(fr["rank"])             # planted: ascending node index only
        z_p = z_for(fr, rows_p, np.zeros((W_S, V)), [], V)
        z_q = z_for(fr, rows_q, np.zeros((W_S, V)), [], V)
        dist, _, _, _ = layer_outcome_distribution(fr, z_p, z_q, blp, blq, W_L, -1.0, 1, fr["node1"], {})
        total = wgt * dist if total is None else total + wgt * dist
    assert np.max(np.abs(total - iid_product(p_ref, W_L))) > 1e-3


def test_inverted_ratio_would_break_the_theorem():
    """The ratio as printed in Section 3.1 / Algorithm 1 (q over p') cannot be the intended one: with it
    even W=1 does not return p.  Planted in a copy of the accept probability, on the CPU."""
    V = 3
    p = ref_joint([0.0], [[0.3, -0.2, 1.0]]).ravel()
    q = ref_joint([0.0], [[1.0, 0.1, -0.5]]).ravel()
    out_good = np.zeros(V)
    out_bad = np.zeros(V)
    res = np.maximum(p - q, 0); res /= res.sum()
    for x in range(V):
        a_good = min(1.0, p[x] / q[x])
        a_bad = min(1.0, q[x] / p[x])
        out_good[x] += q[x] * a_good
        out_good += q[x] * (1 - a_good) * res
        out_bad[x] += q[x] * a_bad
        out_bad += q[x] * (1 - a_bad) * res
    assert np.max(np.abs(out_good - p)) < 1e-14
    assert np.max(np.abs(out_bad - p)) > 1e-2
    # and the oracle follows the good one
    fr = build_forest(1, [(0, 0)])
    z_p = np.array([[0.3, -0.2, 1.0], [0, 0, 0]]); z_q = np.array([[1.0, 0.1, -0.5], [0, 0, 0]])
    _, trace = run(fr, z_p, z_q, [0.0], [0.0], np.zeros(2, dtype=np.float32), 1, -1.0)
    assert abs(trace[0]["tests"][0]["ratio"] - p[0] / q[0]) < 1e-14


@pytest.mark.parametrize("pattern", [(True, False, True), (True, True, False), (False, True, True)])
def test_second_layer_outputs_are_iid_p_beam_over_survivors(pattern):
    """Layer 2: drafts were drawn from q_beam over ALL layer-1 drafts; those under rejected parents are
    pruned.  Conditioned on the layer-1 outcome, the layer-2 outputs must be iid p_beam^(2) over
    (accepted layer-1 beams) x V."""
    W_in, V, W_S, W_L = 2, 2, 3, 2
    layer1 = [(0, 1), (1, 0), (0, 0)]
    for seed in range(50):           # first seed whose logits let the forced layer-1 pattern happen
        rng = np.random.default_rng(seed)
        rows_p = rng.normal(0, 1, (W_in, V)); rows_q = rows_p + rng.normal(0, 0.6, (W_in, V))
        blp = rng.normal(0, 1, W_in); blq = blp + rng.normal(0, 0.4, W_in)
        rows1_p = rng.normal(0, 1, (W_S, V)); rows1_q = rows1_p + rng.normal(0, 0.6, (W_S, V))
        rows2_p = rng.normal(0, 1, (W_S, V)); rows2_q = rng.normal(0, 1, (W_S, V))
        fr = build_forest(W_in, layer1)
        u = np.zeros(len(fr["parent"]), dtype=np.float32)
        for n, a in zip(fr["node1"], pattern):
            u[n] = U_ACC if a else U_REJ
        res, _ = run(fr, z_for(fr, rows_p, rows1_p, [], V), z_for(fr, rows_q, rows1_q, [], V), blp, blq, u, W_L, -1.0)
        if all((res["node_status"][n] == verify.ACCEPTED) == a for n, a in zip(fr["node1"], pattern)):
            break
    else:
        raise AssertionError("no seed realises the pattern")
    lsm = lambda r: torch.log_softmax(torch.tensor(r, dtype=torch.float64), -1).numpy()
    cum1_p = np.array([blp[s] + lsm(rows_p[s])[x] for s, x in layer1])
    cum1_q = np.array([blq[s] + lsm(rows_q[s])[x] for s, x in layer1])
    q2 = ref_joint(cum1_q, rows1_q)                      # what the drafter sampled layer 2 from
    acc_idx = [j for j, a in enumerate(pattern) if a]
    p2_ref = ref_joint(cum1_p[acc_idx], rows1_p[acc_idx])
    total = None
    for tup in itertools.product(range(W_S * V), repeat=W_S):
        wgt = float(np.prod([q2.ravel()[d] for d in tup]))
        fr = build_forest(W_in, layer1, [(d // V, d % V) for d in tup])
        z_p = z_for(fr, rows_p, rows1_p, rows2_p, V)
        z_q = z_for(fr, rows_q, rows1_q, rows2_q, V)
        fixed = {n: (U_ACC if a else U_REJ) for n, a in zip(fr["node1"], pattern)}
        dist, _, I, pb = layer_outcome_distribution(fr, z_p, z_q, blp, blq, W_L, -1.0, 2, fr["node2"], fixed)
        assert dist is not None, "layer 1 did not pass with the forced pattern"
        assert I == [fr["node1"][j] for j in acc_idx]
        assert np.allclose(pb, p2_ref, atol=1e-14)
        total = wgt * dist if total is None else total + wgt * dist
    assert abs(total.sum() - 1.0) < 1e-12
    assert np.max(np.abs(total - iid_product(p2_ref, W_L))) < 1e-12


@pytest.mark.parametrize("W_in,M,V", [(1, 2, 3), (2, 3, 2), (2, 4, 2)])
def test_accept_count_table_is_the_exact_accept_count_distribution(W_in, M, V):
    """Eq. 1-2: P(M,k) must be the probability that exactly k of M iid drafts are accepted when the layer
    never stops early (width above M)."""
    rng = np.random.default_rng(5 + M)
    rows_p = rng.normal(0, 1, (W_in, V)); rows_q = rows_p + rng.normal(0, 1.0, (W_in, V))
    blp = rng.normal(0, 1, W_in); blq = rng.normal(0, 1, W_in)
    q_ref = ref_joint(blq, rows_q)
    p_ref = ref_joint(blp, rows_p)
    hist = np.zeros(M + 1)
    for tup in itertools.product(range(W_in * V), repeat=M):
        wgt = float(np.prod([q_ref.ravel()[d] for d in tup]))
        fr = build_forest(W_in, [(d // V, d % V) for d in tup])
        z_p = z_for(fr, rows_p, np.zeros((M, V)), [], V)
        z_q = z_for(fr, rows_q, np.zeros((M, V)), [], V)
        _, h, _, _ = layer_outcome_distribution(fr, z_p, z_q, blp, blq, M + 1, -1.0, 1, fr["node1"], {})
        hist += wgt * h
    assert abs(hist.sum() - 1.0) < 1e-12
    alpha = verify.acceptance_chain(p_ref, q_ref, M)
    P = verify.accept_count_table(alpha, M)
    assert np.max(np.abs(P[M] - hist)) < 1e-12

    # Eq. 6: W~(t) = the largest K such that at least K of the M drafts are accepted with probability >= t, read off
    # the ENUMERATED accept-count histogram (not the oracle's table), for thresholds just below and just above every
    # tail probability.  Summing from k = 1 as Eq. 4 prints it (instead of from k = 0) adds P(no draft accepted) to
    # every tail and must come out wrong for at least one of these thresholds.
    tails = [float(hist[K:].sum()) for K in range(M + 1)]          # P(at least K accepted), K = 0..M (enumerated)
    assert abs(tails[0] - 1.0) < 1e-12 and all(a >= b for a, b in zip(tails, tails[1:]))
    assert hist[0] > 1e-3                                           # the two readings do differ on this case
    planted_differs = False
    for K in range(1, M + 1):
        for t in (tails[K] - 1e-7, tails[K] + 1e-7):
            if not 0.0 < t < 1.0:
                continue
            want = max(k for k in range(M + 1) if tails[k] >= t)
            got = verify.dynamic_width(p_ref, q_ref, M, t, 1, 16)[1]
            assert got == want, (K, t, got, want)
            # the variant that starts the sum at k = 1
            planted = max(k for k in range(M + 1) if 1.0 - float(hist[1:k].sum()) >= t)
            planted_differs |= planted != want
    assert planted_differs
    # and the floor / the cap around it: W_L = min(W_cap, max(W_min, W~))
    t_mid = 0.5 * (tails[1] + tails[2]) if M >= 2 else 0.5 * tails[1]
    wt = verify.dynamic_width(p_ref, q_ref, M, t_mid, 1, 16)[1]
    assert verify.dynamic_width(p_ref, q_ref, M, t_mid, wt + 1, 16)[0] == wt + 1
    assert verify.dynamic_width(p_ref, q_ref, M, 0.0, 1, M - 1 if M > 1 else 1)[0] == (M - 1 if M > 1 else 1)
