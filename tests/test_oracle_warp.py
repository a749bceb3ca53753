"""Pins of the warping operation T (top-k, top-p) on the beam-sampling joints (Section 2.1; Section 3.1 "Details":
p_beam = T o p/P, q_beam = T o q/Q; appendix "Experiment Configuration": top-k then top-p, k = 10, p = 0.8).

Independent references: the logits warpers of the transformers library applied to the flattened joint, the
degenerate settings, and the exhaustive enumeration of the correctness theorem with warped distributions."""
import itertools

import numpy as np
import pytest
import torch

from enum_util import build_forest, layer_outcome_distribution
from oracle import verify
from test_oracle_theorem import iid_product, ref_joint, z_for


def hf_warp(joint, top_k, top_p):
    from transformers import TopKLogitsWarper, TopPLogitsWarper
    x = torch.log(torch.tensor(joint, dtype=torch.float64).reshape(1, -1))
    if top_k > 0:
        x = TopKLogitsWarper(top_k)(None, x)
    if top_p < 1.0:
        x = TopPLogitsWarper(top_p)(None, x)
    return torch.softmax(x, dim=-1).numpy().reshape(joint.shape)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("top_k,top_p", [(10, 0.8), (3, 1.0), (0, 0.5), (7, 0.35), (1, 0.9), (40, 0.999)])
def test_warp_joint_equals_library_warpers_on_the_flattened_joint(seed, top_k, top_p):
    rng = np.random.default_rng(seed)
    W, V = 3, 37
    joint = ref_joint(rng.normal(0, 1, W), rng.normal(0, 2.0, (W, V)))
    got = verify.warp_joint(joint, top_k, top_p)
    want = hf_warp(joint, top_k, top_p)
    assert np.array_equal(got > 0, want > 0)
    assert np.max(np.abs(got - want)) < 1e-14 and abs(got.sum() - 1.0) < 1e-14


def test_warp_degenerate_settings():
    rng = np.random.default_rng(1)
    joint = ref_joint(rng.normal(0, 1, 2), rng.normal(0, 1, (2, 9)))
    assert np.array_equal(verify.warp_joint(joint, 0, 1.0), joint)                     # both steps off: identity
    assert np.allclose(verify.warp_joint(joint, 18, 1.0), joint, atol=1e-16)           # k covers everything
    one = verify.warp_joint(joint, 1, 1.0)                                             # k = 1: the deterministic case
    assert one.ravel()[np.argmax(joint)] == 1.0 and one.sum() == 1.0
    # "smallest subset whose mass exceeds p": with p below the largest entry a single entry is kept
    assert (verify.warp_joint(joint, 0, float(joint.max()) * 0.99) > 0).sum() == 1
    # ties go to the lower flat index
    tie = np.array([[0.25, 0.25], [0.25, 0.25]])
    assert np.array_equal(verify.warp_joint(tie, 2, 1.0), np.array([[0.5, 0.5], [0.0, 0.0]]))


@pytest.mark.parametrize("W_in,W_S,W_L,V,top_k,top_p,t", [
    (2, 2, 2, 3, 3, 1.0, -1.0),
    (2, 3, 2, 3, 4, 0.8, -1.0),
    (1, 3, 2, 4, 3, 0.9, -1.0),
    (2, 3, 0, 3, 4, 0.7, 0.5),       # dynamic width on the warped joints
])
def test_outputs_are_iid_warped_p_beam_when_drafts_come_from_warped_q_beam(W_in, W_S, W_L, V, top_k, top_p, t):
    """Theorem 3.1 with T in place: drafts iid from T o q_beam, outputs iid from T o p_beam."""
    rng = np.random.default_rng(7 * W_in + W_S + V)
    rows_p = rng.normal(0, 1.0, (W_in, V)); rows_q = rows_p + rng.normal(0, 0.8, (W_in, V))
    blp = rng.normal(0, 1, W_in); blq = blp + rng.normal(0, 0.5, W_in)
    p_ref = hf_warp(ref_joint(blp, rows_p), top_k, top_p)
    q_ref = hf_warp(ref_joint(blq, rows_q), top_k, top_p)
    support = [d for d in range(W_in * V) if q_ref.ravel()[d] > 0]
    total, widths = None, set()
    for tup in itertools.product(support, repeat=W_S):
        wgt = float(np.prod([q_ref.ravel()[d] for d in tup]))
        fr = build_forest(W_in, [(d // V, d % V) for d in tup])
        z_p = z_for(fr, rows_p, np.zeros((W_S, V)), [], V)
        z_q = z_for(fr, rows_q, np.zeros((W_S, V)), [], V)
        dist, _, I, pb = layer_outcome_distribution(fr, z_p, z_q, blp, blq, W_L, t, 1, fr["node1"], {},
                                                    top_k=top_k, top_p=top_p)
        assert np.allclose(pb, p_ref, atol=1e-14)
        widths.add(dist.ndim)
        total = wgt * dist if total is None else total + wgt * dist
    assert len(widths) == 1
    width = widths.pop()
    assert abs(total.sum() - 1.0) < 1e-12
    assert np.max(np.abs(total - iid_product(p_ref, width))) < 1e-12
