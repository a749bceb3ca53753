"""The verification call under HIP graph capture: one capture, several replays on NEW inputs in the same buffers, with
eager work and synchronisations between the replays; every replay is compared with the oracle on its own inputs.
(Exchange slots are told apart by a per-launch tag: a replay repeats the captured launch's arguments, so the tag must
also change from replay to replay, or values a previous replay left in the workspace pass for this one's.)"""
import numpy as np
import pytest
import torch

from dsbd_synth import make_workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("top_k,top_p,static", [(0, 1.0, False), (8, 0.9, False), (0, 1.0, True)])
def test_replays_of_a_captured_verification_on_new_inputs(top_k, top_p, static):
    """static: through the entry point that allocates nothing (its workspace is the library's own device array), the
    one meant for callers under capture."""
    import gpu_util as gu
    import paper_2409_16560_amd as dsbd
    dsbd.dsbd_init()                      # (second stream and events exist before the capture)
    kw = dict(L=1, Hq=1, Hkv=1, D=64, V=6000, draft_top_k=3 if top_k else 0)
    ws_ = [make_workload("c5", seed=40 + r, noise_std=0.6, **kw) for r in range(4)]
    d = gu.DeviceWorkload(ws_[0])
    w0 = ws_[0]
    res = dsbd.VerifyResult.allocate(d.forest, w0.W_cap)
    nx = dsbd.NextBeams.allocate(d.forest, w0.W_cap)
    nb = dsbd.dsbd_verify_forest_workspace_bytes(d.forest, w0.V, 0, 1, w0.W_cap, 0.7, top_k, top_p)
    work = torch.empty(nb, dtype=torch.uint8, device="cuda")
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    if static:
        call = lambda st: dsbd.dsbd_verify_forest_static(d.forest, d.logits_p, d.logits_q, d.blp, d.blq, d.u_accept, d.u_resid,
                                                         d.u_fill, res, W_cap=w0.W_cap, t=0.7, stream=st)
    else:
        call = lambda st: d.verify_select(t=0.7, result=res, next_beams=nx, workspace=work, stream=st, top_k=top_k, top_p=top_p)
    call(None)                            # once eagerly (the library's first-call set-up is not part of the capture)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            call(s)
    torch.cuda.synchronize()
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for r in (1, 2, 3, 0, 2):
        w = ws_[r]
        # the forest is the same (same shape, same seeded trees); tokens, logits, likelihoods and uniforms are new
        assert np.array_equal(w.parent, w0.parent) and np.array_equal(w.tree_off, w0.tree_off)
        d.forest.token.copy_(t(w.token).to(d.forest.token.dtype))
        d.logits_p.copy_(t(w.logits_p)); d.logits_q.copy_(t(w.logits_q))
        d.blp.copy_(t(w.beam_logp_p)); d.blq.copy_(t(w.beam_logp_q))
        d.u_accept.copy_(t(w.u_accept)); d.u_resid.copy_(t(w.u_resid)); d.u_fill.copy_(t(w.u_fill))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ref = gu.oracle_verify(w, t=0.7, top_k=top_k, top_p=top_p)
        gu.compare_verify(res, ref, w)
        _ = torch.randn(1 << 18, device="cuda").square().sum().item()      # eager work between the replays
        print("replay on inputs", r, "ok", flush=True)
