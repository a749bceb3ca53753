"""The entry point that allocates nothing: dsbd_verify_forest_static (workspace = a device array inside the library's
image) must return what dsbd_verify_forest returns with a caller-supplied workspace, on two calls in a row, the second
on a smaller problem (the array keeps what the first call left there).  Collected last: a failure here must not hide
the other GPU tests from a run that stops at the first failure."""
import numpy as np
import pytest
import torch

from dsbd_synth import make_workload

pytestmark = pytest.mark.gpu


def _both(w, t, top_k=0, top_p=1.0):
    import paper_2409_16560_amd as dsbd
    from dsbd_synth.device import DeviceWorkload
    d = DeviceWorkload(w)
    # the static entry point first: in a fresh process it then runs before the library's second stream exists (the
    # statistics pass in front of the layer kernel), after other tests with the stream in place (beside it)
    res = dsbd.VerifyResult.allocate(d.forest, w.W_cap)
    dsbd.dsbd_verify_forest_static(d.forest, d.logits_p, d.logits_q, d.blp, d.blq, d.u_accept, d.u_resid, d.u_fill, res,
                                   W_cap=w.W_cap, t=t, top_k=top_k, top_p=top_p)
    torch.cuda.synchronize()
    ref = d.verify(t=t, top_k=top_k, top_p=top_p)
    torch.cuda.synchronize()
    g = lambda x: x.cpu().numpy()
    assert int(g(res.fault)[0]) == int(g(ref.fault)[0]) == 0
    for name in ("node_status", "l_last", "layer_width", "n_out", "out_parent", "out_token", "out_node", "near_tie_count"):
        assert np.array_equal(g(getattr(res, name)), g(getattr(ref, name))), name
    # the two entry points run the same kernels on the same inputs: floating-point outputs agree bit for bit
    for name in ("out_logp_target", "out_logp_draft", "lse_target", "lse_draft", "node_logp_target", "node_logp_draft"):
        assert np.array_equal(g(getattr(res, name)), g(getattr(ref, name))), name
    return res, d


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    import gpu_util as gu
    import paper_2409_16560_amd as dsbd
    assert dsbd.dsbd_verify_forest_static_capacity() == 32 << 20
    # first call: the benchmark's forest at a reduced vocabulary (8 beams, 248 nodes, 5 layers, 256 workgroups);
    # second call, right behind it on the same array: a smaller batch of several prompts, dynamic width and warping
    w1 = make_workload("c5", L=1, Hq=1, Hkv=1, D=64, V=20000)
    res1, _ = _both(w1, t=-1.0)
    gu.compare_verify(res1, gu.oracle_verify(w1, t=-1.0), w1)
    w2 = make_workload("c4", L=1, Hq=1, Hkv=1, D=64, V=3000, n_prompts=6)
    res2, _ = _both(w2, t=0.7)
    gu.compare_verify(res2, gu.oracle_verify(w2, t=0.7), w2)
    w3 = make_workload("c3", L=1, Hq=1, Hkv=1, D=64, V=5000, draft_top_k=4)
    res3, _ = _both(w3, t=-1.0, top_k=8, top_p=0.9)
    gu.compare_verify(res3, gu.oracle_verify(w3, t=-1.0, top_k=8, top_p=0.9), w3)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import paper_2409_16560_amd as dsbd
    from dsbd_synth.device import DeviceWorkload
    # 16 prompts at the full vocabulary keep their joint slices in the workspace: far beyond the 32 MiB array
    w = make_workload("c4", L=1, Hq=1, Hkv=1, D=64)
    d = DeviceWorkload(w)
    need = dsbd.dsbd_verify_forest_workspace_bytes(d.forest, w.V, 0, 1, w.W_cap, -1.0)
    assert need > dsbd.dsbd_verify_forest_static_capacity()
    res = dsbd.VerifyResult.allocate(d.forest, w.W_cap)
    with pytest.raises(dsbd.DsbdError) as e:
        dsbd.dsbd_verify_forest_static(d.forest, d.logits_p, d.logits_q, d.blp, d.blq, d.u_accept, d.u_resid, d.u_fill, res,
                                       W_cap=w.W_cap)
    assert e.value.code == -3
