"""Verifications issued from several streams without synchronisation in between.  The layer kernel is persistent and
needs its workgroups resident together, so the library orders its layer launches across streams by itself; each call
must return what the same call returns alone."""
import numpy as np
import pytest
import torch

from dsbd_synth import make_workload

pytestmark = pytest.mark.gpu

NAMES = ("node_status", "l_last", "layer_width", "n_out", "out_parent", "out_token", "out_node", "near_tie_count",
         "out_logp_target", "out_logp_draft", "lse_target", "lse_draft", "node_logp_target", "node_logp_draft")


def test_verifications_on_two_streams_do_not_disturb_each_other():
    import gpu_util as gu
    from dsbd_synth.device import DeviceWorkload
    wa = make_workload("c5", L=1, Hq=1, Hkv=1, D=64, V=20000)
    wb = make_workload("c4", L=1, Hq=1, Hkv=1, D=64, V=6000, n_prompts=5, seed=7)
    da, db = DeviceWorkload(wa), DeviceWorkload(wb)
    alone_a, alone_b = da.verify(t=-1.0), db.verify(t=0.8)
    torch.cuda.synchronize()
    gu.compare_verify(alone_a, gu.oracle_verify(wa, t=-1.0), wa)
    gu.compare_verify(alone_b, gu.oracle_verify(wb, t=0.8), wb)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    sa.wait_stream(torch.cuda.current_stream())
    sb.wait_stream(torch.cuda.current_stream())
    got = []
    for _ in range(4):
        with torch.cuda.stream(sa):
            got.append((da.verify(t=-1.0, stream=sa), alone_a))
        with torch.cuda.stream(sb):
            got.append((db.verify(t=0.8, stream=sb), alone_b))
    torch.cuda.synchronize()
    g = lambda x: x.cpu().numpy()
    for i, (res, ref) in enumerate(got):
        assert int(g(res.fault)[0]) == 0, i
        for name in NAMES:
            assert np.array_equal(g(getattr(res, name)), g(getattr(ref, name))), (i, name)
