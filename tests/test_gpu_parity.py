"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on seeded
synthetic inputs.  Sizes are scaled so the oracle finishes in seconds while the kernels still see
several tiles, several KV splits and ragged tails."""
import numpy as np
import pytest
import torch

from dsbd_synth import make_workload

pytestmark = pytest.mark.gpu


def _gu():
    import gpu_util
    return gpu_util


ATTN_CASES = [
    ("c1", {}),                                                   # tiny: D=64, 3-node chains
    ("c1", dict(W=1, tree_nodes=5, L=77)),                        # single chain = causal attention
    ("c2", dict(L=200)),                                          # 7 rows per tree, ragged tail (200 % 32 != 0)
    ("c2", dict(L=0)),                                            # no prefix at all: tree rows only
    ("c3", dict(L=300, shared_len=101)),                          # shared + own segment, both ragged
    ("c4", dict(L=(33, 190), n_prompts=5, Hq=8, Hkv=8)),          # ragged batch, random trees
    ("c5", dict(L=333)),                                          # GQA 32/8: 124 rows per (tree, KV head)
    ("c5", dict(L=96, Hq=16, Hkv=4, tree_nodes=63, tree="binary_bfs")),   # 63-node trees: 252 rows, two row blocks
    ("c3", dict(L=64, shared_len=0, Hq=8, Hkv=4, D=64)),          # D=64 with GQA
]


@pytest.mark.parametrize("cfg,kw", ATTN_CASES)
def test_forest_attention_matches_oracle(cfg, kw):
    gu = _gu()
    w = make_workload(cfg, V=64, **kw)
    print("case", cfg, kw, "N", w.n_nodes, flush=True)
    d = gu.DeviceWorkload(w)
    anc = torch.zeros(w.n_nodes, dtype=torch.int64, device="cuda")
    out, lse, fault = d.attention(anc_mask_out=anc)
    torch.cuda.synchronize()
    assert int(fault.item()) == 0
    from oracle import forest as o_forest
    assert np.array_equal(anc.cpu().numpy().view(np.uint64), o_forest.ancestor_masks(w.parent, w.tree_off))
    ref_out, ref_lse = gu.oracle_attention(w)
    err = gu.compare_attention(w, out, lse, ref_out, ref_lse)
    print("max abs err out/lse", err, flush=True)


def test_shared_prefix_equals_duplicated_prefix():
    gu = _gu()
    w = make_workload("c3", L=160, shared_len=70, V=64)
    a = gu.DeviceWorkload(w, share_prefix=True).attention()
    b = gu.DeviceWorkload(w, share_prefix=False).attention()
    torch.cuda.synchronize()
    assert torch.max(torch.abs(a[0].float() - b[0].float())).item() <= 2e-2


def test_head_major_cache_layout():
    gu = _gu()
    import paper_2409_16560_amd as dsbd
    w = make_workload("c2", L=100, V=64, Hq=8, Hkv=4)
    d = gu.DeviceWorkload(w)
    ref = d.attention()
    k_hm = [gu.bf16_dev(k).permute(1, 0, 2).contiguous() for k in w.k_own]
    v_hm = [gu.bf16_dev(v).permute(1, 0, 2).contiguous() for v in w.v_own]
    kv = dsbd.PrefixKV(k_hm, v_hm, head_major=True)
    out, lse, fault = dsbd.dsbd_forest_attention(d.forest, kv, d.q, d.k_tree, d.v_tree)
    torch.cuda.synchronize()
    assert int(fault.item()) == 0
    assert torch.equal(out, ref[0]) and torch.equal(lse, ref[1])


VERIFY_CASES = [
    ("c1", {}, 0),
    ("c2", dict(V=1000), 0),
    ("c2", dict(V=32000), 0),
    ("c3", dict(V=4001), 0),                                      # V not a multiple of 4: unaligned rows
    ("c3", dict(V=32000), 0),
    ("c4", dict(V=3000, n_prompts=6), 0),
    ("c5", dict(V=20000), 0),
    ("c5", dict(V=20000, draft="indep"), 0),                      # near-total rejection: residual path
    ("c3", dict(V=5000), 3),                                      # explicit W_L below the number of input beams
]


@pytest.mark.parametrize("t", [-1.0, 0.9, 0.7, 0.3])
@pytest.mark.parametrize("cfg,kw,W_L", VERIFY_CASES)
def test_verify_forest_matches_oracle(cfg, kw, W_L, t):
    gu = _gu()
    w = make_workload(cfg, L=1, Hq=1, Hkv=1, D=64, **kw)
    print("case", cfg, kw, "W_L", W_L, "t", t, "N", w.n_nodes, flush=True)
    d = gu.DeviceWorkload(w)
    res = d.verify(W_L=W_L, t=t)
    torch.cuda.synchronize()
    ref = gu.oracle_verify(w, W_L=W_L, t=t)
    near = gu.compare_verify(res, ref, w)
    print("l_last", ref["l_last"].tolist(), "widths", ref["layer_width"].tolist(), "near ties", near, flush=True)
    import paper_2409_16560_amd as dsbd
    from oracle import select as o_select
    for keep_one in (False, True):
        nx = dsbd.dsbd_select_beams(d.forest, res, keep_one=keep_one)
        torch.cuda.synchronize()
        sref = o_select.select_beams(w.tree_off, w.parent, ref["n_out"], ref["out_parent"], ref["out_token"],
                                     ref["out_logp_p"], ref["out_logp_q"], w.max_depth + 1, keep_one=keep_one)
        if near == 0:
            g = lambda x: x.cpu().numpy()
            for name in ("n_next", "src_tree", "src_out", "path_len", "path", "token"):
                assert np.array_equal(g(getattr(nx, name)), sref[name]), name
            assert np.max(np.abs(g(nx.logp_target) - sref["logp_p"])) <= 1e-9


@pytest.mark.parametrize("seed", [11, 12, 13, 14, 15, 16])
@pytest.mark.parametrize("noise", [0.25, 0.5, 0.8, 2.5])
def test_verify_accept_patterns_over_seeds(seed, noise):
    """Many different accept / reject sequences on the benchmark's forest shape: runs of acceptances, rejection
    streaks of several chain entries, layers that fall short at every depth (the draft's distance from the target
    sets the acceptance rate).  Fixed and dynamic width."""
    gu = _gu()
    w = make_workload("c5", L=1, Hq=1, Hkv=1, D=64, V=9000, seed=seed, noise_std=noise)
    d = gu.DeviceWorkload(w)
    for t in (-1.0, 0.6):
        res = d.verify(t=t)
        torch.cuda.synchronize()
        ref = gu.oracle_verify(w, t=t)
        gu.compare_verify(res, ref, w)


def test_verify_with_draft_rank_order():
    gu = _gu()
    w = make_workload("c3", L=1, Hq=1, Hkv=1, D=64, V=3000)
    rng = np.random.default_rng(5)
    rank = rng.permutation(w.n_nodes).astype(np.int32)
    d = gu.DeviceWorkload(w, rank=rank)
    res = d.verify(t=0.7)
    torch.cuda.synchronize()
    ref = gu.oracle_verify(w, t=0.7, rank=rank)
    gu.compare_verify(res, ref, w)


def test_verify_is_deterministic():
    gu = _gu()
    w = make_workload("c4", L=1, Hq=1, Hkv=1, D=64, V=3000, n_prompts=6)
    d = gu.DeviceWorkload(w)
    a = d.verify(t=0.9)
    b = d.verify(t=0.9)
    torch.cuda.synchronize()
    for name in ("node_status", "out_parent", "out_token", "out_node", "l_last", "layer_width", "out_logp_target"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name


def test_device_side_faults_are_reported_not_fatal():
    gu = _gu()
    import paper_2409_16560_amd as dsbd
    w = make_workload("c2", L=40, V=500, Hq=4, Hkv=4)
    # parent pointing outside its tree
    bad = w.parent.copy(); bad[9] = 1
    w2 = make_workload("c2", L=40, V=500, Hq=4, Hkv=4); w2.parent = bad
    d = gu.DeviceWorkload(w2)
    _, _, fault = d.attention()
    res = d.verify()
    torch.cuda.synchronize()
    assert int(fault.item()) & dsbd.DSBD_FAULT_TOPOLOGY
    assert int(res.fault.item()) & dsbd.DSBD_FAULT_TOPOLOGY
    # non-finite logit and token out of range
    w3 = make_workload("c2", L=40, V=500, Hq=4, Hkv=4)
    w3.logits_p[3, 7] = np.inf
    w3.token[5] = 500
    res = gu.DeviceWorkload(w3).verify()
    torch.cuda.synchronize()
    f = int(res.fault.item())
    assert f & dsbd.DSBD_FAULT_NONFINITE and f & dsbd.DSBD_FAULT_TOKEN


def test_a_missing_partner_ends_in_a_fault_bit_not_in_a_hang():
    """Error path of the layer kernel's exchanges, forced from the host: one workgroup withholds its first post
    (test hook), every wait for it is bounded (2 ms here instead of 3 s), so all workgroups give up, the kernel ends
    normally and the call reports DSBD_FAULT_SYNC_TIMEOUT.  The next call on the same workspace works."""
    import os
    gu = _gu()
    import paper_2409_16560_amd as dsbd
    w = make_workload("c5", L=1, Hq=1, Hkv=1, D=64, V=20000)
    d = gu.DeviceWorkload(w)
    nbytes = dsbd.dsbd_verify_forest_workspace_bytes(d.forest, w.V, 0, 1, w.W_cap, -1.0)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    os.environ["DSBD_VERIFY_SYNC_LIMIT_US"] = "2000"
    os.environ["DSBD_VERIFY_TEST_MUTE_WG"] = "5"
    try:
        res = d.verify(workspace=ws)
        torch.cuda.synchronize()
    finally:
        del os.environ["DSBD_VERIFY_SYNC_LIMIT_US"]
        del os.environ["DSBD_VERIFY_TEST_MUTE_WG"]
    assert int(res.fault.item()) & dsbd.DSBD_FAULT_SYNC_TIMEOUT
    res = d.verify(workspace=ws)
    torch.cuda.synchronize()
    gu.compare_verify(res, gu.oracle_verify(w), w)
