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
    ("c3", dict(L=40, shared_len=40, Hq=8, Hkv=2)),               # the whole prefix shared: every beam's own part is empty
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


# The three main kernels: wave-private K/V streams (at most 32 rows per stream, 16 or 32 of them), the register-staged
# shared tile (head size 64), the tile loaded straight into the LDS (head size 128); each with a ragged last tile and
# a shared leading segment whose end falls inside a split.
SPLIT_KERNELS = [
    ("wave-private, 15 rows", "c3", dict(L=777, shared_len=301, Hq=8, Hkv=8)),
    ("wave-private, 30 rows", "c3", dict(L=777, shared_len=301, Hq=8, Hkv=4)),
    ("shared tile, D=64", "c5", dict(L=1100, shared_len=413, Hq=16, Hkv=4, D=64)),
    ("tile into LDS, D=128", "c5", dict(L=1100, shared_len=413, Hq=16, Hkv=4)),
    ("tile into LDS, 63-node trees", "c5", dict(L=600, shared_len=0, Hq=8, Hkv=2, tree_nodes=63, tree="binary_bfs", W=3)),
]


@pytest.mark.parametrize("nsplit", [2, 4, 8])
@pytest.mark.parametrize("name,cfg,kw", SPLIT_KERNELS)
def test_forest_attention_with_pinned_kv_splits(name, cfg, kw, nsplit, knobs):
    """Every main kernel with 2, 4 and 8 KV splits per (tree, KV head, row block) and the merge kernel behind them
    (the plan of the scaled-down cases would otherwise settle on one or two splits)."""
    gu = _gu()
    knobs.set("DSBD_ATTN_NSPLIT", nsplit)
    w = make_workload(cfg, V=64, **kw)
    print("case", name, kw, "nsplit", nsplit, "N", w.n_nodes, flush=True)
    d = gu.DeviceWorkload(w)
    out, lse, fault = d.attention()
    torch.cuda.synchronize()
    assert int(fault.item()) == 0
    ref_out, ref_lse = gu.oracle_attention(w)
    err = gu.compare_attention(w, out, lse, ref_out, ref_lse)
    print("max abs err out/lse", err, flush=True)


def _plant_outlier_keys(w, beta=8.0, seed=7):
    """Overwrites a few keys so that one query row each scores far above everything it has seen: key = beta x that
    row's query (exact in bf16 for a power of two), i.e. beta |q|^2 / sqrt(D) ~ 90 (64 at head size 64) against N(0,1) scores.  Places:
    late in the own prefix segment, at the end of the shared segment, in the first tile, and among the tree rows (an
    ancestor's key).  Returns the (node, head) rows that now have such a key."""
    from dsbd_synth import bf16_bits_to_f32, f32_to_bf16_bits
    rng = np.random.default_rng(seed)
    group = w.Hq // w.Hkv
    hit = []
    qf = bf16_bits_to_f32(w.q)
    for b in range(w.n_trees):
        a0, a1 = int(w.tree_off[b]), int(w.tree_off[b + 1])
        p = int(w.tree_prompt[b])
        own, sh = int(w.own_len[b]), int(w.shared_len[b])
        places = []
        if own > 0:
            places += [("own", own - 1 - int(rng.integers(0, min(own, 40)))), ("own", int(rng.integers(0, own)))]
        if sh > 0 and b == int(np.argmax(w.tree_prompt == p)):
            places += [("shared", sh - 1)]
        if own > 3:
            places += [("own", 2)]
        for kind, pos in places:
            n = int(rng.integers(a0, a1)); h = int(rng.integers(0, w.Hq)); g = h // group
            key = f32_to_bf16_bits(np.float32(beta) * qf[n, h])
            if kind == "own":
                w.k_own[b][pos, g, :] = key
            else:
                w.k_shared[p][pos, g, :] = key
            hit.append((n, h))
        if a1 - a0 >= 2:
            # a tree row: the key of node n's parent, tuned to n's query
            n = int(rng.integers(a0 + 1, a1)); h = int(rng.integers(0, w.Hq)); g = h // group
            w.k_tree[int(w.parent[n]), g, :] = f32_to_bf16_bits(np.float32(beta) * qf[n, h])
            hit.append((n, h))
    return hit


@pytest.mark.parametrize("name,cfg,kw", SPLIT_KERNELS)
@pytest.mark.parametrize("nsplit", [1, 4])
def test_forest_attention_outlier_scores_raise_the_reference(name, cfg, kw, nsplit, knobs):
    """The kernels keep a per-row softmax reference that is only raised when a score exceeds it by 2^40, and then
    rescale what they have accumulated.  Random N(0,1) caches never get there after a row's first step, so keys tuned
    to single query rows are planted late in the prefix, at the end of the shared segment and among the tree rows:
    the reference rises in mid-stream, with non-zero accumulators, inside and across KV splits."""
    gu = _gu()
    knobs.set("DSBD_ATTN_NSPLIT", nsplit)
    w = make_workload(cfg, V=64, **kw)
    hit = _plant_outlier_keys(w)
    d = gu.DeviceWorkload(w)
    out, lse, fault = d.attention()
    torch.cuda.synchronize()
    assert int(fault.item()) == 0
    ref_out, ref_lse = gu.oracle_attention(w)
    # the planted keys do dominate their rows (the case tests what it says): 2^40 is 27.7 in natural units
    assert min(ref_lse[n, h] for n, h in hit) > 35.0
    err = gu.compare_attention(w, out, lse, ref_out, ref_lse)
    print("case", name, "nsplit", nsplit, "rows with a planted key", len(hit), "max abs err out/lse", err, flush=True)


@pytest.mark.parametrize("name,cfg,kw", SPLIT_KERNELS)
@pytest.mark.parametrize("scale", [0.03, 0.25, 2.0])
def test_forest_attention_explicit_scale(name, cfg, kw, scale):
    """A caller-supplied softmax scale instead of 1/sqrt(D): flatter than the default, sharper, and so sharp
    (score deviations of tens of units) that new maxima more than 2^40 above the reference keep turning up along the
    prefix and the softmax is close to one-hot."""
    gu = _gu()
    from oracle import attention as o_attn
    w = make_workload(cfg, V=64, **kw)
    d = gu.DeviceWorkload(w)
    out, lse, fault = d.attention(scale=scale)
    torch.cuda.synchronize()
    assert int(fault.item()) == 0
    pk, pv = zip(*[gu.logical_prefix(w, t) for t in range(w.n_trees)])
    ref_out, ref_lse = o_attn.forest_attention(w.parent, w.tree_off, gu.f64(w.q), gu.f64(w.k_tree), gu.f64(w.v_tree),
                                               list(pk), list(pv), scale=scale)
    # the lse tolerance is absolute on a quantity that now reaches hundreds: bf16 keys and queries are exact inputs on
    # both sides and the scores are fp32 sums of exact products, so the absolute bound still holds up to scale 2
    err = gu.compare_attention(w, out, lse, ref_out, ref_lse)
    print("case", name, "scale", scale, "max abs err out/lse", err, "largest lse", float(np.max(ref_lse)), flush=True)


@pytest.mark.parametrize("sweep", [0, 1])
def test_forest_attention_random_shapes(sweep):
    """Randomized sweep: tree shapes up to 64 nodes, head groupings, both head sizes, prefix lengths from nothing to
    several tiles (equal or ragged within the batch), shared leading segments up to the whole prefix, given to the
    library as a segment of their own or duplicated into every beam's cache."""
    from dsbd_synth.workloads import Spec
    from oracle import forest as o_forest
    gu = _gu()
    rng = np.random.default_rng(2000 + sweep)
    for case in range(30):
        tree = str(rng.choice(["random", "binary_dfs", "binary_bfs", "chain", "fork_chain"]))
        nodes = int(rng.choice([3, 7, 15, 31, 63])) if tree == "binary_dfs" else (1, int(rng.integers(1, 65)))
        Hq, Hkv = [(1, 1), (4, 4), (8, 2), (4, 1), (32, 8), (16, 16)][int(rng.integers(0, 6))]
        Lhi = int(rng.choice([0, 5, 40, 130, 300, 700]))
        L = (0, Lhi) if rng.random() < 0.5 else Lhi
        shared = int(rng.integers(0, (Lhi if isinstance(L, int) else 0) + 1)) if rng.random() < 0.4 else 0
        if case % 10 == 0 and isinstance(L, int):
            shared = L                                   # the whole prefix shared
        spec = Spec("sweep", int(rng.integers(1, 4)), (1, int(rng.integers(1, 6))), tree, nodes, L, shared, Hq, Hkv,
                    int(rng.choice([64, 128])), 64, 3.0, "noise", 0.5, int(rng.integers(0, 1 << 30)))
        w = make_workload(spec)
        d = gu.DeviceWorkload(w, share_prefix=bool(rng.integers(0, 2)))
        anc = torch.zeros(w.n_nodes, dtype=torch.int64, device="cuda")
        out, lse, fault = d.attention(anc_mask_out=anc)
        torch.cuda.synchronize()
        try:
            assert int(fault.item()) == 0
            assert np.array_equal(anc.cpu().numpy().view(np.uint64), o_forest.ancestor_masks(w.parent, w.tree_off))
            ref_out, ref_lse = gu.oracle_attention(w)
            gu.compare_attention(w, out, lse, ref_out, ref_lse)
        except AssertionError as e:
            raise AssertionError("sweep %d case %d (%s): %s" % (sweep, case, spec, e))


@pytest.mark.parametrize("cfg,kw", [("c5", dict(L=333)), ("c5", dict(L=96, Hq=16, Hkv=4, tree_nodes=63, tree="binary_bfs")),
                                    ("c3", dict(L=300, shared_len=101, Hq=8, Hkv=1))])
def test_register_staged_tile_kernel(cfg, kw, knobs):
    """Head size 128 with many rows per K/V stream normally runs the kernel that loads its tiles straight into the
    LDS; the register-staged kernel (what head size 64 uses) is selected by a knob and must give the same."""
    gu = _gu()
    w = make_workload(cfg, V=64, **kw)
    d = gu.DeviceWorkload(w)
    ref_out, ref_lse = gu.oracle_attention(w)
    out, lse, fault = d.attention()
    torch.cuda.synchronize()
    knobs.set("DSBD_ATTN_STAGED", "1")
    out2, lse2, fault2 = d.attention()
    torch.cuda.synchronize()
    assert int(fault.item()) == 0 and int(fault2.item()) == 0
    gu.compare_attention(w, out, lse, ref_out, ref_lse)
    gu.compare_attention(w, out2, lse2, ref_out, ref_lse)
    assert float((out.float() - out2.float()).abs().max()) <= 2e-2


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
    gu.check_verify_select(d, w, ref, W_L=W_L, t=t)        # the same through the one-call form
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
        gu.check_verify_select(d, w, ref, t=t)


@pytest.mark.parametrize("sweep", [0, 1, 2])
def test_verify_random_forests_and_parameters(sweep):
    """Randomized sweep: prompts, beams, tree shapes and sizes, vocabulary sizes (one workgroup per prompt up to
    several per row), draft distance, fixed / dynamic width, W_L above and below the number of beams, warping."""
    from dsbd_synth.workloads import Spec
    gu = _gu()
    rng = np.random.default_rng(1000 + sweep)
    for case in range(25):
        tree = str(rng.choice(["random", "binary_dfs", "chain", "fork_chain"]))
        nodes = int(rng.choice([3, 7, 15, 31])) if tree == "binary_dfs" else (2, int(rng.integers(3, 32)))
        spec = Spec("sweep", int(rng.integers(1, 5)), (1, int(rng.integers(1, 9))), tree, nodes, 1, 0, 1, 1, 64,
                    int(rng.choice([17, 130, 1000, 4097, 12000, 33000])), float(rng.choice([1.0, 3.0])),
                    str(rng.choice(["noise", "indep"])), float(rng.choice([0.25, 0.5, 1.0, 2.5])),
                    int(rng.integers(0, 1 << 30)), int(rng.choice([0, 0, 4])))
        t = float(rng.choice([-1.0, -1.0, 0.3, 0.6, 0.9]))
        W_L = int(rng.choice([0, 0, 2, 5]))
        top_k, top_p = 0, 1.0
        if spec.draft_top_k and rng.random() < 0.7:
            top_k, top_p = int(rng.choice([1, 5, 16, 32])), float(rng.choice([1.0, 0.9, 0.6]))
        w = make_workload(spec)
        d = gu.DeviceWorkload(w)
        res = d.verify(W_L=W_L, t=t, top_k=top_k, top_p=top_p)
        torch.cuda.synchronize()
        ref = gu.oracle_verify(w, W_L=W_L, t=t, top_k=top_k, top_p=top_p)
        try:
            gu.compare_verify(res, ref, w)
            gu.check_verify_select(d, w, ref, W_L=W_L, t=t, top_k=top_k, top_p=top_p)
        except AssertionError as e:
            raise AssertionError("sweep %d case %d (%s, t=%g, W_L=%d, top_k=%d, top_p=%g): %s"
                                 % (sweep, case, spec, t, W_L, top_k, top_p, e))


WARP_CASES = [
    # (config, overrides, top_k, top_p)
    ("c3", dict(V=5000, draft_top_k=4), 16, 1.0),
    ("c3", dict(V=5000, draft_top_k=4), 16, 0.8),
    ("c3", dict(V=5000, draft_top_k=2), 5, 0.6),
    ("c3", dict(V=4001, draft_top_k=8), 32, 0.95),
    ("c2", dict(V=32000, draft_top_k=3), 8, 0.9),
    ("c5", dict(V=20000, draft_top_k=4), 32, 0.9),
    ("c5", dict(V=20000, draft_top_k=4, draft="indep"), 12, 1.0),    # supports that barely overlap
    ("c4", dict(V=3000, n_prompts=6, draft_top_k=4), 10, 0.85),      # several prompts, ragged widths
    ("c1", dict(V=9, draft_top_k=3), 32, 0.9),                       # fewer than top_k entries in I x V
    ("c3", dict(V=5000, draft_top_k=1), 1, 1.0),                     # top_k = 1: one-point joints
]


@pytest.mark.parametrize("t", [-1.0, 0.6])
@pytest.mark.parametrize("cfg,kw,top_k,top_p", WARP_CASES)
def test_verify_with_warping_matches_oracle(cfg, kw, top_k, top_p, t):
    """Warping operation T (top-k, then top-p) on the joints: the decisions, widths and samples agree with the oracle's."""
    gu = _gu()
    w = make_workload(cfg, L=1, Hq=1, Hkv=1, D=64, **kw)
    print("case", cfg, kw, "top_k", top_k, "top_p", top_p, "t", t, flush=True)
    d = gu.DeviceWorkload(w)
    res = d.verify(t=t, top_k=top_k, top_p=top_p)
    torch.cuda.synchronize()
    ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=top_p)
    near = gu.compare_verify(res, ref, w)
    st = ref["node_status"]
    print("l_last", ref["l_last"].tolist(), "accepted", int((st == 1).sum()), "rejected", int((st == 2).sum()),
          "near ties", near, flush=True)


@pytest.mark.parametrize("seed", [21, 22, 23, 24])
def test_verify_with_warping_over_seeds(seed):
    gu = _gu()
    w = make_workload("c5", L=1, Hq=1, Hkv=1, D=64, V=9000, seed=seed, noise_std=0.8, draft_top_k=3)
    d = gu.DeviceWorkload(w)
    for top_k, top_p, t in ((8, 1.0, -1.0), (8, 0.7, 0.6), (24, 0.9, -1.0), (3, 0.5, 0.3)):
        print("seed", seed, "top_k", top_k, "top_p", top_p, "t", t, flush=True)
        res = d.verify(t=t, top_k=top_k, top_p=top_p)
        torch.cuda.synchronize()
        ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=top_p)
        gu.compare_verify(res, ref, w)


@pytest.mark.parametrize("fast", [1, 0])
@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("seed", [31, 32])
def test_warping_selection_in_one_level_and_by_the_tree(seed, G, fast, knobs):
    """The two forms of the top-k selection on the same inputs.  With many workgroups per prompt (forced here on a
    mid-size vocabulary: 8 or 16 pieces per row) the bound comes from the table of the workgroups' largest entries
    and the candidates travel in one exchange; DSBD_WARP_FAST=0 keeps the tree of merges.  top_k 16 on 64 workgroups
    has just the 4 x top_k workgroups the one-level form asks for, top_k 24 has not and takes the tree either way."""
    gu = _gu()
    knobs.set("DSBD_VERIFY_G", G)
    knobs.set("DSBD_WARP_FAST", fast)
    w = make_workload("c5", L=1, Hq=1, Hkv=1, D=64, V=9000, seed=seed, noise_std=0.8, draft_top_k=3)
    d = gu.DeviceWorkload(w)
    for top_k, top_p, t in ((3, 1.0, -1.0), (8, 0.7, 0.6), (16, 0.9, -1.0), (24, 0.8, 0.3), (10, 0.8, -1.0)):
        print("seed", seed, "G", G, "fast", fast, "top_k", top_k, "top_p", top_p, "t", t, flush=True)
        res = d.verify(t=t, top_k=top_k, top_p=top_p)
        torch.cuda.synchronize()
        ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=top_p)
        gu.compare_verify(res, ref, w)


@pytest.mark.parametrize("quantum", ["half", "bf16"])
@pytest.mark.parametrize("G", [2, 3, 16, 64])
def test_warping_with_equal_logits_in_different_pieces_of_a_row(G, quantum, knobs):
    """Logits on a coarse grid (multiples of 0.5, or rounded to bfloat16 as a 16-bit model's are): equal logits of one
    row sit in different workgroups' pieces, whose slice entries are scaled piece by piece.  Equal logits must still give
    equal joint entries, or the order of equal values (by index) that decides the top-k / top-p cut comes out different
    from a row-by-row evaluation: the candidates are ranked by values recomputed from the logits in a form that depends
    on the row alone.  (Found by a randomized sweep: wrong sampled tokens with two or more workgroups per prompt.)"""
    import dataclasses
    gu = _gu()
    knobs.set("DSBD_VERIFY_G", G)
    for seed, n_prompts in ((895529104, 2), (188831134, 2), (5, 1)):
        w = make_workload("c4", n_prompts=n_prompts, W=(1, 6), tree_nodes=(2, 7), L=1, Hq=1, Hkv=1, D=64, V=2000, seed=seed,
                          logit_std=1.0, noise_std=1.0, draft_top_k=4)
        if quantum == "half":
            q = lambda z: (np.round(z * 2) / 2).astype(np.float32)
        else:
            q = lambda z: torch.from_numpy(z).to(torch.bfloat16).to(torch.float32).numpy()
        w = dataclasses.replace(w, logits_p=q(w.logits_p), logits_q=q(w.logits_q))
        d = gu.DeviceWorkload(w)
        for top_k, top_p, t in ((32, 0.6, 0.6), (32, 1.0, -1.0), (10, 0.8, -1.0), (31, 0.6, 0.3)):
            print("seed", seed, "G", G, quantum, "top_k", top_k, "top_p", top_p, "t", t, flush=True)
            res = d.verify(t=t, top_k=top_k, top_p=top_p)
            torch.cuda.synchronize()
            ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=top_p)
            gu.compare_verify(res, ref, w)


@pytest.mark.parametrize("G", [0, 64])
@pytest.mark.parametrize("cfg,kw", [("c3", dict(V=5000)), ("c2", dict(V=700)), ("c4", dict(V=3000, n_prompts=3))])
def test_warping_with_many_equal_entries(cfg, kw, G, knobs):
    """Rows of equal logits: thousands of joint entries tie, the order of equal values (lower flat index first)
    decides which are kept, and the selection has to leave its fast path (more candidates than it can hold).  With 64
    workgroups forced the one-level form is tried first: the candidates do not fit the workgroups' slots and all fall
    back to the tree."""
    import dataclasses
    gu = _gu()
    if G and cfg != "c4":
        knobs.set("DSBD_VERIFY_G", G)
    w = make_workload(cfg, L=1, Hq=1, Hkv=1, D=64, **kw)
    zp, zq = np.zeros_like(w.logits_p), np.zeros_like(w.logits_q)
    zp[1::3] = np.round(w.logits_p[1::3])            # some rows with a few distinct levels instead
    zq[1::3] = np.round(w.logits_q[1::3])
    w = dataclasses.replace(w, logits_p=zp, logits_q=zq)
    d = gu.DeviceWorkload(w)
    for top_k, top_p, t in ((16, 1.0, -1.0), (32, 0.7, 0.5), (3, 0.9, -1.0)):
        print("case", cfg, kw, "top_k", top_k, "top_p", top_p, "t", t, flush=True)
        res = d.verify(t=t, top_k=top_k, top_p=top_p)
        torch.cuda.synchronize()
        ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=top_p)
        gu.compare_verify(res, ref, w)


@pytest.mark.parametrize("cfg,kw,top_k,G", [("c3", dict(V=5000), 0, 0), ("c4", dict(V=3000, n_prompts=6), 0, 0),
                                            ("c5", dict(V=20000, draft_top_k=4), 16, 0), ("c5", dict(V=20000), 0, 0),
                                            # few workgroups: long slices (sampling walks chunks of 64 entries and more)
                                            ("c3", dict(V=5000), 0, 1), ("c3", dict(V=5000), 0, 2),
                                            ("c5", dict(V=20000), 0, 3), ("c3", dict(V=5000, draft="indep"), 0, 2)])
@pytest.mark.parametrize("lds_slice", [0, 1000, 2502])
def test_verify_with_slices_in_the_workspace(cfg, kw, top_k, G, lds_slice, knobs):
    """The same results when the joint slices live in the workspace instead of the LDS, wholly or from entry 1000 or
    2502 on (as they do at large I x V per workgroup): each workgroup's region is private, whatever way the layers
    cut I x V."""
    gu = _gu()
    knobs.set("DSBD_VERIFY_LDS_SLICE", lds_slice)
    if G:
        knobs.set("DSBD_VERIFY_G", G)
    w = make_workload(cfg, L=1, Hq=1, Hkv=1, D=64, **kw)
    d = gu.DeviceWorkload(w)
    for t in (-1.0, 0.6):
        res = d.verify(t=t, top_k=top_k, top_p=0.9 if top_k else 1.0)
        torch.cuda.synchronize()
        ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=0.9 if top_k else 1.0)
        gu.compare_verify(res, ref, w)


def test_duplicate_beams_tie_exactly_as_in_a_row_by_row_evaluation():
    """Beam sampling often returns the same beam twice.  Two input beams with equal logits and equal likelihoods
    have equal joint entries; which of two equal entries the top-k / top-p cut keeps is decided by the index on
    both sides, which needs the library to form equal rows' sums in the same order."""
    import dataclasses
    gu = _gu()
    for cfg, kw in (("c3", dict(V=5000, draft_top_k=4)), ("c5", dict(V=9000, draft_top_k=3))):
        w = make_workload(cfg, L=1, Hq=1, Hkv=1, D=64, **kw)
        zp, zq, bp, bq = w.logits_p.copy(), w.logits_q.copy(), w.beam_logp_p.copy(), w.beam_logp_q.copy()
        n = w.max_tree_nodes                              # all trees have the same shape in these configurations
        for src, dst in ((0, 2), (0, 5), (1, 3)):
            zp[dst * n:(dst + 1) * n], zq[dst * n:(dst + 1) * n] = zp[src * n:(src + 1) * n], zq[src * n:(src + 1) * n]
            bp[dst], bq[dst] = bp[src], bq[src]
        w = dataclasses.replace(w, logits_p=zp, logits_q=zq, beam_logp_p=bp, beam_logp_q=bq)
        d = gu.DeviceWorkload(w)
        for top_k, top_p, t in ((16, 0.8, -1.0), (10, 0.8, 0.6), (7, 1.0, -1.0), (0, 1.0, -1.0)):
            print("case", cfg, "top_k", top_k, "top_p", top_p, "t", t, flush=True)
            res = d.verify(t=t, top_k=top_k, top_p=top_p)
            torch.cuda.synchronize()
            ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=top_p)
            gu.compare_verify(res, ref, w)


@pytest.mark.parametrize("cfg,kw,top_k,top_p", [("c3", dict(V=5000), 0, 1.0), ("c5", dict(V=40000), 0, 1.0),
                                                 ("c3", dict(V=5000, draft_top_k=4), 8, 0.9),
                                                 ("c4", dict(V=3000, n_prompts=5), 0, 1.0)])
def test_one_model_in_both_roles(cfg, kw, top_k, top_p):
    """The same arrays given as target and as draft (what the draft stage does): the library keeps and computes
    the joint once; the result must be what the oracle gives for two equal models (every draft accepted: the
    ratio is one; the additional layer's samples come from the joint itself)."""
    import paper_2409_16560_amd as dsbd
    from oracle import verify as o_verify
    gu = _gu()
    w = make_workload(cfg, L=1, Hq=1, Hkv=1, D=64, **kw)
    d = gu.DeviceWorkload(w)
    for t in (-1.0, 0.7):
        res = dsbd.dsbd_verify_forest(d.forest, d.logits_p, d.logits_p, d.blp, d.blp, d.u_accept, d.u_resid, d.u_fill,
                                      W_L=0, W_min=1, W_cap=w.W_cap, t=t, top_k=top_k, top_p=top_p)
        torch.cuda.synchronize()
        ref = o_verify.verify_forest(w.tree_prompt, w.tree_off, w.parent, w.token, w.logits_p, w.logits_p,
                                     w.beam_logp_p, w.beam_logp_p, w.u_accept, w.u_resid, w.u_fill,
                                     0, 1, w.W_cap, np.float32(t), top_k=top_k, top_p=float(np.float32(top_p)))
        gu.compare_verify(res, ref, w)


def test_warping_switched_off_is_the_plain_path():
    gu = _gu()
    w = make_workload("c3", L=1, Hq=1, Hkv=1, D=64, V=5000)
    d = gu.DeviceWorkload(w)
    a = d.verify(t=0.7)
    b = d.verify(t=0.7, top_k=0, top_p=1.0)
    torch.cuda.synchronize()
    for name in ("node_status", "out_parent", "out_token", "out_node", "l_last", "layer_width", "out_logp_target"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name


@pytest.mark.parametrize("name,kw,W_cap,top_k", [
    ("64 beams of 8 nodes: 512 nodes in one prompt", dict(W=64, tree="binary_bfs", tree_nodes=8, V=700), 64, 0),
    ("64 beams, warped", dict(W=64, tree="fork_chain", tree_nodes=7, V=700, draft_top_k=3), 64, 32),
    ("one chain of 64 nodes: 63 draft layers", dict(W=1, tree="chain", tree_nodes=64, V=300, noise_std=0.05), 16, 0),
    ("one 64-node tree, warped", dict(W=2, tree="random", tree_nodes=64, V=300, draft_top_k=2), 16, 4),
])
def test_verify_at_the_size_limits(name, kw, W_cap, top_k):
    gu = _gu()
    w = make_workload("c3", W_cap=W_cap, L=1, Hq=1, Hkv=1, D=64, **kw)
    print(name, "nodes", w.n_nodes, "depth", w.max_depth, flush=True)
    d = gu.DeviceWorkload(w)
    for t in (-1.0, 0.5):
        res = d.verify(t=t, top_k=top_k, top_p=0.9 if top_k else 1.0)
        torch.cuda.synchronize()
        ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=0.9 if top_k else 1.0)
        gu.compare_verify(res, ref, w)
        print("  t", t, "l_last", ref["l_last"].tolist(), "widths", ref["layer_width"][0][:8].tolist(), flush=True)


def test_a_prompt_without_beams_between_two_others():
    """tree_prompt may skip a prompt: it gets no output beams, its neighbours are verified as usual."""
    import dataclasses
    gu = _gu()
    w = make_workload("c4", L=1, Hq=1, Hkv=1, D=64, V=900, n_prompts=2, seed=4)
    tp = w.tree_prompt.copy()
    tp[tp == 1] = 2                                   # prompts 0 and 2 keep their trees, prompt 1 has none
    u_res = np.concatenate([w.u_resid[:1], w.u_resid[:1], w.u_resid[1:]])
    u_fill = np.concatenate([w.u_fill[:1], w.u_fill[:1], w.u_fill[1:]])
    w3 = dataclasses.replace(w, tree_prompt=tp, n_prompts=3, u_resid=u_res, u_fill=u_fill,
                             k_shared=[w.k_shared[0], None, w.k_shared[1]], v_shared=[w.v_shared[0], None, w.v_shared[1]])
    d = gu.DeviceWorkload(w3)
    res = d.verify(t=0.7)
    torch.cuda.synchronize()
    ref2 = gu.oracle_verify(w, t=0.7)                 # the two real prompts, numbered 0 and 1
    g = lambda x: x.cpu().numpy()
    assert int(res.fault.item()) == 0
    assert g(res.n_out).tolist() == [int(ref2["n_out"][0]), 0, int(ref2["n_out"][1])]
    assert np.array_equal(g(res.node_status), ref2["node_status"])
    for name, key in (("out_parent", "out_parent"), ("out_token", "out_token"), ("l_last", "l_last")):
        got = g(getattr(res, name))
        assert np.array_equal(got[0], ref2[key][0]) and np.array_equal(got[2], ref2[key][1]), name
    assert np.all(g(res.out_parent)[1] == -1) and g(res.l_last)[1] == 0


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
    for model, col in (("logits_q", 3), ("logits_p", 499), ("logits_q", 256)):     # NaN, at places the pass reads in different ways
        w3 = make_workload("c2", L=40, V=500, Hq=4, Hkv=4)
        getattr(w3, model)[2, col] = np.nan
        res = gu.DeviceWorkload(w3).verify()
        torch.cuda.synchronize()
        assert int(res.fault.item()) & dsbd.DSBD_FAULT_NONFINITE, (model, col)
    # -Inf is a masked token and no fault by itself, but a drafted token masked in its parent's row (either model)
    # and a row without any finite logit are
    for model, what in (("logits_p", "drafted"), ("logits_q", "drafted"), ("logits_p", "row"), ("logits_q", "row")):
        w4 = make_workload("c2", L=40, V=500, Hq=4, Hkv=4)
        n = int(np.flatnonzero(w4.parent >= 0)[2])
        if what == "drafted":
            getattr(w4, model)[w4.parent[n], w4.token[n]] = -np.inf
        else:
            getattr(w4, model)[n, :] = -np.inf
        res = gu.DeviceWorkload(w4).verify()
        torch.cuda.synchronize()
        assert int(res.fault.item()) == dsbd.DSBD_FAULT_NONFINITE, (model, what)
    # stored likelihoods: no beam of a prompt with a likelihood above 0 under one model, or one that is no number
    for field, value in (("beam_logp_q", -np.inf), ("beam_logp_p", -np.inf), ("beam_logp_p", np.nan)):
        w5 = make_workload("c2", L=40, V=500, Hq=4, Hkv=4)
        if value != value:
            getattr(w5, field)[1] = value
        else:
            getattr(w5, field)[:] = value
        res = gu.DeviceWorkload(w5).verify()
        torch.cuda.synchronize()
        assert int(res.fault.item()) & dsbd.DSBD_FAULT_NONFINITE, (field, value)      # (other bits may follow from it)


@pytest.mark.parametrize("G", [0, 64])
@pytest.mark.parametrize("pattern", ["tail", "random", "both"])
def test_masked_tokens_with_logit_minus_infinity(pattern, G, knobs):
    """Logit processors forbid tokens by setting their logits to -Inf (padding entries of a vocabulary, banned
    tokens).  Such entries have probability 0 and are no fault: the results are the oracle's, whole pieces of a row
    may be masked (a contiguous tail over many workgroups), and the statistics pass treats them alike."""
    gu = _gu()
    if G:
        knobs.set("DSBD_VERIFY_G", G)
    for cfg, kw in (("c5", dict(V=9000)), ("c4", dict(V=3000, n_prompts=4))):
        w = make_workload(cfg, L=1, Hq=1, Hkv=1, D=64, seed=5, draft_top_k=3, **kw)
        rng = np.random.default_rng(1)
        mask = np.zeros(w.V, dtype=bool)
        if pattern in ("tail", "both"):
            mask[int(0.6 * w.V):] = True
        if pattern in ("random", "both"):
            mask |= rng.random(w.V) < 0.3
        mask[w.token[w.token >= 0]] = False              # drafted tokens stay allowed
        mask[:64] = pattern == "both"                     # (and a masked stretch at the start of every row)
        mask[w.token[w.token >= 0]] = False
        w.logits_p[:, mask] = -np.inf
        w.logits_q[:, mask] = -np.inf
        d = gu.DeviceWorkload(w)
        for top_k, top_p, t in ((0, 1.0, -1.0), (0, 1.0, 0.6), (10, 0.8, -1.0), (32, 0.9, 0.6)):
            print(cfg, pattern, "G", G, "top_k", top_k, "t", t, "masked", int(mask.sum()), "of", w.V, flush=True)
            res = d.verify(t=t, top_k=top_k, top_p=top_p)
            torch.cuda.synchronize()
            with np.errstate(all="ignore"):
                ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=top_p)
            gu.compare_verify(res, ref, w)                # (asserts a zero fault word as well)
            gu.check_verify_select(d, w, ref, t=t, top_k=top_k, top_p=top_p)


@pytest.mark.parametrize("field", ["beam_logp_q", "beam_logp_p"])
def test_an_input_beam_of_probability_zero_under_one_model(field):
    """A stored likelihood of -Inf (what comes back for an output beam whose last token the other model masks): the
    beam has the weight 0 in that model's joints; as long as every layer has another beam, the results are the
    oracle's and no fault is raised."""
    gu = _gu()
    for seed in range(3):
        w = make_workload("c3", L=1, Hq=1, Hkv=1, D=64, V=3000, seed=seed)
        getattr(w, field)[1 + seed % 3] = -np.inf
        d = gu.DeviceWorkload(w)
        for top_k, top_p, t in ((0, 1.0, -1.0), (0, 1.0, 0.6), (10, 0.8, -1.0)):
            with np.errstate(all="ignore"):
                ref = gu.oracle_verify(w, t=t, top_k=top_k, top_p=top_p)
            res = d.verify(t=t, top_k=top_k, top_p=top_p)
            torch.cuda.synchronize()
            gu.compare_verify(res, ref, w)
            gu.check_verify_select(d, w, ref, t=t, top_k=top_k, top_p=top_p)


def test_a_missing_partner_ends_in_a_fault_bit_not_in_a_hang(knobs):
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
    knobs.set("DSBD_VERIFY_SYNC_LIMIT_US", "2000")
    knobs.set("DSBD_VERIFY_TEST_MUTE_WG", "5")
    res = d.verify(workspace=ws)
    torch.cuda.synchronize()
    knobs.clear()
    assert int(res.fault.item()) & dsbd.DSBD_FAULT_SYNC_TIMEOUT
    res = d.verify(workspace=ws)
    torch.cuda.synchronize()
    gu.compare_verify(res, gu.oracle_verify(w), w)


def _commit_case(cfg, kw, keep_one, t, head_major=False, in_place=True):
    """Runs verify -> select -> commit on the device and the oracle chain on the CPU; compares the new caches
    bit for bit.  With in_place the first next beam of every source tree continues in its source buffer."""
    gu = _gu()
    import paper_2409_16560_amd as dsbd
    from oracle import commit as o_commit, select as o_select
    w = make_workload(cfg, **kw)
    d = gu.DeviceWorkload(w, share_prefix=True)
    res = d.verify(t=t)
    nx = dsbd.dsbd_select_beams(d.forest, res, keep_one=keep_one)
    torch.cuda.synchronize()
    ref = gu.oracle_verify(w, t=t)
    near = gu.compare_verify(res, ref, w)
    if near:
        pytest.skip("near tie in the verification: plans may differ")
    sref = o_select.select_beams(w.tree_off, w.parent, ref["n_out"], ref["out_parent"], ref["out_token"],
                                 ref["out_logp_p"], ref["out_logp_q"], w.max_depth + 1, keep_one=keep_one)
    rk, rv, rlen = o_commit.commit_kv(w.k_own, w.v_own, w.k_tree, w.v_tree, sref["n_next"], sref["src_tree"],
                                      sref["path_len"], sref["path"])
    # source caches with room to grow (so that a beam can continue in place), destination buffers for the rest
    grow = w.max_depth + 1
    cap = max(k.shape[0] for k in w.k_own) + grow
    def buf():
        t_ = torch.full((cap, w.Hkv, w.D), -1.0, dtype=torch.bfloat16, device="cuda")
        return t_.permute(1, 0, 2).contiguous().permute(1, 0, 2) if head_major else t_
    src_k, src_v = [], []
    for b in range(w.n_trees):
        kb, vb = buf(), buf()
        kb[:w.k_own[b].shape[0]] = gu.bf16_dev(w.k_own[b]); vb[:w.v_own[b].shape[0]] = gu.bf16_dev(w.v_own[b])
        src_k.append(kb); src_v.append(vb)
    L = [k.shape[0] for k in w.k_own]
    view = lambda t_, n: (t_.permute(1, 0, 2)[:, :n] if head_major else t_[:n])
    kv = dsbd.PrefixKV([view(src_k[b], L[b]) for b in range(w.n_trees)], [view(src_v[b], L[b]) for b in range(w.n_trees)],
                       head_major=head_major)
    dst_k, dst_v, taken = [], [], set()
    for p in range(w.n_prompts):
        for s_ in range(w.W_cap):
            b = int(sref["src_tree"][p, s_]) if s_ < int(sref["n_next"][p]) else -1
            if b >= 0 and in_place and b not in taken:
                taken.add(b); dst_k.append(src_k[b]); dst_v.append(src_v[b])
            else:
                dst_k.append(buf()); dst_v.append(buf())
    to_view = (lambda t_: t_.permute(1, 0, 2)) if head_major else (lambda t_: t_)
    dst = dsbd.KVDst([to_view(t_) for t_ in dst_k], [to_view(t_) for t_ in dst_v], kv, head_major=head_major)
    dlen, fault = dsbd.dsbd_commit_kv(d.forest, kv, d.k_tree, d.v_tree, nx, w.W_cap, dst)
    torch.cuda.synchronize()
    assert int(fault.item()) == 0
    assert np.array_equal(dlen.cpu().numpy(), rlen)
    bits = lambda t_: t_.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    n_checked = 0
    for (p, s_), want in rk.items():
        j = p * w.W_cap + s_
        n = want.shape[0]
        assert np.array_equal(bits(dst_k[j][:n]), want), ("K", p, s_)
        assert np.array_equal(bits(dst_v[j][:n]), rv[(p, s_)]), ("V", p, s_)
        assert bool((dst_k[j][n:] == -1.0).all()) and bool((dst_v[j][n:] == -1.0).all())   # nothing beyond the new length
        n_checked += 1
    assert n_checked == int(sref["n_next"].sum())
    return n_checked


@pytest.mark.parametrize("cfg,kw", [
    ("c1", {}),
    ("c2", dict(L=100, V=500, Hq=8, Hkv=4)),
    ("c3", dict(L=300, V=700, Hq=8, Hkv=2, D=64)),              # shared leading segment stays shared
    ("c4", dict(L=(40, 200), V=300, n_prompts=5, Hq=4, Hkv=4)), # ragged lengths, several prompts
    ("c5", dict(L=333, V=2000)),                                 # GQA 32/8, 31-node trees
])
@pytest.mark.parametrize("keep_one", [False, True])
def test_commit_kv_matches_oracle(cfg, kw, keep_one):
    _commit_case(cfg, kw, keep_one, t=-1.0)


def test_commit_kv_head_major_and_copy_only():
    _commit_case("c2", dict(L=100, V=500, Hq=8, Hkv=4), False, t=0.7, head_major=True)
    _commit_case("c5", dict(L=130, V=2000), False, t=-1.0, in_place=False)


def test_commit_kv_reports_what_does_not_fit():
    gu = _gu()
    import paper_2409_16560_amd as dsbd
    w = make_workload("c2", L=50, V=500, Hq=4, Hkv=4)
    d = gu.DeviceWorkload(w)
    res = d.verify()
    nx = dsbd.dsbd_select_beams(d.forest, res)
    small = [torch.full((52, w.Hkv, w.D), -1.0, dtype=torch.bfloat16, device="cuda") for _ in range(2 * w.n_prompts * w.W_cap)]
    n = w.n_prompts * w.W_cap
    dst = dsbd.KVDst(small[:n], small[n:], d.kv)              # capacity 52 < 50 + path length for deeper beams
    dlen, fault = dsbd.dsbd_commit_kv(d.forest, d.kv, d.k_tree, d.v_tree, nx, w.W_cap, dst)
    torch.cuda.synchronize()
    pl = nx.path_len.cpu().numpy(); nn = nx.n_next.cpu().numpy()
    too_long = [(p, s_) for p in range(w.n_prompts) for s_ in range(int(nn[p])) if 50 + pl[p, s_] > 52]
    assert (int(fault.item()) & dsbd.DSBD_FAULT_BOUNDS != 0) == bool(too_long)
    for p, s_ in too_long:
        assert int(dlen[p, s_]) == 0 and bool((small[p * w.W_cap + s_] == -1.0).all())


@pytest.mark.parametrize("broken", ["null V", "misaligned V", "null K", "source longer than max_len"])
def test_commit_kv_rejects_a_destination_with_one_unusable_plane(broken):
    """A destination whose K buffer is fine and whose V buffer is missing or misaligned (or the other way round) is
    left untouched as a whole: both planes' workgroups take the same decision, the length reads 0 and the bounds
    fault is raised.  The other destinations are copied as usual."""
    gu = _gu()
    import paper_2409_16560_amd as dsbd
    from oracle import commit as o_commit, select as o_select
    w = make_workload("c2", L=50, V=500, Hq=4, Hkv=4)
    d = gu.DeviceWorkload(w)
    res = d.verify()
    nx = dsbd.dsbd_select_beams(d.forest, res)
    torch.cuda.synchronize()
    ref = gu.oracle_verify(w)
    if gu.compare_verify(res, ref, w):
        pytest.skip("near tie in the verification")
    sref = o_select.select_beams(w.tree_off, w.parent, ref["n_out"], ref["out_parent"], ref["out_token"],
                                 ref["out_logp_p"], ref["out_logp_q"], w.max_depth + 1)
    rk, rv, rlen = o_commit.commit_kv(w.k_own, w.v_own, w.k_tree, w.v_tree, sref["n_next"], sref["src_tree"],
                                      sref["path_len"], sref["path"])
    n = w.n_prompts * w.W_cap
    cap = 50 + w.max_depth + 1
    mk = lambda: torch.full((cap + 1, w.Hkv, w.D), -1.0, dtype=torch.bfloat16, device="cuda")
    dst_k, dst_v = [mk() for _ in range(n)], [mk() for _ in range(n)]
    used = int(sref["n_next"][0])
    assert used >= 2
    victim = 1
    dst = dsbd.KVDst([t[:cap] for t in dst_k], [t[:cap] for t in dst_v], d.kv)
    kv = d.kv
    if broken == "null V":
        dst.v_ptr[victim] = 0
    elif broken == "misaligned V":
        dst.v_ptr[victim] += 8
    elif broken == "null K":
        dst.k_ptr[victim] = 0
    else:
        # the lengths array claims more tokens than the max_len the grid was sized for
        victim = None
        kv = dsbd.PrefixKV(d.kv.keep[0], d.kv.keep[1])
        kv.len[int(sref["src_tree"][0, 1])] += 7
    dlen, fault = dsbd.dsbd_commit_kv(d.forest, kv, d.k_tree, d.v_tree, nx, w.W_cap, dst)
    torch.cuda.synchronize()
    assert int(fault.item()) & dsbd.DSBD_FAULT_BOUNDS
    bits = lambda t_: t_.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    hit = 0
    for (p, s_), want in rk.items():
        j = p * w.W_cap + s_
        affected = (j == victim) if victim is not None else int(sref["src_tree"][p, s_]) == int(sref["src_tree"][0, 1])
        if affected:
            hit += 1
            assert int(dlen[p, s_]) == 0
            assert bool((dst_k[j] == -1.0).all()) and bool((dst_v[j] == -1.0).all())     # neither plane was written
        else:
            assert int(dlen[p, s_]) == rlen[p, s_]
            assert np.array_equal(bits(dst_k[j][:want.shape[0]]), want) and np.array_equal(bits(dst_v[j][:want.shape[0]]), rv[(p, s_)])
    assert hit >= 1


def test_select_beams_with_more_trees_than_the_lds_staging_holds():
    """Selection stages tree_off in the LDS for its binary searches; a forest of more than 8192 trees is searched where
    it lies instead.  9000 single-node trees in 9000 prompts (no draft layers: every prompt draws from its root)."""
    import paper_2409_16560_amd as dsbd
    from oracle import select as o_select
    T = 9000
    rng = np.random.default_rng(5)
    tree_off = np.arange(T + 1, dtype=np.int32)
    parent = np.full(T, -1, dtype=np.int32)
    forest = dsbd.Forest(np.arange(T, dtype=np.int32), tree_off, parent, np.zeros(T, dtype=np.int32), None, n_prompts=T,
                         max_tree_nodes=1, max_depth=0, max_prompt_trees=1, device="cuda")
    W_cap = 2
    res = dsbd.VerifyResult.allocate(forest, W_cap)
    n_out = rng.integers(0, 3, T).astype(np.int32)
    out_parent = np.where(np.arange(W_cap)[None, :] < n_out[:, None], np.arange(T, dtype=np.int32)[:, None], -1).astype(np.int32)
    out_token = rng.integers(0, 100, (T, W_cap)).astype(np.int32)
    lp = rng.normal(0, 1, (T, W_cap)); lq = rng.normal(0, 1, (T, W_cap))
    res.n_out.copy_(torch.from_numpy(n_out)); res.out_parent.copy_(torch.from_numpy(out_parent))
    res.out_token.copy_(torch.from_numpy(out_token))
    res.out_logp_target.copy_(torch.from_numpy(lp)); res.out_logp_draft.copy_(torch.from_numpy(lq))
    for keep_one in (False, True):
        nx = dsbd.dsbd_select_beams(forest, res, keep_one=keep_one)
        torch.cuda.synchronize()
        sref = o_select.select_beams(tree_off, parent, n_out, out_parent, out_token, lp, lq, 1, keep_one=keep_one)
        _gu().compare_select(nx, sref)


@pytest.mark.parametrize("n_prompts,t", [(300, -1.0), (300, 0.7), (700, -1.0)])
def test_verify_more_prompts_than_workgroups_fit_the_device(n_prompts, t):
    """Algorithm 1 runs per prompt.  A forest with more prompts than the layer kernel can keep resident at once (one
    workgroup per prompt and compute unit) is verified in groups of prompts, one launch after the other, on the same
    workspace."""
    gu = _gu()
    w = make_workload("c4", n_prompts=n_prompts, W=(1, 2), tree_nodes=(2, 6), L=1, Hq=1, Hkv=1, D=64, V=300, seed=11)
    d = gu.DeviceWorkload(w)
    res = d.verify(t=t)
    torch.cuda.synchronize()
    ref = gu.oracle_verify(w, t=t)
    near = gu.compare_verify(res, ref, w)
    print("prompts", n_prompts, "trees", w.n_trees, "nodes", w.n_nodes, "near ties", near, flush=True)
    gu.check_verify_select(d, w, ref, t=t)
