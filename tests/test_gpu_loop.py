"""The multi-iteration loop over the library's calls against the oracle's loop: the same synthetic model pair and
the same uniforms on both sides; every iteration's forest, verification, plan, attention and caches compared."""
import numpy as np
import pytest
import torch

from dsbd_synth import SyntheticModels, bf16_bits_to_f32, uniform01_f32

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,start,V,W_S,gamma,kw", [
    ("fixed width", [[(5,), (9,)]], 300, 4, 3, dict(W_L=2, t=-1.0)),
    ("two prompts, dynamic width", [[(5,), (9,), (11,)], [(2,)]], 2000, 6, 3, dict(W_L=0, t=0.6, W_min=1)),
    ("warped joints", [[(1, 2, 3), (1, 2, 4), (1, 5, 6)]], 5000, 8, 2, dict(W_L=3, t=-1.0, top_k=10, top_p=0.8)),
    ("one cache kept", [[(7,), (8,)]], 300, 4, 3, dict(W_L=2, t=-1.0, keep_one=True)),
    ("no draft layers", [[(3,), (4,)]], 300, 4, 0, dict(W_L=2, t=-1.0)),
    ("more beams than draws per step", [[(269, 239, 253)]], 300, 1, 1, dict(W_L=3, t=-1.0, W_min=2, top_k=10, top_p=0.5)),
    ("five beams, three draws", [[(4557, 8707)], [(6912, 130)]], 9000, 3, 3, dict(W_L=5, t=-1.0, W_min=2)),
])
def test_loop_matches_the_oracle_loop(name, start, V, W_S, gamma, kw):
    import gpu_util as gu
    from paper_2409_16560_amd.loop import DecodeLoop
    from oracle.loop import OracleLoop
    m = SyntheticModels(V=V, seed=13, Hq=4, Hkv=2, D=64)
    seed, W_cap = 31, 8
    lib = DecodeLoop(m, start, W_S, gamma, lambda n, stream: uniform01_f32(n, seed, stream), W_cap=W_cap, kv_capacity=64, **kw)
    ora = OracleLoop(m, start, W_S, gamma, W_cap=W_cap, seed=seed, **kw)
    g = lambda x: x.cpu().numpy()
    for it in range(5):
        print(name, "iteration", it, "beams", [len(pb) for pb in ora.beams], flush=True)
        a, b = lib.step(), ora.step()
        torch.cuda.synchronize()
        f = b["forest"]
        for field in ("tree_prompt", "tree_off", "parent", "token", "draft_rank"):
            assert np.array_equal(g(getattr(a["forest"], field)), f[field]), field
        assert a["node_seq"] == b["node_seq"]

        class W:
            tree_prompt, tree_off, n_nodes = f["tree_prompt"], f["tree_off"], len(f["parent"])
        near = gu.compare_verify(a["verify"], b["verify"], W)
        assert near == 0, "a near tie: the two loops may part ways (change the seed)"
        for field in ("n_next", "src_tree", "src_out", "path_len", "path", "token"):
            assert np.array_equal(g(getattr(a["next"], field)), b["next"][field]), field
        assert np.max(np.abs(g(a["next"].logp_target) - b["next"]["logp_p"])) <= 1e-9
        assert int(a["attn_fault"].item()) == 0
        err = np.max(np.abs(a["attn_out"].float().cpu().numpy() - b["attn_out"]))
        assert err <= gu.ATOL, err
        assert np.max(np.abs(g(a["attn_lse"]) - b["attn_lse"])) <= gu.ATOL
        # state after the iteration
        assert lib.beams == ora.beams
        assert np.max(np.abs(g(lib.cum_p) - np.concatenate([np.asarray(c) for c in ora.cum_p]))) <= 1e-9
        assert len(lib.k_buf) == len(ora.k_cache)
        bits = lambda t_: t_.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        for j in range(len(ora.k_cache)):
            n = ora.k_cache[j].shape[0]
            assert lib.kv_len[j] == n
            assert np.array_equal(bits(lib.k_buf[j][:n]), ora.k_cache[j]) and np.array_equal(bits(lib.v_buf[j][:n]), ora.v_cache[j])

@pytest.mark.parametrize("sweep", [0, 1])
def test_loop_random_parameters(sweep):
    """Randomized sweep of the whole loop: prompts and input beams, draws per step above and below the number of
    beams, draft depth 0..3, fixed and dynamic width, warping, one-cache mode, head groupings, banned tokens."""
    import gpu_util as gu
    from paper_2409_16560_amd.loop import DecodeLoop
    from oracle.loop import OracleLoop
    rng = np.random.default_rng(3000 + sweep)
    rng_banned = np.random.default_rng(5000 + sweep)
    g = lambda x: x.cpu().numpy()
    bits = lambda t_: t_.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    for case in range(12):
        V = int(rng.choice([50, 300, 2000, 9000]))
        plen = int(rng.integers(1, 4))
        start = [[tuple(int(x) for x in rng.integers(0, V, plen)) for _ in range(int(rng.integers(1, 4)))]
                 for _ in range(int(rng.integers(1, 4)))]
        W_S, gamma = int(rng.integers(1, 9)), int(rng.integers(0, 4))
        kw = dict(W_L=int(rng.choice([0, 1, 2, 3, 5])), t=float(rng.choice([-1.0, -1.0, 0.4, 0.8])), W_min=int(rng.choice([1, 2])))
        if rng.random() < 0.4:
            kw.update(top_k=int(rng.choice([1, 4, 10, 32])), top_p=float(rng.choice([1.0, 0.8, 0.5])))
        if rng.random() < 0.25:
            kw.update(keep_one=True)
        Hq, Hkv = [(4, 2), (2, 2), (8, 1)][int(rng.integers(0, 3))]
        mseed, seed = int(rng.integers(0, 1000)), int(rng.integers(0, 1000))
        what = "sweep %d case %d: V=%d start=%s W_S=%d gamma=%d %s heads %d/%d seeds %d %d" % (
            sweep, case, V, start, W_S, gamma, kw, Hq, Hkv, mseed, seed)
        print(what, flush=True)
        banned = float(rng_banned.choice([0.0, 0.0, 0.3, 0.9]))     # share of the vocabulary at -Inf, per sequence
        what += " banned %g" % banned
        m = SyntheticModels(V=V, seed=mseed, Hq=Hq, Hkv=Hkv, D=64, banned=banned)
        lib = DecodeLoop(m, start, W_S, gamma, lambda n, stream: uniform01_f32(n, seed, stream), W_cap=8, kv_capacity=64, **kw)
        ora = OracleLoop(m, start, W_S, gamma, W_cap=8, seed=seed, **kw)
        for it in range(3):
            a, b = lib.step(), ora.step()
            torch.cuda.synchronize()
            f = b["forest"]
            for field in ("tree_prompt", "tree_off", "parent", "token", "draft_rank"):
                assert np.array_equal(g(getattr(a["forest"], field)), f[field]), (what, it, field)
            assert a["node_seq"] == b["node_seq"], (what, it)

            class W:
                tree_prompt, tree_off, n_nodes = f["tree_prompt"], f["tree_off"], len(f["parent"])
            if gu.compare_verify(a["verify"], b["verify"], W):
                break                                    # a near tie: the two loops may part ways from here on
            for field in ("n_next", "src_tree", "src_out", "path_len", "path", "token"):
                assert np.array_equal(g(getattr(a["next"], field)), b["next"][field]), (what, it, field)
            assert int(a["attn_fault"].item()) == 0
            assert np.max(np.abs(a["attn_out"].float().cpu().numpy() - b["attn_out"])) <= gu.ATOL, (what, it)
            assert lib.beams == ora.beams, (what, it)
            assert len(lib.k_buf) == len(ora.k_cache)
            for j in range(len(ora.k_cache)):
                n = ora.k_cache[j].shape[0]
                assert lib.kv_len[j] == n, (what, it, j)
                assert np.array_equal(bits(lib.k_buf[j][:n]), ora.k_cache[j]), (what, it, j)
                assert np.array_equal(bits(lib.v_buf[j][:n]), ora.v_cache[j]), (what, it, j)
