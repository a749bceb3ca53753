"""Pins of the cache-commit oracle (Section 3.3 last paragraph, Section 3.4).

The cache of a beam is, by definition, one key/value row per token of the beam's sequence, in sequence order.
Rows here carry an identity code of the token occurrence they belong to, so the committed caches can be checked
against sequences rebuilt by walking parent pointers directly, independent of the plan the oracle consumed."""
import numpy as np
import pytest

from dsbd_synth import make_workload
from oracle import commit as o_commit
from oracle import select as o_select
from oracle import verify as o_verify


def coded_rows(w):
    """K/V rows whose first two entries identify the token occurrence: (0, tree, position) for prefix tokens,
    (1, node) for forest nodes; V carries the same code plus a marker."""
    Hkv, D = 2, 4
    k_own, v_own = [], []
    for b in range(w.n_trees):
        L = 3 + b            # different lengths per beam
        k = np.zeros((L, Hkv, D), dtype=np.int64)
        k[:, :, 0] = 0; k[:, :, 1] = b; k[:, :, 2] = np.arange(L)[:, None]; k[:, :, 3] = np.arange(Hkv)[None, :]
        k_own.append(k); v_own.append(k + 1000)
    kt = np.zeros((w.n_nodes, Hkv, D), dtype=np.int64)
    kt[:, :, 0] = 1; kt[:, :, 1] = np.arange(w.n_nodes)[:, None]; kt[:, :, 3] = np.arange(Hkv)[None, :]
    return k_own, v_own, kt, kt + 1000


def run(cfg, keep_one, t=-1.0, **kw):
    w = make_workload(cfg, L=1, Hq=1, Hkv=1, D=64, **kw)
    v = o_verify.verify_forest(w.tree_prompt, w.tree_off, w.parent, w.token, w.logits_p, w.logits_q, w.beam_logp_p,
                               w.beam_logp_q, w.u_accept, w.u_resid, w.u_fill, 0, 1, w.W_cap, np.float32(t))
    s = o_select.select_beams(w.tree_off, w.parent, v["n_out"], v["out_parent"], v["out_token"], v["out_logp_p"],
                              v["out_logp_q"], w.max_depth + 1, keep_one=keep_one)
    return w, v, s


@pytest.mark.parametrize("cfg,kw", [("c1", {}), ("c2", dict(V=500)), ("c3", dict(V=700)), ("c4", dict(V=300, n_prompts=5)),
                                    ("c5", dict(V=900))])
@pytest.mark.parametrize("keep_one", [False, True])
def test_committed_cache_is_the_row_sequence_of_the_new_beam(cfg, kw, keep_one):
    w, v, s = run(cfg, keep_one, **kw)
    k_own, v_own, kt, vt = coded_rows(w)
    dk, dv, dlen = o_commit.commit_kv(k_own, v_own, kt, vt, s["n_next"], s["src_tree"], s["path_len"], s["path"])
    tree_of = np.searchsorted(w.tree_off, np.arange(w.n_nodes), side="right") - 1
    for p in range(w.n_prompts):
        outs = list(range(int(v["n_out"][p])))
        if keep_one and outs:
            outs = [max(outs, key=lambda j: (v["out_logp_p"][p, j], -j))]
        assert int(s["n_next"][p]) == len(outs)
        for slot, j in enumerate(outs):
            # the new beam's sequence, rebuilt by walking parent pointers from the node the output beam hangs from
            chain, n = [], int(v["out_parent"][p, j])
            while n >= 0:
                chain.append(n); n = int(w.parent[n])
            chain.reverse()
            b = int(tree_of[chain[0]])
            assert chain[0] == w.tree_off[b]                      # starts at the root of the source tree
            L = k_own[b].shape[0]
            got = dk[(p, slot)]
            assert got.shape[0] == L + len(chain) == int(dlen[p, slot])
            assert np.array_equal(got[:L], k_own[b])                               # the beam's prefix, in order
            assert [int(r[0, 1]) for r in got[L:]] == chain and np.all(got[L:, :, 0] == 1)   # then its tree rows
            assert np.array_equal(dv[(p, slot)], got + 1000)                       # V follows K row for row
    assert np.all(dlen[np.arange(w.W_cap)[None, :] >= s["n_next"][:, None]] == 0)


def test_single_chain_is_the_speculative_decoding_cache_update():
    """W = 1 and a chain-shaped tree is vanilla speculative decoding (Section 2.2): the new cache is the old one
    plus the rows of the root and of the accepted draft tokens, nothing else."""
    w, v, s = run("c1", False, W=1)
    k_own, v_own, kt, vt = coded_rows(w)
    dk, _, dlen = o_commit.commit_kv(k_own, v_own, kt, vt, s["n_next"], s["src_tree"], s["path_len"], s["path"])
    acc = [n for n in range(w.n_nodes) if v["node_status"][n] == o_verify.ACCEPTED]
    l_last = int(v["l_last"][0])
    # the output beam hangs from the node at depth l_last - 1: root + (l_last - 1) accepted drafts
    assert int(dlen[0, 0]) == k_own[0].shape[0] + l_last
    rows = [int(r[0, 1]) for r in dk[(0, 0)][k_own[0].shape[0]:]]
    assert rows[0] == 0 and rows[1:] == [n for n in acc if n < l_last][:l_last - 1]


def test_sources_are_left_untouched_and_one_cache_survives_in_the_reduced_variant():
    w, v, s = run("c3", True, V=700)
    k_own, v_own, kt, vt = coded_rows(w)
    before = [k.copy() for k in k_own]
    dk, dv, dlen = o_commit.commit_kv(k_own, v_own, kt, vt, s["n_next"], s["src_tree"], s["path_len"], s["path"])
    assert all(np.array_equal(a, b) for a, b in zip(before, k_own))
    assert len(dk) == int(s["n_next"].sum()) == w.n_prompts            # Section 3.4: one beam, one cache per prompt
