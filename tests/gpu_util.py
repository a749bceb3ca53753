"""Shared helpers of the GPU parity tests: upload a synthetic workload, run the HIP path through the
binding, run the CPU oracle on the same inputs, compare."""
import numpy as np
import torch

import paper_2409_16560_amd as dsbd
from dsbd_synth import bf16_bits_to_f32
from oracle import attention as o_attn
from oracle import forest as o_forest
from oracle import select as o_select
from oracle import verify as o_verify

ATOL = 2e-2     # absolute tolerance on attention outputs and log-probabilities (bf16 inputs, fp32 accumulate)


def bf16_dev(bits, dev="cuda"):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)


def f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


class DeviceWorkload:
    """Device copies of a dsbd_synth Workload."""

    def __init__(self, w, share_prefix=True, rank=None, dev="cuda"):
        self.w = w
        self.forest = dsbd.Forest(w.tree_prompt, w.tree_off, w.parent, w.token, rank, n_prompts=w.n_prompts,
                                  max_tree_nodes=w.max_tree_nodes, max_depth=w.max_depth,
                                  max_prompt_trees=w.max_prompt_trees, device=dev)
        has_shared = any(k is not None for k in w.k_shared)
        ks = [None if k is None else bf16_dev(k, dev) for k in w.k_shared]
        vs = [None if v is None else bf16_dev(v, dev) for v in w.v_shared]
        if has_shared and share_prefix:
            k_own = [bf16_dev(k, dev) for k in w.k_own]
            v_own = [bf16_dev(v, dev) for v in w.v_own]
            self.kv = dsbd.PrefixKV(k_own, v_own, [ks[int(p)] for p in w.tree_prompt], [vs[int(p)] for p in w.tree_prompt])
        else:
            k_all, v_all = [], []
            for t in range(w.n_trees):
                p = int(w.tree_prompt[t])
                if w.k_shared[p] is not None:
                    k_all.append(bf16_dev(np.concatenate([w.k_shared[p], w.k_own[t]], 0), dev))
                    v_all.append(bf16_dev(np.concatenate([w.v_shared[p], w.v_own[t]], 0), dev))
                else:
                    k_all.append(bf16_dev(w.k_own[t], dev))
                    v_all.append(bf16_dev(w.v_own[t], dev))
            self.kv = dsbd.PrefixKV(k_all, v_all)
        self.q, self.k_tree, self.v_tree = bf16_dev(w.q, dev), bf16_dev(w.k_tree, dev), bf16_dev(w.v_tree, dev)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.logits_p, self.logits_q = t(w.logits_p), t(w.logits_q)
        self.blp, self.blq = t(w.beam_logp_p), t(w.beam_logp_q)
        self.u_accept, self.u_resid, self.u_fill = t(w.u_accept), t(w.u_resid), t(w.u_fill)

    def attention(self, **kw):
        return dsbd.dsbd_forest_attention(self.forest, self.kv, self.q, self.k_tree, self.v_tree, **kw)

    def verify(self, W_L=0, W_min=1, t=-1.0, **kw):
        return dsbd.dsbd_verify_forest(self.forest, self.logits_p, self.logits_q, self.blp, self.blq, self.u_accept,
                                       self.u_resid, self.u_fill, W_L=W_L, W_min=W_min, W_cap=self.w.W_cap, t=t, **kw)


def logical_prefix(w, t):
    p = int(w.tree_prompt[t])
    ks, vs = [], []
    if w.k_shared[p] is not None:
        ks.append(f64(w.k_shared[p])); vs.append(f64(w.v_shared[p]))
    ks.append(f64(w.k_own[t])); vs.append(f64(w.v_own[t]))
    return np.concatenate(ks, 0), np.concatenate(vs, 0)


def oracle_attention(w):
    pk, pv = zip(*[logical_prefix(w, t) for t in range(w.n_trees)])
    return o_attn.forest_attention(w.parent, w.tree_off, f64(w.q), f64(w.k_tree), f64(w.v_tree), list(pk), list(pv))


def oracle_verify(w, W_L=0, W_min=1, t=-1.0, rank=None, top_k=0, top_p=1.0):
    # top_p reaches the library as a 32-bit float: the oracle takes the same value
    return o_verify.verify_forest(w.tree_prompt, w.tree_off, w.parent, w.token, w.logits_p, w.logits_q,
                                  w.beam_logp_p, w.beam_logp_q, w.u_accept, w.u_resid, w.u_fill,
                                  W_L, W_min, w.W_cap, np.float32(t), rank=rank, top_k=top_k,
                                  top_p=float(np.float32(top_p)))


def compare_attention(w, out, lse, ref_out, ref_lse, rows=None):
    o = out.float().cpu().numpy().astype(np.float64)
    l = lse.cpu().numpy().astype(np.float64)
    if rows is None:
        err_o = np.max(np.abs(o - ref_out))
        err_l = np.max(np.abs(l - ref_lse))
    else:
        err_o = max(np.max(np.abs(o[n, h] - ref_out[i])) for i, (n, h) in enumerate(rows))
        err_l = max(abs(l[n, h] - ref_lse[i]) for i, (n, h) in enumerate(rows))
    assert np.isfinite(o).all() and np.isfinite(l).all()
    assert err_o <= ATOL, "attention output error %g" % err_o
    assert err_l <= ATOL, "attention lse error %g" % err_l
    return err_o, err_l


def compare_verify(res, ref, w):
    """Bit-exact decisions, tolerance on log-probabilities.  Returns the number of near ties reported."""
    g = lambda t: t.cpu().numpy()
    assert int(g(res.fault)[0]) == ref["fault"] == 0
    near = g(res.near_tie_count)
    assert np.array_equal(near, ref["near_tie"])
    # a prompt with a near tie may legitimately differ; everything else must match exactly
    clean = near == 0
    prompt_of_node = np.asarray(w.tree_prompt)[o_forest.tree_of_node(w.tree_off, w.n_nodes)]
    node_ok = clean[prompt_of_node]
    assert np.array_equal(g(res.node_status)[node_ok], ref["node_status"][node_ok])
    for name, key in (("l_last", "l_last"), ("layer_width", "layer_width"), ("n_out", "n_out"),
                      ("out_parent", "out_parent"), ("out_token", "out_token"), ("out_node", "out_node")):
        got, want = g(getattr(res, name))[clean], ref[key][clean]
        if not np.array_equal(got, want):
            bad = np.argwhere(got != want)
            raise AssertionError("%s differs at (clean prompt, ...) %s: got %s, expected %s"
                                 % (name, bad[:8].tolist(), got[got != want][:8].tolist(), want[got != want][:8].tolist()))
    for name, key in (("lse_target", "lse_p"), ("lse_draft", "lse_q"), ("node_logp_target", "node_logp_p"),
                      ("node_logp_draft", "node_logp_q")):
        err = np.max(np.abs(g(getattr(res, name)).astype(np.float64) - ref[key]))
        assert err <= ATOL, (name, err)
    for name, key in (("out_logp_target", "out_logp_p"), ("out_logp_draft", "out_logp_q")):
        err = np.max(np.abs(g(getattr(res, name))[clean] - ref[key][clean]))
        assert err <= 1e-9, (name, err)
    return int(near.sum())


def compare_select(nx, ref):
    g = lambda t: t.cpu().numpy()
    assert int(g(nx.fault)[0]) == 0
    for name, key in (("n_next", "n_next"), ("src_tree", "src_tree"), ("src_out", "src_out"), ("path_len", "path_len"),
                      ("path", "path"), ("token", "token")):
        assert np.array_equal(g(getattr(nx, name)), ref[key]), name
    assert np.array_equal(g(nx.logp_target), ref["logp_p"]) and np.array_equal(g(nx.logp_draft), ref["logp_q"])
