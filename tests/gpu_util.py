"""Shared helpers of the GPU parity tests: run the CPU oracle on the inputs of a synthetic workload and compare its
results with what the HIP path returned (the uploader itself is dsbd_synth.device: it knows nothing of the oracle)."""
import numpy as np
import torch

import paper_2409_16560_amd as dsbd
from dsbd_synth import bf16_bits_to_f32
from dsbd_synth.device import DeviceWorkload, bf16_dev          # noqa: F401  (the uploader lives beside the generators)
from oracle import attention as o_attn
from oracle import forest as o_forest
from oracle import select as o_select
from oracle import verify as o_verify

ATOL = 2e-2     # absolute tolerance on attention outputs and log-probabilities (bf16 inputs, fp32 accumulate)


def f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


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


def max_abs_err(got, want):
    """Largest |got - want|, where entries that are the same infinity on both sides (the log-probability of a
    masked token) count as equal."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    same_inf = np.isinf(got) & (got == want)
    with np.errstate(invalid="ignore"):
        err = np.where(same_inf, 0.0, np.abs(got - want))
    return float(np.max(np.where(np.isnan(err), np.inf, err), initial=0.0))


def compare_verify(res, ref, w):
    """Bit-exact decisions, tolerance on log-probabilities.  Returns the number of near ties reported."""
    g = lambda t: t.cpu().numpy()
    assert int(g(res.fault)[0]) == ref["fault"] == 0, ("fault", int(g(res.fault)[0]), ref["fault"])
    near = g(res.near_tie_count)
    assert np.array_equal(near, ref["near_tie"]), ("near_tie_count", near.tolist(), ref["near_tie"].tolist())
    # a prompt with a near tie may legitimately differ; everything else must match exactly
    clean = near == 0
    prompt_of_node = np.asarray(w.tree_prompt)[o_forest.tree_of_node(w.tree_off, w.n_nodes)]
    node_ok = clean[prompt_of_node]
    assert np.array_equal(g(res.node_status)[node_ok], ref["node_status"][node_ok]), "node_status"
    for name, key in (("l_last", "l_last"), ("layer_width", "layer_width"), ("n_out", "n_out"),
                      ("out_parent", "out_parent"), ("out_token", "out_token"), ("out_node", "out_node")):
        got, want = g(getattr(res, name))[clean], ref[key][clean]
        if not np.array_equal(got, want):
            bad = np.argwhere(got != want)
            raise AssertionError("%s differs at (clean prompt, ...) %s: got %s, expected %s"
                                 % (name, bad[:8].tolist(), got[got != want][:8].tolist(), want[got != want][:8].tolist()))
    for name, key in (("lse_target", "lse_p"), ("lse_draft", "lse_q"), ("node_logp_target", "node_logp_p"),
                      ("node_logp_draft", "node_logp_q")):
        err = max_abs_err(g(getattr(res, name)), ref[key])
        assert err <= ATOL, (name, err)
    for name, key in (("out_logp_target", "out_logp_p"), ("out_logp_draft", "out_logp_q")):
        err = max_abs_err(g(getattr(res, name))[clean], ref[key][clean])
        assert err <= 1e-9, (name, err)
    return int(near.sum())


def compare_select(nx, ref):
    g = lambda t: t.cpu().numpy()
    assert int(g(nx.fault)[0]) == 0
    for name, key in (("n_next", "n_next"), ("src_tree", "src_tree"), ("src_out", "src_out"), ("path_len", "path_len"),
                      ("path", "path"), ("token", "token")):
        assert np.array_equal(g(getattr(nx, name)), ref[key]), name
    assert np.array_equal(g(nx.logp_target), ref["logp_p"]) and np.array_equal(g(nx.logp_draft), ref["logp_q"])


def check_verify_select(d, w, ref, **verify_args):
    """The one-call form (dsbd_verify_forest_select) against the oracle: the verification outputs as compare_verify
    holds them, and the next-beam plan against the oracle's selection from the oracle's own verification, for both
    values of keep_one.  The plan is compared for prompts without a near tie (a near tie may change the output beams)."""
    g = lambda x: x.cpu().numpy()
    for keep_one in (False, True):
        res, nx = d.verify_select(keep_one=keep_one, **verify_args)
        torch.cuda.synchronize()
        compare_verify(res, ref, w)
        logp_p = ref["out_logp_p"]
        if keep_one:
            # Likelihoods of different output beams that are equal in exact arithmetic (equal steps in another order,
            # beams with equal rows) differ in the last bit, and not in the same way on both sides.  Where the
            # library's choice is within the comparison's tolerance of the oracle's best, the choice is valid and the
            # plan is compared with the oracle's selection of that beam.
            logp_p = logp_p.copy()
            for p in range(len(ref["n_out"])):
                n, j = int(ref["n_out"][p]), int(g(nx.src_out)[p, 0])
                if n > 1 and 0 <= j < n and logp_p[p, j] >= logp_p[p, :n].max() - 1e-9:
                    logp_p[p, j] = logp_p[p, :n].max() + 1e-8
        sref = o_select.select_beams(w.tree_off, w.parent, ref["n_out"], ref["out_parent"], ref["out_token"],
                                     logp_p, ref["out_logp_q"], w.max_depth + 1, keep_one=keep_one)
        clean = ref["near_tie"] == 0
        for name in ("n_next", "src_tree", "src_out", "path_len", "path", "token"):
            got, want = g(getattr(nx, name))[clean], sref[name][clean]
            assert np.array_equal(got, want), (name, "keep_one", keep_one, got[got != want][:8], want[got != want][:8])
        for name, key in (("logp_target", "logp_p"), ("logp_draft", "logp_q")):
            err = max_abs_err(g(getattr(nx, name))[clean], sref[key][clean])
            assert err <= (2e-8 if keep_one and name == "logp_target" else 1e-9), (name, "keep_one", keep_one, err)
