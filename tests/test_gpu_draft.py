"""GPU parity of the draft stage (dsbd_draft_layer, dsbd_build_forest) against oracle/draft.py: sampled (parent,
token) pairs and forest arrays bit for bit, log-likelihoods to 1e-9."""
import numpy as np
import pytest
import torch

from dsbd_synth import uniform01_f32

pytestmark = pytest.mark.gpu


def _mods():
    import paper_2409_16560_amd as dsbd
    from oracle import draft as o_draft
    return dsbd, o_draft


def layer_inputs(seed, beams_per_prompt, V, W_S, std=3.0):
    rng = np.random.Generator(np.random.Philox(key=[seed, 77]))
    beam_off = np.concatenate([[0], np.cumsum(beams_per_prompt)]).astype(np.int32)
    B, P = int(beam_off[-1]), len(beams_per_prompt)
    z = (rng.standard_normal((B, V), dtype=np.float32) * np.float32(std)).astype(np.float32)
    cum = -3.0 * rng.random(B)
    u = uniform01_f32(P * W_S, seed, 201).reshape(P, W_S)
    return beam_off, z, cum, u


def run_draft_layer(beam_off, z, cum, u, W_S, top_k=0, top_p=1.0):
    dsbd, _ = _mods()
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    par, tok, lp, fault = dsbd.dsbd_draft_layer(t(beam_off), t(z), t(cum), t(u), W_S,
                                                max_prompt_beams=int(np.diff(beam_off).max()), top_k=top_k, top_p=top_p)
    torch.cuda.synchronize()
    return par.cpu().numpy(), tok.cpu().numpy(), lp.cpu().numpy(), int(fault.item())


def oracle_draft_layer(beam_off, z, cum, u, top_k=0, top_p=1.0):
    _, o_draft = _mods()
    P = len(beam_off) - 1
    par, tok, lp = [], [], []
    for p in range(P):
        a, b = int(beam_off[p]), int(beam_off[p + 1])
        pp, tt, ll = o_draft.draft_layer(z[a:b], cum[a:b], u[p], top_k, float(np.float32(top_p)))
        par.append(pp + a); tok.append(tt); lp.append(ll)
    return np.stack(par), np.stack(tok), np.stack(lp)


DRAFT_CASES = [
    # beams per prompt, V, W_S, top_k, top_p
    ([2], 256, 4, 0, 1.0),
    ([8], 32000, 16, 0, 1.0),
    ([1], 5000, 8, 0, 1.0),                      # a single input beam (first step of the first iteration)
    ([16], 20000, 16, 0, 1.0),                   # a later step: W_S beams in, W_S out
    ([3, 1, 8, 5], 3000, 6, 0, 1.0),             # several prompts, ragged
    ([64], 1000, 64, 0, 1.0),                    # the largest width
    ([4], 4001, 1, 0, 1.0),                      # one draw; V not a multiple of 4
    ([8], 32000, 16, 10, 0.8),                   # the paper's warping setting
    ([16, 16], 9000, 16, 32, 0.9),
    ([5], 300, 7, 3, 1.0),
    ([2], 9, 5, 32, 0.7),                        # fewer entries than top_k
]


@pytest.mark.parametrize("beams,V,W_S,top_k,top_p", DRAFT_CASES)
def test_draft_layer_matches_oracle(beams, V, W_S, top_k, top_p):
    print("case", beams, V, W_S, top_k, top_p, flush=True)
    beam_off, z, cum, u = layer_inputs(len(beams) * 1000 + V, beams, V, W_S)
    par, tok, lp, fault = run_draft_layer(beam_off, z, cum, u, W_S, top_k, top_p)
    rpar, rtok, rlp = oracle_draft_layer(beam_off, z, cum, u, top_k, top_p)
    assert fault == 0
    assert np.array_equal(par, rpar) and np.array_equal(tok, rtok)
    assert np.max(np.abs(lp - rlp)) <= 1e-9


def test_draft_layer_full_vocabulary():
    """The benchmark's shape: 16 beams of the step before, vocabulary 128256, 16 draws; plain and warped."""
    beam_off, z, cum, u = layer_inputs(5, [16], 128256, 16)
    for top_k, top_p in ((0, 1.0), (10, 0.8)):
        par, tok, lp, fault = run_draft_layer(beam_off, z, cum, u, 16, top_k, top_p)
        rpar, rtok, rlp = oracle_draft_layer(beam_off, z, cum, u, top_k, top_p)
        assert fault == 0
        assert np.array_equal(par, rpar) and np.array_equal(tok, rtok)
        assert np.max(np.abs(lp - rlp)) <= 1e-9


@pytest.mark.parametrize("top_k,top_p", [(0, 1.0), (10, 0.8)])
def test_draft_layer_with_masked_tokens(top_k, top_p):
    """Logits of -Inf are tokens of probability 0 (never drawn), not a fault: a masked tail, masks per row, and a row
    with a single allowed token."""
    beam_off, z, cum, u = layer_inputs(11, [6, 3], 9000, 8)
    rng = np.random.default_rng(2)
    z[:, 5000:] = -np.inf
    z[rng.random(z.shape) < 0.3] = -np.inf
    z[4, :] = -np.inf; z[4, 123] = 0.5
    z[np.arange(z.shape[0]), rng.integers(0, 5000, z.shape[0])] = 1.0
    par, tok, lp, fault = run_draft_layer(beam_off, z, cum, u, 8, top_k, top_p)
    with np.errstate(all="ignore"):
        rpar, rtok, rlp = oracle_draft_layer(beam_off, z, cum, u, top_k, top_p)
    assert fault == 0
    assert np.array_equal(par, rpar) and np.array_equal(tok, rtok)
    assert np.isfinite(z[par, tok]).all()
    assert np.max(np.abs(lp - rlp)) <= 1e-9


def test_draft_layer_skips_beams_of_probability_zero():
    """Beams with a stored likelihood of -Inf are never continued; the draws are the oracle's."""
    for top_k, top_p in ((0, 1.0), (10, 0.8)):
        beam_off, z, cum, u = layer_inputs(2, [5, 3], 4000, 8)
        cum[1] = -np.inf
        cum[6] = -np.inf
        with np.errstate(all="ignore"):
            rpar, rtok, rlp = oracle_draft_layer(beam_off, z, cum, u, top_k, top_p)
        par, tok, lp, fault = run_draft_layer(beam_off, z, cum, u, 8, top_k, top_p)
        assert fault == 0 and not np.isin(par, [1, 6]).any()
        assert np.array_equal(par, rpar) and np.array_equal(tok, rtok)
        assert np.max(np.abs(lp - rlp)) <= 1e-9


def test_draft_layer_reports_bad_inputs():
    beam_off, z, cum, u = layer_inputs(3, [3, 2], 500, 4)
    z_bad = z.copy(); z_bad[1, 17] = np.inf
    assert run_draft_layer(beam_off, z_bad, cum, u, 4)[3] & 4            # non-finite logit
    off_bad = beam_off.copy(); off_bad[-1] = 4                           # does not cover the rows
    assert run_draft_layer(off_bad, z, cum, u, 4)[3] & 1


# ------------------------------------------------------------------------------------------- forest layout
def random_layers(rng, root_off, gamma, W_S, V, lopsided=False):
    P = len(root_off) - 1
    lp = np.zeros((gamma, P * W_S), dtype=np.int32)
    lt = rng.integers(0, V, (gamma, P * W_S)).astype(np.int32)
    for l in range(1, gamma + 1):
        for p in range(P):
            lo, hi = (root_off[p], root_off[p + 1]) if l == 1 else (p * W_S, (p + 1) * W_S)
            lp[l - 1, p * W_S:(p + 1) * W_S] = lo if lopsided else rng.integers(lo, hi, W_S)
    return lp, lt


def run_build(root_off, lp, lt, root_token=None):
    dsbd, _ = _mods()
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    f, nroot, nof, mx, fault = dsbd.dsbd_build_forest(t(root_off), t(lp), t(lt), t(root_token), n_roots=int(root_off[-1]),
                                                      max_prompt_trees=int(np.diff(root_off).max()))
    torch.cuda.synchronize()
    g = lambda x: x.cpu().numpy()
    return f, g(nroot), g(nof), int(mx.item()), int(fault.item())


@pytest.mark.parametrize("seed,root_off,gamma,W_S", [(0, [0, 2], 3, 4), (1, [0, 1, 4, 6], 2, 5), (2, [0, 3], 1, 2),
                                                     (3, [0, 4, 5], 4, 3), (4, [0, 8], 4, 16), (5, [0, 64], 7, 64),
                                                     (6, list(range(0, 17)), 5, 8), (7, [0, 5], 0, 0),
                                                     # more input beams than draws per step: a root's own index exceeds W_S
                                                     (8, [0, 3], 1, 1), (9, [0, 6, 14], 3, 2), (10, [0, 8], 2, 3), (11, [0, 5, 10], 3, 3)])
def test_build_forest_matches_oracle(seed, root_off, gamma, W_S):
    _, o_draft = _mods()
    rng = np.random.default_rng(seed)
    root_off = np.asarray(root_off, dtype=np.int32)
    if gamma:
        lp, lt = random_layers(rng, root_off, gamma, W_S, 32000)
    else:
        lp, lt = np.zeros((0, 0), dtype=np.int32), np.zeros((0, 0), dtype=np.int32)
    root_token = rng.integers(0, 32000, int(root_off[-1])).astype(np.int32)
    f, nroot, nof, mx, fault = run_build(root_off, lp, lt, root_token)
    ref = o_draft.build_forest(root_off, list(lp), list(lt), root_token)
    sizes = np.diff(ref["tree_off"])
    assert fault == (16 if sizes.max() > 64 else 0)
    g = lambda x: x.cpu().numpy()
    for name in ("tree_prompt", "tree_off", "parent", "token", "draft_rank"):
        assert np.array_equal(g(getattr(f, name)), ref[name]), name
    assert np.array_equal(nroot, ref["node_of"][0])
    for l in range(gamma):
        assert np.array_equal(nof[l], ref["node_of"][l + 1])
    assert mx == sizes.max()
    assert f.max_depth == gamma and f.n_nodes == len(ref["parent"])


def test_build_forest_reports_what_the_other_calls_cannot_take():
    root_off = np.asarray([0, 2], dtype=np.int32)
    lp, lt = random_layers(np.random.default_rng(0), root_off, 4, 16, 100, lopsided=True)      # one tree of 65 nodes
    assert run_build(root_off, lp, lt)[4] & 16
    lp, lt = random_layers(np.random.default_rng(1), root_off, 2, 4, 100)
    lp[1, 2] = 9                                                                                # parent row outside the prompt
    assert run_build(root_off, lp, lt)[4] & 1


# ------------------------------------------------------------------------------------------- the whole draft stage
@pytest.mark.parametrize("beams,V,W_S,gamma,top_k,top_p", [([2], 300, 4, 3, 0, 1.0), ([8], 20000, 16, 3, 0, 1.0),
                                                           ([3, 1, 5], 3000, 6, 2, 10, 0.8)])
def test_draft_stage_then_verification(beams, V, W_S, gamma, top_k, top_p):
    """gamma steps of the small model's beam sampling (synthetic logits per step), the forest built from them, and
    the verification of that forest: library and oracle agree at every stage."""
    import gpu_util as gu
    dsbd, o_draft = _mods()
    from oracle import verify as o_verify
    rng = np.random.Generator(np.random.Philox(key=[len(beams), V]))
    P = len(beams)
    root_off = np.concatenate([[0], np.cumsum(beams)]).astype(np.int32)
    T = int(root_off[-1])
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    # logits of both models at the beams of every layer (a model would produce them from the sequences)
    rows = [T] + [P * W_S] * gamma
    zq = [(rng.standard_normal((r, V), dtype=np.float32) * np.float32(3.0)) for r in rows]
    zp = [(z + rng.standard_normal(z.shape, dtype=np.float32) * np.float32(0.5)).astype(np.float32) for z in zq]
    cum_q0 = -3.0 * rng.random(T)
    cum_p0 = cum_q0 + 0.25 * rng.standard_normal(T)
    off_l = np.arange(P + 1, dtype=np.int32) * W_S
    # library
    cum, off = t(cum_q0), t(root_off)
    lpar, ltok = [], []
    for l in range(1, gamma + 1):
        u = uniform01_f32(P * W_S, 900 + l, 202).reshape(P, W_S)
        par, tok, lp, fault = dsbd.dsbd_draft_layer(off, t(zq[l - 1]), cum, t(u), W_S,
                                                    max_prompt_beams=max(max(beams), W_S), top_k=top_k, top_p=top_p)
        assert int(fault.item()) == 0
        lpar.append(par.reshape(-1)); ltok.append(tok.reshape(-1))
        cum, off = lp.reshape(-1).contiguous(), t(off_l)
    f, nroot, nof, mx, fault = dsbd.dsbd_build_forest(t(root_off), torch.stack(lpar), torch.stack(ltok), None, n_roots=T,
                                                      max_prompt_trees=max(beams))
    torch.cuda.synchronize()
    # oracle
    cum_o, off_o = cum_q0, root_off
    opar, otok = [], []
    for l in range(1, gamma + 1):
        u = uniform01_f32(P * W_S, 900 + l, 202).reshape(P, W_S)
        a, b, c = oracle_draft_layer(off_o, zq[l - 1], cum_o, u, top_k, top_p)
        opar.append(a.reshape(-1)); otok.append(b.reshape(-1))
        cum_o, off_o = c.reshape(-1), off_l
    ref_f = o_draft.build_forest(root_off, opar, otok)
    g = lambda x: x.cpu().numpy()
    for l in range(gamma):
        assert np.array_equal(g(lpar[l]), opar[l]) and np.array_equal(g(ltok[l]), otok[l])
    for name in ("tree_prompt", "tree_off", "parent", "token", "draft_rank"):
        assert np.array_equal(g(getattr(f, name)), ref_f[name]), name
    if int(mx.item()) > 64:
        pytest.skip("a tree of this run exceeds the 64 nodes the attention and verification calls take")
    # logits in forest order, then the verification on both sides
    N = f.n_nodes
    order = [ref_f["node_of"][0]] + [ref_f["node_of"][l] for l in range(1, gamma + 1)]
    logits_p, logits_q = np.zeros((N, V), dtype=np.float32), np.zeros((N, V), dtype=np.float32)
    for l in range(gamma + 1):
        logits_p[order[l]], logits_q[order[l]] = zp[l], zq[l]
    W_cap = 16
    u_acc = uniform01_f32(N, 7, 101)
    u_res = uniform01_f32(P * (gamma + 2), 7, 102).reshape(P, gamma + 2)
    u_fill = uniform01_f32(P * (gamma + 2) * W_cap, 7, 103).reshape(P, gamma + 2, W_cap)
    res = dsbd.dsbd_verify_forest(f, t(logits_p), t(logits_q), t(cum_p0), t(cum_q0), t(u_acc), t(u_res), t(u_fill),
                                  W_L=0, W_min=1, W_cap=W_cap, t=-1.0, top_k=top_k, top_p=top_p)
    torch.cuda.synchronize()
    ref = o_verify.verify_forest(ref_f["tree_prompt"], ref_f["tree_off"], ref_f["parent"], ref_f["token"], logits_p,
                                 logits_q, cum_p0, cum_q0, u_acc, u_res, u_fill, 0, 1, W_cap, np.float32(-1.0),
                                 rank=ref_f["draft_rank"], top_k=top_k, top_p=float(np.float32(top_p)))

    class W:      # what compare_verify wants to know about the workload
        tree_prompt, tree_off, n_nodes = ref_f["tree_prompt"], ref_f["tree_off"], N
    gu.compare_verify(res, ref, W)
    st = ref["node_status"]
    print("l_last", ref["l_last"].tolist(), "accepted", int((st == 1).sum()), "rejected", int((st == 2).sum()), flush=True)
