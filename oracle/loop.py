"""Several iterations of the method, end to end, on the CPU (test infrastructure, not the product path).

One iteration (Section 3.1 "Overview", Algorithm 1; Section 3.3): the small model extends the input beams by gamma
beam-sampling steps of width W_S (draft.draft_layer), the steps form the draft forest (draft.build_forest), both
models score every node of the forest in one pass (here: a callback that returns logits and attention rows for
token sequences), the layers are verified (verify.verify_forest), the output beams of the additional layer
become the next input beams (select.select_beams) and the key/value caches follow them (commit.commit_kv).
An iteration yields l_last new tokens per beam: its accepted layers plus the additional one (Section 3.2 counts
these steps per iteration).

Readings: the uniforms of iteration `it` come from fixed streams (accept tests 4*it+0, residual 4*it+1, additional
layer 4*it+2, draft step l: 1000*(it+1)+l), so two implementations given the same seed draw the same numbers; a
beam's cache covers all its tokens but the last (whose row is produced when it becomes a tree's root).
"""
import numpy as np

from dsbd_synth import bf16_bits_to_f32, uniform01_f32

from . import attention as o_attn
from . import commit as o_commit
from . import draft as o_draft
from . import select as o_select
from . import verify as o_verify


class OracleLoop:
    def __init__(self, models, beams, W_S, gamma, W_L=0, W_min=1, W_cap=16, t=-1.0, top_k=0, top_p=1.0,
                 keep_one=False, seed=0, with_kv=True):
        """beams: per prompt, the list of input beams (tuples of token ids; equal lengths within a prompt)."""
        self.m, self.W_S, self.gamma = models, W_S, gamma
        self.W_L, self.W_min, self.W_cap, self.t = W_L, W_min, W_cap, t
        self.top_k, self.top_p, self.keep_one, self.seed, self.with_kv = top_k, top_p, keep_one, seed, with_kv
        self.beams = [[tuple(b) for b in pb] for pb in beams]
        self.cum_p = [[0.0] * len(pb) for pb in beams]
        self.cum_q = [[0.0] * len(pb) for pb in beams]
        self.it = 0
        self.k_cache = self.v_cache = None
        if with_kv:           # caches of all tokens but the last, one per beam
            self.k_cache, self.v_cache = [], []
            for pb in self.beams:
                for b in pb:
                    _, k, v = self.m.qkv([b[:i + 1] for i in range(len(b) - 1)])
                    self.k_cache.append(k); self.v_cache.append(v)

    def step(self):
        """One iteration.  Returns a record of everything it produced (for comparison with another implementation)."""
        P, W_S, gamma, it = len(self.beams), self.W_S, self.gamma, self.it
        root_off = np.concatenate([[0], np.cumsum([len(pb) for pb in self.beams])]).astype(np.int32)
        T = int(root_off[-1])
        seqs = [[b for pb in self.beams for b in pb]]                # sequences of the rows of every layer
        cum = np.asarray([c for pc in self.cum_q for c in pc], dtype=np.float64)
        off = root_off
        lpar, ltok = [], []
        for l in range(1, gamma + 1):
            _, zq = self.m.logits(seqs[l - 1])
            u = uniform01_f32(P * W_S, self.seed, 1000 * (it + 1) + l).reshape(P, W_S)
            par = np.zeros(P * W_S, dtype=np.int32); tok = np.zeros(P * W_S, dtype=np.int32); lp = np.zeros(P * W_S)
            for p in range(P):
                a, b = int(off[p]), int(off[p + 1])
                pp, tt, ll = o_draft.draft_layer(zq[a:b], cum[a:b], u[p], self.top_k, float(np.float32(self.top_p)))
                par[p * W_S:(p + 1) * W_S], tok[p * W_S:(p + 1) * W_S], lp[p * W_S:(p + 1) * W_S] = pp + a, tt, ll
            lpar.append(par); ltok.append(tok)
            seqs.append([seqs[l - 1][int(par[r])] + (int(tok[r]),) for r in range(P * W_S)])
            cum, off = lp, np.arange(P + 1, dtype=np.int32) * W_S
        f = o_draft.build_forest(root_off, lpar, ltok, [b[-1] for b in seqs[0]])
        N = len(f["parent"])
        node_seq = [None] * N
        for l in range(gamma + 1):
            for r, n in enumerate(f["node_of"][l]):
                node_seq[int(n)] = seqs[l][r]
        zp, zq = self.m.logits(node_seq)
        rec = {"forest": f, "logits_p": zp, "logits_q": zq, "node_seq": node_seq}
        if self.with_kv:
            q, k, v = self.m.qkv(node_seq)
            rec.update(q=q, k_tree=k, v_tree=v)
            f64 = lambda bits: bf16_bits_to_f32(bits).astype(np.float64)
            rec["attn_out"], rec["attn_lse"] = o_attn.forest_attention(
                f["parent"], f["tree_off"], f64(q), f64(k), f64(v), [f64(c) for c in self.k_cache], [f64(c) for c in self.v_cache])
        u_acc = uniform01_f32(N, self.seed, 4 * it)
        u_res = uniform01_f32(P * (gamma + 2), self.seed, 4 * it + 1).reshape(P, gamma + 2)
        u_fill = uniform01_f32(P * (gamma + 2) * self.W_cap, self.seed, 4 * it + 2).reshape(P, gamma + 2, self.W_cap)
        blp = np.asarray([c for pc in self.cum_p for c in pc], dtype=np.float64)
        blq = np.asarray([c for pc in self.cum_q for c in pc], dtype=np.float64)
        ver = o_verify.verify_forest(f["tree_prompt"], f["tree_off"], f["parent"], f["token"], zp, zq, blp, blq,
                                     u_acc, u_res, u_fill, self.W_L, self.W_min, self.W_cap, np.float32(self.t),
                                     rank=f["draft_rank"], top_k=self.top_k, top_p=float(np.float32(self.top_p)))
        nxt = o_select.select_beams(f["tree_off"], f["parent"], ver["n_out"], ver["out_parent"], ver["out_token"],
                                    ver["out_logp_p"], ver["out_logp_q"], gamma + 1, keep_one=self.keep_one)
        rec.update(verify=ver, next=nxt, u=(u_acc, u_res, u_fill), beam_logp=(blp, blq))
        # the next input beams
        beams, cum_p, cum_q = [], [], []
        for p in range(P):
            n = int(nxt["n_next"][p])
            beams.append([node_seq[int(ver["out_parent"][p, int(nxt["src_out"][p, s])])] + (int(nxt["token"][p, s]),)
                          for s in range(n)])
            cum_p.append([float(nxt["logp_p"][p, s]) for s in range(n)])
            cum_q.append([float(nxt["logp_q"][p, s]) for s in range(n)])
        if self.with_kv:
            dk, dv, dlen = o_commit.commit_kv(self.k_cache, self.v_cache, rec["k_tree"], rec["v_tree"], nxt["n_next"],
                                              nxt["src_tree"], nxt["path_len"], nxt["path"])
            self.k_cache = [dk[(p, s)] for p in range(P) for s in range(int(nxt["n_next"][p]))]
            self.v_cache = [dv[(p, s)] for p in range(P) for s in range(int(nxt["n_next"][p]))]
            rec["cache_len"] = dlen
        self.beams, self.cum_p, self.cum_q = beams, cum_p, cum_q
        self.it += 1
        return rec
