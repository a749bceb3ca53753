"""Several iterations of the method over the library's calls (Section 3.1 "Overview"; Algorithm 1; Section 3.3).

One iteration: gamma calls of dsbd_draft_layer (the small model's beam sampling), dsbd_build_forest, one pass of
both models over the forest's nodes (a callback: `models.logits(seqs)`, `models.qkv(seqs)` for token sequences;
this package holds no model), dsbd_forest_attention, dsbd_verify_forest_select (verification and selection in one
call), dsbd_commit_kv.
The loop itself only moves data between the calls and keeps the token sequences on the host for the callback.

Uniforms come from `uniforms(n, stream) -> float32[n]`; the streams of iteration `it` are 4*it (accept tests),
4*it+1 (residual draws), 4*it+2 (additional layer) and 1000*(it+1)+l (draft step l).
"""
import numpy as np
import torch

from . import binding as B


class DecodeLoop:
    def __init__(self, models, beams, W_S, gamma, uniforms, W_L=0, W_min=1, W_cap=16, t=-1.0, top_k=0, top_p=1.0,
                 keep_one=False, with_kv=True, kv_capacity=256, device="cuda"):
        """beams: per prompt, the list of input beams (tuples of token ids, equal lengths within a prompt)."""
        self.m, self.W_S, self.gamma, self.uniforms = models, int(W_S), int(gamma), uniforms
        self.W_L, self.W_min, self.W_cap, self.t = W_L, W_min, W_cap, t
        self.top_k, self.top_p, self.keep_one, self.with_kv = top_k, top_p, keep_one, with_kv
        self.dev, self.cap = device, int(kv_capacity)
        self.beams = [[tuple(b) for b in pb] for pb in beams]
        n = sum(len(pb) for pb in beams)
        self.cum_p = torch.zeros(n, dtype=torch.float64, device=device)
        self.cum_q = torch.zeros(n, dtype=torch.float64, device=device)
        self.it = 0
        self.k_buf, self.v_buf, self.kv_len = [], [], []
        if with_kv:
            for pb in self.beams:
                for b in pb:
                    _, k, v = models.qkv([b[:i + 1] for i in range(len(b) - 1)])
                    kb, vb = self._buffer(), self._buffer()
                    kb[:k.shape[0]] = self._bf16(k); vb[:v.shape[0]] = self._bf16(v)
                    self.k_buf.append(kb); self.v_buf.append(vb); self.kv_len.append(k.shape[0])

    def _buffer(self):
        return torch.zeros((self.cap, self.m.Hkv, self.m.D), dtype=torch.bfloat16, device=self.dev)

    def _bf16(self, bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(self.dev).view(torch.bfloat16)

    def _dev(self, a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)

    def step(self):
        """One iteration; returns what it produced (device tensors) for inspection."""
        P, W_S, gamma, it, dev = len(self.beams), self.W_S, self.gamma, self.it, self.dev
        counts = [len(pb) for pb in self.beams]
        root_off_h = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        T = int(root_off_h[-1])
        root_off = self._dev(root_off_h)
        layer_off = self._dev(np.arange(P + 1, dtype=np.int32) * W_S)
        # ---- draft stage
        seqs = [[b for pb in self.beams for b in pb]]
        cum, off, width = self.cum_q, root_off, max(counts)
        lpar, ltok = [], []
        for l in range(1, gamma + 1):
            _, zq = self.m.logits(seqs[l - 1])
            u = self._dev(self.uniforms(P * W_S, 1000 * (it + 1) + l).reshape(P, W_S))
            par, tok, lp, fault = B.dsbd_draft_layer(off, self._dev(zq), cum, u, W_S, max_prompt_beams=width,
                                                     top_k=self.top_k, top_p=self.top_p)
            if int(fault.item()):
                raise B.DsbdError(int(fault.item()), "dsbd_draft_layer (fault bits)")
            lpar.append(par.reshape(-1)); ltok.append(tok.reshape(-1))
            ph, th = lpar[-1].cpu().numpy(), ltok[-1].cpu().numpy()
            seqs.append([seqs[l - 1][int(ph[r])] + (int(th[r]),) for r in range(P * W_S)])
            cum, off, width = lp.reshape(-1).contiguous(), layer_off, W_S
        root_token = self._dev(np.asarray([b[-1] for b in seqs[0]], dtype=np.int32))
        empty = torch.zeros((0, 0), dtype=torch.int32, device=dev)
        forest, node_of_root, node_of, mx, fault = B.dsbd_build_forest(
            root_off, torch.stack(lpar) if gamma else empty, torch.stack(ltok) if gamma else empty, root_token,
            n_roots=T, max_prompt_trees=max(counts))
        if int(fault.item()):
            raise B.DsbdError(int(fault.item()), "dsbd_build_forest (fault bits)")
        N = forest.n_nodes
        node_seq = [None] * N
        nr, no = node_of_root.cpu().numpy(), node_of.cpu().numpy()
        for r in range(T):
            node_seq[int(nr[r])] = seqs[0][r]
        for l in range(1, gamma + 1):
            for r in range(P * W_S):
                node_seq[int(no[l - 1, r])] = seqs[l][r]
        # ---- both models over the forest, then the hot path
        zp, zq = self.m.logits(node_seq)
        rec = {"forest": forest, "node_seq": node_seq}
        if self.with_kv:
            q, k, v = self.m.qkv(node_seq)
            q, k_tree, v_tree = self._bf16(q), self._bf16(k), self._bf16(v)
            kv = B.PrefixKV([self.k_buf[b][:self.kv_len[b]] for b in range(T)], [self.v_buf[b][:self.kv_len[b]] for b in range(T)])
            out, lse, afault = B.dsbd_forest_attention(forest, kv, q, k_tree, v_tree)
            rec.update(attn_out=out, attn_lse=lse, attn_fault=afault)
        u_acc = self._dev(self.uniforms(N, 4 * it))
        u_res = self._dev(self.uniforms(P * (gamma + 2), 4 * it + 1))
        u_fill = self._dev(self.uniforms(P * (gamma + 2) * self.W_cap, 4 * it + 2))
        ver, nxt = B.dsbd_verify_forest_select(forest, self._dev(zp), self._dev(zq), self.cum_p, self.cum_q, u_acc,
                                               u_res, u_fill, W_L=self.W_L, W_min=self.W_min, W_cap=self.W_cap,
                                               t=self.t, keep_one=self.keep_one, top_k=self.top_k, top_p=self.top_p)
        rec.update(verify=ver, next=nxt)
        # ---- the next input beams
        n_next = nxt.n_next.cpu().numpy()
        src_out = nxt.src_out.view(P, -1).cpu().numpy()
        src_tree = nxt.src_tree.view(P, -1).cpu().numpy()
        token = nxt.token.view(P, -1).cpu().numpy()
        out_parent = ver.out_parent.view(P, -1).cpu().numpy()
        if int(ver.fault.item()) or int(nxt.fault.item()):
            raise B.DsbdError(int(ver.fault.item()) | int(nxt.fault.item()), "verification / selection (fault bits)")
        beams, keep = [], []
        for p in range(P):
            beams.append([node_seq[int(out_parent[p, int(src_out[p, s])])] + (int(token[p, s]),) for s in range(int(n_next[p]))])
            keep += [p * self.W_cap + s for s in range(int(n_next[p]))]
        keep_t = torch.tensor(keep, dtype=torch.int64, device=dev)
        new_cum_p = nxt.logp_target.reshape(-1)[keep_t].contiguous()
        new_cum_q = nxt.logp_draft.reshape(-1)[keep_t].contiguous()
        if self.with_kv:
            # the first next beam of a source tree continues in that tree's buffer, the others get fresh ones
            dst_k, dst_v, taken = [None] * (P * self.W_cap), [None] * (P * self.W_cap), set()
            for p in range(P):
                for s in range(int(n_next[p])):
                    b = int(src_tree[p, s])
                    if b not in taken:
                        taken.add(b); dst_k[p * self.W_cap + s], dst_v[p * self.W_cap + s] = self.k_buf[b], self.v_buf[b]
                    else:
                        dst_k[p * self.W_cap + s], dst_v[p * self.W_cap + s] = self._buffer(), self._buffer()
            dst = B.KVDst(dst_k, dst_v, kv)
            dlen, cfault = B.dsbd_commit_kv(forest, kv, k_tree, v_tree, nxt, self.W_cap, dst)
            if int(cfault.item()):
                raise B.DsbdError(int(cfault.item()), "dsbd_commit_kv (fault bits)")
            dl = dlen.reshape(-1).cpu().numpy()
            self.k_buf = [dst_k[j] for j in keep]
            self.v_buf = [dst_v[j] for j in keep]
            self.kv_len = [int(dl[j]) for j in keep]
        self.beams, self.cum_p, self.cum_q = beams, new_cum_p, new_cum_q
        self.it += 1
        return rec
