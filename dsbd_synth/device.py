"""Device copies of a synthetic workload and the calls of the HIP library on them (argument marshalling only).

Serves the GPU tests, the smoke run and the benchmark's timed region.  Imports the library binding and nothing of the
CPU oracle; it is not imported by the package's __init__, so the oracle's tests never load the library through it."""
import numpy as np
import torch

import paper_2409_16560_amd as dsbd


def bf16_dev(bits, dev="cuda"):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)


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

    def verify_select(self, W_L=0, W_min=1, t=-1.0, **kw):
        """Verification with the next-beam plan written in the same call; returns (VerifyResult, NextBeams)."""
        return dsbd.dsbd_verify_forest_select(self.forest, self.logits_p, self.logits_q, self.blp, self.blq,
                                              self.u_accept, self.u_resid, self.u_fill, W_L=W_L, W_min=W_min,
                                              W_cap=self.w.W_cap, t=t, **kw)
