"""Seeded synthetic workloads shaped like the five benchmark configurations.

Everything here is input generation: forest topologies (parent arrays), random
bf16 Q/K/V, random fp32 logits, draft tokens drawn from the draft logits, stored
beam log-likelihoods and the uniform draws the verification consumes.  None of
the method's arithmetic lives here.

Stand-in statement: the paper measures on SQuAD / Spider / MT-Bench prompts with
Llama-2-13B, Llama-3.1-8B and OPT-13B.  Neither datasets nor weights are used;
only the tensor shapes of those models (32 heads x 128, vocabulary 32000 or
128256, GQA 32/8) are reproduced with random values.
"""
from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple, Union

import numpy as np

from .bf16 import f32_to_bf16_bits
from .philox import uniform01_f32

IntOrRange = Union[int, Tuple[int, int]]


@dataclass(frozen=True)
class Spec:
    name: str
    n_prompts: int
    W: IntOrRange                 # input beams (= trees) per prompt
    tree: str                     # 'chain', 'fork_chain', 'binary_bfs', 'binary_dfs', 'random'
    tree_nodes: IntOrRange        # nodes per tree (incl. root)
    L: IntOrRange                 # prefix tokens per beam (equal within a prompt)
    shared_len: int               # leading prefix tokens common to the beams of a prompt
    Hq: int
    Hkv: int
    D: int
    V: int
    logit_std: float
    draft: str                    # 'indep' (independent N(0,std)) or 'noise' (target + N(0,noise_std))
    noise_std: float = 0.5
    seed: int = 0
    draft_top_k: int = 0          # > 0: draft tokens come from the draft_top_k largest draft logits of the parent's row


CONFIGS = {
    # W=2 chains of 3 nodes, L=32, 4 heads x 64, V=256, independent logits N(0,2)
    "c1": Spec("c1", 1, 2, "chain", 3, 32, 0, 4, 4, 64, 256, 2.0, "indep"),
    # W=4, 7-node trees (root, 2 children, each continued as a chain), L=512, 32x128, V=32000
    "c2": Spec("c2", 1, 4, "fork_chain", 7, 512, 0, 32, 32, 128, 32000, 3.0, "noise"),
    # W=8, complete binary trees of 15 nodes, L=2048 with the first 1024 shared, draft = target + N(0,0.5)
    "c3": Spec("c3", 1, 8, "binary_bfs", 15, 2048, 1024, 32, 32, 128, 32000, 3.0, "noise"),
    # 16 prompts, W~U{1..8}, random trees of 4..16 nodes, L~U{1024..4096}
    "c4": Spec("c4", 16, (1, 8), "random", (4, 16), (1024, 4096), 0, 32, 32, 128, 32000, 3.0, "noise"),
    # W=8, complete binary trees of 31 nodes, L=8192, GQA 32/8, V=128256
    "c5": Spec("c5", 1, 8, "binary_dfs", 31, 8192, 0, 32, 8, 128, 128256, 3.0, "noise"),
}


@dataclass
class Workload:
    spec: Spec
    n_prompts: int
    n_trees: int
    n_nodes: int
    tree_prompt: np.ndarray        # [T] i32
    tree_off: np.ndarray           # [T+1] i32
    parent: np.ndarray             # [N] i32 global index, -1 at roots
    token: np.ndarray              # [N] i32
    max_depth: int                 # deepest node (roots are depth 0)
    max_tree_nodes: int
    max_prompt_trees: int
    own_len: np.ndarray            # [T] i32 tokens in the beam's own prefix segment
    shared_len: np.ndarray         # [T] i32 tokens in the prompt-shared leading segment
    k_own: List[np.ndarray]        # per tree [own_len,Hkv,D] bf16 bits
    v_own: List[np.ndarray]
    k_shared: List[Optional[np.ndarray]]   # per prompt [shared_len,Hkv,D] bf16 bits or None
    v_shared: List[Optional[np.ndarray]]
    q: np.ndarray                  # [N,Hq,D] bf16 bits
    k_tree: np.ndarray             # [N,Hkv,D] bf16 bits
    v_tree: np.ndarray
    logits_p: np.ndarray           # [N,V] f32 target
    logits_q: np.ndarray           # [N,V] f32 draft
    beam_logp_p: np.ndarray        # [T] f64
    beam_logp_q: np.ndarray
    u_accept: np.ndarray           # [N] f32
    u_resid: np.ndarray            # [P, max_depth+2] f32
    u_fill: np.ndarray             # [P, max_depth+2, W_cap] f32
    W_cap: int
    extra: dict = field(default_factory=dict)

    @property
    def Hq(self):
        return self.spec.Hq

    @property
    def Hkv(self):
        return self.spec.Hkv

    @property
    def D(self):
        return self.spec.D

    @property
    def V(self):
        return self.spec.V


def _draw(rng, v: IntOrRange) -> int:
    if isinstance(v, tuple):
        return int(rng.integers(v[0], v[1] + 1))
    return int(v)


def tree_parents(kind: str, n: int, rng) -> List[int]:
    """Local parent indices (root = -1, parent < child) of one tree of n nodes."""
    if kind == "chain":
        return [-1] + list(range(n - 1))
    if kind == "fork_chain":
        # root, two children, each child continued as a chain
        return ([-1, 0, 0] + [i - 2 for i in range(3, n)])[:n]
    if kind == "binary_bfs":
        return [-1] + [(i - 1) // 2 for i in range(1, n)]
    if kind == "binary_dfs":
        # complete binary tree numbered in depth-first (pre-order) order
        out: List[int] = []

        def rec(par, size):
            me = len(out)
            out.append(par)
            sub = (size - 1) // 2
            if sub > 0:
                rec(me, sub)
                rec(me, sub)

        rec(-1, n)
        assert len(out) == n, "binary_dfs needs n = 2^k - 1"
        return out
    if kind == "random":
        return [-1] + [int(rng.integers(0, i)) for i in range(1, n)]
    raise ValueError(kind)


def _depths(parent):
    d = np.zeros(len(parent), dtype=np.int32)
    for i, p in enumerate(parent):
        d[i] = 0 if p < 0 else d[p] + 1
    return d


def _normal_bf16(rng, shape):
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32)).reshape(shape)


def make_workload(config: Union[str, Spec], W_cap: Optional[int] = None, **overrides) -> Workload:
    """Build the seeded workload of a named configuration (or an explicit Spec).

    overrides: any Spec field (e.g. L=64, V=512) to get a scaled-down variant.
    """
    spec = CONFIGS[config] if isinstance(config, str) else config
    if overrides:
        spec = replace(spec, **overrides)
    seed = spec.seed
    topo = np.random.Generator(np.random.Philox(key=[seed, 1]))
    P = spec.n_prompts

    tree_prompt, tree_off, parent = [], [0], []
    own_len, shared_len = [], []
    for p in range(P):
        W = _draw(topo, spec.W)
        L = _draw(topo, spec.L)
        Ls = min(spec.shared_len, L)
        for _ in range(W):
            n = _draw(topo, spec.tree_nodes)
            base = tree_off[-1]
            loc = tree_parents(spec.tree, n, topo)
            parent.extend([-1 if a < 0 else a + base for a in loc])
            tree_off.append(base + n)
            tree_prompt.append(p)
            own_len.append(L - Ls)
            shared_len.append(Ls)
    T, N = len(tree_prompt), len(parent)
    parent = np.asarray(parent, dtype=np.int32)
    tree_off = np.asarray(tree_off, dtype=np.int32)
    tree_prompt = np.asarray(tree_prompt, dtype=np.int32)
    depth = _depths(parent)
    max_depth = int(depth.max())
    max_tree_nodes = int(np.diff(tree_off).max())
    max_prompt_trees = int(np.bincount(tree_prompt, minlength=P).max())
    if W_cap is None:
        # room for every candidate of the widest layer of a prompt to be accepted
        W_cap = max(max_prompt_trees, 16)

    Hq, Hkv, D, V = spec.Hq, spec.Hkv, spec.D, spec.V
    kvr = np.random.Generator(np.random.Philox(key=[seed, 2]))
    k_shared: List[Optional[np.ndarray]] = []
    v_shared: List[Optional[np.ndarray]] = []
    first_tree = {int(p): int(np.argmax(tree_prompt == p)) for p in range(P)}
    for p in range(P):
        Ls = shared_len[first_tree[p]]
        if Ls > 0:
            k_shared.append(_normal_bf16(kvr, (Ls, Hkv, D)))
            v_shared.append(_normal_bf16(kvr, (Ls, Hkv, D)))
        else:
            k_shared.append(None)
            v_shared.append(None)
    k_own = [_normal_bf16(kvr, (own_len[t], Hkv, D)) for t in range(T)]
    v_own = [_normal_bf16(kvr, (own_len[t], Hkv, D)) for t in range(T)]
    q = _normal_bf16(kvr, (N, Hq, D))
    k_tree = _normal_bf16(kvr, (N, Hkv, D))
    v_tree = _normal_bf16(kvr, (N, Hkv, D))

    lr = np.random.Generator(np.random.Philox(key=[seed, 3]))
    logits_p = lr.standard_normal((N, V), dtype=np.float32) * np.float32(spec.logit_std)
    if spec.draft == "noise":
        logits_q = logits_p + lr.standard_normal((N, V), dtype=np.float32) * np.float32(spec.noise_std)
    elif spec.draft == "indep":
        logits_q = lr.standard_normal((N, V), dtype=np.float32) * np.float32(spec.logit_std)
    else:
        raise ValueError(spec.draft)
    logits_q = np.ascontiguousarray(logits_q, dtype=np.float32)

    # draft tokens: token[n] ~ softmax(logits_q[parent[n]]) iid (Gumbel-max draw), optionally restricted to the
    # row's draft_top_k largest logits (a draft model that samples with a top-k cut); roots arbitrary
    tr = np.random.Generator(np.random.Philox(key=[seed, 4]))
    token = np.zeros(N, dtype=np.int32)
    for n in range(N):
        if parent[n] < 0:
            token[n] = int(tr.integers(0, V))
        elif spec.draft_top_k > 0:
            row = logits_q[parent[n]].astype(np.float64)
            best = np.argsort(-row, kind="stable")[:spec.draft_top_k]
            g = tr.gumbel(size=len(best))
            token[n] = int(best[np.argmax(row[best] + g)])
        else:
            g = tr.gumbel(size=V)
            token[n] = int(np.argmax(logits_q[parent[n]].astype(np.float64) + g))
    # stored beam log-likelihoods: only differences within a prompt matter; the draft model's
    # likelihoods track the target's (as the per-token logits do) with a small mismatch
    beam_logp_p = -3.0 * tr.random(T)
    beam_logp_q = beam_logp_p + 0.25 * tr.standard_normal(T) if spec.draft == "noise" else -3.0 * tr.random(T)

    u_accept = uniform01_f32(N, seed, 101)
    u_resid = uniform01_f32(P * (max_depth + 2), seed, 102).reshape(P, max_depth + 2)
    u_fill = uniform01_f32(P * (max_depth + 2) * W_cap, seed, 103).reshape(P, max_depth + 2, W_cap)

    return Workload(
        spec=spec, n_prompts=P, n_trees=T, n_nodes=N,
        tree_prompt=tree_prompt, tree_off=tree_off, parent=parent, token=token,
        max_depth=max_depth, max_tree_nodes=max_tree_nodes, max_prompt_trees=max_prompt_trees,
        own_len=np.asarray(own_len, dtype=np.int32), shared_len=np.asarray(shared_len, dtype=np.int32),
        k_own=k_own, v_own=v_own, k_shared=k_shared, v_shared=v_shared,
        q=q, k_tree=k_tree, v_tree=v_tree,
        logits_p=logits_p, logits_q=logits_q,
        beam_logp_p=beam_logp_p.astype(np.float64), beam_logp_q=beam_logp_q.astype(np.float64),
        u_accept=u_accept, u_resid=u_resid, u_fill=u_fill, W_cap=W_cap,
    )


def algorithmic_bytes(w: Workload, share_prefix: bool = True):
    """Bytes the method must move once: (attention, verify).

    attention = unique prefix K/V tokens + tree K/V + Q + O, all bf16;
    verify    = both fp32 logit arrays once.
    """
    Hkv, Hq, D = w.Hkv, w.Hq, w.D
    tok_bytes = 2 * Hkv * D * 2
    uniq = int(w.own_len.sum())
    first = {}
    for t in range(w.n_trees):
        p = int(w.tree_prompt[t])
        if share_prefix:
            first.setdefault(p, int(w.shared_len[t]))
        else:
            uniq += int(w.shared_len[t])
    uniq += sum(first.values())
    attn = uniq * tok_bytes + w.n_nodes * tok_bytes + 2 * w.n_nodes * Hq * D * 2
    verify = 2 * w.n_nodes * w.V * 4
    return attn, verify
