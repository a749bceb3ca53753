"""A stand-in for the two language models: next-token logits and attention rows as exact, seeded functions of the
token sequence.

Only an input generator (no part of the method): the multi-iteration loops on both sides ask it for the logits
of the sequences they have built.  Values are sums of four 24-bit uniforms of a counter-based generator keyed by
a hash of the sequence (integer arithmetic up to one final scaling), so they are reproducible bit for bit.
"""
import numpy as np

from .bf16 import f32_to_bf16_bits
from .philox import philox4x32_10

_MASK64 = (1 << 64) - 1


def _seq_key(seq):
    h = 0xCBF29CE484222325                      # FNV-1a over the token ids
    for tok in seq:
        h = ((h ^ (int(tok) + 1)) * 0x100000001B3) & _MASK64
    return h


class SyntheticModels:
    """target: logits ~ std * N(0,1) per (sequence, token); draft: target + noise * N(0,1).
    context_free=True: every sequence gets the logits of the empty one (the same p and q at every step).
    banned > 0: after every sequence about that share of the vocabulary is forbidden (the same tokens in both models,
    another set per sequence; token 0 always stays): their logits are -Inf, as a logit processor leaves them."""

    def __init__(self, V, seed=0, std=3.0, noise=0.5, context_free=False, Hq=4, Hkv=2, D=64, banned=0.0):
        self.V, self.seed, self.std, self.noise, self.context_free = int(V), int(seed), float(std), float(noise), context_free
        self.Hq, self.Hkv, self.D = Hq, Hkv, D
        self.banned = float(banned)

    def _normal(self, seq, stream, n):
        """n approximately normal values (Irwin-Hall of four uniforms, unit variance), float64."""
        h = _seq_key(() if self.context_free and stream < 3 else seq) ^ (self.seed * 0x9E3779B97F4A7C15 & _MASK64)
        ctr = np.zeros((n, 4), dtype=np.uint32)
        ctr[:, 0] = np.arange(n, dtype=np.uint32)
        ctr[:, 1] = stream
        w = philox4x32_10(ctr, (h & 0xFFFFFFFF, h >> 32))
        s = (w >> np.uint32(8)).astype(np.int64).sum(axis=1)
        return (s.astype(np.float64) * 2.0 ** -24 - 2.0) * np.sqrt(3.0)

    def logits(self, seqs):
        """(target [n,V], draft [n,V]) float32 logits after each of the sequences."""
        zp = np.zeros((len(seqs), self.V), dtype=np.float32)
        zq = np.zeros((len(seqs), self.V), dtype=np.float32)
        for i, s in enumerate(seqs):
            a = self.std * self._normal(s, 1, self.V)
            zp[i] = a.astype(np.float32)
            zq[i] = (a + self.noise * self._normal(s, 2, self.V)).astype(np.float32)
            if self.banned > 0.0:
                # (four 24-bit uniforms summed, shifted and scaled as in _normal: their fractional parts are uniform)
                gone = np.mod(self._normal(s, 6, self.V) * 1000.0, 1.0) < self.banned
                gone[0] = False
                zp[i, gone] = -np.inf
                zq[i, gone] = -np.inf
        return zp, zq

    def qkv(self, seqs):
        """bf16 bit patterns: query [n,Hq,D], key [n,Hkv,D], value [n,Hkv,D] of the sequences' last tokens."""
        n = len(seqs)
        q = np.zeros((n, self.Hq, self.D), dtype=np.uint16)
        k = np.zeros((n, self.Hkv, self.D), dtype=np.uint16)
        v = np.zeros((n, self.Hkv, self.D), dtype=np.uint16)
        for i, s in enumerate(seqs):
            q[i] = f32_to_bf16_bits(self._normal(s, 3, self.Hq * self.D).astype(np.float32)).reshape(self.Hq, self.D)
            k[i] = f32_to_bf16_bits(self._normal(s, 4, self.Hkv * self.D).astype(np.float32)).reshape(self.Hkv, self.D)
            v[i] = f32_to_bf16_bits(self._normal(s, 5, self.Hkv * self.D).astype(np.float32)).reshape(self.Hkv, self.D)
        return q, k, v
