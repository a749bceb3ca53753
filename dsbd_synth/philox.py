"""Philox4x32-10 counter-based generator (Salmon et al., SC'11), vectorised in numpy.

Used only to produce the uniform draws that are handed, as plain arrays, to both
the CPU oracle and the HIP path, so neither side owns a random-number generator.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)


def philox4x32_10(counter, key):
    """counter: uint32 [n,4]; key: (k0, k1) python ints. Returns uint32 [n,4]."""
    c = np.ascontiguousarray(counter, dtype=np.uint32).astype(np.uint64)
    c0, c1, c2, c3 = c[:, 0], c[:, 1], c[:, 2], c[:, 3]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        n0 = (p1 >> _SH) ^ c1 ^ np.uint64(k0)
        n1 = p1 & _MASK
        n2 = (p0 >> _SH) ^ c3 ^ np.uint64(k1)
        n3 = p0 & _MASK
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=1).astype(np.uint32)


def random_words(n, seed, stream):
    """n uint32 words of stream `stream` under `seed` (key = (seed, stream))."""
    nblk = (n + 3) // 4
    ctr = np.zeros((nblk, 4), dtype=np.uint32)
    idx = np.arange(nblk, dtype=np.uint64)
    ctr[:, 0] = (idx & _MASK).astype(np.uint32)
    ctr[:, 1] = (idx >> _SH).astype(np.uint32)
    return philox4x32_10(ctr, (seed, stream)).reshape(-1)[:n]


def uniform01_f32(n, seed, stream):
    """n float32 uniforms in [0,1): the top 24 bits of each word times 2^-24."""
    w = random_words(n, seed, stream)
    return ((w >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float32)
