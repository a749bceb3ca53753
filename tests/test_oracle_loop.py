"""Pins of the multi-iteration oracle loop: its book-keeping against quantities rebuilt from the token sequences
alone (lengths, caches, sequence likelihoods), and the number of steps per iteration against the efficiency
theorem of Section 3.2 in the case where the theorem's acceptance rate is a constant of the two models."""
import numpy as np
import pytest
from scipy.special import log_softmax, softmax

from dsbd_synth import SyntheticModels
from oracle.loop import OracleLoop


def sequence_logp(models, seq, start, which):
    """log-likelihood of seq[start:] given seq[:start] under one of the two models, token by token."""
    total = 0.0
    for i in range(start, len(seq)):
        z = models.logits([seq[:i]])[which][0].astype(np.float64)
        total += log_softmax(z)[seq[i]]
    return total


@pytest.mark.parametrize("kw", [dict(W_L=2, t=-1.0), dict(W_L=0, t=0.6, W_min=1), dict(W_L=3, t=-1.0, top_k=6, top_p=0.8),
                                dict(W_L=2, t=-1.0, keep_one=True)])
def test_loop_bookkeeping_over_iterations(kw):
    m = SyntheticModels(V=40, seed=3, Hq=2, Hkv=1, D=8)
    start = [[(5,), (9,), (11,)], [(2,)]]
    lp = OracleLoop(m, start, W_S=4, gamma=3, W_cap=8, seed=9, **kw)
    lens = [[1] * len(pb) for pb in start]
    for it in range(5):
        before = [list(pb) for pb in lp.beams]
        rec = lp.step()
        ver, nxt = rec["verify"], rec["next"]
        c = 0
        for p, pb in enumerate(lp.beams):
            assert len(pb) == int(nxt["n_next"][p]) >= 1
            if kw.get("keep_one"):
                assert len(pb) == 1
            for s, b in enumerate(pb):
                # every beam grew by the iteration's number of steps, out of one of the input beams
                src = before[p][int(nxt["src_tree"][p, s]) - sum(len(x) for x in before[:p])]
                assert len(b) == len(src) + int(ver["l_last"][p]) and b[:len(src)] == src
                # the stored likelihoods are those of the whole continuation, under the unwarped models
                first = len(start[p][0])
                assert abs(lp.cum_p[p][s] - sequence_logp(m, b, first, 0)) < 1e-9
                assert abs(lp.cum_q[p][s] - sequence_logp(m, b, first, 1)) < 1e-9
                # the cache holds the rows of all tokens but the last, bit for bit
                _, k, v = m.qkv([b[:i + 1] for i in range(len(b) - 1)])
                assert np.array_equal(lp.k_cache[c], k) and np.array_equal(lp.v_cache[c], v)
                c += 1
        assert c == len(lp.k_cache)


def test_loop_is_reproducible():
    m = SyntheticModels(V=30, seed=1)
    a = OracleLoop(m, [[(1,), (2,)]], W_S=3, gamma=2, W_L=2, W_cap=4, seed=4, with_kv=False)
    b = OracleLoop(m, [[(1,), (2,)]], W_S=3, gamma=2, W_L=2, W_cap=4, seed=4, with_kv=False)
    for _ in range(4):
        a.step(); b.step()
    assert a.beams == b.beams and a.cum_p == b.cum_p


@pytest.mark.parametrize("gamma,noise", [(4, 0.8), (2, 1.5)])
def test_steps_per_iteration_follow_the_efficiency_theorem(gamma, noise):
    """One beam, one draft per layer, the same two distributions at every step: a layer is accepted with the
    constant probability alpha = sum min(p, q), and the expected number of steps per iteration is
    (1 - alpha^(gamma+1)) / (1 - alpha)."""
    m = SyntheticModels(V=12, seed=2, std=1.5, noise=noise, context_free=True)
    zp, zq = m.logits([()])
    alpha = float(np.minimum(softmax(zp[0].astype(np.float64)), softmax(zq[0].astype(np.float64))).sum())
    want = (1 - alpha ** (gamma + 1)) / (1 - alpha)
    lp = OracleLoop(m, [[(0,)]], W_S=1, gamma=gamma, W_L=1, W_cap=2, seed=21, with_kv=False)
    n = 4000
    steps = np.array([int(lp.step()["verify"]["l_last"][0]) for _ in range(n)])
    assert 1 <= steps.min() and steps.max() <= gamma + 1
    assert abs(steps.mean() - want) <= 4.5 * steps.std() / np.sqrt(n)
    # and the number of accepted layers is geometric, cut at gamma
    for k in range(gamma):
        pk = alpha ** k * (1 - alpha)
        assert abs((steps == k + 1).mean() - pk) <= 4.5 * np.sqrt(pk * (1 - pk) / n) + 1e-3


@pytest.mark.parametrize("kw", [dict(W_L=2, t=-1.0), dict(W_L=0, t=0.6, W_min=1), dict(W_L=3, t=-1.0, top_k=6, top_p=0.8)])
def test_banned_tokens_never_enter_a_beam(kw):
    """Models that forbid half of the vocabulary after every sequence (logits of -Inf): no beam ever continues with
    a forbidden token, and the stored likelihoods stay those of the sequences."""
    m = SyntheticModels(V=40, seed=3, Hq=2, Hkv=1, D=8, banned=0.5)
    start = [[(5,), (9,)], [(2,)]]
    with np.errstate(all="ignore"):
        lp = OracleLoop(m, start, W_S=4, gamma=3, W_cap=8, seed=9, with_kv=False, **kw)
        for it in range(5):
            lp.step()
    grown = 0
    for p, pb in enumerate(lp.beams):
        for s, b in enumerate(pb):
            for i in range(1, len(b)):
                assert np.isfinite(m.logits([b[:i]])[0][0, b[i]]), (p, s, i)
            grown += len(b) - 1
            with np.errstate(all="ignore"):
                assert abs(lp.cum_p[p][s] - sequence_logp(m, b, 1, 0)) < 1e-9
    assert grown > 10
