"""Input generators: Philox known answers, bf16 packing, workload shapes and byte counts."""
import os

import numpy as np

from dsbd_synth import bf16_bits_to_f32, f32_to_bf16_bits, make_workload, philox4x32_10, uniform01_f32
from dsbd_synth.workloads import algorithmic_bytes, tree_parents

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = philox4x32_10(np.array([v[0:4]], dtype=np.uint32), (v[4], v[5]))[0]
        assert [int(x) for x in out] == v[6:10]


def test_uniform_range_and_determinism():
    a = uniform01_f32(100003, 0, 7)
    b = uniform01_f32(100003, 0, 7)
    c = uniform01_f32(100003, 0, 8)
    assert a.dtype == np.float32 and (a >= 0).all() and (a < 1).all()
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert abs(float(a.mean()) - 0.5) < 0.01
    # 24-bit grid
    assert np.all(a * np.float32(2 ** 24) == np.round(a * np.float32(2 ** 24)))


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, -2.5, 3.140625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -9], dtype=np.float32)
    bits = f32_to_bf16_bits(x)
    y = bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: rounds to even (1.0); 1 + 3*2^-9 rounds up to 1 + 2^-7
    assert y.tolist() == [1.0, -2.5, 3.140625, 1.0, 1.0 + 2 ** -7]
    r = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    assert np.max(np.abs(bf16_bits_to_f32(f32_to_bf16_bits(r)) - r) / np.abs(r)) <= 2 ** -8


def test_tree_shapes():
    assert tree_parents("chain", 3, None) == [-1, 0, 1]
    assert tree_parents("fork_chain", 7, None) == [-1, 0, 0, 1, 2, 3, 4]
    assert tree_parents("fork_chain", 2, None) == [-1, 0] and tree_parents("fork_chain", 1, None) == [-1]
    assert tree_parents("binary_bfs", 7, None) == [-1, 0, 0, 1, 1, 2, 2]
    assert tree_parents("binary_dfs", 7, None) == [-1, 0, 1, 1, 0, 4, 4]


def test_small_configs_shapes_and_bytes():
    w = make_workload("c1")
    assert (w.n_trees, w.n_nodes, w.max_depth) == (2, 6, 2)
    assert algorithmic_bytes(w) == (77824, 12288)
    w = make_workload("c2")
    assert (w.n_trees, w.n_nodes, w.max_depth, w.max_tree_nodes) == (4, 28, 3, 7)
    a, v = algorithmic_bytes(w)
    assert v == 2 * 28 * 32000 * 4 and a == 4 * 512 * 16384 + 28 * 16384 + 2 * 28 * 32 * 128 * 2
    assert w.q.dtype == np.uint16 and w.logits_p.dtype == np.float32
    assert (w.token >= 0).all() and (w.token < w.V).all()


def test_scaled_down_variants_keep_structure():
    w = make_workload("c5", L=96, V=1000)
    assert w.n_nodes == 248 and w.Hq == 32 and w.Hkv == 8 and w.max_depth == 4
    assert all(k.shape == (96, 8, 128) for k in w.k_own)
    w = make_workload("c3", L=64, shared_len=24, V=500)
    assert w.shared_len.tolist() == [24] * 8 and w.own_len.tolist() == [40] * 8
    assert w.k_shared[0].shape == (24, 32, 128)
    w = make_workload("c4", L=(16, 48), V=300)
    assert w.n_prompts == 16 and 16 <= w.n_trees <= 128
    assert np.all(np.diff(w.tree_prompt) >= 0)


def test_synthetic_models_are_functions_of_the_sequence_and_ban_the_same_tokens_in_both():
    from dsbd_synth import SyntheticModels
    m = SyntheticModels(V=500, seed=7, banned=0.4)
    zp, zq = m.logits([(1, 2, 3), (4,), (1, 2, 3)])
    assert np.array_equal(zp[0], zp[2]) and np.array_equal(zq[0], zq[2])          # same sequence, same logits
    gone = np.isneginf(zp)
    assert np.array_equal(gone, np.isneginf(zq)) and not gone[:, 0].any()
    assert 0.3 < gone.mean() < 0.5 and (gone[0] != gone[1]).any()                   # another set per sequence
    assert np.isfinite(zp[~gone]).all() and np.isfinite(zq[~gone]).all()
    plain = SyntheticModels(V=500, seed=7)
    zp0, zq0 = plain.logits([(1, 2, 3)])
    assert np.array_equal(zp0[0][~gone[0]], zp[0][~gone[0]])                      # banning changes nothing else
