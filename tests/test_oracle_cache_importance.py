"""Pins for the oracle's cache_importance (the per-layer score vector taken from the
decode-time cache).  None of them repeats its loop: a hand-worked fixture, the
dense special case (a library column sum), conservation of mass in exact
arithmetic, invariance under the order of slots, and agreement with the
separately pinned prefill functions on a cache that has not evicted anything."""
import os

import numpy as np
import pytest

from oracle import xkv_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _fixture():
    heads, rows = [], {}
    for line in open(os.path.join(HERE, "golden", "cache_importance_hand_example.txt")):
        if line.startswith("head"):
            toks = [t.split(":") for t in line.split(":", 1)[1].split()]
            heads.append((np.array([int(a) for a, _ in toks]), np.array([float(b) for _, b in toks], np.float32)))
        elif line.startswith("w"):
            name, vals = line.split(":")
            rows[name] = np.array([float(v) for v in vals.split()], np.float32)
    return heads, rows


def test_hand_example():
    heads, rows = _fixture()
    pos, score = [h[0] for h in heads], [h[1] for h in heads]
    assert np.array_equal(orc.cache_importance(pos, score, 6), rows["w"])
    assert np.array_equal(orc.cache_importance(pos, score, 4), rows["w4"])


def test_dense_cache_is_the_column_sum():
    """Nothing evicted, slot = position: the vector is the sum of the heads' score
    rows.  Scores are small integers times 2^-6, so every order of adding is exact."""
    r = np.random.default_rng(0)
    H, n = 5, 300
    sc = (r.integers(0, 64, size=(H, n)) / 64.0).astype(np.float32)
    w = orc.cache_importance([np.arange(n)] * H, list(sc), n)
    assert np.array_equal(w, sc.sum(axis=0, dtype=np.float64).astype(np.float32))


@pytest.mark.parametrize("seed", range(6))
def test_mass_is_conserved_and_slot_order_does_not_matter(seed):
    r = np.random.default_rng(seed)
    H, n_pos = int(r.integers(1, 6)), int(r.integers(1, 200))
    pos, score = [], []
    for _ in range(H):
        k = int(r.integers(0, n_pos + 1))
        pos.append(r.permutation(n_pos)[:k])
        score.append((r.integers(0, 1024, size=k) / 1024.0).astype(np.float32))
    w = orc.cache_importance(pos, score, n_pos)
    assert w.shape == (n_pos,) and w.dtype == np.float32
    total = sum(float(s.astype(np.float64).sum()) for s in score)
    assert float(w.astype(np.float64).sum()) == total            # exact: dyadic values
    held = np.zeros(n_pos, bool)
    for p in pos:
        held[p] = True
    assert not w[~held].any()                                    # positions no head holds
    shuffled_pos, shuffled_score = [], []
    for p, s in zip(pos, score):
        perm = r.permutation(p.size)
        shuffled_pos.append(p[perm])
        shuffled_score.append(s[perm])
    assert np.array_equal(orc.cache_importance(shuffled_pos, shuffled_score, n_pos), w)


def test_positions_outside_the_range_are_left_out_and_duplicates_refused():
    w = orc.cache_importance([np.array([-1, 0, 7, 3])], [np.array([9.0, 1.0, 9.0, 2.0], np.float32)], 4)
    assert w.tolist() == [1.0, 0.0, 0.0, 2.0]
    with pytest.raises(ValueError):
        orc.cache_importance([np.array([2, 2])], [np.array([1.0, 1.0], np.float32)], 4)


def test_agrees_with_the_prefill_functions_before_any_eviction():
    """A cache filled by the prefill-phase eviction with a budget that keeps every
    token holds, per head, score = the window's mass on each position.  Its
    position-indexed vector must then be the head-merged mass vector that
    window_importance (pool 1) returns for the candidates."""
    r = np.random.default_rng(3)
    Hkv, G, ows, d, t = 3, 2, 4, 16, 40
    q_win = r.standard_normal((Hkv, G, ows, d)).astype(np.float32)
    K = r.standard_normal((Hkv, t, d)).astype(np.float32)
    V = r.standard_normal((Hkv, t, d)).astype(np.float32)
    pos, score = [], []
    for h in range(Hkv):
        _, _, s, p, _ = orc.prefill_evict(q_win[h], K[h], V[h], budget=t, ows=ows)
        pos.append(p)
        score.append(s)
    w = orc.cache_importance(pos, score, t)
    ref = orc.window_importance(q_win, K, pool_size=1)
    assert np.max(np.abs(w[:t - ows].astype(np.float64) - ref)) <= 1e-6 * np.max(ref)
