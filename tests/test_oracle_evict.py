"""Pins for the oracle's pooling, top-k selection and hole-fill compaction
(Alg. 2 steps 4-7)."""
import itertools

import numpy as np
import pytest

from oracle import xkv_oracle as orc


def _unit(n, d, seed, ties=False):
    r = np.random.default_rng(seed)
    K = r.standard_normal((n, d)).astype(np.float32)
    V = r.standard_normal((n, d)).astype(np.float32)
    if ties:
        score = r.integers(0, 4, size=n).astype(np.float32) * 0.25
    else:
        score = r.random(n).astype(np.float32)
    pos = r.permutation(n + 5)[:n].astype(np.int32)
    return K, V, score, pos


# ---- selection ------------------------------------------------------------
def test_hand_cases():
    # keys 0.5 0.1 0.5 0.3, keep 2 -> slots 0 and 2; keep 3 -> plus slot 3
    s = np.array([0.5, 0.1, 0.5, 0.3], np.float32)
    p = np.arange(4, dtype=np.int32)
    assert orc.select_keep(s, p, 2).tolist() == [0, 2]
    assert orc.select_keep(s, p, 3).tolist() == [0, 2, 3]
    # a tie at the cut goes to the lower slot
    s = np.array([0.2, 0.7, 0.2, 0.2], np.float32)
    assert orc.select_keep(s, p, 2).tolist() == [0, 1]
    assert orc.select_keep(s, p, 3).tolist() == [0, 1, 2]
    # all equal -> the first k slots
    assert orc.select_keep(np.ones(6, np.float32), np.arange(6), 4).tolist() == [0, 1, 2, 3]
    # k >= n keeps everything, k = 0 nothing
    assert orc.select_keep(s, p, 9).tolist() == [0, 1, 2, 3]
    assert orc.select_keep(s, p, 0).tolist() == []


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_over_all_subsets(seed):
    """Among all C(n, k) subsets, the kept set has the largest key sum and is,
    among those, the lexicographically smallest index tuple."""
    r = np.random.default_rng(seed)
    n = int(r.integers(4, 10))
    k = int(r.integers(1, n))
    score = (r.integers(0, 5, size=n) * 0.125).astype(np.float32)      # many ties, exact sums
    best = None
    for comb in itertools.combinations(range(n), k):
        tot = float(np.sum(score[list(comb)].astype(np.float64)))
        cand = (-tot, comb)
        if best is None or cand < best:
            best = cand
    assert tuple(orc.select_keep(score, np.arange(n), k).tolist()) == best[1]


@pytest.mark.parametrize("ties", [False, True])
def test_threshold_invariant(ties):
    K, V, score, pos = _unit(500, 4, 11, ties)
    for k in (1, 7, 250, 499):
        keep = orc.select_keep(score, pos, k)
        assert keep.size == k and np.all(np.diff(keep) > 0)
        ev = np.setdiff1d(np.arange(500), keep)
        lo, hi = score[keep].min(), score[ev].max()
        assert lo >= hi
        if lo == hi:   # equal keys: every kept one has a lower slot than every evicted one
            assert keep[score[keep] == lo].max() < ev[score[ev] == hi].min()


def test_protected_window():
    K, V, score, pos = _unit(64, 4, 12)
    pos = np.random.default_rng(0).permutation(64).astype(np.int32)
    score[:] = np.linspace(1.0, 2.0, 64)
    recent = np.flatnonzero(pos >= 64 - 8)
    score[recent] = 0.0                       # lowest scores, but inside the window
    keep = orc.select_keep(score, pos, 20, n_protect=8)
    assert set(recent.tolist()) <= set(keep.tolist())
    rest = np.setdiff1d(keep, recent)
    others = np.setdiff1d(np.arange(64), recent)
    top = others[np.argsort(-score[others], kind="stable")[:12]]
    assert sorted(rest.tolist()) == sorted(top.tolist())


# ---- pooling --------------------------------------------------------------
def test_pooling_identity_constant_and_convolve():
    s = np.random.default_rng(1).random(100).astype(np.float32)
    np.testing.assert_array_equal(orc.pooled_keys(s, 1), s)
    c = np.full(20, 0.5, np.float32)
    key = orc.pooled_keys(c, 7)
    assert np.all(key[3:-3] == 3.5)
    assert key[0] == 2.0 and key[1] == 2.5 and key[2] == 3.0 and key[-1] == 2.0
    for ps in (3, 7, 9):
        ref = np.convolve(s.astype(np.float64), np.ones(ps), "same")
        np.testing.assert_allclose(orc.pooled_keys(s, ps), ref, rtol=1e-6)
    with pytest.raises(ValueError):
        orc.pooled_keys(s, 4)


def test_pooling_order_is_left_to_right_fp32():
    s = np.array([1.0, 2.0 ** -24, 2.0 ** -24, 0.0], np.float32)
    # window of slot 1: (1 + 2^-24) + 2^-24 in fp32 = 1 (each add rounds to even),
    # whereas right-to-left would give 1 + 2^-23.
    assert orc.pooled_keys(s, 3)[1] == np.float32(1.0)
    # window of slot 2: (2^-24 + 2^-24) + 0 is exact
    assert orc.pooled_keys(s, 3)[2] == np.float32(2.0 ** -23)


def test_pooling_changes_selection():
    s = np.zeros(16, np.float32)
    s[5] = 1.0
    s[12] = 0.9
    s[11] = 0.2
    p = np.arange(16, dtype=np.int32)
    assert orc.select_keep(s, p, 3, pool_size=1).tolist() == [5, 11, 12]
    # width 3: keys at 10..13 = 0.2, 1.1, 1.1, 0.9 ; at 4..6 = 1, 1, 1
    assert orc.select_keep(s, p, 3, pool_size=3).tolist() == [4, 11, 12]


# ---- compaction -----------------------------------------------------------
@pytest.mark.parametrize("n,k", [(10, 4), (10, 9), (100, 50), (257, 1), (64, 64), (64, 100), (5, 0)])
def test_hole_fill_properties(n, k):
    K, V, score, pos = _unit(n, 8, 20 + n + k, ties=True)
    keep = orc.select_keep(score, pos, k)
    K2, V2, s2, p2, kept_idx = orc.evict_compact(K, V, score, pos, k)
    kk = min(k, n)
    assert K2.shape[0] == kk == kept_idx.shape[0]
    # the same set of tokens survives
    assert sorted(kept_idx.tolist()) == keep.tolist()
    assert sorted(p2.tolist()) == sorted(pos[keep].tolist())
    # every row carries its K, V, score, pos together
    np.testing.assert_array_equal(K2, K[kept_idx])
    np.testing.assert_array_equal(V2, V[kept_idx])
    np.testing.assert_array_equal(s2, score[kept_idx])
    np.testing.assert_array_equal(p2, pos[kept_idx])
    # a kept token below k' never moves; movers come from >= k' in ascending order
    moved = np.flatnonzero(kept_idx != np.arange(kk))
    assert np.all(kept_idx[moved] >= kk)
    assert np.all(np.diff(kept_idx[moved]) > 0)
    assert moved.size <= min(kk, n - kk)
    for s in range(kk):
        if s in set(keep.tolist()):
            assert kept_idx[s] == s


def test_steady_state_moves_at_most_one_row():
    K, V, score, pos = _unit(33, 8, 40)
    score[7] = -0.0 + 0.0
    score[7] = 0.0                            # slot 7 is the minimum
    _, _, _, _, kept_idx = orc.evict_compact(K, V, score, pos, 32)
    assert kept_idx[7] == 32 and np.count_nonzero(kept_idx != np.arange(32)) == 1
    score[:] = 1.0
    score[32] = 0.0                           # the newest token is the minimum: nothing moves
    _, _, _, _, kept_idx = orc.evict_compact(K, V, score, pos, 32)
    np.testing.assert_array_equal(kept_idx, np.arange(32))


def test_retention_ratio_eq4():
    w = np.random.default_rng(2).random(50)
    r = [orc.retention_ratio(w, n) for n in range(51)]
    assert r[0] == 0.0 and abs(r[50] - 1.0) < 1e-15
    d = np.diff(r)
    assert np.all(d >= 0) and np.all(np.diff(d) <= 1e-15)      # non-decreasing, concave
    assert abs(r[3] - (np.sort(w)[-3:].sum() / w.sum())) < 1e-15
