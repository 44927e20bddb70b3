"""Pins for the oracle's prefill-phase eviction (Alg. 2 as written, Sec. 4.1):
checked against a full causal attention matrix built independently, closed
forms, the already pinned decode function, invariants and brute force."""
import itertools

import numpy as np
import pytest
from scipy.special import softmax

from oracle import xkv_oracle as orc


def full_causal_attention(Q, K, scale):
    """W_attn of Eq. 2 for a whole prompt: t x t, row i sees columns 0..i."""
    t = K.shape[0]
    S = scale * (Q @ K.T)
    S[np.triu_indices(t, k=1)] = -np.inf
    return softmax(S, axis=1)


@pytest.mark.parametrize("t,ows,G,d", [(9, 3, 1, 4), (20, 8, 2, 8), (33, 1, 4, 16), (12, 12, 1, 4)])
def test_mass_is_select_and_merge_of_the_full_matrix(t, ows, G, d):
    """The attention processing module: t x t matrix, last ows rows, first
    t - ows columns, merged over rows (and heads)."""
    r = np.random.default_rng(t * 100 + ows)
    Q = r.normal(size=(G, t, d))
    K = r.normal(size=(t, d))
    scale = 1.0 / np.sqrt(d)
    w = orc.window_attention_mass(Q[:, t - ows:, :].astype(np.float32), K.astype(np.float32), scale)
    Qf, Kf = Q.astype(np.float32).astype(np.float64), K.astype(np.float32).astype(np.float64)
    ref = np.zeros(t)
    for g in range(G):
        W = full_causal_attention(Qf[g], Kf, scale)
        block = W[t - ows:, :]                     # Select the window rows
        ref += block.sum(axis=0)                   # Merge
    assert np.allclose(w, ref, rtol=1e-12, atol=1e-15)
    assert abs(w.sum() - G * ows) < 1e-9           # every row of W_attn sums to one
    # nothing after a row's own position: the last column only hears the last row
    W_last = sum(full_causal_attention(Qf[g], Kf, scale)[t - 1, t - 1] for g in range(G))
    assert abs(w[t - 1] - W_last) < 1e-12


def test_uniform_keys_closed_form():
    """Equal keys give uniform rows: row r spreads 1 over t - ows + r + 1 columns."""
    t, ows, d = 10, 4, 4
    K = np.ones((t, d), np.float32)
    q = np.random.default_rng(0).normal(size=(1, ows, d)).astype(np.float32)
    w = orc.window_attention_mass(q, K)
    for j in range(t):
        expect = sum(1.0 / (t - ows + r + 1) for r in range(ows) if j <= t - ows + r)
        assert abs(w[j] - expect) < 1e-12


def test_hand_example_two_rows():
    """t = 3, ows = 2, d = 1, scale 1, keys (0, ln 2, ln 3), queries 1 and 1:
    row 0 sees e^0 : e^ln2 = 1 : 2, row 1 sees 1 : 2 : 3."""
    K = np.array([[0.0], [np.log(2.0)], [np.log(3.0)]])
    q = np.ones((1, 2, 1))
    w = orc.window_attention_mass(q, K, scale=1.0)
    assert np.allclose(w, [1 / 3 + 1 / 6, 2 / 3 + 2 / 6, 3 / 6], atol=1e-15)


def test_single_row_window_is_the_decode_probability():
    """ows = 1: the window row is a decode query over the whole prompt."""
    r = np.random.default_rng(5)
    t, d, G = 40, 8, 2
    K = r.normal(size=(t, d)).astype(np.float32)
    q = r.normal(size=(G, d)).astype(np.float32)
    _, _, p = orc.attend_score(q, K, K, np.zeros(t, np.float32))
    w = orc.window_attention_mass(q[:, None, :], K)
    assert np.allclose(w, p.sum(axis=0), rtol=1e-13)


def brute_force_selection(key, m):
    """The m-subset with the largest key sum; among equals the lexicographically
    smallest index tuple (what "equal keys by lower position" means)."""
    best, best_sum = None, None
    for c in itertools.combinations(range(len(key)), m):
        s = float(np.sum(key[list(c)].astype(np.float64)))
        if best is None or s > best_sum + 1e-300 or (s == best_sum and c < best):
            best, best_sum = c, s
    return np.array(best, dtype=np.int64)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("ps", [1, 3])
def test_selection_against_exhaustive_search(seed, ps):
    r = np.random.default_rng(seed)
    t, ows, budget = 11, 3, 7
    w = (r.integers(0, 5, size=t) * 0.25).astype(np.float32) if seed % 2 else r.random(t).astype(np.float32)
    keep = orc.prefill_select(w, ows, budget, ps)
    tc = t - ows
    assert np.array_equal(keep[-ows:], np.arange(tc, t))           # the window is always kept
    key = orc.pooled_keys(w[:tc], ps)
    # keys here are multiples of 2^-k or generic: the fp64 sums of the search are exact enough
    assert np.array_equal(keep[:-ows], brute_force_selection(key, budget - ows))
    assert len(keep) == budget and np.all(np.diff(keep) > 0)


def test_window_never_leaks_into_candidate_keys():
    """Pooling runs on the candidate vector alone: a huge window mass next to the
    boundary must not lift the last candidate."""
    w = np.array([0.3, 0.2, 0.1, 0.05, 100.0, 100.0], np.float32)   # ows = 2
    keep = orc.prefill_select(w, 2, 3, pool_size=3)
    # pooled candidates: [0.5, 0.6, 0.35, 0.15] -> position 1
    assert keep.tolist() == [1, 4, 5]


def test_budget_rules():
    w = np.arange(8, dtype=np.float32)
    assert orc.prefill_select(w, 2, 100).tolist() == list(range(8))      # budget >= t keeps all
    assert orc.prefill_select(w, 2, 2).tolist() == [6, 7]                # only the window
    with pytest.raises(ValueError):
        orc.prefill_select(w, 3, 2)


def test_evict_gathers_rows_scores_and_positions():
    r = np.random.default_rng(11)
    t, d, ows, budget = 30, 8, 4, 12
    K = r.normal(size=(t, d)).astype(np.float32)
    V = r.normal(size=(t, d)).astype(np.float32)
    q = r.normal(size=(2, ows, d)).astype(np.float32)
    K2, V2, s2, p2, w = orc.prefill_evict(q, K, V, budget, ows, pool_size=7)
    assert w.dtype == np.float32 and len(p2) == budget and np.all(np.diff(p2) > 0)
    assert np.array_equal(K2, K[p2]) and np.array_equal(V2, V[p2]) and np.array_equal(s2, w[p2])
    # the kept candidates carry at least as much pooled mass as any evicted one
    key = orc.pooled_keys(w[:t - ows], 7)
    kept_c = p2[:-ows]
    evicted = np.setdiff1d(np.arange(t - ows), kept_c)
    assert key[kept_c].min() >= key[evicted].max()
    # a caller-supplied mass vector replaces the function's own
    w_alt = w.copy()
    w_alt[:5] = 9.0
    _, _, _, p3, _ = orc.prefill_evict(q, K, V, budget, ows, pool_size=1, w=w_alt)
    assert set(range(5)) <= set(p3.tolist())


def test_window_importance_merges_heads_then_pools():
    """Against the full causal matrices of every head and a convolution with ones."""
    r = np.random.default_rng(21)
    Hkv, G, t, ows, d, ps = 3, 2, 26, 4, 8, 5
    Q = r.normal(size=(Hkv, G, t, d)).astype(np.float32)
    K = r.normal(size=(Hkv, t, d)).astype(np.float32)
    got = orc.window_importance(Q[:, :, t - ows:, :], K, ps)
    scale = 1.0 / np.sqrt(d)
    merged = np.zeros(t - ows)
    for h in range(Hkv):
        for g in range(G):
            W = full_causal_attention(Q[h, g].astype(np.float64), K[h].astype(np.float64), scale)
            merged += W[t - ows:, :t - ows].sum(axis=0)
    ref = np.convolve(merged, np.ones(ps), mode="same")        # zero padding, same length
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-15)
    # without pooling the vector carries everything the windows did not spend on themselves
    w1 = orc.window_importance(Q[:, :, t - ows:, :], K, 1)
    own = sum(orc.window_attention_mass(Q[h, :, t - ows:, :], K[h])[t - ows:].sum() for h in range(Hkv))
    assert abs(w1.sum() + own - Hkv * G * ows) < 1e-9


# ---- the window rows' normalisers (Eq. 2), for callers that already hold them ----

@pytest.mark.parametrize("t,ows,G,d", [(9, 3, 1, 4), (20, 8, 2, 8), (33, 1, 4, 16), (12, 12, 1, 4)])
def test_row_lse_against_the_full_logit_matrix(t, ows, G, d):
    """lse of window row r = logsumexp of row t - ows + r of the causally masked
    t x t logit matrix, built independently and reduced with SciPy's routine."""
    from scipy.special import logsumexp
    r = np.random.default_rng(t * 7 + ows)
    Q = r.normal(size=(G, t, d)).astype(np.float32)
    K = (3.0 * r.normal(size=(t, d))).astype(np.float32)
    scale = 0.37
    lse = orc.window_row_lse(Q[:, t - ows:, :], K, scale)
    for g in range(G):
        S = scale * (Q[g].astype(np.float64) @ K.astype(np.float64).T)
        S[np.triu_indices(t, k=1)] = -np.inf
        assert np.allclose(lse[g], logsumexp(S[t - ows:], axis=1), rtol=1e-13, atol=1e-13)


def test_row_lse_closed_forms():
    """Zero keys: every logit is 0 and row r sees t - ows + r + 1 of them.  And the
    hand example (keys 0, ln 2, ln 3; queries 1): normalisers 3 and 6."""
    t, ows, d = 10, 4, 4
    q = np.random.default_rng(1).normal(size=(2, ows, d)).astype(np.float32)
    lse = orc.window_row_lse(q, np.zeros((t, d), np.float32))
    assert np.allclose(lse, np.log(np.arange(t - ows + 1, t + 1))[None, :].repeat(2, 0), atol=1e-15)
    K = np.array([[0.0], [np.log(2.0)], [np.log(3.0)]])
    assert np.allclose(orc.window_row_lse(np.ones((1, 2, 1)), K, scale=1.0), [[np.log(3.0), np.log(6.0)]], atol=1e-15)


def test_mass_with_given_normalisers():
    """With the rows' own lse the masses are the softmax masses; with every lse
    raised by ln 2 they are halved (the given normaliser is used as it is); and a
    large common shift of the logits changes nothing (no overflow in lse)."""
    r = np.random.default_rng(9)
    G, ows, t, d = 2, 5, 60, 8
    q = r.normal(size=(G, ows, d)).astype(np.float32)
    K = r.normal(size=(t, d)).astype(np.float32)
    w = orc.window_attention_mass(q, K)
    lse = orc.window_row_lse(q, K)
    assert np.allclose(orc.window_attention_mass(q, K, lse=lse), w, rtol=1e-12, atol=1e-16)
    assert np.allclose(orc.window_attention_mass(q, K, lse=lse + np.log(2.0)), 0.5 * w, rtol=1e-12, atol=1e-16)
    big = orc.window_row_lse(1000.0 * q, K, scale=1.0)
    assert np.all(np.isfinite(big))
    with pytest.raises(ValueError):
        orc.window_attention_mass(q, K, lse=lse[:, :2])
