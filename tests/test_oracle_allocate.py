"""Pins for the oracle's budget allocator (Alg. 1; objectives Eq. 17, Eq. 18)."""
import itertools
import os

import numpy as np
import pytest

from oracle import xkv_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def ravg_of(w, alloc):
    """Objective of Eq. 17 evaluated from its definition (Eq. 4 per layer)."""
    return float(np.mean([orc.retention_ratio(w_l, n) if n > 0 else 0.0 for w_l, n in zip(w, alloc)]))


def compositions(N, lo, hi):
    ranges = [range(a, b + 1) for a, b in zip(lo, hi)]
    for c in itertools.product(*ranges):
        if sum(c) == N:
            yield c


def exchange_invariant(w, alloc, lo=None, hi=None):
    """No single token moved from one layer to another can raise R_avg
    (marginal gain of the (n+1)-th token = Sort(w)[-(n+1)]/Sum(w), Eq. 21)."""
    L = len(w)
    lo = [0] * L if lo is None else lo
    hi = [len(x) for x in w] if hi is None else hi
    p = [np.sort(np.asarray(x, np.float64))[::-1] / max(float(np.sum(np.asarray(x, np.float64))), 1e-300) for x in w]
    last_taken = [p[l][alloc[l] - 1] for l in range(L) if alloc[l] > lo[l]]
    next_free = [p[l][alloc[l]] for l in range(L) if alloc[l] < hi[l]]
    if not last_taken or not next_free:
        return True
    return min(last_taken) >= max(next_free) - 1e-15


def test_hand_example_from_golden():
    w, cases = [], []
    for line in open(os.path.join(GOLD, "alloc_hand_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        tag, *v = line.split()
        if tag == "w":
            w.append(np.array([float(x) for x in v], np.float32))
        else:
            cases.append((int(v[0]), [int(v[1]), int(v[2])], float(v[3])))
    for N, alloc, ravg in cases:
        got, r = orc.allocate_budgets(w, total_size=N)
        assert got.tolist() == alloc, (N, got)
        assert abs(r - ravg) < 1e-12


@pytest.mark.parametrize("seed", range(8))
def test_exhaustive_optimum(seed):
    r = np.random.default_rng(seed)
    L = int(r.integers(2, 5))
    w = [r.integers(0, 6, size=int(r.integers(2, 8))).astype(np.float32) for _ in range(L)]
    for x in w:
        x[0] = max(x[0], 1.0)                 # no all-zero layer here
    lens = [len(x) for x in w]
    for N in range(0, sum(lens) + 1):
        got, ravg = orc.allocate_budgets(w, total_size=N)
        assert int(got.sum()) == N and all(0 <= g <= t for g, t in zip(got, lens))
        best = max(ravg_of(w, c) for c in compositions(N, [0] * L, lens))
        assert abs(ravg - best) < 1e-12
        assert abs(ravg - ravg_of(w, got)) < 1e-12


@pytest.mark.parametrize("seed", range(4))
def test_exhaustive_optimum_with_floors_and_caps(seed):
    r = np.random.default_rng(100 + seed)
    L = 3
    w = [r.random(int(r.integers(4, 8))).astype(np.float32) for _ in range(L)]
    lens = [len(x) for x in w]
    lo = [int(r.integers(0, 3)) for _ in range(L)]
    hi = [int(r.integers(l + 1, t + 1)) for l, t in zip(lo, lens)]
    for N in range(sum(lo), sum(hi) + 1):
        got, ravg = orc.allocate_budgets(w, total_size=N, min_budget=lo, max_budget=hi)
        assert int(got.sum()) == N and all(a <= g <= b for a, g, b in zip(lo, got, hi))
        best = max(ravg_of(w, c) for c in compositions(N, lo, hi))
        assert abs(ravg - best) < 1e-12
    with pytest.raises(ValueError):
        orc.allocate_budgets(w, total_size=sum(lo) - 1, min_budget=lo, max_budget=hi)
    with pytest.raises(ValueError):
        orc.allocate_budgets(w, total_size=sum(hi) + 1, min_budget=lo, max_budget=hi)


def test_equals_global_sort_of_all_contributions():
    """Taking the N largest normalised values over all layers, ties by (layer,
    rank): a library sort, not the wait-list loop."""
    r = np.random.default_rng(5)
    L, T = 6, 300
    w = [np.round(r.random(T) ** 3, 2).astype(np.float32) for _ in range(L)]     # many ties
    trip = []
    for l in range(L):
        a = np.sort(w[l]).astype(np.float64)
        tot = float(np.add.accumulate(a)[-1])
        pl = a[::-1] / tot
        trip += [(-pl[k], l, k) for k in range(T)]
    trip.sort()
    for N in (0, 1, 57, 600, 1799, 1800):
        cnt = np.zeros(L, dtype=np.int64)
        for _, l, _ in trip[:N]:
            cnt[l] += 1
        got, _ = orc.allocate_budgets(w, total_size=N)
        np.testing.assert_array_equal(got, cnt)
        assert exchange_invariant(w, got)


def test_zipf_closed_form_brackets_the_answer():
    """p_l[r] = (r+1)^-s_l / H_l: the N largest are those above a threshold
    tau, so n_l = floor((tau * H_l)^(-1/s_l)) up to one token at the cut."""
    T, L = 4096, 8
    s = np.linspace(0.6, 1.4, L)
    w = [np.power(np.arange(1, T + 1, dtype=np.float64), -sl).astype(np.float32) for sl in s]
    N = int(0.3 * L * T)
    got, ravg = orc.allocate_budgets(w, total_size=N)
    H = [float(np.sum(x.astype(np.float64))) for x in w]
    lo_t, hi_t = 1e-12, 1.0
    for _ in range(200):                      # bisection on the threshold
        tau = np.sqrt(lo_t * hi_t)
        tot = sum(min(T, int(np.floor((tau * H[l]) ** (-1.0 / s[l])))) for l in range(L))
        if tot > N:
            lo_t = tau
        else:
            hi_t = tau
    closed = [min(T, int(np.floor((hi_t * H[l]) ** (-1.0 / s[l])))) for l in range(L)]
    assert np.all(np.abs(got - np.array(closed)) <= 2), (got, closed)
    assert exchange_invariant(w, got)
    assert got[0] != got[-1]                  # layers differ: the point of the method


def test_zero_layer_and_ties_go_to_lowest_index():
    w = [np.zeros(4, np.float32), np.array([1, 1, 1, 1], np.float32), np.array([2, 2, 2, 2], np.float32)]
    got, r = orc.allocate_budgets(w, total_size=5)
    # layers 1 and 2 both offer 0.25 per token: lowest index first, all of layer 1, then layer 2
    assert got.tolist() == [0, 4, 1]
    got, r = orc.allocate_budgets(w, total_size=9)
    assert got.tolist() == [1, 4, 4] and abs(r - 2.0 / 3.0) < 1e-12
    with pytest.raises(ValueError):
        orc.allocate_budgets([np.array([1.0, -1.0], np.float32)], total_size=1)
    with pytest.raises(ValueError):
        orc.allocate_budgets([np.array([1.0, np.nan], np.float32)], total_size=1)


@pytest.mark.parametrize("seed", range(4))
def test_target_mode_is_smallest_total_reaching_target(seed):
    r = np.random.default_rng(200 + seed)
    L = 3
    w = [r.random(int(r.integers(3, 7))).astype(np.float32) for _ in range(L)]
    lens = [len(x) for x in w]
    prev = -1
    for target in (0.0, 0.2, 0.5, 0.77, 0.95, 1.0):
        got, ravg = orc.allocate_budgets(w, target_ravg=target)
        tot = int(got.sum())
        assert tot >= prev                    # monotone in the target
        prev = tot
        if tot < sum(lens):
            assert ravg >= target - 1e-12
        # brute force: no smaller total reaches the target
        for N in range(0, tot):
            best = max(ravg_of(w, c) for c in compositions(N, [0] * L, lens))
            assert best < target + 1e-12
        # and it agrees with the total-size mode at the size it returns
        same, r2 = orc.allocate_budgets(w, total_size=tot)
        np.testing.assert_array_equal(same, got)
        assert abs(r2 - ravg) < 1e-12
