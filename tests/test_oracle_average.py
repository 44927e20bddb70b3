"""Pins for the oracle's averaged allocation list (Sec. 4.3)."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import xkv_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))
SAMPLES = np.array([[10, 5, 3, 2], [8, 6, 4, 2], [9, 4, 4, 3]])


def test_hand_example():
    for line in open(os.path.join(HERE, "golden", "average_allocations_hand_example.txt")):
        if line.startswith("total"):
            left, right = line.split("->")
            total = int(left.split()[1])
            assert orc.average_allocations(SAMPLES, total).tolist() == [int(v) for v in right.split()]


def test_identical_samples_come_back_unchanged():
    one = np.array([[7, 0, 12, 1]])
    assert orc.average_allocations(np.repeat(one, 5, axis=0), 20).tolist() == [7, 0, 12, 1]


@pytest.mark.parametrize("seed", range(8))
def test_rounding_is_the_closest_integer_list(seed):
    """Largest-remainder rounding minimises the distance to the exact averages
    among all integer lists with the right total (brute force on tiny cases)."""
    r = np.random.default_rng(seed)
    L, S = 4, int(r.integers(1, 5))
    lists = r.integers(0, 6, size=(S, L))
    if lists.sum() == 0:
        lists[0, 0] = 1
    N = int(r.integers(0, 15))
    got = orc.average_allocations(lists, N)
    assert got.sum() == N and np.all(got >= 0)
    col = lists.sum(axis=0)
    x = [Fraction(int(c) * N, int(col.sum())) for c in col]
    dist = lambda n: sum(abs(Fraction(int(a)) - b) for a, b in zip(n, x))
    best = min(dist(n) for n in itertools.product(range(N + 1), repeat=L) if sum(n) == N)
    assert dist(got) == best
    assert all(abs(Fraction(int(a)) - b) < 1 for a, b in zip(got, x))


def test_bounds_are_met_and_total_kept():
    lists = np.array([[50, 30, 15, 5], [40, 40, 10, 10]])
    got = orc.average_allocations(lists, 100, min_budget=[0, 0, 20, 8], max_budget=[40, 100, 100, 100])
    assert got.sum() == 100 and got[0] <= 40 and got[2] >= 20 and got[3] >= 8
    # averages 45 35 12.5 7.5: layer 0 loses 5 to its cap, layers 2 and 3 are lifted to their
    # floors (+7.5, +0.5), so 3 tokens too many: they come off layer 1, the only one above its target
    assert got.tolist() == [40, 32, 20, 8]
    with pytest.raises(ValueError):
        orc.average_allocations(lists, 10, min_budget=[5, 5, 5, 5])
    with pytest.raises(ValueError):
        orc.average_allocations(np.zeros((2, 3), int), 4)
