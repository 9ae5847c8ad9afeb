"""Pins of the replica-balancing oracle."""
import heapq
import itertools
from fractions import Fraction

import numpy as np
import pytest

from oracle import plan as oplan
from oracle import replicas as orep


def test_two_way_differencing_worked_example():
    # the classic illustration of the differencing method: 8 7 6 5 4 -> {8, 6} and {7, 5, 4}, difference 2
    rep, sums = orep.karmarkar_karp([8, 7, 6, 5, 4], 2)
    assert sorted(sums) == [14, 16]
    groups = [sorted(v for v, r in zip([8, 7, 6, 5, 4], rep) if r == k) for k in range(2)]
    assert sorted(groups) == [[4, 5, 7], [6, 8]]


def _numbers_only_difference(t):
    # the two-way method on bare numbers: replace the two largest by their difference until one is left
    h = [-x for x in t]
    heapq.heapify(h)
    while len(h) > 1:
        a, b = -heapq.heappop(h), -heapq.heappop(h)
        heapq.heappush(h, -(a - b))
    return -h[0] if h else 0


@pytest.mark.parametrize("seed", range(20))
def test_two_way_set_bookkeeping_matches_bare_numbers(seed):
    rng = np.random.default_rng(seed)
    t = [int(x) for x in rng.integers(1, 1000, int(rng.integers(1, 30)))]
    rep, sums = orep.karmarkar_karp(t, 2)
    assert abs(sums[0] - sums[1]) == _numbers_only_difference(t)
    assert sums[0] + sums[1] == sum(t)
    assert abs(sums[0] - sums[1]) <= max(t)                 # the method's guarantee for two sets


def _optimum(t, k):
    best = None
    for assign in itertools.product(range(k), repeat=len(t)):
        s = [0] * k
        for x, r in zip(t, assign):
            s[r] += x
        m = max(s)
        best = m if best is None else min(best, m)
    return best


@pytest.mark.parametrize("seed", range(12))
def test_multiway_is_valid_and_near_optimal_on_tiny_inputs(seed):
    rng = np.random.default_rng(100 + seed)
    k = int(rng.integers(2, 5))
    t = [int(x) for x in rng.integers(1, 60, int(rng.integers(1, 9)))]
    rep, sums = orep.karmarkar_karp(t, k)
    assert len(rep) == len(t) and all(0 <= r < k for r in rep)
    assert sums == [sum(x for x, r in zip(t, rep) if r == j) for j in range(k)]
    assert sums == sorted(sums, reverse=True)
    opt = _optimum(t, k)
    assert opt <= max(sums) <= Fraction(4, 3) * opt          # list-scheduling-class bound; the optimum is a floor


def test_special_cases():
    assert orep.karmarkar_karp([], 3) == ([], [0, 0, 0])
    rep, sums = orep.karmarkar_karp([5, 5, 5, 5, 5, 5], 3)
    assert sums == [10, 10, 10]
    rep, sums = orep.karmarkar_karp([9, 4, 7], 5)                # more replicas than items: everyone alone
    assert sorted(sums) == [0, 0, 4, 7, 9] and len(set(rep)) == 3
    rep, sums = orep.karmarkar_karp([3, 1, 2], 1)
    assert rep == [0, 0, 0] and sums == [6]


def _brute(lengths, cap, c, D, fixed, lin):
    """argmin over all contiguous partitions of the sorted list of (c-1)*max t + (1/D)*sum t, exact rationals."""
    order = sorted(range(len(lengths)), key=lambda i: (lengths[i], i))
    ls = [int(lengths[i]) for i in order]
    n = len(ls)
    best = None
    for mask in range(1 << (n - 1)):
        cuts = [0] + [i + 1 for i in range(n - 1) if mask >> i & 1] + [n]
        ts, ok = [], True
        for a, b in zip(cuts[:-1], cuts[1:]):
            L = max(ls[a:b])
            if (b - a) * L > cap:
                ok = False
                break
            ts.append(fixed + (b - a) * L * (lin + L))
        if not ok:
            continue
        J = (c - 1) * max(ts) + Fraction(sum(ts), D)
        key = (J, max(ts), tuple(-x for x in reversed(cuts[:-1])))   # same total order as the partition oracle's pins
        if best is None or key < best[0]:
            best = (key, cuts)
    return best


@pytest.mark.parametrize("seed", range(10))
def test_scaled_objective_is_the_papers_objective(seed):
    rng = np.random.default_rng(200 + seed)
    n = int(rng.integers(2, 10))
    lengths = rng.integers(4, 120, n).astype(np.int32)
    c, D = int(rng.integers(2, 6)), int(rng.integers(2, 5))
    fixed = int(rng.integers(0, 5000))
    cap = int(rng.integers(int(lengths.max()), 4 * int(lengths.max())))
    p = orep.plan_replicas(lengths, cap, c, D, fixed=fixed, lin=64)
    key, cuts = _brute(lengths, cap, c, D, fixed, 64)
    assert list(p["cuts"]) == cuts
    assert Fraction(int(p["objective"]), D) == key[0]
    assert sum(p["replica_time"]) == sum(p["mb_cost"]) and len(p["replica_of_mb"]) == len(cuts) - 1
