"""Pins for the partition oracle (oracle/plan_oracle.c): brute force over all contiguous
partitions (n <= 12), the closed form that holds for a cost with no fixed term, invariants and
special cases.  Nothing here calls the product."""
import itertools

import numpy as np
import pytest

from oracle import plan as oplan

INF = float("inf")


def _sorted_order(lens, tgts=None):
    idx = list(range(len(lens)))
    if tgts is None:
        idx.sort(key=lambda i: (lens[i], i))
    else:
        idx.sort(key=lambda i: (lens[i], tgts[i], i))
    return idx


def brute(lens, cap, c, cost, tgts=None):
    """Enumerate every cut set of the ordered list; return the best by (J, max t, reversed starts)."""
    order = _sorted_order(lens, tgts)
    n = len(order)
    best = None
    for mask in range(1 << (n - 1)):
        cuts = [0] + [k + 1 for k in range(n - 1) if mask >> k & 1] + [n]
        ts = []
        ok = True
        for a, b in zip(cuts[:-1], cuts[1:]):
            L = max(lens[order[k]] for k in range(a, b))
            Lt = max(tgts[order[k]] for k in range(a, b)) if tgts is not None else 0
            if (b - a) * L > cap:
                ok = False
                break
            ts.append(cost(b - a, L, Lt))
        if not ok:
            continue
        J = (c - 1) * max(ts) + sum(ts)
        key = (J, max(ts), tuple(reversed(cuts[:-1])))
        if best is None or key < best[0]:
            best = (key, cuts)
    return order, best


def test_brute_force_table_costs():
    rng = np.random.default_rng(7)
    for trial in range(300):
        n = int(rng.integers(1, 10))
        lmax = int(rng.integers(2, 9))
        lens = rng.integers(1, lmax + 1, size=n).astype(np.int32)
        table = rng.integers(1, 60, size=(n, lmax)).astype(np.int64)
        cap = int(rng.integers(lmax, 4 * lmax + 1))
        c = int(rng.choice([1, 2, 4, 8]))
        order, best = brute(list(lens), cap, c, lambda b, L, Lt: int(table[b - 1, L - 1]))
        got = oplan.plan(lens, cap, c, kind=oplan.COST_TABLE, table=table)
        assert list(got["perm"]) == order
        assert best is not None
        assert got["objective"] == best[0][0], (trial, lens, cap, c)
        assert got["t_max"] == best[0][1]
        assert list(got["cuts"]) == best[1], (trial, lens, cap, c)


def test_brute_force_n12_poly_with_fixed_term():
    rng = np.random.default_rng(11)
    for trial in range(6):
        n = 12
        lens = rng.integers(1, 40, size=n).astype(np.int32)
        fixed, lin = int(rng.integers(0, 3000)), int(rng.integers(1, 64))
        cap = int(rng.integers(40, 200))
        c = int(rng.choice([1, 2, 4, 8]))
        order, best = brute(list(lens), cap, c, lambda b, L, Lt: fixed + b * L * (lin + L))
        got = oplan.plan(lens, cap, c, fixed=fixed, lin=lin)
        assert got["objective"] == best[0][0]
        assert list(got["cuts"]) == best[1]


def test_brute_force_encoder_decoder_cost():
    rng = np.random.default_rng(13)
    for trial in range(80):
        n = int(rng.integers(1, 9))
        lens = rng.integers(1, 30, size=n).astype(np.int32)
        tgts = rng.integers(1, 12, size=n).astype(np.int32)
        fixed, lin = int(rng.integers(0, 500)), int(rng.integers(1, 40))
        cap = int(rng.integers(30, 120))
        c = int(rng.choice([1, 2, 4]))
        cost = lambda b, L, Lt: fixed + b * L * (lin + L) + b * Lt * (lin + Lt + L)
        order, best = brute(list(lens), cap, c, cost, list(tgts))
        got = oplan.plan(lens, cap, c, lengths_tgt=tgts, kind=oplan.COST_POLY_T5, fixed=fixed, lin=lin)
        assert list(got["perm"]) == order
        assert got["objective"] == best[0][0]
        assert list(got["cuts"]) == best[1]


def test_closed_form_no_fixed_term():
    """t(b,L) = b*g(L) with g increasing and no per-micro-batch term: singletons minimise both
    the sum and the max, so J* = (c-1) g(l_max) + sum_i g(l_i), the plan has zero padding and no
    micro-batch costs more than g(l_max)."""
    rng = np.random.default_rng(3)
    g = lambda l: l * (2048 + l)
    for trial in range(20):
        n = int(rng.integers(1, 80))
        lens = np.clip(np.rint(rng.lognormal(4.5, 0.8, size=n)), 8, 512).astype(np.int32)
        c = int(rng.choice([1, 4, 8]))
        got = oplan.plan(lens, 4096, c)
        assert got["objective"] == (c - 1) * g(int(lens.max())) + sum(g(int(l)) for l in lens)
        assert got["t_max"] <= g(int(lens.max()))
        srt = lens[got["perm"]]
        for a, b in zip(got["cuts"][:-1], got["cuts"][1:]):
            assert srt[a] == srt[b - 1]                      # zero padding: equal lengths only
            assert (b - a) * g(int(srt[a])) <= g(int(lens.max()))


def test_invariants_and_monotone_in_cap():
    rng = np.random.default_rng(5)
    for trial in range(40):
        n = int(rng.integers(2, 40))
        lens = rng.integers(1, 100, size=n).astype(np.int32)
        fixed = int(rng.integers(100, 20000))
        c = int(rng.choice([1, 2, 4]))
        prev = None
        for cap in (int(lens.max()), 2 * int(lens.max()), 8 * int(lens.max()), 10 ** 6):
            got = oplan.plan(lens, cap, c, fixed=fixed, lin=16)
            cuts = got["cuts"]
            assert cuts[0] == 0 and cuts[-1] == n and all(b > a for a, b in zip(cuts[:-1], cuts[1:]))
            assert sorted(got["perm"]) == list(range(n))
            srt = lens[got["perm"]]
            assert all(srt[i] <= srt[i + 1] for i in range(n - 1))
            ts = []
            for a, b in zip(cuts[:-1], cuts[1:]):
                L = int(srt[a:b].max())
                assert (b - a) * L <= cap
                ts.append(fixed + (b - a) * L * (16 + L))
            assert got["objective"] == (c - 1) * max(ts) + sum(ts)
            assert got["t_max"] == max(ts)
            if prev is not None:
                assert got["objective"] <= prev                 # a looser cap never hurts
            prev = got["objective"]


def test_special_cases():
    # one sequence
    got = oplan.plan([17], 17, 4)
    assert list(got["cuts"]) == [0, 1] and got["objective"] == 4 * 17 * (2048 + 17)
    # all-equal lengths, big fixed term: merge as far as the cap allows, longest slice last
    got = oplan.plan([10] * 7, 30, 1, fixed=10 ** 6, lin=1)
    assert list(got["cuts"]) == [0, 1, 4, 7]
    # stable ties: equal lengths keep original order
    got = oplan.plan([5, 3, 5, 3], 100, 2)
    assert list(got["perm"]) == [1, 3, 0, 2]
    # a sequence longer than the cap: no admissible partition
    with pytest.raises(oplan.OraclePlanError) as e:
        oplan.plan([4, 50], 49, 4)
    assert e.value.code == -2
    # bad arguments
    for bad in ([0, 3], [-1]):
        with pytest.raises(oplan.OraclePlanError) as e:
            oplan.plan(bad, 10, 4)
        assert e.value.code == -1
    with pytest.raises(oplan.OraclePlanError):
        oplan.plan([3], 10, 0)
    # overflow of the 64-bit cost
    with pytest.raises(oplan.OraclePlanError) as e:
        oplan.plan([2 ** 30, 2 ** 30], 2 ** 40, 4, lin=2 ** 62)
    assert e.value.code == -4


def test_candidate_count_bound():
    """At most N(N+1)/2 distinct single-micro-batch costs exist (section "Micro-batch Construction")."""
    lens = np.arange(1, 21, dtype=np.int32)
    vals = set()
    for i in range(20):
        for j in range(i + 1, 21):
            vals.add((j - i) * int(lens[j - 1]) * (2048 + int(lens[j - 1])))
    assert len(vals) <= 20 * 21 // 2
