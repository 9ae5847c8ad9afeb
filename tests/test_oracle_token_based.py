"""Pins of the token-based micro-batching oracle (the paper's TB baseline)."""
import itertools

import numpy as np
import pytest

from oracle import token_based as otb


def test_example_worked_by_hand():
    # sorted: 1 2 3 4 4 5 (original indices 1 2 0 4 5 3); budget 8 padded tokens
    #   [1 2] = 2 x 2 = 4, adding 3 gives 3 x 3 = 9 > 8      -> cut after 2 samples
    #   [3 4] = 2 x 4 = 8, adding 4 gives 3 x 4 = 12 > 8     -> cut after 4
    #   [4]   = 4,         adding 5 gives 2 x 5 = 10 > 8     -> cut after 5
    #   [5]
    r = otb.plan([3, 1, 2, 5, 4, 4], 8)
    assert r["perm"] == [1, 2, 0, 4, 5, 3]
    assert r["cuts"] == [0, 2, 4, 5, 6]


def test_encoder_decoder_order_and_input_side_budget():
    # equal input lengths are ordered by target length, then by index; the budget counts input tokens only
    r = otb.plan([4, 4, 2, 4], 8, lengths_tgt=[9, 1, 50, 1])
    assert r["perm"] == [2, 1, 3, 0]
    assert r["cuts"] == [0, 2, 4]           # [2 4] = 2 x 4 = 8; [4 4] = 8


def _admissible(ls, cuts, budget):
    return all((b - a) * max(ls[a:b]) <= budget for a, b in zip(cuts[:-1], cuts[1:]))


def _all_partitions(n):
    for k in range(n):
        for inner in itertools.combinations(range(1, n), k):
            yield [0] + list(inner) + [n]


@pytest.mark.parametrize("seed", range(40))
def test_brute_force_fewest_micro_batches_and_largest_cut_list(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 11))
    lens = rng.integers(1, 30, n)
    budget = int(rng.integers(int(lens.max()), 4 * int(lens.max()) + 1))
    r = otb.plan(lens, budget)
    ls = [int(lens[i]) for i in r["perm"]]
    assert ls == sorted(ls)
    ok = [c for c in _all_partitions(n) if _admissible(ls, c, budget)]
    assert r["cuts"] in ok
    assert len(r["cuts"]) == min(len(c) for c in ok)
    assert r["cuts"][1:] == max(c[1:] + [n] * (n + 1 - len(c)) for c in ok)[:len(r["cuts"]) - 1]


@pytest.mark.parametrize("seed", range(20))
def test_every_micro_batch_admissible_and_not_extensible(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 300))
    lens = np.clip(np.rint(rng.lognormal(4.5, 0.9, n)), 4, 2048).astype(np.int64)
    tgts = rng.integers(1, 100, n) if seed % 2 else None
    budget = int(rng.integers(int(lens.max()), 8 * int(lens.max())))
    r = otb.plan(lens, budget, lengths_tgt=tgts)
    ls = [int(lens[i]) for i in r["perm"]]
    cuts = r["cuts"]
    assert sorted(r["perm"]) == list(range(n)) and cuts[0] == 0 and cuts[-1] == n
    for a, b in zip(cuts[:-1], cuts[1:]):
        assert b > a and (b - a) * max(ls[a:b]) <= budget
        if b < n:
            assert (b + 1 - a) * max(ls[a:b + 1]) > budget


def test_closed_forms():
    # equal lengths l: micro-batches of floor(budget / l) samples, the last one takes the rest
    r = otb.plan([7] * 23, 30)
    assert r["cuts"] == [0, 4, 8, 12, 16, 20, 23]
    # a budget that binds nowhere: one micro-batch; one that binds everywhere: one sample each
    assert otb.plan([5, 9, 2, 6], 4 * 9)["cuts"] == [0, 4]
    assert otb.plan([5, 9, 6, 7], 9)["cuts"] == [0, 1, 2, 3, 4]
    # a sample longer than the budget cannot be placed
    assert otb.plan([5, 9, 2], 8) is None
    assert otb.plan([4], 4)["cuts"] == [0, 1]
