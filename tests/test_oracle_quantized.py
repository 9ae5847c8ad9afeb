"""Pins of the sampled-t_max oracle."""
import numpy as np
import pytest

from oracle import plan as oplan
from oracle import quantized as oq


def _case(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 14))
    lens = rng.integers(4, 200, n).astype(np.int32)
    cap = int(rng.integers(int(lens.max()), 5 * int(lens.max())))
    return lens, cap, int(rng.integers(1, 7)), int(rng.integers(0, 40000))


@pytest.mark.parametrize("seed", range(15))
def test_unit_interval_is_the_exact_procedure(seed):
    lens, cap, c, fixed = _case(seed)
    a = oq.plan(lens, cap, c, 1, fixed=fixed, lin=64)
    b = oplan.plan(lens, cap, c, fixed=fixed, lin=64)
    assert list(a["cuts"]) == list(b["cuts"]) and a["objective"] == b["objective"] and a["t_max"] == b["t_max"]


@pytest.mark.parametrize("seed", range(15))
def test_loss_is_bounded_by_the_interval(seed):
    lens, cap, c, fixed = _case(100 + seed)
    exact = oplan.plan(lens, cap, c, fixed=fixed, lin=64)
    for q in (7, 1000, 50000, 10 ** 7):
        s = oq.plan(lens, cap, c, q, fixed=fixed, lin=64)
        # never better than the optimum, and within (c-1) * q of it: the optimal t_max rounds up by less than q
        assert exact["objective"] <= s["objective"] < exact["objective"] + (c - 1) * q + 1
        assert s["t_max"] <= s["sampled_t_max"]


@pytest.mark.parametrize("seed", range(8))
def test_changes_only_grid_equals_full_grid(seed):
    lens, cap, c, fixed = _case(200 + seed)
    lens = np.minimum(lens, 40)                                   # keep the full grid short
    cap = max(cap // 4, int(lens.max()))
    for q in (50, 333):
        a = oq.plan(lens, cap, c, q, fixed=fixed % 2000, lin=16)
        b = oq.plan(lens, cap, c, q, fixed=fixed % 2000, lin=16, full_grid=True)
        assert list(a["cuts"]) == list(b["cuts"]) and a["sampled_t_max"] == b["sampled_t_max"]


def test_one_huge_interval_minimises_the_sum():
    lens = np.array([10, 12, 50, 51, 200], np.int32)
    s = oq.plan(lens, 400, 4, 10 ** 12, fixed=5000, lin=64)
    # a single candidate admits every slice: the plan is the sum-optimal one, whatever its largest micro-batch
    best = min(
        (sum(5000 + (b - a) * max(sorted(lens)[a:b]) * (64 + max(sorted(lens)[a:b])) for a, b in zip(cuts[:-1], cuts[1:])), cuts)
        for cuts in ([0] + [i + 1 for i in range(4) if m >> i & 1] + [5] for m in range(16))
        if all((b - a) * max(sorted(lens)[a:b]) <= 400 for a, b in zip(cuts[:-1], cuts[1:])))
    assert sum(5000 + (b - a) * int(max(sorted(lens)[a:b])) * (64 + int(max(sorted(lens)[a:b]))) for a, b in zip(s["cuts"][:-1], s["cuts"][1:])) == best[0]
