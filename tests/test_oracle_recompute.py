"""Pins of the dynamic-recomputation oracle (oracle/recompute.py) against things fixed outside it:
timelines worked out by hand from Alg. 1's rules, the single-stage closed form, and invariants.
Paper: section "Implementation", paragraph "Dynamic recomputation"."""
import numpy as np
import pytest

from oracle import plan as oplan
from oracle import recompute as orc


def poly(lin, act, fwd=(1, 4)):
    return dict(kind=oplan.COST_POLY_GPT, fixed=0, lin=lin, table=None, act_per_row=act, fwd_num=fwd[0], fwd_den=fwd[1])


# Two samples of 10 and 20 tokens, two stages, t(b, L) = b * L * (lin + L), forward = t / 4.
# Scheme A (nothing recomputed): lin 10 -> t = 200, 600 (forward 50, 150; backward 150, 450); 2 memory units per row.
# Scheme B (recomputing):        lin 20 -> t = 300, 800 (forward 75, 200; backward 225, 600); 1 unit per row.
A, B = poly(10, 2), poly(20, 1)
LENS = np.array([20, 10], dtype=np.int32)        # given unsorted on purpose


def test_unconstrained_timeline_by_hand():
    # ample memory: stage 0 runs F0 F1 B0 B1, stage 1 runs F0 B0 F1 B1 (one backward, then one forward per cycle)
    # stage 0: F0 [0,50] F1 [50,200]; stage 1: F0 [50,100] B0 [100,250] F1 [250,400] B1 [400,850];
    # stage 0: B0 [250,400] B1 [850,1300].  Memory (2/row): stage 0 holds 20 + 40 = 60, stage 1 at most 40.
    e = orc.evaluate_scheme(LENS, A, 10_000, 2)
    assert e["feasible"] and e["t"] == [200, 600] and e["rows"] == [10, 20]
    assert e["makespan"] == 1300 and e["peak"] == 60
    # scheme B alone: stage 0 F0 [0,75] F1 [75,275]; stage 1 F0 [75,150] B0 [150,375] F1 [375,575] B1 [575,1175];
    # stage 0 B0 [375,600] B1 [1175,1775]
    e = orc.evaluate_scheme(LENS, B, 10_000, 2)
    assert e["makespan"] == 1775 and e["peak"] == 30


def test_memory_limit_delays_forward_then_excludes_scheme():
    # limit 50: under A the second forward (20 + 40 < 50 is false) waits for B0 on stage 0:
    # stage 0 F0 [0,50], stage 1 F0 [50,100] B0 [100,250], stage 0 B0 [250,400] F1 [400,550],
    # stage 1 F1 [550,700] B1 [700,1150], stage 0 B1 [1150,1600].  B is not delayed (10 + 20 < 50): 1775.
    idx, res = orc.choose_scheme(LENS, [A, B], 50, 2)
    assert [r["makespan"] for r in res] == [1600, 1775] and idx == 0
    assert res[0]["peak"] == 40 and res[1]["peak"] == 30
    # limit 41: cap under A = 40 // 2 = 20, the 20-token sample still fits (40 < 41)
    idx, res = orc.choose_scheme(LENS, [A, B], 41, 2)
    assert idx == 0 and res[0]["makespan"] == 1600
    # limit 40: cap under A = 39 // 2 = 19 < 20: A cannot hold the long sample, B is chosen
    idx, res = orc.choose_scheme(LENS, [A, B], 40, 2)
    assert idx == 1 and not res[0]["feasible"] and res[1]["makespan"] == 1775
    # limit 20: cap under B = 19 < 20 as well
    with pytest.raises(orc.RecomputeError):
        orc.choose_scheme(LENS, [A, B], 20, 2)


def test_forward_share_matters():
    # forward = 3/4 instead of 1/4 (a swapped share) gives a different timeline: stage 0 F0 [0,150] F1 [150,600];
    # stage 1 F0 [150,300] B0 [300,350] F1 [600,1050] B1 [1050,1200]; stage 0 B0 [600,650] B1 [1200,1350]
    e = orc.evaluate_scheme(LENS, poly(10, 2, fwd=(3, 4)), 10_000, 2)
    assert e["makespan"] == 1350


def test_equal_times_go_to_the_first_scheme():
    idx, _ = orc.choose_scheme(LENS, [poly(10, 1), poly(10, 2)], 10_000, 2)
    assert idx == 0
    idx, _ = orc.choose_scheme(LENS, [poly(10, 2), poly(10, 1)], 10_000, 2)
    assert idx == 0


@pytest.mark.parametrize("seed", range(6))
def test_single_stage_closed_form(seed):
    # one stage: the device is never idle, so the iteration takes sum of t; with no fixed cost per micro-batch the
    # optimal partition has no padding, so sum of t = sum_i l_i * (lin + l_i) whatever was merged; Alg. 1 on one
    # stage runs B_m before F_(m+1) in the same cycle, so at most one micro-batch is held: peak = a * largest rows
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 9))
    lens = rng.choice(np.arange(3, 200), size=n, replace=False).astype(np.int32)     # distinct: nothing merges
    lin, a = int(rng.integers(1, 300)), int(rng.integers(1, 5))
    e = orc.evaluate_scheme(lens, poly(lin, a, fwd=(1, 3)), a * int(lens.max()) + 1, 1)
    assert e["feasible"]
    assert e["makespan"] == int(sum(int(l) * (lin + int(l)) for l in lens))
    assert e["peak"] == a * int(lens.max())
    # one unit less of memory and the longest sample no longer satisfies a * l < limit
    assert not orc.evaluate_scheme(lens, poly(lin, a), a * int(lens.max()), 1)["feasible"]


@pytest.mark.parametrize("seed", range(8))
def test_invariants_on_random_inputs(seed):
    rng = np.random.default_rng(100 + seed)
    n, C = int(rng.integers(2, 10)), int(rng.integers(1, 4))
    lens = rng.integers(4, 120, size=n).astype(np.int32)
    schemes = [poly(64, 4), dict(poly(96, 2), fixed=500), poly(160, 1)]
    limit = int(rng.integers(int(lens.max()) + 1, 6 * int(lens.sum())))
    try:
        idx, res = orc.choose_scheme(lens, schemes, limit, C)
    except orc.RecomputeError:
        assert all((limit - 1) // s["act_per_row"] < int(lens.max()) for s in schemes)
        return
    for s, e in zip(schemes, res):
        cap = (limit - 1) // s["act_per_row"]
        if cap < int(lens.max()):
            assert not e["feasible"]
            continue
        assert e["feasible"]                                    # Alg. 1 always completes when every micro-batch fits alone
        assert sorted(e["perm"]) == list(range(n)) and e["cuts"][0] == 0 and e["cuts"][-1] == n
        assert all(r <= cap for r in e["rows"])
        assert e["peak"] < limit
        assert sum(e["t"]) <= e["makespan"] <= C * sum(e["t"])  # stage 0 runs every op; a chain of C ops per unit of work
    feas = [k for k, e in enumerate(res) if e["feasible"]]
    best = min(res[k]["makespan"] for k in feas)
    assert res[idx]["makespan"] == best and idx == min(k for k in feas if res[k]["makespan"] == best)
