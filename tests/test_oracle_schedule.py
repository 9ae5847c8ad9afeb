"""Pins of the schedule oracle: hand-derived orders, closed forms, invariants."""
import numpy as np
import pytest

from oracle import schedule as osch

F, B = osch.F, osch.B


def _uniform(C, M, v=1):
    return [[v] * C for _ in range(M)]


def test_adaptive_two_stages_three_micro_batches_by_hand():
    # unlimited memory: stage 1 injects every cycle, stage 2 alternates as work arrives (derived cycle by cycle)
    O, cycles = osch.adaptive(2, 3, _uniform(2, 3), [100, 100])
    assert O[0] == [(0, F), (1, F), (2, F), (0, B), (1, B), (2, B)]
    assert O[1] == [(0, F), (0, B), (1, F), (1, B), (2, F), (2, B)]
    assert cycles == 6
    # limit 2.5 activations (strict test m + a < l: two micro-batches may be live): forward 2 waits for backward 0
    O, cycles = osch.adaptive(2, 3, _uniform(2, 3, 2), [5, 5])
    assert O[0] == [(0, F), (1, F), (0, B), (2, F), (1, B), (2, B)]
    assert O[1] == [(0, F), (0, B), (1, F), (1, B), (2, F), (2, B)]
    assert cycles == 7


def test_one_f_one_b_by_hand():
    O = osch.one_f_one_b(2, 3)
    assert O[0] == [(0, F), (1, F), (0, B), (2, F), (1, B), (2, B)]
    assert O[1] == [(0, F), (0, B), (1, F), (1, B), (2, F), (2, B)]
    O = osch.one_f_one_b(4, 2)                       # fewer micro-batches than stages
    assert O[0] == [(0, F), (1, F), (0, B), (1, B)] and O[3] == [(0, F), (0, B), (1, F), (1, B)]


@pytest.mark.parametrize("C,M", [(1, 1), (2, 5), (4, 7), (4, 16), (8, 8), (3, 20)])
def test_uniform_times_closed_form(C, M):
    # equal micro-batches: iteration time (C - 1) * t + M * t with t = t_f + t_b (Eq1 with all t equal)
    a = _uniform(C, M)
    tf, tb = _uniform(C, M, 3), _uniform(C, M, 5)
    for O in (osch.one_f_one_b(C, M), osch.adaptive(C, M, a, [10 ** 9] * C)[0]):
        sim = osch.simulate(C, M, O, tf, tb, a)
        assert sim["makespan"] == (C - 1) * 8 + M * 8
        assert sim["idle"][C - 1] == (C - 1) * 8     # the last stage idles exactly for the fill and the drain
    # 1F1B keeps at most C + 1 - n micro-batches on stage n
    sim = osch.simulate(C, M, osch.one_f_one_b(C, M), tf, tb, a)
    assert sim["peak"] == [min(C - j, M) for j in range(C)]


@pytest.mark.parametrize("seed", range(15))
def test_adaptive_invariants(seed):
    rng = np.random.default_rng(seed)
    C, M = int(rng.integers(1, 6)), int(rng.integers(1, 12))
    a = rng.integers(1, 50, (M, C)).tolist()
    l = [int(max(a[i][j] for i in range(M)) + rng.integers(1, 120)) for j in range(C)]
    O, _ = osch.adaptive(C, M, a, l)
    for j in range(C):
        assert sorted(O[j]) == sorted([(i, F) for i in range(M)] + [(i, B) for i in range(M)])   # every op once
        mem = 0
        for i, kind in O[j]:
            mem += a[i][j] if kind == F else -a[i][j]
            assert 0 <= mem < l[j]                   # the limit is never reached
        assert [i for i, k in O[j] if k == F] == list(range(M))     # injection order is kept
    tf = rng.integers(1, 30, (M, C)).tolist()
    tb = rng.integers(1, 60, (M, C)).tolist()
    sim = osch.simulate(C, M, O, tf, tb, a)          # executable: no deadlock
    assert all(p < l[j] for j, p in enumerate(sim["peak"]))
    lower = max(sum(tf[i][j] + tb[i][j] for i in range(M)) for j in range(C))
    assert sim["makespan"] >= lower
    assert sim["makespan"] >= sum(tf[0][j] + tb[0][j] for j in range(C))   # one micro-batch's round trip


def test_adaptive_errors():
    with pytest.raises(osch.ScheduleError):
        osch.adaptive(2, 2, [[5, 5], [9, 1]], [9, 9])          # 9 < 9 fails: can never run
    with pytest.raises(osch.ScheduleError):
        osch.simulate(2, 1, [[(0, B), (0, F)], [(0, F), (0, B)]], [[1, 1]], [[1, 1]], [[1, 1]])


def test_more_safety_stock_helps_under_variance():
    # one slow micro-batch: injecting early (adaptive, enough memory) is never worse than 1F1B here
    C, M = 4, 8
    a = _uniform(C, M)
    tf = [[2] * C for _ in range(M)]
    tb = [[4] * C for _ in range(M)]
    tf[2], tb[2] = [10] * C, [20] * C
    m1 = osch.simulate(C, M, osch.one_f_one_b(C, M), tf, tb, a)["makespan"]
    m2 = osch.simulate(C, M, osch.adaptive(C, M, a, [M + 1] * C)[0], tf, tb, a)["makespan"]
    assert m2 <= m1


@pytest.mark.parametrize("seed", range(10))
def test_comm_plan_invariants(seed):
    rng = np.random.default_rng(40 + seed)
    C, M = int(rng.integers(2, 6)), int(rng.integers(1, 10))
    a = _uniform(C, M)
    tf = rng.integers(1, 30, (M, C)).tolist()
    tb = rng.integers(1, 60, (M, C)).tolist()
    O = osch.adaptive(C, M, a, [int(rng.integers(2, M + 2))] * C)[0] if seed % 2 else osch.one_f_one_b(C, M)
    sim = osch.simulate(C, M, O, tf, tb, a)
    queue, stream = osch.comm_plan(C, M, O, sim)
    for j in range(C - 1):
        # the pairs on link j <-> j+1 appear in the same order on both ends (what rules out deadlock)
        lo = [("act", i) if c == osch.SEND_ACT else ("grad", i) for c, i in queue[j] if c in (osch.SEND_ACT, osch.RECV_GRAD)]
        hi = [("act", i) if c == osch.RECV_ACT else ("grad", i) for c, i in queue[j + 1] if c in (osch.RECV_ACT, osch.SEND_GRAD)]
        assert lo == hi and len(lo) == 2 * M
    for j in range(C):
        st = stream[j]
        assert [x for x in st if x[0] in (osch.FWD, osch.BWD)] == [(osch.FWD if k == F else osch.BWD, i) for i, k in O[j]]
        assert [x for x in st if x[0] in (osch.SEND_ACT, osch.RECV_ACT, osch.SEND_GRAD, osch.RECV_GRAD)] == queue[j]
        idx = {x: n for n, x in enumerate(st)}
        for i in range(M):
            if j > 0:
                assert idx[(osch.RECV_ACT, i)] < idx[(osch.WAIT_ACT, i)] == idx[(osch.FWD, i)] - 1
                assert idx[(osch.BWD, i)] < idx[(osch.SEND_GRAD, i)]
            if j + 1 < C:
                assert idx[(osch.RECV_GRAD, i)] < idx[(osch.WAIT_GRAD, i)] == idx[(osch.BWD, i)] - 1
                assert idx[(osch.FWD, i)] < idx[(osch.SEND_ACT, i)]


def _golden(name):
    import os
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, *v = line.split()
                out[k] = [int(x) for x in v]
    return out


def test_paper_example_of_safety_stocks():
    """The figures the paper states for its 7-micro-batch example (tests/golden/safety_stock_example.txt), with
    equal micro-batches (the text gives no sizes): how many micro-batches the first stage takes in before its first
    backward under 1F1B and under the adaptive schedule, the activations held, and which micro-batches a limit of
    three activations holds back."""
    g = _golden("safety_stock_example.txt")
    C, M = g["stages"][0], g["micro_batches"][0]
    a = [[1] * C for _ in range(M)]

    def leading_forwards(order):
        n = 0
        for _, kind in order:
            if kind != osch.F:
                break
            n += 1
        return n

    assert leading_forwards(osch.one_f_one_b(C, M)[0]) == g["injected_at_start_1f1b"][0]
    O, _ = osch.adaptive(C, M, a, [10 ** 6] * C)
    assert leading_forwards(O[0]) == g["injected_at_start_adaptive"][0]
    tf, tb = [[1] * C for _ in range(M)], [[2] * C for _ in range(M)]
    assert max(osch.simulate(C, M, O, tf, tb, a)["peak"]) == g["peak_adaptive_unlimited"][0]
    # a limit of three activations (Alg. 1's test is strict: m + a < l, so l = 3 + 1)
    lim = g["peak_adaptive_limited"][0]
    O, _ = osch.adaptive(C, M, a, [lim + 1] * C)
    sim = osch.simulate(C, M, O, tf, tb, a)
    assert max(sim["peak"]) == lim
    # held back = forwards on the first stage that start after the stage sat idle (since its previous forward)
    held, idle = [], False
    for k, (i, kind) in enumerate(O[0]):
        if k and sim["start"][0][k] > sim["end"][0][k - 1]:
            idle = True
        if kind == osch.F:
            if idle:
                held.append(i)
            idle = False
    assert held == g["held_back"]


def test_comm_plan_two_stages_two_micro_batches_worked_by_hand():
    """1F1B on 2 stages x 2 micro-batches, every forward 1 and every backward 2 time units, derived on paper.
    Orders: stage 0 = F0 F1 B0 B1, stage 1 = F0 B0 F1 B1.  Timeline: stage 0 F0 [0,1] F1 [1,2]; stage 1 F0 [1,2]
    B0 [2,4] F1 [4,5] B1 [5,7]; stage 0 B0 [4,6] B1 [7,9].  Transfers in order of the producing op's end: act 0 (t=1),
    act 1 (t=2), grad 0 (t=4), grad 1 (t=7); each start goes before the first compute op of its stage that starts at or
    after that time, each wait right before its consumer."""
    C, M = 2, 2
    O = osch.one_f_one_b(C, M)
    assert O == [[(0, F), (1, F), (0, B), (1, B)], [(0, F), (0, B), (1, F), (1, B)]]
    one, two = [[1] * C for _ in range(M)], [[2] * C for _ in range(M)]
    sim = osch.simulate(C, M, O, one, two, one)
    assert sim["start"] == [[0, 1, 4, 7], [1, 2, 4, 5]] and sim["end"] == [[1, 2, 6, 9], [2, 4, 5, 7]]
    assert sim["makespan"] == 9 and sim["idle"] == [3, 3] and sim["peak"] == [2, 1]
    queue, stream = osch.comm_plan(C, M, O, sim)
    S = osch
    assert queue[0] == [(S.SEND_ACT, 0), (S.SEND_ACT, 1), (S.RECV_GRAD, 0), (S.RECV_GRAD, 1)]
    assert queue[1] == [(S.RECV_ACT, 0), (S.RECV_ACT, 1), (S.SEND_GRAD, 0), (S.SEND_GRAD, 1)]
    assert stream[0] == [(S.FWD, 0), (S.SEND_ACT, 0), (S.FWD, 1), (S.SEND_ACT, 1), (S.RECV_GRAD, 0), (S.WAIT_GRAD, 0),
                         (S.BWD, 0), (S.RECV_GRAD, 1), (S.WAIT_GRAD, 1), (S.BWD, 1)]
    assert stream[1] == [(S.RECV_ACT, 0), (S.WAIT_ACT, 0), (S.FWD, 0), (S.RECV_ACT, 1), (S.BWD, 0), (S.SEND_GRAD, 0),
                         (S.WAIT_ACT, 1), (S.FWD, 1), (S.BWD, 1), (S.SEND_GRAD, 1)]
