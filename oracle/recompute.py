"""TEST INFRASTRUCTURE: dynamic recomputation, from the paper's text (not part of the product path).

Section "Implementation", paragraph "Dynamic recomputation": the peak memory of an iteration varies
with its micro-batches, so for every iteration the recomputation scheme is chosen anew, by repeating
micro-batch partitioning and scheduling once per scheme, each under that scheme's own cost model, and
keeping the scheme with the least computation overhead that does not run out of memory.

Plain Python over the other oracle modules (partitioning: the exact DP of section "Micro-batch
Construction"; schedule and timeline: Alg. 1 and the simulator of section "Pipeline Execution
Schedule"), in the paper's order: for every scheme partition, schedule, simulate; then choose.

A scheme r is (cost model t_r(b, L) of forward + backward including what r recomputes, a_r = units
of activation memory one padded row of a micro-batch holds on a stage between its forward and its
backward, and the forward's share of t_r as a fraction).  Readings (the text leaves these open):
* memory: a micro-batch of b sequences padded to L (and L_tgt) holds a_r * b * (L + L_tgt) on every
  stage; every stage has the same limit l.  Alg. 1 admits a forward only if m + a < l, so one
  micro-batch alone needs a_r * b * L_pad < l: the partitioner's token cap under scheme r is
  (l - 1) // a_r.  A sample longer than that makes the scheme infeasible, and so does a schedule
  Alg. 1 cannot complete.
* times: all stages are alike (one stage's cost model stands for each); a micro-batch's forward takes
  t * fwd_num // fwd_den, its backward the rest, so forward + backward is exactly t.
* "least computation overhead without running out of memory": the feasible scheme whose simulated
  iteration time (makespan) is smallest; equal times go to the scheme listed first (list the schemes
  in ascending order of recomputation).  No feasible scheme is an error.
"""
from . import plan as oplan
from . import replicas as orep
from . import schedule as osched


class RecomputeError(Exception):
    pass


def evaluate_scheme(lengths, scheme, mem_limit, num_stages, lengths_tgt=None):
    """One scheme: partition under its cost model and cap, schedule with Alg. 1, simulate.
    scheme: dict(kind, fixed, lin, table, act_per_row, fwd_num, fwd_den).
    -> dict(feasible, makespan, peak, cuts, perm, t, rows) (makespan/peak None when infeasible)."""
    a_r = int(scheme["act_per_row"])
    if a_r <= 0 or mem_limit <= 0:
        raise RecomputeError("activation size and memory limit must be positive")
    cap = (int(mem_limit) - 1) // a_r
    bad = dict(feasible=False, makespan=None, peak=None, cuts=None, perm=None, t=None, rows=None)
    if cap < int(max(lengths)):
        return bad
    kind, fixed, lin, table = scheme["kind"], scheme.get("fixed", 0), scheme.get("lin", 2048), scheme.get("table")
    try:
        p = oplan.plan(lengths, cap, num_stages, lengths_tgt=lengths_tgt, kind=kind, fixed=fixed, lin=lin, table=table)
    except oplan.OraclePlanError:
        return bad
    perm, cuts = p["perm"], p["cuts"]
    M, C = len(cuts) - 1, int(num_stages)
    t, rows = [], []
    for m in range(M):
        idx = perm[cuts[m]:cuts[m + 1]]
        b = len(idx)
        L = int(max(lengths[i] for i in idx))
        Lt = 0 if lengths_tgt is None else int(max(lengths_tgt[i] for i in idx))
        t.append(int(orep.cost(kind, fixed, lin, table, b, L, Lt)))
        rows.append(b * (L + Lt))
    tf = [[t[m] * int(scheme["fwd_num"]) // int(scheme["fwd_den"])] * C for m in range(M)]
    tb = [[t[m] - tf[m][0]] * C for m in range(M)]
    a = [[a_r * rows[m]] * C for m in range(M)]
    try:
        O, _ = osched.adaptive(C, M, a, [int(mem_limit)] * C)
    except osched.ScheduleError:
        return bad
    sim = osched.simulate(C, M, O, tf, tb, a)
    return dict(feasible=True, makespan=sim["makespan"], peak=max(sim["peak"]), cuts=[int(c) for c in cuts],
                perm=[int(i) for i in perm], t=t, rows=rows)


def choose_scheme(lengths, schemes, mem_limit, num_stages, lengths_tgt=None):
    """-> (index of the chosen scheme, [evaluate_scheme result per scheme])."""
    res = [evaluate_scheme(lengths, s, mem_limit, num_stages, lengths_tgt) for s in schemes]
    best = None
    for r, e in enumerate(res):
        if e["feasible"] and (best is None or e["makespan"] < res[best]["makespan"]):
            best = r
    if best is None:
        raise RecomputeError("no recomputation scheme fits the memory limit")
    return best, res
