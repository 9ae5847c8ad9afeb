"""TEST INFRASTRUCTURE: data-parallel replica balancing, written out from the paper's statement.

Section "Micro-batch Construction", paragraph "Balance data parallel model replicas": with |D|
replicas the planner minimises  (c-1) * max_m t(M_m) + (1/|D|) * sum_m t(M_m)  with the same
dynamic programme, then splits the micro-batches among the replicas with the Karmarkar-Karp
differencing method so that the largest per-replica sum is small.

Readings (the paper names the method and no more):
* the objective is kept exact by scaling with |D|:  |D|*(c-1)*max t + sum t ; this is the plain
  partition oracle run with (c-1)*|D| in place of (c-1);
* Karmarkar-Karp for more than two sets is the largest differencing method on partial partitions:
  every micro-batch starts as a partial partition with one non-empty set; the two partial
  partitions with the largest spread (largest set sum - smallest set sum) are merged by joining
  the first's sets in descending order of sum with the second's in ascending order; repeat until
  one is left;
* ties, fixed so that results are reproducible: sets inside a partial partition are ordered by
  (sum descending, smallest member index ascending, an empty set counting as index +infinity), the
  ascending order is the exact reverse; partial partitions of equal spread are taken in the order
  they were created (the initial ones in order of descending time, then ascending index);
* replica r receives the r-th set of the final partial partition in that order.
"""
import heapq

from . import plan as oplan

_BIG = 1 << 62


def cost(kind, fixed, lin, table, b, L, Lt=0):
    if kind == oplan.COST_POLY_GPT:
        return fixed + b * L * (lin + L)
    if kind == oplan.COST_POLY_T5:
        return fixed + b * L * (lin + L) + b * Lt * (lin + Lt + L)
    return int(table[b - 1][L - 1])


def _canon(sets):
    return sorted(sets, key=lambda s: (-s[0], min(s[1]) if s[1] else _BIG))


def karmarkar_karp(t, k):
    """-> (replica_of[i], replica_time[r]) for item times t (non-negative ints) and k replicas."""
    n = len(t)
    order = sorted(range(n), key=lambda i: (-t[i], i))
    heap, seq = [], 0
    for i in order:
        sets = _canon([(t[i], [i])] + [(0, [])] * (k - 1))
        heapq.heappush(heap, (-(sets[0][0] - sets[-1][0]), seq, sets))
        seq += 1
    if not heap:
        return [], [0] * k
    while len(heap) > 1:
        _, _, a = heapq.heappop(heap)
        _, _, b = heapq.heappop(heap)
        rb = list(reversed(b))
        merged = _canon([(a[p][0] + rb[p][0], a[p][1] + rb[p][1]) for p in range(k)])
        heapq.heappush(heap, (-(merged[0][0] - merged[-1][0]), seq, merged))
        seq += 1
    final = heap[0][2]
    replica_of = [0] * n
    for r, (_, members) in enumerate(final):
        for i in members:
            replica_of[i] = r
    return replica_of, [s for s, _ in final]


def plan_replicas(lengths, cap, num_stages, n_replicas, lengths_tgt=None, kind=oplan.COST_POLY_GPT, fixed=0, lin=2048,
                  table=None):
    """The scaled-objective partition plus the replica assignment.  Returns the plan dict extended with
    mb_cost, replica_of_mb, replica_time."""
    p = oplan.plan(lengths, cap, (num_stages - 1) * n_replicas + 1, lengths_tgt=lengths_tgt, kind=kind, fixed=fixed, lin=lin,
                   table=table)
    perm, cuts = p["perm"], p["cuts"]
    costs = []
    for m in range(len(cuts) - 1):
        idx = perm[cuts[m]:cuts[m + 1]]
        L = max(int(lengths[i]) for i in idx)
        Lt = max(int(lengths_tgt[i]) for i in idx) if lengths_tgt is not None else 0
        costs.append(cost(kind, fixed, lin, table, len(idx), L, Lt))
    rep, sums = karmarkar_karp(costs, n_replicas)
    out = dict(p)
    out.update(mb_cost=costs, replica_of_mb=rep, replica_time=sums)
    return out
