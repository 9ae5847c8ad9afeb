"""TEST INFRASTRUCTURE: the partition DP with t_max sampled at fixed intervals.

Section "Micro-batch Construction", last paragraph of "Dynamic programming": many candidate t_max
values are close to each other, so the paper only considers t_max values a fixed interval apart (5 us
in its evaluation).  Reading taken here: the candidates are the multiples q, 2q, 3q, ... of the
interval q; for each candidate T Eq2 is run over the slices with t <= T and the candidate minimising
(c-1)*T + f(N; T) wins (smallest T on equal value, smallest split index inside Eq2, as in the exact
procedure); the returned objective and t_max are those of the partition actually chosen,
(c-1)*max t + sum t and max t.  Decoder-only polynomial and table costs.

full_grid=True walks every multiple (the definition); the default visits only the multiples at which
the set of admitted slices changes, which cannot change the result (between two of them f is
constant and (c-1)*T grows); a test checks the two against each other.
"""
import numpy as np


def plan(lengths, cap, num_stages, quantum, fixed=0, lin=2048, table=None, full_grid=False):
    n = len(lengths)
    perm = sorted(range(n), key=lambda i: (int(lengths[i]), i))
    ls = [int(lengths[i]) for i in perm]
    INF = float("inf")
    t = {}
    for i in range(n):
        for j in range(i + 1, n + 1):
            b, L = j - i, max(ls[i:j])
            if b * L > cap:
                continue
            t[(i, j)] = int(table[b - 1][L - 1]) if table is not None else fixed + b * L * (lin + L)
    if not t:
        return None
    q = int(quantum)
    top = -(-max(t.values()) // q) * q
    cands = range(q, top + 1, q) if full_grid else sorted({-(-v // q) * q for v in t.values()})
    best = None
    for T in cands:
        f = [INF] * (n + 1)
        arg = [-1] * (n + 1)
        f[0] = 0
        for nn in range(1, n + 1):
            for i in range(nn):
                v = t.get((i, nn))
                if v is None or v > T or f[i] == INF:
                    continue
                if f[i] + v < f[nn]:
                    f[nn], arg[nn] = f[i] + v, i
        if f[n] == INF:
            continue
        J = (num_stages - 1) * T + f[n]
        if best is None or J < best[0]:
            best = (J, T, arg)
    if best is None:
        return None
    _, T, arg = best
    cuts, pos = [n], n
    while pos > 0:
        pos = arg[pos]
        cuts.append(pos)
    cuts.reverse()
    costs = [t[(a, b)] for a, b in zip(cuts[:-1], cuts[1:])]
    return dict(perm=np.array(perm, np.int32), cuts=np.array(cuts, np.int32), sampled_t_max=T,
                t_max=max(costs), objective=(num_stages - 1) * max(costs) + sum(costs))
