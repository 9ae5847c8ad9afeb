"""TEST INFRASTRUCTURE: pipeline execution schedules and communication order, from the paper's text.

Section "Pipeline Execution Schedule": the memory-aware adaptive schedule (Alg. 1), the 1F1B order
it is compared with, and a device timeline under given op times (what section "Communication
Planning" simulates); section "Communication Planning": the order of send / receive starts and the
late waits.  Plain Python, the paper's notation: C stages, M micro-batches, a[i][j] activation
memory of micro-batch i on stage j, l[j] memory limit, O[j] execution order of stage j.

Readings (the text leaves these open):
* Alg. 1 is followed as printed: per cycle every stage, in stage order, takes at most one backward op
  and then at most one forward op from the head of its buffers; a forward op runs only if
  m_j + a < l_j (strict), otherwise it goes back to the head and nothing behind it is tried; ops
  unlocked in a cycle join the buffers at the end of that cycle.  After the last stage's forward the
  backward of the same micro-batch is unlocked on that stage.
* A micro-batch whose activation alone does not satisfy a < l_j can never run: reported as an error
  instead of looping for ever; so is a cycle in which nothing ran while work was left.
* 1F1B: stage j (1-based) runs min(C + 1 - j, M) forwards, then alternates one backward, one
  forward while forwards are left, then the remaining backwards; micro-batches in index order.
* Timeline: a stage executes its ops in the given order; an op starts when the stage is free and
  its predecessor has ended (forward of the same micro-batch on the previous stage; backward on the
  next stage, or the forward on the last stage).  Communication takes no time (the paper calls it
  very small for pipeline parallelism).  Memory of a stage rises by a at a forward's start and
  falls by a at the backward's end.
* Communication order: ops are visited in ascending end time (ties: lower stage first, then the
  order on that stage); a forward on stage j < C appends SendActStart to stage j's queue and
  RecvActStart to stage j+1's; a backward on stage j > 1 appends SendGradStart to j's and
  RecvGradStart to j-1's.  The instruction stream of a stage lists its compute ops in order, every
  queued start before the first compute op of that stage that starts at or after the start's time
  (so a stage's own sends follow their producer and a receive is started before its consumer),
  and the wait for a received tensor immediately before the op that consumes it.
"""

F, B = 0, 1
FWD, BWD, SEND_ACT, RECV_ACT, SEND_GRAD, RECV_GRAD, WAIT_ACT, WAIT_GRAD = range(8)


class ScheduleError(Exception):
    pass


def adaptive(C, M, a, l):
    O = [[] for _ in range(C)]
    Sf = [[] for _ in range(C)]
    Sb = [[] for _ in range(C)]
    m = [0] * C
    for i in range(M):
        for j in range(C):
            if not a[i][j] < l[j]:
                raise ScheduleError("micro-batch %d cannot fit stage %d" % (i, j))
    Sf[0] = list(range(M))
    cycles = 0
    while any(Sf[j] or Sb[j] for j in range(C)):
        Nf = [[] for _ in range(C)]
        Nb = [[] for _ in range(C)]
        ran = False
        for j in range(C):
            if Sb[j]:
                i = Sb[j].pop(0)
                m[j] -= a[i][j]
                O[j].append((i, B))
                ran = True
                if j > 0:
                    Nb[j - 1].append(i)
            if Sf[j]:
                i = Sf[j].pop(0)
                if m[j] + a[i][j] < l[j]:
                    m[j] += a[i][j]
                    O[j].append((i, F))
                    ran = True
                    if j + 1 < C:
                        Nf[j + 1].append(i)
                    else:
                        Nb[j].append(i)
                else:
                    Sf[j].insert(0, i)
        for j in range(C):
            Sf[j] += Nf[j]
            Sb[j] += Nb[j]
        cycles += 1
        if not ran:
            raise ScheduleError("no op could run")
    return O, cycles


def one_f_one_b(C, M):
    O = []
    for j in range(C):
        warm = min(C - j, M)
        o = [(i, F) for i in range(warm)]
        nf, nb = warm, 0
        while nb < M:
            o.append((nb, B))
            nb += 1
            if nf < M:
                o.append((nf, F))
                nf += 1
        O.append(o)
    return O


def simulate(C, M, O, tf, tb, a):
    """-> dict(makespan, start[j][k], end[j][k], idle[j], peak[j]) for per-op times tf[i][j], tb[i][j]."""
    pos = [0] * C
    free = [0] * C
    endF = [[None] * C for _ in range(M)]
    endB = [[None] * C for _ in range(M)]
    start = [[None] * len(O[j]) for j in range(C)]
    end = [[None] * len(O[j]) for j in range(C)]
    done, total = 0, sum(len(o) for o in O)
    while done < total:
        progressed = False
        for j in range(C):
            while pos[j] < len(O[j]):
                i, kind = O[j][pos[j]]
                if kind == F:
                    dep = 0 if j == 0 else endF[i][j - 1]
                else:
                    dep = endF[i][j] if j == C - 1 else endB[i][j + 1]
                    if endF[i][j] is None:
                        dep = None
                if dep is None:
                    break
                s = max(free[j], dep)
                e = s + (tf[i][j] if kind == F else tb[i][j])
                start[j][pos[j]], end[j][pos[j]] = s, e
                (endF if kind == F else endB)[i][j] = e
                free[j] = e
                pos[j] += 1
                done += 1
                progressed = True
        if not progressed:
            raise ScheduleError("the order deadlocks")
    makespan = max(free)
    idle, peak = [], []
    for j in range(C):
        busy = sum(end[j][k] - start[j][k] for k in range(len(O[j])))
        idle.append(makespan - busy)
        ev = []
        for k, (i, kind) in enumerate(O[j]):
            ev.append((start[j][k], 1, a[i][j]) if kind == F else (end[j][k], 0, -a[i][j]))
        cur = pk = 0
        for _, _, dm in sorted(ev):                      # at equal times memory is freed before it is taken
            cur += dm
            pk = max(pk, cur)
        peak.append(pk)
    return dict(makespan=makespan, start=start, end=end, idle=idle, peak=peak)


def comm_plan(C, M, O, sim):
    """-> (queue[j] of (code, micro-batch), stream[j] of (code, micro-batch))."""
    ops = []
    for j in range(C):
        for k, (i, kind) in enumerate(O[j]):
            ops.append((sim["end"][j][k], j, k, i, kind))
    ops.sort()
    queue = [[] for _ in range(C)]
    timed = [[] for _ in range(C)]                       # (time, code, micro-batch) of the starts of each stage
    for e, j, k, i, kind in ops:
        if kind == F and j + 1 < C:
            queue[j].append((SEND_ACT, i)); timed[j].append((e, SEND_ACT, i))
            queue[j + 1].append((RECV_ACT, i)); timed[j + 1].append((e, RECV_ACT, i))
        if kind == B and j > 0:
            queue[j].append((SEND_GRAD, i)); timed[j].append((e, SEND_GRAD, i))
            queue[j - 1].append((RECV_GRAD, i)); timed[j - 1].append((e, RECV_GRAD, i))
    stream = []
    for j in range(C):
        out, q = [], 0
        for k, (i, kind) in enumerate(O[j]):
            # starts whose time is not after this op's start come before it
            while q < len(timed[j]) and timed[j][q][0] <= sim["start"][j][k]:
                out.append((timed[j][q][1], timed[j][q][2]))
                q += 1
            if kind == F and j > 0:
                out.append((WAIT_ACT, i))
            if kind == B and j + 1 < C:
                out.append((WAIT_GRAD, i))
            out.append((FWD if kind == F else BWD, i))
        while q < len(timed[j]):
            out.append((timed[j][q][1], timed[j][q][2]))
            q += 1
        stream.append(out)
    return queue, stream
