// Pipeline execution schedules and communication order (host only): the memory-aware adaptive
// schedule (section "Pipeline Execution Schedule", Alg. 1), the 1F1B order it is compared with, a
// device timeline under given op times, and the order of communication starts and waits (section
// "Communication Planning").  Semantics are stated with the declarations in dynastage.h.
//
// How the three are computed here.
//  * Adaptive schedule.  Every buffer of ready ops of the algorithm is fed by exactly one producer (a stage's
//    forward buffer by the previous stage's forwards, its backward buffer by the next stage's backwards, the last
//    stage's by its own forwards) and gets at most one op per cycle, so ops leave every buffer in the order the
//    micro-batches entered the pipeline.  A stage's state is therefore two counters (forwards done, backwards
//    done) and its held memory; the buffers themselves are replaced by tables of the cycle from which each op is
//    ready.  The scan over cycles stops when all ops are done, or when a cycle changes nothing (then no later
//    cycle can: nothing new became ready).
//  * Timeline.  The ops form a DAG (each op follows the previous op of its stage and its cross-stage
//    producer); start times are longest paths, evaluated in a topological order that a work list produces;
//    ops never reached mean the given orders contain a cycle (they deadlock).
//  * Communication plan.  The transfers a stage takes part in are produced by its own ops and by the ops of
//    its two neighbours; each of these three sequences is already ordered by end time, so the stage's queue of
//    starts is a three-way merge under the key (end time, producing stage, position), and every start is placed
//    by a binary search over the stage's op start times.
#include "../../include/dynastage.h"

#include <algorithm>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

namespace {

struct StageOps {                       // the ops of all stages, flattened: node id = j * 2M + k
    int32_t C = 0, M = 0;
    std::vector<int32_t> mb, kind;      // per node
    std::vector<int32_t> node_of;       // [j][mb][kind] -> node id
    size_t id(int32_t j, int32_t k) const { return (size_t)j * 2 * M + k; }
    int32_t find(int32_t j, int32_t i, int32_t kd) const { return node_of[((size_t)j * M + i) * 2 + kd]; }
};

// false: some stage's list is not a permutation of its 2M ops
bool load_orders(int32_t C, int32_t M, const int32_t* order_mb, const int32_t* order_kind, StageOps& g) {
    g.C = C;
    g.M = M;
    const size_t n = (size_t)2 * M * C;
    g.mb.assign(order_mb, order_mb + n);
    g.kind.assign(order_kind, order_kind + n);
    g.node_of.assign(n, -1);
    for (size_t v = 0; v < n; ++v) {
        const int32_t i = g.mb[v], kd = g.kind[v];
        if (i < 0 || i >= M || (kd != DS_OP_FWD && kd != DS_OP_BWD)) return false;
        int32_t& slot = g.node_of[((v / (2 * (size_t)M)) * M + i) * 2 + kd];
        if (slot >= 0) return false;
        slot = (int32_t)v;
    }
    return true;
}

// Longest-path start / end times of every op.  DS_EINVAL when the orders deadlock.
ds_status longest_paths(const StageOps& g, const int64_t* tf, const int64_t* tb, std::vector<int64_t>& start,
                        std::vector<int64_t>& end) {
    const int32_t C = g.C, M = g.M;
    const size_t n = (size_t)2 * M * C;
    // the cross-stage producer of node v, or -1
    auto producer = [&](size_t v) -> int32_t {
        const int32_t j = (int32_t)(v / (2 * (size_t)M)), i = g.mb[v];
        if (g.kind[v] == DS_OP_FWD) return j == 0 ? -1 : g.find(j - 1, i, DS_OP_FWD);
        return j == C - 1 ? g.find(j, i, DS_OP_FWD) : g.find(j + 1, i, DS_OP_BWD);
    };
    // a backward also needs its own stage's forward of the same micro-batch (it releases what that forward took)
    auto own_forward = [&](size_t v) -> int32_t {
        const int32_t j = (int32_t)(v / (2 * (size_t)M));
        return g.kind[v] == DS_OP_BWD ? g.find(j, g.mb[v], DS_OP_FWD) : -1;
    };
    std::vector<int32_t> waiting(n, 0);
    std::vector<std::vector<int32_t>> unlocks(n);
    for (size_t v = 0; v < n; ++v) {
        const bool first_of_stage = v % (2 * (size_t)M) == 0;
        if (!first_of_stage) { unlocks[v - 1].push_back((int32_t)v); ++waiting[v]; }
        const int32_t p = producer(v), f = own_forward(v);
        if (p >= 0) { unlocks[p].push_back((int32_t)v); ++waiting[v]; }
        if (f >= 0 && f != p) { unlocks[f].push_back((int32_t)v); ++waiting[v]; }
    }
    start.assign(n, 0);
    end.assign(n, 0);
    std::vector<int32_t> work;
    for (size_t v = 0; v < n; ++v)
        if (waiting[v] == 0) work.push_back((int32_t)v);
    size_t reached = 0;
    while (!work.empty()) {
        const int32_t v = work.back();
        work.pop_back();
        ++reached;
        const int32_t j = (int32_t)((size_t)v / (2 * (size_t)M));
        const size_t ij = (size_t)g.mb[v] * C + j;
        // start[v] already holds the latest end among the predecessors that constrain the start time (the stage's
        // previous op and the producer; the own forward only orders, its end never exceeds the producer's)
        if (__builtin_add_overflow(start[v], g.kind[v] == DS_OP_FWD ? tf[ij] : tb[ij], &end[v])) return DS_EOVERFLOW;
        for (int32_t u : unlocks[v]) {
            start[u] = std::max(start[u], end[v]);
            if (--waiting[u] == 0) work.push_back(u);
        }
    }
    return reached == n ? DS_OK : DS_EINVAL;
}

}  // namespace

extern "C" ds_status ds_schedule_adaptive(int32_t C, int32_t M, const int64_t* act, const int64_t* limit, int32_t* order_mb,
                                          int32_t* order_kind, int32_t* n_cycles) {
    if (C < 1 || M < 1 || !act || !limit || !order_mb || !order_kind) return DS_EINVAL;
    for (int32_t i = 0; i < M; ++i)
        for (int32_t j = 0; j < C; ++j) {
            if (act[(size_t)i * C + j] < 0) return DS_EINVAL;
            if (!(act[(size_t)i * C + j] < limit[j])) return DS_EINFEASIBLE;
        }
    try {
        constexpr int32_t kNever = std::numeric_limits<int32_t>::max();
        // cycle from which the forward / backward of micro-batch i is ready on stage j
        std::vector<int32_t> ready_f((size_t)C * M, kNever), ready_b((size_t)C * M, kNever);
        for (int32_t i = 0; i < M; ++i) ready_f[i] = 0;                 // stage 0 holds every micro-batch from the start
        std::vector<int32_t> n_fwd(C, 0), n_bwd(C, 0);                  // ops done; also the next micro-batch of each kind
        std::vector<int64_t> held(C, 0);
        size_t left = (size_t)2 * M * C;
        int32_t cycle = 0;
        for (; left > 0; ++cycle) {
            const size_t before = left;
            for (int32_t j = 0; j < C; ++j) {
                int32_t* const slot_mb = order_mb + (size_t)j * 2 * M + n_fwd[j] + n_bwd[j];
                int32_t* const slot_kind = order_kind + (size_t)j * 2 * M + n_fwd[j] + n_bwd[j];
                int32_t wrote = 0;
                const int32_t ib = n_bwd[j];
                if (ib < M && ready_b[(size_t)j * M + ib] <= cycle) {   // at most one backward, first: it frees memory
                    held[j] -= act[(size_t)ib * C + j];
                    slot_mb[wrote] = ib;
                    slot_kind[wrote++] = DS_OP_BWD;
                    ++n_bwd[j];
                    if (j > 0) ready_b[(size_t)(j - 1) * M + ib] = cycle + 1;
                }
                const int32_t jf = n_fwd[j];
                if (jf < M && ready_f[(size_t)j * M + jf] <= cycle && held[j] + act[(size_t)jf * C + j] < limit[j]) {
                    held[j] += act[(size_t)jf * C + j];
                    slot_mb[wrote] = jf;
                    slot_kind[wrote++] = DS_OP_FWD;
                    ++n_fwd[j];
                    if (j + 1 < C) ready_f[(size_t)(j + 1) * M + jf] = cycle + 1;
                    else ready_b[(size_t)j * M + jf] = cycle + 1;
                }
                left -= wrote;
            }
            if (left == before) return DS_EINFEASIBLE;                  // a cycle that changed nothing: no later one can
        }
        if (n_cycles) *n_cycles = cycle;
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    }
}

extern "C" ds_status ds_schedule_1f1b(int32_t C, int32_t M, int32_t* order_mb, int32_t* order_kind) {
    if (C < 1 || M < 1 || !order_mb || !order_kind) return DS_EINVAL;
    for (int32_t j = 0; j < C; ++j) {
        // position k of stage j: the first `warm` are forwards; after that backward b sits at warm + 2b while forwards
        // remain to alternate with (b < M - warm), and the last `warm` backwards close the list
        const int32_t warm = std::min(C - j, M);
        int32_t* const mb = order_mb + (size_t)j * 2 * M;
        int32_t* const kd = order_kind + (size_t)j * 2 * M;
        for (int32_t i = 0; i < M; ++i) {
            const int32_t pos_f = i < warm ? i : warm + 2 * (i - warm) + 1;
            const int32_t pos_b = i < M - warm ? warm + 2 * i : M + i;
            mb[pos_f] = i; kd[pos_f] = DS_OP_FWD;
            mb[pos_b] = i; kd[pos_b] = DS_OP_BWD;
        }
    }
    return DS_OK;
}

extern "C" ds_status ds_schedule_simulate(int32_t C, int32_t M, const int32_t* order_mb, const int32_t* order_kind,
                                          const int64_t* t_fwd, const int64_t* t_bwd, const int64_t* act, int64_t* makespan,
                                          int64_t* idle, int64_t* peak, int64_t* op_start, int64_t* op_end) {
    if (C < 1 || M < 1 || !order_mb || !order_kind || !t_fwd || !t_bwd || !makespan) return DS_EINVAL;
    if (peak && !act) return DS_EINVAL;
    for (size_t x = 0; x < (size_t)M * C; ++x)
        if (t_fwd[x] < 0 || t_bwd[x] < 0 || (act && act[x] < 0)) return DS_EINVAL;
    try {
        StageOps g;
        if (!load_orders(C, M, order_mb, order_kind, g)) return DS_EINVAL;
        std::vector<int64_t> start, end;
        const ds_status st = longest_paths(g, t_fwd, t_bwd, start, end);
        if (st != DS_OK) return st;
        const size_t n = start.size();
        int64_t span = 0;
        for (size_t v = 0; v < n; ++v) span = std::max(span, end[v]);
        *makespan = span;
        if (op_start) std::copy(start.begin(), start.end(), op_start);
        if (op_end) std::copy(end.begin(), end.end(), op_end);
        for (int32_t j = 0; j < C; ++j) {
            const size_t v0 = g.id(j, 0), v1 = v0 + 2 * (size_t)M;
            if (idle) {
                int64_t busy = 0;
                for (size_t v = v0; v < v1; ++v) busy += end[v] - start[v];
                idle[j] = span - busy;
            }
            if (peak) {
                // memory changes: +a at a forward's start, -a at a backward's end.  Both sequences are already in time
                // order along the stage's list (ops of a stage do not overlap), so a two-pointer sweep replaces a sort;
                // at equal times the release goes first.
                std::vector<size_t> takes, frees;
                for (size_t v = v0; v < v1; ++v) (g.kind[v] == DS_OP_FWD ? takes : frees).push_back(v);
                size_t a = 0, b = 0;
                int64_t cur = 0, top = 0;
                while (a < takes.size()) {
                    if (b < frees.size() && end[frees[b]] <= start[takes[a]]) {
                        cur -= act[(size_t)g.mb[frees[b]] * C + j];
                        ++b;
                    } else {
                        cur += act[(size_t)g.mb[takes[a]] * C + j];
                        top = std::max(top, cur);
                        ++a;
                    }
                }
                peak[j] = top;
            }
        }
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    }
}

extern "C" ds_status ds_comm_plan(int32_t C, int32_t M, const int32_t* order_mb, const int32_t* order_kind,
                                  const int64_t* t_fwd, const int64_t* t_bwd, int32_t* stream_code, int32_t* stream_mb,
                                  int32_t* stream_len) {
    if (C < 1 || M < 1 || !order_mb || !order_kind || !t_fwd || !t_bwd || !stream_code || !stream_mb || !stream_len)
        return DS_EINVAL;
    for (size_t x = 0; x < (size_t)M * C; ++x)
        if (t_fwd[x] < 0 || t_bwd[x] < 0) return DS_EINVAL;
    try {
        StageOps g;
        if (!load_orders(C, M, order_mb, order_kind, g)) return DS_EINVAL;
        std::vector<int64_t> start, end;
        const ds_status st = longest_paths(g, t_fwd, t_bwd, start, end);
        if (st != DS_OK) return st;
        const size_t cap = (size_t)8 * M;
        struct Xfer { int64_t t; int32_t code, mb; };
        // the transfer starts stage j sees that are caused by the ops of stage p (p = j-1, j or j+1), in p's op order,
        // which is their time order
        auto caused_by = [&](int32_t j, int32_t p, std::vector<Xfer>& out) {
            out.clear();
            if (p < 0 || p >= C) return;
            for (size_t v = g.id(p, 0); v < g.id(p, 0) + 2 * (size_t)M; ++v) {
                const bool fwd = g.kind[v] == DS_OP_FWD;
                if (p == j) {
                    if (fwd && j + 1 < C) out.push_back({end[v], DS_INSTR_SEND_ACT_START, g.mb[v]});
                    if (!fwd && j > 0) out.push_back({end[v], DS_INSTR_SEND_GRAD_START, g.mb[v]});
                } else if (p == j - 1) {
                    if (fwd) out.push_back({end[v], DS_INSTR_RECV_ACT_START, g.mb[v]});
                } else {
                    if (!fwd) out.push_back({end[v], DS_INSTR_RECV_GRAD_START, g.mb[v]});
                }
            }
        };
        std::vector<Xfer> src[3], queue;
        std::vector<int32_t> slot_count;
        for (int32_t j = 0; j < C; ++j) {
            for (int s = 0; s < 3; ++s) caused_by(j, j - 1 + s, src[s]);
            // three-way merge; equal times: the lower producing stage first (src index ascending)
            queue.clear();
            size_t at[3] = {0, 0, 0};
            for (;;) {
                int pick = -1;
                for (int s = 0; s < 3; ++s)
                    if (at[s] < src[s].size() && (pick < 0 || src[s][at[s]].t < src[pick][at[pick]].t)) pick = s;
                if (pick < 0) break;
                queue.push_back(src[pick][at[pick]++]);
            }
            // a start goes before the first compute op of the stage that starts at or after its time
            const int64_t* s0 = start.data() + g.id(j, 0);
            slot_count.assign(2 * (size_t)M + 1, 0);
            std::vector<int32_t> slot_of(queue.size());
            for (size_t q = 0; q < queue.size(); ++q) {
                slot_of[q] = (int32_t)(std::lower_bound(s0, s0 + 2 * (size_t)M, queue[q].t) - s0);
                ++slot_count[slot_of[q]];
            }
            size_t n = 0, q = 0;
            auto put = [&](int32_t code, int32_t mb) {
                stream_code[(size_t)j * cap + n] = code;
                stream_mb[(size_t)j * cap + n] = mb;
                ++n;
            };
            for (int32_t k = 0; k <= 2 * M; ++k) {
                for (int32_t c = 0; c < slot_count[k]; ++c, ++q) put(queue[q].code, queue[q].mb);
                if (k == 2 * M) break;
                const size_t v = g.id(j, k);
                const bool fwd = g.kind[v] == DS_OP_FWD;
                if (fwd && j > 0) put(DS_INSTR_WAIT_RECV_ACT, g.mb[v]);
                if (!fwd && j + 1 < C) put(DS_INSTR_WAIT_RECV_GRAD, g.mb[v]);
                put(fwd ? DS_INSTR_FORWARD : DS_INSTR_BACKWARD, g.mb[v]);
            }
            stream_len[j] = (int32_t)n;
        }
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    }
}
