// Pipeline execution schedules and communication order (host only): the memory-aware adaptive
// schedule (section "Pipeline Execution Schedule", Alg. 1), the 1F1B order it is compared with, a
// device timeline under given op times, and the order of communication starts and waits (section
// "Communication Planning").  Semantics are stated with the declarations in dynastage.h.
#include "../../include/dynastage.h"

#include <algorithm>
#include <cstdint>
#include <deque>
#include <new>
#include <vector>

namespace {
struct Op {
    int32_t mb, kind;   // kind: DS_OP_FWD / DS_OP_BWD
};
bool read_orders(int32_t C, int32_t M, const int32_t* order_mb, const int32_t* order_kind, std::vector<std::vector<Op>>& O) {
    O.assign(C, {});
    for (int32_t j = 0; j < C; ++j) {
        std::vector<char> seen(2 * (size_t)M, 0);
        for (int32_t k = 0; k < 2 * M; ++k) {
            const int32_t i = order_mb[(size_t)j * 2 * M + k], kind = order_kind[(size_t)j * 2 * M + k];
            if (i < 0 || i >= M || (kind != DS_OP_FWD && kind != DS_OP_BWD) || seen[2 * (size_t)i + kind]) return false;
            seen[2 * (size_t)i + kind] = 1;
            O[j].push_back({i, kind});
        }
    }
    return true;
}
struct Timeline {
    std::vector<std::vector<int64_t>> start, end;
    int64_t makespan = 0;
};
// list scheduling of the given per-stage orders; false when the orders deadlock
ds_status run_timeline(int32_t C, int32_t M, const std::vector<std::vector<Op>>& O, const int64_t* tf, const int64_t* tb,
                       Timeline& tl) {
    std::vector<int32_t> pos(C, 0);
    std::vector<int64_t> free_at(C, 0);
    std::vector<int64_t> endF((size_t)M * C, -1), endB((size_t)M * C, -1);
    tl.start.assign(C, std::vector<int64_t>(2 * (size_t)M, 0));
    tl.end = tl.start;
    size_t done = 0;
    const size_t total = (size_t)2 * M * C;
    while (done < total) {
        bool progressed = false;
        for (int32_t j = 0; j < C; ++j) {
            while (pos[j] < 2 * M) {
                const Op op = O[j][pos[j]];
                const size_t ij = (size_t)op.mb * C + j;
                int64_t dep;
                if (op.kind == DS_OP_FWD) {
                    dep = j == 0 ? 0 : endF[ij - 1];
                } else {
                    dep = j == C - 1 ? endF[ij] : endB[ij + 1];
                    if (endF[ij] < 0) dep = -1;
                }
                if (dep < 0) break;
                const int64_t s = std::max(free_at[j], dep);
                int64_t e;
                if (__builtin_add_overflow(s, op.kind == DS_OP_FWD ? tf[ij] : tb[ij], &e)) return DS_EOVERFLOW;
                tl.start[j][pos[j]] = s;
                tl.end[j][pos[j]] = e;
                (op.kind == DS_OP_FWD ? endF : endB)[ij] = e;
                free_at[j] = e;
                ++pos[j];
                ++done;
                progressed = true;
            }
        }
        if (!progressed) return DS_EINVAL;
    }
    tl.makespan = *std::max_element(free_at.begin(), free_at.end());
    return DS_OK;
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
        std::vector<std::deque<int32_t>> Sf(C), Sb(C);
        std::vector<std::vector<int32_t>> Nf(C), Nb(C);
        std::vector<int64_t> m(C, 0);
        std::vector<int32_t> filled(C, 0);
        for (int32_t i = 0; i < M; ++i) Sf[0].push_back(i);
        auto record = [&](int32_t j, int32_t i, int32_t kind) {
            order_mb[(size_t)j * 2 * M + filled[j]] = i;
            order_kind[(size_t)j * 2 * M + filled[j]] = kind;
            ++filled[j];
        };
        int32_t cycles = 0;
        for (;;) {
            bool left = false;
            for (int32_t j = 0; j < C; ++j) left = left || !Sf[j].empty() || !Sb[j].empty();
            if (!left) break;
            bool ran = false;
            for (int32_t j = 0; j < C; ++j) {
                if (!Sb[j].empty()) {                           // schedule a backward op
                    const int32_t i = Sb[j].front();
                    Sb[j].pop_front();
                    m[j] -= act[(size_t)i * C + j];
                    record(j, i, DS_OP_BWD);
                    ran = true;
                    if (j > 0) Nb[j - 1].push_back(i);
                }
                if (!Sf[j].empty()) {                           // schedule a forward op, memory permitting
                    const int32_t i = Sf[j].front();
                    const int64_t a = act[(size_t)i * C + j];
                    if (m[j] + a < limit[j]) {
                        Sf[j].pop_front();
                        m[j] += a;
                        record(j, i, DS_OP_FWD);
                        ran = true;
                        if (j + 1 < C) Nf[j + 1].push_back(i);
                        else Nb[j].push_back(i);
                    }
                }
            }
            for (int32_t j = 0; j < C; ++j) {
                for (int32_t i : Nf[j]) Sf[j].push_back(i);
                for (int32_t i : Nb[j]) Sb[j].push_back(i);
                Nf[j].clear();
                Nb[j].clear();
            }
            ++cycles;
            if (!ran) return DS_EINFEASIBLE;
        }
        if (n_cycles) *n_cycles = cycles;
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    }
}

extern "C" ds_status ds_schedule_1f1b(int32_t C, int32_t M, int32_t* order_mb, int32_t* order_kind) {
    if (C < 1 || M < 1 || !order_mb || !order_kind) return DS_EINVAL;
    for (int32_t j = 0; j < C; ++j) {
        int32_t k = 0;
        auto put = [&](int32_t i, int32_t kind) {
            order_mb[(size_t)j * 2 * M + k] = i;
            order_kind[(size_t)j * 2 * M + k] = kind;
            ++k;
        };
        const int32_t warm = std::min(C - j, M);
        for (int32_t i = 0; i < warm; ++i) put(i, DS_OP_FWD);
        int32_t nf = warm;
        for (int32_t nb = 0; nb < M; ++nb) {
            put(nb, DS_OP_BWD);
            if (nf < M) put(nf++, DS_OP_FWD);
        }
    }
    return DS_OK;
}

extern "C" ds_status ds_schedule_simulate(int32_t C, int32_t M, const int32_t* order_mb, const int32_t* order_kind,
                                          const int64_t* t_fwd, const int64_t* t_bwd, const int64_t* act, int64_t* makespan,
                                          int64_t* idle, int64_t* peak, int64_t* op_start, int64_t* op_end) {
    if (C < 1 || M < 1 || !order_mb || !order_kind || !t_fwd || !t_bwd || !makespan) return DS_EINVAL;
    for (size_t x = 0; x < (size_t)M * C; ++x)
        if (t_fwd[x] < 0 || t_bwd[x] < 0 || (act && act[x] < 0)) return DS_EINVAL;
    try {
        std::vector<std::vector<Op>> O;
        if (!read_orders(C, M, order_mb, order_kind, O)) return DS_EINVAL;
        Timeline tl;
        ds_status st = run_timeline(C, M, O, t_fwd, t_bwd, tl);
        if (st != DS_OK) return st;
        *makespan = tl.makespan;
        for (int32_t j = 0; j < C; ++j) {
            int64_t busy = 0;
            for (int32_t k = 0; k < 2 * M; ++k) {
                busy += tl.end[j][k] - tl.start[j][k];
                if (op_start) op_start[(size_t)j * 2 * M + k] = tl.start[j][k];
                if (op_end) op_end[(size_t)j * 2 * M + k] = tl.end[j][k];
            }
            if (idle) idle[j] = tl.makespan - busy;
            if (peak) {
                if (!act) return DS_EINVAL;
                struct Ev { int64_t t; int32_t take; int64_t dm; };
                std::vector<Ev> ev;
                for (int32_t k = 0; k < 2 * M; ++k) {
                    const Op op = O[j][k];
                    const int64_t a = act[(size_t)op.mb * C + j];
                    if (op.kind == DS_OP_FWD) ev.push_back({tl.start[j][k], 1, a});
                    else ev.push_back({tl.end[j][k], 0, -a});
                }
                std::stable_sort(ev.begin(), ev.end(), [](const Ev& x, const Ev& y) {
                    if (x.t != y.t) return x.t < y.t;
                    return x.take < y.take;                     // at equal times memory is freed before it is taken
                });
                int64_t cur = 0, pk = 0;
                for (const Ev& e : ev) { cur += e.dm; pk = std::max(pk, cur); }
                peak[j] = pk;
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
        std::vector<std::vector<Op>> O;
        if (!read_orders(C, M, order_mb, order_kind, O)) return DS_EINVAL;
        Timeline tl;
        ds_status st = run_timeline(C, M, O, t_fwd, t_bwd, tl);
        if (st != DS_OK) return st;
        struct Done { int64_t end; int32_t j, k; };
        std::vector<Done> ops;
        for (int32_t j = 0; j < C; ++j)
            for (int32_t k = 0; k < 2 * M; ++k) ops.push_back({tl.end[j][k], j, k});
        std::sort(ops.begin(), ops.end(), [](const Done& a, const Done& b) {
            if (a.end != b.end) return a.end < b.end;
            if (a.j != b.j) return a.j < b.j;
            return a.k < b.k;
        });
        struct Start { int64_t t; int32_t code, mb; };
        std::vector<std::vector<Start>> timed(C);
        for (const Done& d : ops) {
            const Op op = O[d.j][d.k];
            if (op.kind == DS_OP_FWD && d.j + 1 < C) {
                timed[d.j].push_back({d.end, DS_INSTR_SEND_ACT_START, op.mb});
                timed[d.j + 1].push_back({d.end, DS_INSTR_RECV_ACT_START, op.mb});
            }
            if (op.kind == DS_OP_BWD && d.j > 0) {
                timed[d.j].push_back({d.end, DS_INSTR_SEND_GRAD_START, op.mb});
                timed[d.j - 1].push_back({d.end, DS_INSTR_RECV_GRAD_START, op.mb});
            }
        }
        const size_t cap = (size_t)8 * M;
        for (int32_t j = 0; j < C; ++j) {
            size_t n = 0, q = 0;
            auto put = [&](int32_t code, int32_t mb) {
                stream_code[(size_t)j * cap + n] = code;
                stream_mb[(size_t)j * cap + n] = mb;
                ++n;
            };
            for (int32_t k = 0; k < 2 * M; ++k) {
                while (q < timed[j].size() && timed[j][q].t <= tl.start[j][k]) {
                    put(timed[j][q].code, timed[j][q].mb);
                    ++q;
                }
                const Op op = O[j][k];
                if (op.kind == DS_OP_FWD && j > 0) put(DS_INSTR_WAIT_RECV_ACT, op.mb);
                if (op.kind == DS_OP_BWD && j + 1 < C) put(DS_INSTR_WAIT_RECV_GRAD, op.mb);
                put(op.kind == DS_OP_FWD ? DS_INSTR_FORWARD : DS_INSTR_BACKWARD, op.mb);
            }
            for (; q < timed[j].size(); ++q) put(timed[j][q].code, timed[j][q].mb);
            stream_len[j] = (int32_t)n;
        }
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    }
}
