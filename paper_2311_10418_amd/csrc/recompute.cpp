// Dynamic recomputation (section "Implementation", paragraph "Dynamic recomputation"), host only: micro-batch
// partitioning and scheduling are repeated once per recomputation scheme, each under the scheme's own cost model and
// activation size, and the scheme with the shortest simulated iteration that stays inside the memory limit is kept.
// Built from the library's own entry points (dp_plan, ds_schedule_adaptive, ds_schedule_simulate); semantics are
// stated with the declaration in dynastage.h.
#include "../../include/dynastage.h"

#include <cstddef>
#include <cstdint>
#include <new>
#include <vector>

namespace {
// makespan / peak of one scheme; DS_EINFEASIBLE when the scheme cannot hold the batch
ds_status evaluate(const int32_t* len, const int32_t* len_tgt, int32_t n, const ds_recompute_scheme& sc, int64_t mem_limit,
                   int32_t C, ds_layout** layout, int64_t* makespan, int64_t* peak) {
    *layout = nullptr;
    if (sc.act_per_row <= 0 || sc.fwd_den <= 0 || sc.fwd_num < 0 || sc.fwd_num > sc.fwd_den) return DS_EINVAL;
    // Alg. 1 admits a forward only while held + own < limit: one micro-batch alone needs act_per_row * rows < limit
    const int64_t cap = (mem_limit - 1) / sc.act_per_row;
    if (cap < 1) return DS_EINFEASIBLE;
    ds_layout* lo = nullptr;
    ds_status st = dp_plan(len, len_tgt, n, &sc.cm, cap, C, &lo);
    if (st != DS_OK) return st;
    ds_layout_view v;
    st = ds_layout_get(lo, &v);
    if (st != DS_OK || !v.mb_cost) {
        ds_layout_free(lo);
        return st != DS_OK ? st : DS_EINVAL;
    }
    const int32_t M = v.n_mb;
    std::vector<int64_t> tf((size_t)M * C), tb((size_t)M * C), act((size_t)M * C), limit(C, mem_limit);
    for (int32_t m = 0; m < M; ++m) {
        const int64_t t = v.mb_cost[m];
        if (t < 0 || (sc.fwd_num > 0 && t > INT64_MAX / sc.fwd_num)) {
            ds_layout_free(lo);
            return DS_EOVERFLOW;
        }
        const int64_t f = t * sc.fwd_num / sc.fwd_den;
        const int64_t rows = (int64_t)v.mb_nrows[m] + (v.mb_nrows_tgt ? (int64_t)v.mb_nrows_tgt[m] : 0);
        if (rows > INT64_MAX / sc.act_per_row) {
            ds_layout_free(lo);
            return DS_EOVERFLOW;
        }
        for (int32_t j = 0; j < C; ++j) {
            tf[(size_t)m * C + j] = f;
            tb[(size_t)m * C + j] = t - f;
            act[(size_t)m * C + j] = sc.act_per_row * rows;
        }
    }
    std::vector<int32_t> order_mb((size_t)C * 2 * M), order_kind((size_t)C * 2 * M);
    std::vector<int64_t> pk(C);
    st = ds_schedule_adaptive(C, M, act.data(), limit.data(), order_mb.data(), order_kind.data(), nullptr);
    if (st == DS_OK)
        st = ds_schedule_simulate(C, M, order_mb.data(), order_kind.data(), tf.data(), tb.data(), act.data(), makespan,
                                  nullptr, pk.data(), nullptr, nullptr);
    if (st != DS_OK) {
        ds_layout_free(lo);
        return st;
    }
    *peak = 0;
    for (int32_t j = 0; j < C; ++j)
        if (pk[j] > *peak) *peak = pk[j];
    *layout = lo;
    return DS_OK;
}
}  // namespace

extern "C" ds_status ds_plan_recompute(const int32_t* len, const int32_t* len_tgt, int32_t n,
                                       const ds_recompute_scheme* schemes, int32_t n_schemes, int64_t mem_limit,
                                       int32_t num_stages, int32_t* chosen, ds_layout** out, int64_t* makespan,
                                       int64_t* peak) {
    if (out) *out = nullptr;
    if (!len || n < 1 || !schemes || n_schemes < 1 || mem_limit < 1 || num_stages < 1 || !chosen || !out) return DS_EINVAL;
    try {
        ds_layout* best = nullptr;
        int32_t best_r = -1;
        int64_t best_time = 0;
        for (int32_t r = 0; r < n_schemes; ++r) {
            ds_layout* lo = nullptr;
            int64_t ms = -1, pk = -1;
            const ds_status st = evaluate(len, len_tgt, n, schemes[r], mem_limit, num_stages, &lo, &ms, &pk);
            if (st != DS_OK && st != DS_EINFEASIBLE) {
                ds_layout_free(best);
                return st;
            }
            if (st == DS_EINFEASIBLE) ms = pk = -1;
            if (makespan) makespan[r] = ms;
            if (peak) peak[r] = pk;
            if (st == DS_OK && (best_r < 0 || ms < best_time)) {         // equal times: the scheme listed first stays
                ds_layout_free(best);
                best = lo;
                best_r = r;
                best_time = ms;
            } else {
                ds_layout_free(lo);
            }
        }
        if (best_r < 0) return DS_EINFEASIBLE;
        *chosen = best_r;
        *out = best;
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    }
}
