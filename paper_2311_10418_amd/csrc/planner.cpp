// Host-side micro-batch planner: sample ordering, the t_max-parameterised dynamic programme of
// the paper's section "Micro-batch Construction" (Eq1, Eq2, memory cap), and layout builders
// for the padding and packing baselines of section "Background".
//
// Design notes.  The candidate set of t_max is every distinct admissible slice cost.  Slices
// are sorted by cost once; as t_max grows, newly admissible slices are switched on
// incrementally, so each candidate only re-runs the O(N^2) recurrence, with one exactness-
// preserving cut-off: f(N; t_max) never increases with t_max, so once
// (c-1)*t_max + f(N; +inf) can no longer beat the incumbent objective the scan stops.
#include "../../include/dynastage.h"
#include "layout.hpp"

#include <algorithm>
#include <limits>
#include <climits>
#include <cmath>
#include <memory>
#include <new>
#include <numeric>

namespace {

constexpr int64_t kInf = std::numeric_limits<int64_t>::max();

std::atomic<uint64_t> g_uid{1};

struct CostEval {
    const ds_cost_model* cm;
    // returns DS_OK and sets *t, or an error status
    ds_status operator()(int64_t b, int64_t L, int64_t Lt, int64_t* t) const {
        int64_t a, s, r;
        switch (cm->kind) {
        case DS_COST_POLY_GPT:
            if (__builtin_add_overflow(cm->lin, L, &s) || __builtin_mul_overflow(b, L, &a) ||
                __builtin_mul_overflow(a, s, &a) || __builtin_add_overflow(a, cm->fixed, &r))
                return DS_EOVERFLOW;
            *t = r;
            return DS_OK;
        case DS_COST_POLY_T5: {
            int64_t e, d;
            if (__builtin_add_overflow(cm->lin, L, &s) || __builtin_mul_overflow(b, L, &e) ||
                __builtin_mul_overflow(e, s, &e))
                return DS_EOVERFLOW;
            if (__builtin_add_overflow(cm->lin, Lt, &s) || __builtin_add_overflow(s, L, &s) ||
                __builtin_mul_overflow(b, Lt, &d) || __builtin_mul_overflow(d, s, &d))
                return DS_EOVERFLOW;
            if (__builtin_add_overflow(e, d, &r) || __builtin_add_overflow(r, cm->fixed, &r))
                return DS_EOVERFLOW;
            *t = r;
            return DS_OK;
        }
        case DS_COST_TABLE:
            if (b > cm->tb || L > cm->tl) return DS_EINVAL;
            *t = cm->table[(b - 1) * (int64_t)cm->tl + (L - 1)];
            if (*t < 0 || *t == kInf) return DS_EINVAL;
            return DS_OK;
        }
        return DS_EINVAL;
    }
};

ds_status check_cost_model(const ds_cost_model* cm, bool has_tgt) {
    if (!cm) return DS_EINVAL;
    switch (cm->kind) {
    case DS_COST_POLY_GPT:
        return (cm->fixed >= 0 && cm->lin >= 0) ? DS_OK : DS_EINVAL;
    case DS_COST_POLY_T5:
        return (cm->fixed >= 0 && cm->lin >= 0 && has_tgt) ? DS_OK : DS_EINVAL;
    case DS_COST_TABLE:
        return (cm->table && cm->tb > 0 && cm->tl > 0 && !has_tgt) ? DS_OK : DS_EINVAL;
    }
    return DS_EINVAL;
}

ds_status check_lengths(const int32_t* len, const int32_t* len_tgt, int32_t n) {
    if (!len || n <= 0) return DS_EINVAL;
    for (int32_t i = 0; i < n; ++i) {
        if (len[i] <= 0) return DS_EINVAL;
        if (len_tgt && len_tgt[i] <= 0) return DS_EINVAL;
    }
    return DS_OK;
}

// Fill rows / offsets of a layout whose perm, mb_start, mb_count, mb_lpad (and mb_ltgt) are set.
ds_status place_padded(ds_layout& lo, const int32_t* len, const int32_t* len_tgt) {
    const int32_t n = lo.n_seq;
    lo.seq_row.assign(n, 0);
    lo.seq_len.assign(n, 0);
    lo.mb_row.assign(lo.n_mb, 0);
    lo.mb_nrows.assign(lo.n_mb, 0);
    if (lo.has_tgt) {
        lo.seq_row_tgt.assign(n, 0);
        lo.seq_len_tgt.assign(n, 0);
        lo.mb_row_tgt.assign(lo.n_mb, 0);
        lo.mb_nrows_tgt.assign(lo.n_mb, 0);
    }
    int64_t row = 0, row_t = 0;
    lo.total_tokens = lo.total_tokens_tgt = 0;
    for (int32_t m = 0; m < lo.n_mb; ++m) {
        const int64_t b = lo.mb_count[m], L = lo.mb_lpad[m];
        if (row + b * L > std::numeric_limits<int32_t>::max()) return DS_EOVERFLOW;
        lo.mb_row[m] = (int32_t)row;
        lo.mb_nrows[m] = (int32_t)(b * L);
        for (int32_t j = 0; j < b; ++j) {
            const int32_t s = lo.mb_start[m] + j;
            lo.seq_row[s] = (int32_t)(row + j * L);
            lo.seq_len[s] = len[lo.perm[s]];
            lo.total_tokens += lo.seq_len[s];
        }
        row += b * L;
        if (lo.has_tgt) {
            const int64_t Lt = lo.mb_ltgt[m];
            if (row_t + b * Lt > std::numeric_limits<int32_t>::max()) return DS_EOVERFLOW;
            lo.mb_row_tgt[m] = (int32_t)row_t;
            lo.mb_nrows_tgt[m] = (int32_t)(b * Lt);
            for (int32_t j = 0; j < b; ++j) {
                const int32_t s = lo.mb_start[m] + j;
                lo.seq_row_tgt[s] = (int32_t)(row_t + j * Lt);
                lo.seq_len_tgt[s] = len_tgt[lo.perm[s]];
                lo.total_tokens_tgt += lo.seq_len_tgt[s];
            }
            row_t += b * Lt;
        }
    }
    lo.total_rows = (int32_t)row;
    lo.total_rows_tgt = (int32_t)row_t;
    return DS_OK;
}

// Objective of an already-built padded layout under a cost model (Eq1).
ds_status score(ds_layout& lo, const ds_cost_model* cm, int32_t num_stages) {
    lo.objective = lo.t_max = 0;
    lo.mb_cost.clear();
    if (!cm) return DS_OK;
    CostEval cost{cm};
    int64_t sum = 0, mx = 0;
    for (int32_t m = 0; m < lo.n_mb; ++m) {
        int64_t t;
        ds_status st = cost(lo.mb_count[m], lo.mb_lpad[m], lo.has_tgt ? lo.mb_ltgt[m] : 0, &t);
        if (st != DS_OK) return st;
        lo.mb_cost.push_back(t);
        if (__builtin_add_overflow(sum, t, &sum)) return DS_EOVERFLOW;
        mx = std::max(mx, t);
    }
    int64_t J;
    if (__builtin_mul_overflow((int64_t)(num_stages - 1), mx, &J) || __builtin_add_overflow(J, sum, &J))
        return DS_EOVERFLOW;
    lo.objective = J;
    lo.t_max = mx;
    return DS_OK;
}

struct Slice {
    int64_t t;
    int32_t i, j;   // sorted positions [i, j)
};

}  // namespace

uint64_t ds_next_layout_uid() { return g_uid.fetch_add(1); }

// The dynamic programme of Eq2 over every candidate t_max, minimising  w * max_m t + sum_m t  (Eq1 with
// w = num_stages - 1; the data-parallel variant passes w = n_replicas * (num_stages - 1)).
// quantum > 0: t_max is sampled at the multiples of quantum (a slice cost t admits the slice from the candidate
// ceil(t / quantum) * quantum on); the layout then reports the objective and t_max of the partition chosen.
static ds_status plan_impl(const int32_t* len, const int32_t* len_tgt, int32_t n, const ds_cost_model* cm, int64_t cap,
                           int64_t w, ds_layout** out, int64_t quantum = 0) {
    if (!out) return DS_EINVAL;
    *out = nullptr;
    ds_status st = check_lengths(len, len_tgt, n);
    if (st != DS_OK) return st;
    if (w < 0 || cap <= 0) return DS_EINVAL;
    st = check_cost_model(cm, len_tgt != nullptr);
    if (st != DS_OK) return st;

    try {
        std::unique_ptr<ds_layout> lo(new ds_layout());
        lo->n_seq = n;
        lo->has_tgt = len_tgt != nullptr;
        lo->uid = ds_next_layout_uid();

        // 1. ordering: ascending (len, len_tgt), ties by original index
        lo->perm.resize(n);
        std::iota(lo->perm.begin(), lo->perm.end(), 0);
        std::stable_sort(lo->perm.begin(), lo->perm.end(), [&](int32_t a, int32_t b) {
            if (len[a] != len[b]) return len[a] < len[b];
            if (len_tgt && len_tgt[a] != len_tgt[b]) return len_tgt[a] < len_tgt[b];
            return false;
        });

        // 2. admissible slices and their costs
        CostEval cost{cm};
        std::vector<Slice> slices;
        slices.reserve((size_t)n * (n + 1) / 2);
        for (int32_t i = 0; i < n; ++i) {
            int64_t L = 0, Lt = 0;
            for (int32_t j = i + 1; j <= n; ++j) {
                const int32_t s = lo->perm[j - 1];
                L = std::max<int64_t>(L, len[s]);
                if (len_tgt) Lt = std::max<int64_t>(Lt, len_tgt[s]);
                const int64_t b = j - i;
                if (b * L > cap) continue;
                int64_t t;
                st = cost(b, L, Lt, &t);
                if (st != DS_OK) return st;
                slices.push_back({t, i, j});
            }
        }
        std::sort(slices.begin(), slices.end(), [](const Slice& a, const Slice& b) {
            if (a.t != b.t) return a.t < b.t;
            if (a.j != b.j) return a.j < b.j;
            return a.i < b.i;
        });

        // active[j] = slices ending at j admitted so far, as (i, t); kept unsorted, scanned fully.
        std::vector<std::vector<std::pair<int32_t, int64_t>>> active(n + 1);
        std::vector<int64_t> f(n + 1);
        std::vector<int32_t> arg(n + 1), best_arg;

        // lower bound of the sum term: f(N; +inf)
        int64_t f_inf = kInf;
        {
            std::vector<std::vector<std::pair<int32_t, int64_t>>> all(n + 1);
            for (const Slice& s : slices) all[s.j].push_back({s.i, s.t});
            f[0] = 0;
            for (int32_t nn = 1; nn <= n; ++nn) {
                int64_t bv = kInf;
                for (auto& e : all[nn]) {
                    if (f[e.first] == kInf) continue;
                    int64_t v;
                    if (__builtin_add_overflow(f[e.first], e.second, &v)) return DS_EOVERFLOW;
                    bv = std::min(bv, v);
                }
                f[nn] = bv;
            }
            f_inf = f[n];
            if (f_inf == kInf) return DS_EINFEASIBLE;
        }

        int64_t bestJ = kInf, bestT = 0;
        bool found = false;
        size_t k = 0;
        while (k < slices.size()) {
            int64_t T = slices[k].t;
            if (quantum > 0) {
                const int64_t up = T / quantum + (T % quantum != 0);
                if (__builtin_mul_overflow(up, quantum, &T)) return DS_EOVERFLOW;
            }
            while (k < slices.size() && slices[k].t <= T) {
                active[slices[k].j].push_back({slices[k].i, slices[k].t});
                ++k;
            }
            // cut-off: no t_max >= T can strictly improve on the incumbent
            if (found) {
                int64_t lb;
                if (__builtin_mul_overflow(w, T, &lb) || __builtin_add_overflow(lb, f_inf, &lb))
                    return DS_EOVERFLOW;
                if (lb >= bestJ) break;
            }
            // recurrence (Eq2)
            f[0] = 0;
            for (int32_t nn = 1; nn <= n; ++nn) {
                int64_t bv = kInf;
                int32_t bi = -1;
                for (auto& e : active[nn]) {
                    const int64_t fi = f[e.first];
                    if (fi == kInf) continue;
                    int64_t v;
                    if (__builtin_add_overflow(fi, e.second, &v)) return DS_EOVERFLOW;
                    if (v < bv || (v == bv && e.first < bi)) { bv = v; bi = e.first; }
                }
                f[nn] = bv;
                arg[nn] = bi;
            }
            if (f[n] == kInf) continue;
            int64_t J;
            if (__builtin_mul_overflow(w, T, &J) || __builtin_add_overflow(J, f[n], &J))
                return DS_EOVERFLOW;
            if (!found || J < bestJ) {
                found = true;
                bestJ = J;
                bestT = T;
                best_arg = arg;
            }
        }
        if (!found) return DS_EINFEASIBLE;

        // 3. backtrack
        std::vector<int32_t> ends;
        for (int32_t pos = n; pos > 0; pos = best_arg[pos]) ends.push_back(pos);
        std::reverse(ends.begin(), ends.end());
        lo->n_mb = (int32_t)ends.size();
        lo->mb_start.resize(lo->n_mb);
        lo->mb_count.resize(lo->n_mb);
        lo->mb_lpad.resize(lo->n_mb);
        if (lo->has_tgt) lo->mb_ltgt.resize(lo->n_mb);
        int32_t start = 0;
        for (int32_t m = 0; m < lo->n_mb; ++m) {
            lo->mb_start[m] = start;
            lo->mb_count[m] = ends[m] - start;
            int32_t L = 0, Lt = 0;
            for (int32_t s = start; s < ends[m]; ++s) {
                L = std::max(L, len[lo->perm[s]]);
                if (len_tgt) Lt = std::max(Lt, len_tgt[lo->perm[s]]);
            }
            lo->mb_lpad[m] = L;
            if (lo->has_tgt) lo->mb_ltgt[m] = Lt;
            start = ends[m];
        }
        st = place_padded(*lo, len, len_tgt);
        if (st != DS_OK) return st;
        for (int32_t m = 0; m < lo->n_mb; ++m) {
            int64_t t;
            st = cost(lo->mb_count[m], lo->mb_lpad[m], lo->has_tgt ? lo->mb_ltgt[m] : 0, &t);
            if (st != DS_OK) return st;
            lo->mb_cost.push_back(t);
        }
        lo->objective = bestJ;
        lo->t_max = bestT;
        if (quantum > 0) {                                   // report the chosen partition itself, not the sampled bound
            int64_t mx = 0, sum = 0, J;
            for (int64_t t : lo->mb_cost) {
                mx = std::max(mx, t);
                if (__builtin_add_overflow(sum, t, &sum)) return DS_EOVERFLOW;
            }
            if (__builtin_mul_overflow(w, mx, &J) || __builtin_add_overflow(J, sum, &J)) return DS_EOVERFLOW;
            lo->objective = J;
            lo->t_max = mx;
        }
        *out = lo.release();
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    } catch (...) {
        return DS_EINVAL;
    }
}

extern "C" ds_status dp_plan(const int32_t* len, const int32_t* len_tgt, int32_t n,
                             const ds_cost_model* cm, int64_t cap, int32_t c, ds_layout** out) {
    if (out) *out = nullptr;
    if (c < 1) return DS_EINVAL;
    return plan_impl(len, len_tgt, n, cm, cap, (int64_t)c - 1, out);
}

extern "C" ds_status dp_plan_sampled(const int32_t* len, const int32_t* len_tgt, int32_t n, const ds_cost_model* cm,
                                     int64_t cap, int32_t c, int64_t t_max_interval, ds_layout** out) {
    if (out) *out = nullptr;
    if (c < 1 || t_max_interval < 1) return DS_EINVAL;
    return plan_impl(len, len_tgt, n, cm, cap, (int64_t)c - 1, out, t_max_interval);
}

// ------------------------------------------------------------------------------------ replica balancing
namespace {
struct KkSet {
    int64_t sum;
    int32_t min_idx;                    // smallest member index; INT32_MAX for an empty set
    std::vector<int32_t> items;
};
struct KkPart {
    std::vector<KkSet> sets;            // canonical order: sum descending, then smallest member index ascending
    int64_t spread;
    int64_t seq;                        // creation number
};
void kk_canon(KkPart& p) {
    std::sort(p.sets.begin(), p.sets.end(), [](const KkSet& a, const KkSet& b) {
        if (a.sum != b.sum) return a.sum > b.sum;
        return a.min_idx < b.min_idx;
    });
    p.spread = p.sets.front().sum - p.sets.back().sum;
}
}  // namespace

extern "C" ds_status ds_assign_replicas(const int64_t* t, int32_t n_items, int32_t k, int32_t* replica_of,
                                        int64_t* replica_time) {
    if (n_items < 0 || k < 1 || !replica_time || (n_items > 0 && (!t || !replica_of))) return DS_EINVAL;
    int64_t total = 0;
    for (int32_t i = 0; i < n_items; ++i) {
        if (t[i] < 0) return DS_EINVAL;
        if (__builtin_add_overflow(total, t[i], &total)) return DS_EOVERFLOW;
    }
    for (int32_t r = 0; r < k; ++r) replica_time[r] = 0;
    if (n_items == 0) return DS_OK;
    try {
        std::vector<int32_t> order(n_items);
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return t[a] > t[b]; });
        // largest spread first, then earliest created
        auto later = [](const KkPart& a, const KkPart& b) {
            if (a.spread != b.spread) return a.spread < b.spread;
            return a.seq > b.seq;
        };
        std::vector<KkPart> heap;
        heap.reserve(n_items);
        int64_t seq = 0;
        for (int32_t i : order) {
            KkPart p;
            p.sets.resize(k);
            for (KkSet& s : p.sets) { s.sum = 0; s.min_idx = INT32_MAX; }
            p.sets[0].sum = t[i];
            p.sets[0].min_idx = i;
            p.sets[0].items.push_back(i);
            p.seq = seq++;
            kk_canon(p);
            heap.push_back(std::move(p));
            std::push_heap(heap.begin(), heap.end(), later);
        }
        while (heap.size() > 1) {
            std::pop_heap(heap.begin(), heap.end(), later);
            KkPart a = std::move(heap.back());
            heap.pop_back();
            std::pop_heap(heap.begin(), heap.end(), later);
            KkPart b = std::move(heap.back());
            heap.pop_back();
            for (int32_t p = 0; p < k; ++p) {            // a descending with b ascending
                KkSet& dst = a.sets[p];
                KkSet& src = b.sets[k - 1 - p];
                dst.sum += src.sum;
                dst.min_idx = std::min(dst.min_idx, src.min_idx);
                dst.items.insert(dst.items.end(), src.items.begin(), src.items.end());
            }
            a.seq = seq++;
            kk_canon(a);
            heap.push_back(std::move(a));
            std::push_heap(heap.begin(), heap.end(), later);
        }
        const KkPart& fin = heap.front();
        for (int32_t r = 0; r < k; ++r) {
            replica_time[r] = fin.sets[r].sum;
            for (int32_t i : fin.sets[r].items) replica_of[i] = r;
        }
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    }
}

extern "C" ds_status dp_plan_replicas(const int32_t* len, const int32_t* len_tgt, int32_t n, const ds_cost_model* cm,
                                      int64_t cap, int32_t c, int32_t n_replicas, ds_layout** out, int32_t* replica_of_mb,
                                      int64_t* replica_time) {
    if (out) *out = nullptr;
    if (c < 1 || n_replicas < 1 || !replica_of_mb || !replica_time) return DS_EINVAL;
    int64_t w;
    if (__builtin_mul_overflow((int64_t)c - 1, (int64_t)n_replicas, &w)) return DS_EOVERFLOW;
    ds_status st = plan_impl(len, len_tgt, n, cm, cap, w, out);
    if (st != DS_OK) return st;
    st = ds_assign_replicas((*out)->mb_cost.data(), (*out)->n_mb, n_replicas, replica_of_mb, replica_time);
    if (st != DS_OK) {
        delete *out;
        *out = nullptr;
    }
    return st;
}

extern "C" ds_status ds_layout_from_cuts(const int32_t* len, const int32_t* len_tgt, int32_t n,
                                         const int32_t* perm, const int32_t* cuts, int32_t n_mb,
                                         int32_t pad_to, int32_t pad_to_tgt,
                                         const ds_cost_model* cm, int32_t num_stages, ds_layout** out) {
    if (!out) return DS_EINVAL;
    *out = nullptr;
    ds_status st = check_lengths(len, len_tgt, n);
    if (st != DS_OK) return st;
    if (!cuts || n_mb <= 0 || n_mb > n || pad_to < 0 || pad_to_tgt < 0) return DS_EINVAL;
    if (cm) {
        st = check_cost_model(cm, len_tgt != nullptr);
        if (st != DS_OK) return st;
        if (num_stages < 1) return DS_EINVAL;
    }
    if (cuts[0] != 0 || cuts[n_mb] != n) return DS_EINVAL;
    for (int32_t m = 0; m < n_mb; ++m)
        if (cuts[m + 1] <= cuts[m]) return DS_EINVAL;
    try {
        std::unique_ptr<ds_layout> lo(new ds_layout());
        lo->n_seq = n;
        lo->n_mb = n_mb;
        lo->has_tgt = len_tgt != nullptr;
        lo->uid = ds_next_layout_uid();
        lo->perm.resize(n);
        if (perm) {
            std::vector<char> seen(n, 0);
            for (int32_t i = 0; i < n; ++i) {
                if (perm[i] < 0 || perm[i] >= n || seen[perm[i]]) return DS_EINVAL;
                seen[perm[i]] = 1;
                lo->perm[i] = perm[i];
            }
        } else {
            std::iota(lo->perm.begin(), lo->perm.end(), 0);
        }
        lo->mb_start.resize(n_mb);
        lo->mb_count.resize(n_mb);
        lo->mb_lpad.resize(n_mb);
        if (lo->has_tgt) lo->mb_ltgt.resize(n_mb);
        for (int32_t m = 0; m < n_mb; ++m) {
            lo->mb_start[m] = cuts[m];
            lo->mb_count[m] = cuts[m + 1] - cuts[m];
            int32_t L = 0, Lt = 0;
            for (int32_t s = cuts[m]; s < cuts[m + 1]; ++s) {
                L = std::max(L, len[lo->perm[s]]);
                if (len_tgt) Lt = std::max(Lt, len_tgt[lo->perm[s]]);
            }
            if (pad_to) { if (pad_to < L) return DS_EINVAL; L = pad_to; }
            if (lo->has_tgt && pad_to_tgt) { if (pad_to_tgt < Lt) return DS_EINVAL; Lt = pad_to_tgt; }
            lo->mb_lpad[m] = L;
            if (lo->has_tgt) lo->mb_ltgt[m] = Lt;
        }
        st = place_padded(*lo, len, len_tgt);
        if (st != DS_OK) return st;
        st = score(*lo, cm, num_stages);
        if (st != DS_OK) return st;
        *out = lo.release();
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    } catch (...) {
        return DS_EINVAL;
    }
}

extern "C" ds_status ds_layout_token_based(const int32_t* len, const int32_t* len_tgt, int32_t n, int64_t token_budget,
                                            const ds_cost_model* cm, int32_t num_stages, ds_layout** out) {
    if (!out) return DS_EINVAL;
    *out = nullptr;
    ds_status st = check_lengths(len, len_tgt, n);
    if (st != DS_OK) return st;
    if (token_budget <= 0) return DS_EINVAL;
    try {
        // the dynamic programme's order: ascending (input length, target length), equal keys by original index
        std::vector<int32_t> perm(n);
        std::iota(perm.begin(), perm.end(), 0);
        std::stable_sort(perm.begin(), perm.end(), [&](int32_t a, int32_t b) {
            if (len[a] != len[b]) return len[a] < len[b];
            return len_tgt && len_tgt[a] < len_tgt[b];
        });
        // ascending lengths: the longest sample of a micro-batch is its last one, so "one more sample fits" is a
        // test on the candidate alone
        std::vector<int32_t> cuts{0};
        int32_t start = 0;
        for (int32_t k = 0; k < n; ++k) {
            const int64_t l = len[perm[k]];
            if (l > token_budget) return DS_EINFEASIBLE;
            if ((int64_t)(k + 1 - start) * l > token_budget) {
                cuts.push_back(k);
                start = k;
            }
        }
        cuts.push_back(n);
        return ds_layout_from_cuts(len, len_tgt, n, perm.data(), cuts.data(), (int32_t)cuts.size() - 1, 0, 0, cm, num_stages, out);
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    }
}

extern "C" ds_status ds_layout_packed(const int32_t* len, int32_t n, int32_t row_len, int32_t rows_per_mb,
                                      ds_layout** out) {
    if (!out) return DS_EINVAL;
    *out = nullptr;
    ds_status st = check_lengths(len, nullptr, n);
    if (st != DS_OK) return st;
    if (row_len <= 0 || rows_per_mb <= 0) return DS_EINVAL;
    for (int32_t i = 0; i < n; ++i)
        if (len[i] > row_len) return DS_EINVAL;
    try {
        // first-fit: each sequence goes into the first row with enough room
        std::vector<int32_t> used;                 // tokens used per row
        std::vector<int32_t> row_of(n), off_of(n);
        for (int32_t i = 0; i < n; ++i) {
            size_t r = 0;
            while (r < used.size() && used[r] + len[i] > row_len) ++r;
            if (r == used.size()) used.push_back(0);
            row_of[i] = (int32_t)r;
            off_of[i] = used[r];
            used[r] += len[i];
        }
        const int64_t n_rows = (int64_t)used.size();
        const int64_t n_mb = (n_rows + rows_per_mb - 1) / rows_per_mb;
        if (n_mb * rows_per_mb * (int64_t)row_len > std::numeric_limits<int32_t>::max()) return DS_EOVERFLOW;
        std::unique_ptr<ds_layout> lo(new ds_layout());
        lo->n_seq = n;
        lo->n_mb = (int32_t)n_mb;
        lo->uid = ds_next_layout_uid();
        // order sequences by (row, offset) so that micro-batches hold consecutive positions
        lo->perm.resize(n);
        std::iota(lo->perm.begin(), lo->perm.end(), 0);
        std::stable_sort(lo->perm.begin(), lo->perm.end(), [&](int32_t a, int32_t b) {
            if (row_of[a] != row_of[b]) return row_of[a] < row_of[b];
            return off_of[a] < off_of[b];
        });
        lo->mb_start.assign(n_mb, 0);
        lo->mb_count.assign(n_mb, 0);
        lo->mb_lpad.assign(n_mb, row_len);
        lo->mb_row.resize(n_mb);
        lo->mb_nrows.assign(n_mb, rows_per_mb * row_len);
        for (int64_t m = 0; m < n_mb; ++m) lo->mb_row[m] = (int32_t)(m * rows_per_mb * row_len);
        lo->seq_row.resize(n);
        lo->seq_len.resize(n);
        for (int32_t s = 0; s < n; ++s) {
            const int32_t i = lo->perm[s];
            const int32_t m = row_of[i] / rows_per_mb;
            if (lo->mb_count[m] == 0) lo->mb_start[m] = s;
            lo->mb_count[m]++;
            lo->seq_row[s] = row_of[i] * row_len + off_of[i];
            lo->seq_len[s] = len[i];
            lo->total_tokens += len[i];
        }
        lo->total_rows = (int32_t)(n_mb * rows_per_mb * row_len);
        *out = lo.release();
        return DS_OK;
    } catch (const std::bad_alloc&) {
        return DS_ENOMEM;
    } catch (...) {
        return DS_EINVAL;
    }
}

extern "C" ds_status ds_layout_get(const ds_layout* lo, ds_layout_view* v) {
    if (!lo || !v) return DS_EINVAL;
    auto p = [](const std::vector<int32_t>& a) { return a.empty() ? nullptr : a.data(); };
    v->n_seq = lo->n_seq;
    v->n_mb = lo->n_mb;
    v->total_rows = lo->total_rows;
    v->total_rows_tgt = lo->total_rows_tgt;
    v->total_tokens = lo->total_tokens;
    v->total_tokens_tgt = lo->total_tokens_tgt;
    v->objective = lo->objective;
    v->t_max = lo->t_max;
    v->perm = p(lo->perm);
    v->mb_start = p(lo->mb_start);
    v->mb_count = p(lo->mb_count);
    v->mb_lpad = p(lo->mb_lpad);
    v->mb_ltgt = p(lo->mb_ltgt);
    v->mb_cost = lo->mb_cost.empty() ? nullptr : lo->mb_cost.data();
    v->mb_row = p(lo->mb_row);
    v->mb_nrows = p(lo->mb_nrows);
    v->mb_row_tgt = p(lo->mb_row_tgt);
    v->mb_nrows_tgt = p(lo->mb_nrows_tgt);
    v->seq_row = p(lo->seq_row);
    v->seq_len = p(lo->seq_len);
    v->seq_row_tgt = p(lo->seq_row_tgt);
    v->seq_len_tgt = p(lo->seq_len_tgt);
    return DS_OK;
}

extern "C" void ds_layout_free(ds_layout* lo) { delete lo; }

// ------------------------------------------------------------------------------------ profiled cost table
namespace {
// index i with grid[i] <= x <= grid[i+1] and the weight of grid[i+1]; weight 0 when x is a grid point
bool bracket(const int32_t* grid, int n, int x, int& i, double& w) {
    for (int k = 0; k < n; ++k)
        if (grid[k] == x) { i = k; w = 0.0; return true; }
    for (int k = 0; k + 1 < n; ++k)
        if (grid[k] < x && x < grid[k + 1]) {
            i = k;
            w = ((double)x - (double)grid[k]) / ((double)grid[k + 1] - (double)grid[k]);
            return true;
        }
    return false;
}
}  // namespace

extern "C" ds_status ds_cost_table_build(const int32_t* b_grid, int32_t nb, const int32_t* l_grid, int32_t nl,
                                         const double* t, double scale, int32_t tb, int32_t tl, int64_t inf_cost,
                                         int64_t* table) {
    if (!b_grid || !l_grid || !t || !table || nb < 1 || nl < 1 || tb < 1 || tl < 1) return DS_EINVAL;
    if (!(scale > 0.0) || inf_cost < 1) return DS_EINVAL;
    for (int i = 0; i < nb; ++i)
        if (b_grid[i] < 1 || (i > 0 && b_grid[i] <= b_grid[i - 1])) return DS_EINVAL;
    for (int j = 0; j < nl; ++j)
        if (l_grid[j] < 1 || (j > 0 && l_grid[j] <= l_grid[j - 1])) return DS_EINVAL;
    for (int k = 0; k < nb * nl; ++k)
        if (t[k] < 0.0) return DS_EINVAL;                       // NaN compares false: allowed
    for (int b = 1; b <= tb; ++b) {
        int i = 0;
        double u = 0.0;
        const bool b_in = b >= b_grid[0] && b <= b_grid[nb - 1] && bracket(b_grid, nb, b, i, u);
        for (int L = 1; L <= tl; ++L) {
            int64_t& out = table[(size_t)(b - 1) * tl + (L - 1)];
            if (!b_in || L > l_grid[nl - 1]) { out = inf_cost; continue; }
            const int Lc = L < l_grid[0] ? l_grid[0] : L;
            int j = 0;
            double v = 0.0;
            if (!bracket(l_grid, nl, Lc, j, v)) { out = inf_cost; continue; }
            auto along_b = [&](int jj) {
                const double lo = t[(size_t)i * nl + jj];
                if (u == 0.0) return lo;
                const double hi = t[(size_t)(i + 1) * nl + jj];
                return lo + u * (hi - lo);
            };
            const double near = along_b(j);
            double val = near;
            if (v != 0.0) {
                const double far = along_b(j + 1);
                val = near + v * (far - near);
            }
            if (val != val) { out = inf_cost; continue; }       // an unprofiled grid point was needed
            const double scaled = std::floor(val * scale + 0.5);
            if (scaled >= (double)inf_cost) return DS_EOVERFLOW;
            out = scaled < 1.0 ? 1 : (int64_t)scaled;
        }
    }
    return DS_OK;
}
