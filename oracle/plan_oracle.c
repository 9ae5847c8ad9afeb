/*
 * TEST INFRASTRUCTURE — CPU oracle for the micro-batch partitioner.
 *
 * This file is the slow, plain reference that the product planner is checked
 * against.  Only tests, the smoke check and the CPU-baseline leg of the
 * benchmark may call it; the product never does, and it shares no code with
 * the product.
 *
 * What it computes (paper section "Micro-batch Construction"):
 *   - samples are put in ascending length order (decoder-only: by length;
 *     encoder-decoder: by input length, then target length), ties keeping the
 *     original order;
 *   - the ordered list is cut into consecutive micro-batches so that the
 *     iteration-time model  (c-1)*max_i t(M_i) + sum_i t(M_i)   (Eq1)
 *     is minimal, by running the recurrence
 *       f(n; t_max) = min_i { f(i; t_max) + t(M[i+1..n]) : t(M[i+1..n]) <= t_max }  (Eq2)
 *     once for every distinct cost a single micro-batch can have (the O(N^2)
 *     candidate values of t_max, no sampling), and keeping the t_max that
 *     minimises (c-1)*t_max + f(N; t_max);
 *   - a micro-batch is admissible only when it is under the per-micro-batch
 *     memory limit (paragraph "Limit memory consumption"); here the limit is
 *     given in tokens: b * L_pad <= cap.
 *
 * Readings where the paper is silent:
 *   - f(0; t_max) = 0 and the split point i ranges over 0..n-1, so that "the
 *     first n samples as one micro-batch" is a legal last slice;
 *   - among equally good results: candidates are scanned in ascending t_max
 *     and only a strictly smaller objective replaces the incumbent; inside
 *     Eq2 the smallest i (the longest last micro-batch) is kept on equal value.
 *
 * Cost models t(b, L) (all exact 64-bit integers):
 *   kind 0 (decoder-only polynomial): fixed + b * L * (lin + L)
 *   kind 1 (encoder-decoder polynomial):
 *          fixed + b * Lin * (lin + Lin) + b * Ltgt * (lin + Ltgt + Lin)
 *   kind 2 (table, decoder-only): table[(b-1) * tl + (L-1)], b <= tb, L <= tl
 * where L (Lin, Ltgt) is the longest sequence in the slice.
 *
 * Return: 0 ok, -1 bad argument, -2 no admissible partition, -4 overflow.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define OR_INF INT64_MAX

static int mul_ovf(int64_t a, int64_t b, int64_t *r) { return __builtin_mul_overflow(a, b, r); }
static int add_ovf(int64_t a, int64_t b, int64_t *r) { return __builtin_add_overflow(a, b, r); }

/* cost of one micro-batch of b sequences padded to (lin_pad, ltgt_pad); *ok = 0 on overflow / out of table */
static int64_t slice_cost(int kind, int64_t fixed, int64_t lin, const int64_t *table, int tb, int tl,
                          int64_t b, int64_t L, int64_t Lt, int *ok)
{
    int64_t r = 0, a, s;
    *ok = 1;
    if (kind == 0) {
        if (add_ovf(lin, L, &s) || mul_ovf(b, L, &a) || mul_ovf(a, s, &a) || add_ovf(a, fixed, &r)) *ok = 0;
        return r;
    }
    if (kind == 1) {
        int64_t e, d;
        if (add_ovf(lin, L, &s) || mul_ovf(b, L, &e) || mul_ovf(e, s, &e)) { *ok = 0; return 0; }
        if (add_ovf(lin, Lt, &s) || add_ovf(s, L, &s) || mul_ovf(b, Lt, &d) || mul_ovf(d, s, &d)) { *ok = 0; return 0; }
        if (add_ovf(e, d, &r) || add_ovf(r, fixed, &r)) *ok = 0;
        return r;
    }
    /* table */
    if (b > tb || L > tl) { *ok = -1; return 0; }
    return table[(b - 1) * (int64_t)tl + (L - 1)];
}

static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

int oracle_plan(const int32_t *len, const int32_t *len_tgt, int32_t n,
                int32_t kind, int64_t fixed, int64_t lin,
                const int64_t *table, int32_t tb, int32_t tl,
                int64_t cap, int32_t c,
                int32_t *perm_out,      /* [n]   sorted position -> original index */
                int32_t *cuts_out,      /* [n+1] micro-batch m covers sorted positions cuts[m]..cuts[m+1]-1 */
                int32_t *n_mb_out, int64_t *objective_out, int64_t *tmax_out)
{
    if (!len || n <= 0 || c < 1 || cap <= 0 || !perm_out || !cuts_out || !n_mb_out) return -1;
    if (kind < 0 || kind > 2) return -1;
    if (kind == 1 && !len_tgt) return -1;
    if (kind == 2 && (!table || tb <= 0 || tl <= 0 || len_tgt)) return -1;
    if (kind != 2 && (lin < 0 || fixed < 0)) return -1;
    for (int i = 0; i < n; i++) {
        if (len[i] <= 0) return -1;
        if (len_tgt && len_tgt[i] <= 0) return -1;
    }

    /* ordering: stable insertion sort, ascending by (len, len_tgt) */
    for (int i = 0; i < n; i++) perm_out[i] = i;
    for (int i = 1; i < n; i++) {
        int32_t p = perm_out[i];
        int j = i - 1;
        while (j >= 0) {
            int32_t q = perm_out[j];
            int greater = len[q] > len[p] || (len[q] == len[p] && len_tgt && len_tgt[q] > len_tgt[p]);
            if (!greater) break;
            perm_out[j + 1] = q;
            j--;
        }
        perm_out[j + 1] = p;
    }

    /* t[i][j] = cost of the slice holding sorted positions i..j-1 (j > i); OR_INF when not admissible */
    size_t np1 = (size_t)n + 1;
    int64_t *t = (int64_t *)malloc(np1 * np1 * sizeof(int64_t));
    int64_t *cand = (int64_t *)malloc(((size_t)n * (n + 1) / 2 + 1) * sizeof(int64_t));
    int64_t *f = (int64_t *)malloc(np1 * sizeof(int64_t));
    int32_t *arg = (int32_t *)malloc(np1 * sizeof(int32_t));
    int32_t *best_arg = (int32_t *)malloc(np1 * sizeof(int32_t));
    if (!t || !cand || !f || !arg || !best_arg) { free(t); free(cand); free(f); free(arg); free(best_arg); return -3; }

    int rc = 0;
    size_t ncand = 0;
    for (int i = 0; i < n && rc == 0; i++) {
        int64_t L = 0, Lt = 0;
        for (int j = i + 1; j <= n; j++) {
            int32_t s = perm_out[j - 1];
            if (len[s] > L) L = len[s];
            if (len_tgt && len_tgt[s] > Lt) Lt = len_tgt[s];
            int64_t b = j - i;
            int64_t v = OR_INF;
            if (b * L <= cap) {
                int ok;
                v = slice_cost(kind, fixed, lin, table, tb, tl, b, L, Lt, &ok);
                if (ok == 0) { rc = -4; break; }
                if (ok < 0 || v < 0 || v == OR_INF) { rc = -1; break; }
                cand[ncand++] = v;
            }
            t[(size_t)i * np1 + j] = v;
        }
    }
    if (rc != 0) goto done;

    qsort(cand, ncand, sizeof(int64_t), cmp_i64);
    {   /* distinct values */
        size_t m = 0;
        for (size_t k = 0; k < ncand; k++)
            if (m == 0 || cand[k] != cand[m - 1]) cand[m++] = cand[k];
        ncand = m;
    }

    int64_t bestJ = OR_INF, bestT = 0;
    int found = 0;
    for (size_t k = 0; k < ncand; k++) {
        int64_t T = cand[k];
        f[0] = 0;
        for (int nn = 1; nn <= n; nn++) {
            int64_t bv = OR_INF;
            int32_t bi = -1;
            for (int i = 0; i < nn; i++) {
                int64_t tc = t[(size_t)i * np1 + nn];
                if (tc == OR_INF || tc > T || f[i] == OR_INF) continue;
                int64_t v;
                if (add_ovf(f[i], tc, &v)) { rc = -4; goto done; }
                if (v < bv) { bv = v; bi = i; }      /* strict: the smallest i wins a tie */
            }
            f[nn] = bv;
            arg[nn] = bi;
        }
        if (f[n] == OR_INF) continue;
        int64_t J;
        if (mul_ovf((int64_t)(c - 1), T, &J) || add_ovf(J, f[n], &J)) { rc = -4; goto done; }
        if (!found || J < bestJ) {
            found = 1; bestJ = J; bestT = T;
            memcpy(best_arg, arg, np1 * sizeof(int32_t));
        }
    }
    if (!found) { rc = -2; goto done; }

    {   /* backtrack */
        int32_t m = 0, pos = n;
        while (pos > 0) { cuts_out[m++] = pos; pos = best_arg[pos]; }   /* ends, right to left */
        cuts_out[m] = 0;
        for (int a = 0, b2 = m; a < b2; a++, b2--) { int32_t tmp = cuts_out[a]; cuts_out[a] = cuts_out[b2]; cuts_out[b2] = tmp; }
        *n_mb_out = m;
    }
    if (objective_out) *objective_out = bestJ;
    if (tmax_out) *tmax_out = bestT;

done:
    free(t); free(cand); free(f); free(arg); free(best_arg);
    return rc;
}
