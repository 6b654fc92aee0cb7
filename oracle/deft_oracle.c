/*
 * CPU oracle for the batched exact 0/1 multiple-knapsack solver.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP path is checked against.  It shares no code with the HIP path, is never
 * called by it, and may be used only by the tests, the smoke check and the
 * benchmark's cpu_baseline leg.
 *
 * What it follows (DeFT, arXiv 2503.16815):
 *   - Section III.B, Problem 1: one 0/1 knapsack, items = bucket communication
 *     times, capacity = a merged computation window, constraint inclusive.
 *     The paper's "NaiveKnapsack" (Algorithm 1) is never spelled out; it is
 *     read here as the textbook exact DP over integer capacities.
 *   - Section III.A/III.B (Cases 1-4, coverage ratio N:M): backward and forward
 *     windows of successive iterations each take what is left over by the
 *     previous window -> m knapsacks filled one after the other in a given
 *     order; each stage is solved exactly on the items still unplaced.
 *   - Section III.C, Problem 2: two knapsacks (links), each item in at most
 *     one; generalised to a separate weight per link (the paper's single c_j
 *     with a capacity scaled by mu is the case w1 == w2).
 *   - Section III.B, Algorithm 1 (RecursiveKnapsack): the knapsack over the whole
 *     list with the remaining time, against the same procedure on the list
 *     without its last item and with that item's time taken off the remaining
 *     time; the shallower answer wins only if its sum is strictly greater.
 *   - Section III.C, the greedy heuristic of the paper's own Solver: capacities
 *     and bucket times are sorted, then the knapsacks are gone through from the
 *     smallest capacity up and each takes, longest bucket first, whatever still
 *     fits.
 *   - Section IV.C, the feedback mechanism: when a schedule fails the convergence
 *     test the knapsack capacity is raised and the problem solved again, up to
 *     ten times -> one instance = one item list and several capacities, each an
 *     independent Problem 1.
 *   - Section III.B, the current and the future task queue and Cases 1-4: which item
 *     list and which capacity each forward and backward stage solves, over several
 *     iterations, and when parameter updates fire (deft_oracle_simulate).
 *
 * Conventions the paper leaves open, fixed here:
 *   - an item is taken at capacity c only if it strictly improves the value;
 *     traceback runs from the last item down.  Among all optimal selections
 *     this yields the one with the smallest mask sum_t x_t 2^t.
 *   - joint DP: per item the order of tests is skip, link 0, link 1, each
 *     replacing the incumbent only if strictly greater.
 *   - values and weights are separate arrays (value == weight is Problem 1).
 *   - greedy heuristic: both sorts are stable (equal capacities: lower knapsack
 *     id first; equal times: lower item index first); with one time per link,
 *     each link goes through the items in the order of its own times.
 *   - Algorithm 1: the time taken off when an item leaves the list is an input
 *     per item; a list met with a negative remaining time schedules nothing;
 *     the sums compared are the values.
 *
 * Arithmetic: int64 accumulators; inputs int32.  No blocking, no bit packing:
 * the keep table is one byte per (item, capacity cell).
 *
 * Pins: tests/test_oracle_*.py (brute force over all 2^n / 3^n selections,
 * the bitset subset-sum recurrence, closed forms, invariants, the Table II
 * bucket times as a worked vector; for Algorithm 1: enumeration of every
 * level and subset, reductions to Problem 1, a case worked by hand).
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ST_OK = 0, ST_INVALID = 1, ST_LIMIT = 2, ST_OVERFLOW = 3, ST_OOM = 4 };

#define VALUE_SUM_LIMIT ((int64_t)1 << 31)

/* Problem 1 on the items listed in act[0..A) (ascending original index).
 * Returns the optimal value; marks chosen[t] and returns the placed weight. */
static int single_stage(int A, const int32_t *aw, const int32_t *av, int32_t C,
                        int64_t *value, int64_t *load, uint8_t *chosen,
                        int64_t *touched, int64_t *table)
{
    size_t cells = (size_t)C + 1;
    int64_t *row = (int64_t *)calloc(cells, sizeof(int64_t));
    uint8_t *keep = (uint8_t *)calloc((size_t)(A > 0 ? A : 1) * cells, 1);
    if (!row || !keep) { free(row); free(keep); return ST_OOM; }

    for (int t = 0; t < A; ++t) {
        int64_t w = aw[t], v = av[t];
        *table += (int64_t)cells;
        if (w <= C) *touched += (int64_t)C - w + 1;
        for (int64_t c = C; c >= w; --c) {
            int64_t cand = row[c - w] + v;
            if (cand > row[c]) {
                row[c] = cand;
                keep[(size_t)t * cells + (size_t)c] = 1;
            }
        }
    }
    *value = row[C];

    int64_t c = C;
    for (int t = A - 1; t >= 0; --t) {
        chosen[t] = 0;
        if (keep[(size_t)t * cells + (size_t)c]) {
            chosen[t] = 1;
            c -= aw[t];
        }
    }
    *load = (int64_t)C - c;
    free(row);
    free(keep);
    return ST_OK;
}

static void clear_outputs(int32_t n_slots, int32_t m_slots, int64_t *total,
                          int32_t *knap_value, int32_t *knap_load, int32_t *assign)
{
    *total = 0;
    for (int j = 0; j < m_slots; ++j) { knap_value[j] = 0; knap_load[j] = 0; }
    for (int i = 0; i < n_slots; ++i) assign[i] = -1;
}

/*
 * Sequential multiple knapsack for one instance.
 * order may be NULL (= 0,1,2,...).  cap_limit < 0 means "no limit".
 * assign has item_stride slots, knap_* have knap_stride slots; all are
 * written (unused slots: -1 / 0).
 */
int deft_oracle_sequential(int32_t n, int32_t item_stride, const int32_t *w, const int32_t *v,
                           int32_t m, int32_t knap_stride, const int32_t *cap,
                           const int32_t *order, int32_t cap_limit,
                           int64_t *total, int32_t *knap_value, int32_t *knap_load,
                           int32_t *assign, int64_t *touched_cells, int64_t *table_cells)
{
    int64_t touched = 0, table = 0;
    clear_outputs(item_stride, knap_stride, total, knap_value, knap_load, assign);
    if (touched_cells) *touched_cells = 0;
    if (table_cells) *table_cells = 0;

    if (n < 0 || n > item_stride || m < 0 || m > knap_stride) return ST_INVALID;
    for (int i = 0; i < n; ++i)
        if (w[i] < 1 || v[i] < 0) return ST_INVALID;
    for (int j = 0; j < m; ++j)
        if (cap[j] < 0) return ST_INVALID;
    if (order) {
        uint8_t *seen = (uint8_t *)calloc((size_t)(m > 0 ? m : 1), 1);
        if (!seen) return ST_OOM;
        for (int s = 0; s < m; ++s) {
            int32_t j = order[s];
            if (j < 0 || j >= m || seen[j]) { free(seen); return ST_INVALID; }
            seen[j] = 1;
        }
        free(seen);
    }
    if (cap_limit >= 0)
        for (int j = 0; j < m; ++j)
            if (cap[j] > cap_limit) return ST_LIMIT;
    int64_t vsum = 0;
    for (int i = 0; i < n; ++i) vsum += v[i];
    if (vsum >= VALUE_SUM_LIMIT) return ST_OVERFLOW;

    int32_t *act = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    int32_t *aw = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    int32_t *av = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    uint8_t *chosen = (uint8_t *)malloc((size_t)(n > 0 ? n : 1));
    int rc = ST_OK;
    if (!act || !aw || !av || !chosen) rc = ST_OOM;

    int64_t sum = 0;
    for (int s = 0; s < m && rc == ST_OK; ++s) {
        int32_t j = order ? order[s] : s;
        int A = 0;
        for (int i = 0; i < n; ++i)
            if (assign[i] == -1) { act[A] = i; aw[A] = w[i]; av[A] = v[i]; ++A; }
        int64_t value = 0, load = 0;
        rc = single_stage(A, aw, av, cap[j], &value, &load, chosen, &touched, &table);
        if (rc != ST_OK) break;
        for (int t = 0; t < A; ++t)
            if (chosen[t]) assign[act[t]] = j;
        knap_value[j] = (int32_t)value;
        knap_load[j] = (int32_t)load;
        sum += value;
    }
    free(act); free(aw); free(av); free(chosen);
    if (rc != ST_OK) {
        clear_outputs(item_stride, knap_stride, total, knap_value, knap_load, assign);
        return rc;
    }
    *total = sum;
    if (touched_cells) *touched_cells = touched;
    if (table_cells) *table_cells = table;
    return ST_OK;
}

/*
 * Joint two-link DP (Problem 2 with per-link weights) for one instance.
 * w1 = weights on link 0 (capacity cap[0]), w2 = weights on link 1 (cap[1]).
 * assign: 0 / 1 / -1.  knap_value[j] = value placed on link j.
 */
int deft_oracle_joint2(int32_t n, int32_t item_stride, const int32_t *w1, const int32_t *w2,
                       const int32_t *v, int32_t m, int32_t knap_stride, const int32_t *cap,
                       int32_t c1_limit, int32_t c2_limit,
                       int64_t *total, int32_t *knap_value, int32_t *knap_load,
                       int32_t *assign, int64_t *touched_cells, int64_t *table_cells)
{
    clear_outputs(item_stride, knap_stride, total, knap_value, knap_load, assign);
    if (touched_cells) *touched_cells = 0;
    if (table_cells) *table_cells = 0;

    if (n < 0 || n > item_stride || m != 2 || knap_stride < 2) return ST_INVALID;
    for (int i = 0; i < n; ++i)
        if (w1[i] < 1 || w2[i] < 1 || v[i] < 0) return ST_INVALID;
    if (cap[0] < 0 || cap[1] < 0) return ST_INVALID;
    if ((c1_limit >= 0 && cap[0] > c1_limit) || (c2_limit >= 0 && cap[1] > c2_limit)) return ST_LIMIT;
    int64_t vsum = 0;
    for (int i = 0; i < n; ++i) vsum += v[i];
    if (vsum >= VALUE_SUM_LIMIT) return ST_OVERFLOW;

    int64_t C1 = cap[0], C2 = cap[1];
    size_t cols = (size_t)C2 + 1, cells = ((size_t)C1 + 1) * cols;
    int64_t *old = (int64_t *)calloc(cells, sizeof(int64_t));
    int64_t *cur = (int64_t *)calloc(cells, sizeof(int64_t));
    uint8_t *code = (uint8_t *)calloc((size_t)(n > 0 ? n : 1) * cells, 1);
    if (!old || !cur || !code) { free(old); free(cur); free(code); return ST_OOM; }

    for (int i = 0; i < n; ++i) {
        int64_t a1 = w1[i], a2 = w2[i], val = v[i];
        for (int64_t a = 0; a <= C1; ++a) {
            for (int64_t b = 0; b <= C2; ++b) {
                size_t at = (size_t)a * cols + (size_t)b;
                int64_t best = old[at];
                uint8_t how = 0;
                if (a >= a1) {
                    int64_t cand = old[(size_t)(a - a1) * cols + (size_t)b] + val;
                    if (cand > best) { best = cand; how = 1; }
                }
                if (b >= a2) {
                    int64_t cand = old[(size_t)a * cols + (size_t)(b - a2)] + val;
                    if (cand > best) { best = cand; how = 2; }
                }
                cur[at] = best;
                code[(size_t)i * cells + at] = how;
            }
        }
        int64_t *tmp = old; old = cur; cur = tmp;
    }
    int64_t opt = old[(size_t)C1 * cols + (size_t)C2];

    int64_t a = C1, b = C2, val0 = 0, val1 = 0;
    for (int i = n - 1; i >= 0; --i) {
        uint8_t how = code[(size_t)i * cells + (size_t)a * cols + (size_t)b];
        if (how == 1) { assign[i] = 0; a -= w1[i]; val0 += v[i]; }
        else if (how == 2) { assign[i] = 1; b -= w2[i]; val1 += v[i]; }
    }
    knap_value[0] = (int32_t)val0;
    knap_value[1] = (int32_t)val1;
    knap_load[0] = (int32_t)(C1 - a);
    knap_load[1] = (int32_t)(C2 - b);
    *total = opt;
    if (touched_cells) *touched_cells = (int64_t)n * (int64_t)cells;
    if (table_cells) *table_cells = (int64_t)n * (int64_t)cells;
    free(old); free(cur); free(code);
    return ST_OK;
}

/*
 * Algorithm 1 (RecursiveKnapsack) for one instance.
 * Items 0 .. n-1 are the list in generation order; drop[i] is the time taken off the
 * remaining time when item i, then the last of the list, is left off it.  The procedure
 * nests: the answer for a list is the knapsack over that list unless the answer for the
 * list without its last item is at least as good.  Unrolled from the innermost call
 * outwards that is a walk over the prefixes of the list, shortest first: the empty list
 * answers "nothing", and each longer prefix, solved with the remaining time it is left
 * with, replaces the incumbent only when its sum is strictly greater.  A prefix met with
 * a negative remaining time schedules nothing.
 * Outputs: assign[i] = 0 for scheduled items else -1; knap_value[0] / knap_load[0] =
 * value and weight scheduled; knap_value[1] = number of items dropped from the end of
 * the list at the level whose answer was returned (n if nothing is scheduled at any
 * level), knap_load[1] = the remaining time of that level (0 if none).
 */
typedef struct { int64_t value, load, remain; int len; uint8_t *chosen; } rec_result_t;

static int recursive_knapsack(int n, const int32_t *w, const int32_t *v, const int32_t *drop,
                              int64_t remain_full, rec_result_t *out, int64_t *touched, int64_t *table)
{
    out->value = 0; out->load = 0; out->remain = 0; out->len = 0;   /* the empty list's answer */
    if (n == 0) return ST_OK;
    uint8_t *trial = (uint8_t *)calloc((size_t)n, 1);
    int64_t *remain = (int64_t *)calloc((size_t)n + 1, sizeof(int64_t));
    if (!trial || !remain) { free(trial); free(remain); return ST_OOM; }
    /* remaining time of the prefix of each length: the full time minus what the items
     * behind the prefix take off */
    remain[n] = remain_full;
    for (int len = n - 1; len >= 0; --len) remain[len] = remain[len + 1] - drop[len];
    int rc = ST_OK;
    for (int len = 1; len <= n && rc == ST_OK; ++len) {
        int64_t value = 0, load = 0;
        if (remain[len] < 0) continue;
        rc = single_stage(len, w, v, (int32_t)remain[len], &value, &load, trial, touched, table);
        if (rc == ST_OK && value > out->value) {
            memcpy(out->chosen, trial, (size_t)len);
            out->value = value; out->load = load; out->remain = remain[len]; out->len = len;
        }
    }
    free(trial); free(remain);
    return rc;
}

int deft_oracle_recursive(int32_t n, int32_t item_stride, const int32_t *w, const int32_t *v,
                          const int32_t *drop, int32_t m, int32_t knap_stride, const int32_t *cap,
                          int32_t cap_limit, int64_t *total, int32_t *knap_value, int32_t *knap_load,
                          int32_t *assign, int64_t *touched_cells, int64_t *table_cells)
{
    int64_t touched = 0, table = 0;
    clear_outputs(item_stride, knap_stride, total, knap_value, knap_load, assign);
    if (touched_cells) *touched_cells = 0;
    if (table_cells) *table_cells = 0;
    if (n < 0 || n > item_stride || m != 1 || knap_stride < 2) return ST_INVALID;
    for (int i = 0; i < n; ++i)
        if (w[i] < 1 || v[i] < 0 || drop[i] < 0) return ST_INVALID;
    if (cap[0] < 0) return ST_INVALID;
    if (cap_limit >= 0 && cap[0] > cap_limit) return ST_LIMIT;
    int64_t vsum = 0;
    for (int i = 0; i < n; ++i) vsum += v[i];
    if (vsum >= VALUE_SUM_LIMIT) return ST_OVERFLOW;

    rec_result_t res = { 0, 0, 0, 0, NULL };
    res.chosen = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!res.chosen) return ST_OOM;
    int rc = recursive_knapsack(n, w, v, drop, cap[0], &res, &touched, &table);
    if (rc != ST_OK) { free(res.chosen); return rc; }
    if (res.value == 0) res.len = 0;             /* nothing scheduled at any level: the empty order */
    for (int i = 0; i < res.len; ++i)
        if (res.chosen[i]) assign[i] = 0;
    knap_value[0] = (int32_t)res.value;
    knap_load[0] = (int32_t)res.load;
    knap_value[1] = n - res.len;
    knap_load[1] = res.len > 0 ? (int32_t)res.remain : 0;
    *total = res.value;
    if (touched_cells) *touched_cells = touched;
    if (table_cells) *table_cells = table;
    free(res.chosen);
    return ST_OK;
}

/*
 * The greedy heuristic of Section III.C for one instance.
 * per_link = 0: one time per item (w[0..n)), m knapsacks.
 * per_link = 1: the two-link layout, w[j * item_stride + i] = time of item i on link j,
 *               m must be 2; link j looks at the items in the order of its own times.
 * Step 1: knapsack ids sorted by capacity, ascending, stable.
 * Step 2: item indices sorted by time, descending, stable.
 * Step 3: for each knapsack in step 1's order, for each item in step 2's order:
 *         an item not placed yet whose time fits what is left of the knapsack is placed.
 */
static void stable_sort_ids(int count, int32_t *ids, const int32_t *key, int descending)
{
    for (int a = 1; a < count; ++a) {          /* insertion sort: stable, plain */
        int32_t id = ids[a];
        int b = a - 1;
        while (b >= 0 && (descending ? key[ids[b]] < key[id] : key[ids[b]] > key[id])) {
            ids[b + 1] = ids[b];
            --b;
        }
        ids[b + 1] = id;
    }
}

int deft_oracle_greedy(int32_t n, int32_t item_stride, const int32_t *w, int per_link, const int32_t *v,
                       int32_t m, int32_t knap_stride, const int32_t *cap, int32_t cap_limit,
                       int32_t c1_limit, int32_t c2_limit, int64_t *total, int32_t *knap_value,
                       int32_t *knap_load, int32_t *assign)
{
    clear_outputs(item_stride, knap_stride, total, knap_value, knap_load, assign);
    if (n < 0 || n > item_stride || m < 0 || m > knap_stride) return ST_INVALID;
    if (per_link && (m != 2 || knap_stride < 2)) return ST_INVALID;
    for (int i = 0; i < n; ++i)
        if (w[i] < 1 || v[i] < 0 || (per_link && w[item_stride + i] < 1)) return ST_INVALID;
    for (int j = 0; j < m; ++j)
        if (cap[j] < 0) return ST_INVALID;
    for (int j = 0; j < m; ++j) {
        int32_t lim = per_link ? (j == 0 ? c1_limit : c2_limit) : cap_limit;
        if (lim >= 0 && cap[j] > lim) return ST_LIMIT;
    }
    int64_t vsum = 0;
    for (int i = 0; i < n; ++i) vsum += v[i];
    if (vsum >= VALUE_SUM_LIMIT) return ST_OVERFLOW;

    int32_t *knaps = (int32_t *)malloc(sizeof(int32_t) * (size_t)(m > 0 ? m : 1));
    int32_t *items = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (!knaps || !items) { free(knaps); free(items); return ST_OOM; }
    for (int j = 0; j < m; ++j) knaps[j] = j;
    stable_sort_ids(m, knaps, cap, 0);
    for (int s = 0; s < m; ++s) {
        int j = knaps[s];
        const int32_t *time = per_link ? w + (size_t)j * item_stride : w;
        if (s == 0 || per_link) {                /* one sort serves every knapsack unless times differ per link */
            for (int i = 0; i < n; ++i) items[i] = i;
            stable_sort_ids(n, items, time, 1);
        }
        int64_t left = cap[j], load = 0, value = 0;
        for (int t = 0; t < n; ++t) {
            int i = items[t];
            if (assign[i] == -1 && time[i] <= left) {
                assign[i] = j;
                left -= time[i];
                load += time[i];
                value += v[i];
            }
        }
        knap_load[j] = (int32_t)load;
        knap_value[j] = (int32_t)value;
        *total += value;
    }
    free(knaps);
    free(items);
    return ST_OK;
}

/*
 * Capacity sweep for one instance (the Solver called again with a larger capacity,
 * Section IV.C): cap[0..m) are m capacities of ONE knapsack; each is Problem 1 over the
 * whole item list, solved on its own from scratch.
 * Outputs: knap_value[j] / knap_load[j] = value and weight scheduled at capacity cap[j];
 * assign[i] = bit mask over j of the capacities at which item i is scheduled (0 if none;
 * slots >= n also 0); total = the value at the largest capacity.  m <= 31.
 */
int deft_oracle_capacity_sweep(int32_t n, int32_t item_stride, const int32_t *w, const int32_t *v,
                               int32_t m, int32_t knap_stride, const int32_t *cap, int32_t cap_limit,
                               int64_t *total, int32_t *knap_value, int32_t *knap_load, int32_t *assign,
                               int64_t *touched_cells, int64_t *table_cells)
{
    int64_t touched = 0, table = 0;
    clear_outputs(item_stride, knap_stride, total, knap_value, knap_load, assign);
    for (int i = 0; i < item_stride; ++i) assign[i] = 0;      /* masks, not knapsack ids */
    if (touched_cells) *touched_cells = 0;
    if (table_cells) *table_cells = 0;
    if (n < 0 || n > item_stride || m < 0 || m > knap_stride || m > 31) return ST_INVALID;
    for (int i = 0; i < n; ++i)
        if (w[i] < 1 || v[i] < 0) return ST_INVALID;
    for (int j = 0; j < m; ++j)
        if (cap[j] < 0) return ST_INVALID;
    for (int j = 0; j < m; ++j)
        if (cap_limit >= 0 && cap[j] > cap_limit) return ST_LIMIT;
    int64_t vsum = 0;
    for (int i = 0; i < n; ++i) vsum += v[i];
    if (vsum >= VALUE_SUM_LIMIT) return ST_OVERFLOW;

    uint8_t *chosen = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!chosen) return ST_OOM;
    int32_t largest = -1;
    for (int j = 0; j < m; ++j) {
        int64_t value = 0, load = 0;
        int rc = single_stage(n, w, v, cap[j], &value, &load, chosen, &touched, &table);
        if (rc != ST_OK) {
            free(chosen);
            clear_outputs(item_stride, knap_stride, total, knap_value, knap_load, assign);
            for (int i = 0; i < item_stride; ++i) assign[i] = 0;
            return rc;
        }
        knap_value[j] = (int32_t)value;
        knap_load[j] = (int32_t)load;
        for (int i = 0; i < n; ++i)
            if (chosen[i]) assign[i] |= (int32_t)(1u << j);
        if (cap[j] > largest) { largest = cap[j]; *total = value; }
    }
    free(chosen);
    if (touched_cells) *touched_cells = touched;
    if (table_cells) *table_cells = table;
    return ST_OK;
}

/* ---- batch driver: instances split statically over nthreads ------------- */

typedef struct {
    int32_t mode, batch, item_stride, knap_stride;
    const int32_t *n_items, *n_knapsacks, *weights, *values, *capacities, *fill_order, *drop_time;
    int32_t cap_limit, c1_limit, c2_limit;
    int64_t *total;
    int32_t *knap_value, *knap_load, *assign, *status;
    int64_t *touched, *table;
} batch_args_t;

typedef struct { const batch_args_t *a; int lo, hi; } slice_t;

static void solve_one(const batch_args_t *a, int b)
{
    size_t is = (size_t)a->item_stride, ks = (size_t)a->knap_stride;
    int64_t touched = 0, table = 0;
    int st;
    if (a->mode == 0) {
        st = deft_oracle_sequential(a->n_items[b], a->item_stride, a->weights + b * is,
                                    a->values + b * is, a->n_knapsacks[b], a->knap_stride,
                                    a->capacities + b * ks,
                                    a->fill_order ? a->fill_order + b * ks : NULL, a->cap_limit,
                                    a->total + b, a->knap_value + b * ks, a->knap_load + b * ks,
                                    a->assign + b * is, &touched, &table);
    } else if (a->mode == 2) {
        st = deft_oracle_recursive(a->n_items[b], a->item_stride, a->weights + b * is, a->values + b * is,
                                   a->drop_time + b * is, a->n_knapsacks[b], a->knap_stride,
                                   a->capacities + b * ks, a->cap_limit, a->total + b,
                                   a->knap_value + b * ks, a->knap_load + b * ks, a->assign + b * is,
                                   &touched, &table);
    } else if (a->mode == 5) {
        st = deft_oracle_capacity_sweep(a->n_items[b], a->item_stride, a->weights + b * is, a->values + b * is,
                                        a->n_knapsacks[b], a->knap_stride, a->capacities + b * ks, a->cap_limit,
                                        a->total + b, a->knap_value + b * ks, a->knap_load + b * ks,
                                        a->assign + b * is, &touched, &table);
    } else if (a->mode == 3 || a->mode == 4) {
        int per_link = a->mode == 4;
        st = deft_oracle_greedy(a->n_items[b], a->item_stride, a->weights + b * (per_link ? 2 : 1) * is, per_link,
                                a->values + b * is, a->n_knapsacks[b], a->knap_stride, a->capacities + b * ks,
                                a->cap_limit, a->c1_limit, a->c2_limit, a->total + b, a->knap_value + b * ks,
                                a->knap_load + b * ks, a->assign + b * is);
    } else {
        st = deft_oracle_joint2(a->n_items[b], a->item_stride, a->weights + b * 2 * is,
                                a->weights + b * 2 * is + is, a->values + b * is,
                                a->n_knapsacks[b], a->knap_stride, a->capacities + b * ks,
                                a->c1_limit, a->c2_limit, a->total + b, a->knap_value + b * ks,
                                a->knap_load + b * ks, a->assign + b * is, &touched, &table);
    }
    a->status[b] = st;
    if (a->touched) a->touched[b] = touched;
    if (a->table) a->table[b] = table;
}

static void *worker(void *p)
{
    const slice_t *s = (const slice_t *)p;
    for (int b = s->lo; b < s->hi; ++b) solve_one(s->a, b);
    return NULL;
}

/* Returns the number of threads actually used (>= 1), or -1 on bad arguments. */
int deft_oracle_solve_batch(int32_t mode, int32_t batch, int32_t item_stride, int32_t knap_stride,
                            const int32_t *n_items, const int32_t *n_knapsacks,
                            const int32_t *weights, const int32_t *values,
                            const int32_t *capacities, const int32_t *fill_order,
                            const int32_t *drop_time,
                            int32_t cap_limit, int32_t c1_limit, int32_t c2_limit,
                            int64_t *total, int32_t *knap_value, int32_t *knap_load,
                            int32_t *assign, int32_t *status, int64_t *touched, int64_t *table,
                            int32_t nthreads)
{
    if (mode < 0 || mode > 5 || (mode == 2 && !drop_time) || batch < 0 || item_stride < 0 || knap_stride < 0)
        return -1;
    batch_args_t a = { mode, batch, item_stride, knap_stride, n_items, n_knapsacks, weights,
                       values, capacities, fill_order, drop_time, cap_limit, c1_limit, c2_limit, total,
                       knap_value, knap_load, assign, status, touched, table };
    if (nthreads < 1) nthreads = 1;
    if (nthreads > batch) nthreads = batch > 0 ? batch : 1;
    if (nthreads == 1) {
        for (int b = 0; b < batch; ++b) solve_one(&a, b);
        return 1;
    }
    pthread_t *tid = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
    slice_t *sl = (slice_t *)malloc(sizeof(slice_t) * (size_t)nthreads);
    char *live = (char *)calloc((size_t)nthreads, 1);
    if (!tid || !sl || !live) { free(tid); free(sl); free(live); return -1; }
    int started = 0;
    for (int t = 0; t < nthreads; ++t) {
        sl[t].a = &a;
        sl[t].lo = (int)((int64_t)batch * t / nthreads);
        sl[t].hi = (int)((int64_t)batch * (t + 1) / nthreads);
        if (pthread_create(&tid[t], NULL, worker, &sl[t]) != 0) {
            worker(&sl[t]);                 /* run the slice inline if no thread */
        } else {
            live[t] = 1;
            ++started;
        }
    }
    for (int t = 0; t < nthreads; ++t)
        if (live[t]) pthread_join(tid[t], NULL);
    free(tid); free(sl); free(live);
    return started > 0 ? nthreads : 1;
}

/* ---- the two task queues over several iterations (Section III.B, Cases 1-4) ---- */
/*
 * One candidate schedule simulated for `iterations` iterations.  Every iteration has a
 * forward stage (window fwd) and then a backward stage (window bwd) during which its n
 * buckets are generated; bucket i takes comm[i] to synchronise, and leaving it off the
 * end of Algorithm 1's list takes drop[i] off the remaining time.
 *
 * State: the current task queue (a subset of the n buckets, holding the gradients of cur_k
 * iterations merged together), the future task queue (empty, or all n buckets holding
 * fut_k iterations), and done_k = iterations whose buckets are all synchronised but not
 * yet applied.
 *   Forward stage, current queue not empty (Case 1): plain knapsack over the current
 *     queue with capacity fwd.
 *   Backward stage, current queue not empty, its total time above bwd (Case 2): plain
 *     knapsack over the current queue with capacity bwd; the new buckets join the future
 *     queue (merged with what waits there).
 *   Backward stage, current queue not empty and fits (Case 3): all of it is synchronised;
 *     the new buckets join the future queue; Algorithm 1 over the future queue with what
 *     is left of bwd; what it leaves becomes the current queue.
 *   Backward stage, current queue empty (Case 4): the new buckets merged with the future
 *     queue; Algorithm 1 over them with bwd; what it leaves becomes the current queue.
 *   A queue that empties is complete; at the end of each iteration every complete set is
 *   applied in one update, update_k[t] = iterations of gradients it carries (0 = none).
 * Outputs per iteration t and stage s (0 forward, 1 backward):
 *   stage_case[2t+s]  0 = nothing to do, else the case number
 *   stage_count[2t+s] buckets synchronised in the stage, stage_time[2t+s] their time
 *   update_k[t]
 *   tail[0..2) = cur_k, fut_k after the last iteration;  *sweep_cells = sum over solved
 *   stages of sum over listed buckets of max(0, capacity - comm + 1).
 */
int deft_oracle_simulate(int32_t n, int32_t iterations, const int32_t *comm, const int32_t *drop,
                         int32_t fwd, int32_t bwd, int32_t cap_limit,
                         int32_t *stage_case, int32_t *stage_count, int32_t *stage_time,
                         int32_t *update_k, int32_t *tail, int64_t *sweep_cells)
{
    for (int x = 0; x < 2 * iterations; ++x) { stage_case[x] = 0; stage_count[x] = 0; stage_time[x] = 0; }
    for (int t = 0; t < iterations; ++t) update_k[t] = 0;
    tail[0] = tail[1] = 0;
    *sweep_cells = 0;
    if (n < 1 || iterations < 0 || fwd < 0 || bwd < 0) return ST_INVALID;
    int64_t sum = 0;
    for (int i = 0; i < n; ++i) {
        if (comm[i] < 1 || drop[i] < 0) return ST_INVALID;
        sum += comm[i];
    }
    if (cap_limit >= 0 && (fwd > cap_limit || bwd > cap_limit)) return ST_LIMIT;
    if (sum >= VALUE_SUM_LIMIT) return ST_OVERFLOW;

    uint8_t *cur = (uint8_t *)calloc((size_t)n, 1);       /* in the current task queue? */
    uint8_t *chosen = (uint8_t *)calloc((size_t)n, 1);
    int32_t *lw = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);   /* the stage's item list */
    int32_t *lid = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    if (!cur || !chosen || !lw || !lid) { free(cur); free(chosen); free(lw); free(lid); return ST_OOM; }
    int cur_k = 0, fut_k = 0, done_k = 0, rc = ST_OK;
    int64_t touched = 0, table = 0;

    for (int t = 0; t < iterations && rc == ST_OK; ++t) {
        for (int stage = 0; stage < 2 && rc == ST_OK; ++stage) {
            int32_t *o_case = &stage_case[2 * t + stage], *o_count = &stage_count[2 * t + stage];
            int32_t *o_time = &stage_time[2 * t + stage];
            int in_cur = 0;
            int64_t cur_time = 0;
            for (int i = 0; i < n; ++i)
                if (cur[i]) { ++in_cur; cur_time += comm[i]; }
            int32_t window = stage == 0 ? fwd : bwd;

            if (in_cur > 0 && (stage == 0 || cur_time > window)) {
                /* Case 1 / Case 2: NaiveKnapsack over the current task queue */
                int A = 0;
                for (int i = 0; i < n; ++i)
                    if (cur[i]) { lw[A] = comm[i]; lid[A] = i; ++A; }
                for (int a = 0; a < A; ++a)
                    if (lw[a] <= window) *sweep_cells += (int64_t)window - lw[a] + 1;
                int64_t value = 0, load = 0;
                rc = single_stage(A, lw, lw, window, &value, &load, chosen, &touched, &table);
                if (rc != ST_OK) break;
                int got = 0;
                for (int a = 0; a < A; ++a)
                    if (chosen[a]) { cur[lid[a]] = 0; ++got; }
                *o_case = stage == 0 ? 1 : 2;
                *o_count = got;
                *o_time = (int32_t)load;
                if (stage == 1) ++fut_k;                  /* the new buckets wait in the future queue */
                if (got == in_cur) { done_k += cur_k; cur_k = 0; }
            } else if (stage == 1) {
                /* Case 3 (the current queue fits: all of it goes first) or Case 4 (it is empty) */
                int64_t remain = window;
                if (in_cur > 0) {
                    *o_case = 3;
                    *o_count = in_cur;
                    *o_time = (int32_t)cur_time;
                    remain -= cur_time;
                    for (int i = 0; i < n; ++i) cur[i] = 0;
                    done_k += cur_k;
                } else {
                    *o_case = 4;
                }
                int list_k = fut_k + 1;                   /* this iteration's buckets merged with the future queue */
                fut_k = 0;
                for (int i = 0; i < n; ++i)
                    if (comm[i] <= remain) *sweep_cells += remain - comm[i] + 1;
                rec_result_t res = { 0, 0, 0, 0, chosen };
                memset(chosen, 0, (size_t)n);
                rc = recursive_knapsack(n, comm, comm, drop, remain, &res, &touched, &table);
                if (rc != ST_OK) break;
                if (res.value == 0) res.len = 0;
                int got = 0;
                for (int i = 0; i < n; ++i) {
                    int take = i < res.len && chosen[i];
                    cur[i] = (uint8_t)!take;              /* what Algorithm 1 leaves is the new current queue */
                    got += take;
                }
                *o_count += got;
                *o_time += (int32_t)res.load;
                cur_k = list_k;
                if (got == n) { done_k += cur_k; cur_k = 0; }
            }
            if (stage == 1) {                             /* end of the iteration: apply what is complete */
                update_k[t] = done_k;
                done_k = 0;
            }
        }
    }
    tail[0] = cur_k;
    tail[1] = fut_k;
    free(cur); free(chosen); free(lw); free(lid);
    return rc;
}

typedef struct {
    int32_t n, iterations, cap_limit, lo, hi;
    const int32_t *comm, *drop, *fwd, *bwd;
    int32_t *stage_case, *stage_count, *stage_time, *update_k, *tail, *status;
    int64_t *sweep_cells;
} sim_slice_t;

static void *sim_worker(void *p)
{
    sim_slice_t *s = (sim_slice_t *)p;
    for (int b = s->lo; b < s->hi; ++b) {
        size_t sn = (size_t)b * (size_t)s->n, si = (size_t)b * (size_t)s->iterations;
        s->status[b] = deft_oracle_simulate(s->n, s->iterations, s->comm + sn, s->drop + sn, s->fwd[b], s->bwd[b],
                                            s->cap_limit, s->stage_case + 2 * si, s->stage_count + 2 * si,
                                            s->stage_time + 2 * si, s->update_k + si, s->tail + 2 * (size_t)b,
                                            s->sweep_cells + b);
    }
    return NULL;
}

/* Batch of candidate schedules; arrays are [batch][n], [batch], [batch][iterations][2], [batch][iterations], [batch][2]. */
int deft_oracle_simulate_batch(int32_t batch, int32_t n, int32_t iterations, const int32_t *comm, const int32_t *drop,
                               const int32_t *fwd, const int32_t *bwd, int32_t cap_limit, int32_t *stage_case,
                               int32_t *stage_count, int32_t *stage_time, int32_t *update_k, int32_t *tail,
                               int32_t *status, int64_t *sweep_cells, int32_t nthreads)
{
    if (batch < 0 || n < 1 || iterations < 0) return -1;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > batch) nthreads = batch > 0 ? batch : 1;
    pthread_t *tid = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
    sim_slice_t *sl = (sim_slice_t *)malloc(sizeof(sim_slice_t) * (size_t)nthreads);
    char *live = (char *)calloc((size_t)nthreads, 1);
    if (!tid || !sl || !live) { free(tid); free(sl); free(live); return -1; }
    for (int t = 0; t < nthreads; ++t) {
        sim_slice_t s = { n, iterations, cap_limit, (int)((int64_t)batch * t / nthreads),
                          (int)((int64_t)batch * (t + 1) / nthreads), comm, drop, fwd, bwd, stage_case, stage_count,
                          stage_time, update_k, tail, status, sweep_cells };
        sl[t] = s;
        if (nthreads > 1 && pthread_create(&tid[t], NULL, sim_worker, &sl[t]) == 0) live[t] = 1;
        else sim_worker(&sl[t]);
    }
    for (int t = 0; t < nthreads; ++t)
        if (live[t]) pthread_join(tid[t], NULL);
    free(tid); free(sl); free(live);
    return nthreads;
}
