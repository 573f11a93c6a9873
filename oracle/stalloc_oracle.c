/*
 * CPU oracle for spatio-temporal allocation planning.
 *
 * THIS IS TEST INFRASTRUCTURE, not a product path: it exists so that the GPU
 * library can be compared against something slow and obviously correct.  Only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, headers, tables or helpers with the GPU library.
 *
 * What is computed (problem statement of Sec. 5.1):
 *   a request is a rectangle  s bytes x [t_s, t_e)  (Sec. 4, request event m);
 *   a plan gives every request a start address a (decision d = m + (a));
 *   two decisions may not conflict in lifespan AND in address range at once;
 *   the extent of a plan is max(d.a + d.s)  (Eq. 2, Eq. 6);
 *   memory efficiency is M_a / M_r (Eq. 1): M_a = max over time of live bytes,
 *   M_r = the plan's extent.
 *
 * Placement rule: requests are taken in a given order and each is put at the
 * lowest address at which it conflicts with no request placed before it
 * ("lowest available address", Sec. 5.1 HomoPhase fusion; larger-first so that
 * smaller requests fill the unused intervals, Sec. 5.1 Global Planning).
 * For a fixed order the result is unique.
 *
 * Readings taken where the text is silent:
 *   - lifetimes are half-open [t_s, t_e): a request released at t and one
 *     allocated at t do not conflict;
 *   - address ranges are half-open [a, a+s): touching ranges do not conflict;
 *   - no alignment is applied;
 *   - among plans of equal extent the lowest plan index wins.
 *
 * Pins (tests/test_oracle_*.py): closed forms for time-cliques and
 * time-disjoint traces, the equal-size case against Algorithm 1's layer count,
 * stack-discipline traces, exhaustive search over all orders for n <= 8 against
 * an independent exact search, a quadratic no-conflict check, a minimality
 * re-derivation, and hand-worked examples under tests/golden/.
 * No value printed in the paper exists for a placement (its worked figures are
 * images), so parity with printed values is unpinned.
 *
 * Dynamic reusable space (Sec. 5.2): oracle_reusable_space, pinned by a
 * byte-by-byte occupancy map on small pools, closed forms and a hand-worked
 * example (tests/test_oracle_reusable.py); no printed values exist for it either.
 *
 * Memory-layer construction (Sec. 5.1, Algorithm 1): oracle_memory_layers, pinned by a
 * hand-worked example, the optimum of interval partitioning (as many layers as
 * requests of the size are ever alive at once), structural invariants, closed forms
 * and the validity of the plan that the layers expand to (tests/test_oracle_layers.py).
 *
 * Candidate placement orders: oracle_make_orders, pinned by the published outputs of
 * SplitMix64, the sorting rules checked on the result, agreement with the numpy input
 * generator of workloads/ and the statistics of the two random families
 * (tests/test_oracle_orders.py).
 *
 * Fusion of two HomoPhase groups (Sec. 5.1, HomoPhase Group Planning): oracle_fuse_groups,
 * pinned by a hand-worked example with an accepted and a rejected fusion, closed forms
 * (disjoint lifetimes: the smaller plan disappears inside the larger; one common lifetime:
 * the plans end up stacked and the fusion is rejected), the no-conflict invariant, the
 * equivalence of its integer accept test with the TMP values of Eq. 2, and planted mistakes
 * (tests/test_oracle_fusion.py).  The paper's worked figure is an image: unpinned by printed values.
 *
 * The time-memory product of a plan (Eq. 2) is a ratio of exact integers and lives in
 * the Python part of the oracle (oracle/__init__.py, tmp), pinned by closed forms, the
 * area bound, unit invariances and an instant-by-instant count (tests/test_oracle_tmp.py).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_OK = 0, ORC_INVALID_ARG = 1, ORC_BAD_TRACE = 2, ORC_OVERFLOW = 3, ORC_NOMEM = 4 };

static int lifetimes_conflict(uint32_t ts_a, uint32_t te_a, uint32_t ts_b, uint32_t te_b)
{
    return ts_a < te_b && ts_b < te_a;
}

static int ranges_conflict(uint64_t a_a, uint64_t s_a, uint64_t a_b, uint64_t s_b)
{
    return a_a < a_b + s_b && a_b < a_a + s_a;
}

/* Trace sanity: sizes > 0, t_s < t_e <= t_end, sum of sizes below 2^63. */
int oracle_check_trace(uint32_t n, uint32_t t_end, const uint64_t *size,
                       const uint32_t *t_s, const uint32_t *t_e)
{
    if (n == 0 || !size || !t_s || !t_e) return ORC_INVALID_ARG;
    uint64_t sum = 0;
    for (uint32_t i = 0; i < n; ++i) {
        if (size[i] == 0 || t_s[i] >= t_e[i] || t_e[i] > t_end) return ORC_BAD_TRACE;
        if (size[i] >= (1ull << 63) || sum + size[i] >= (1ull << 63)) return ORC_OVERFLOW;
        sum += size[i];
    }
    return ORC_OK;
}

typedef struct { uint64_t a; uint64_t end; } span_t;

static int span_by_address(const void *pa, const void *pb)
{
    const span_t *x = (const span_t *)pa, *y = (const span_t *)pb;
    if (x->a != y->a) return x->a < y->a ? -1 : 1;
    if (x->end != y->end) return x->end < y->end ? -1 : 1;
    return 0;
}

/* Lowest address x such that [x, x+s) meets none of the k spans. */
static uint64_t lowest_free_address(span_t *spans, size_t k, uint64_t s)
{
    qsort(spans, k, sizeof(span_t), span_by_address);
    uint64_t x = 0;
    for (size_t c = 0; c < k; ++c) {
        if (spans[c].a >= x + s) break;      /* the hole [x, spans[c].a) is large enough */
        if (spans[c].end > x) x = spans[c].end;
    }
    return x;
}

/*
 * One plan, every earlier request examined for every placement.
 * order: permutation of 0..n-1.  a[i] receives request i's address.
 */
int oracle_plan_allpairs(uint32_t n, const uint64_t *size, const uint32_t *t_s,
                         const uint32_t *t_e, const uint32_t *order,
                         uint64_t *a, uint64_t *extent)
{
    if (n == 0 || !order || !a || !extent) return ORC_INVALID_ARG;
    span_t *spans = (span_t *)malloc((size_t)n * sizeof(span_t));
    if (!spans) return ORC_NOMEM;
    uint64_t top = 0;
    for (uint32_t k = 0; k < n; ++k) {
        uint32_t i = order[k];
        size_t m = 0;
        for (uint32_t q = 0; q < k; ++q) {
            uint32_t j = order[q];
            if (lifetimes_conflict(t_s[i], t_e[i], t_s[j], t_e[j])) {
                spans[m].a = a[j];
                spans[m].end = a[j] + size[j];
                ++m;
            }
        }
        a[i] = lowest_free_address(spans, m, size[i]);
        if (a[i] + size[i] > top) top = a[i] + size[i];
    }
    free(spans);
    *extent = top;
    return ORC_OK;
}

/*
 * Lists, for every request, the requests whose lifetime conflicts with it
 * (both directions).  Call with nbr == NULL to obtain the counts in
 * nbr_begin[0..n] (as prefix sums), then again with storage.
 */
int oracle_conflict_lists(uint32_t n, const uint32_t *t_s, const uint32_t *t_e,
                          uint64_t *nbr_begin, uint32_t *nbr)
{
    if (n == 0 || !nbr_begin) return ORC_INVALID_ARG;
    uint64_t *fill = NULL;
    if (nbr) {
        fill = (uint64_t *)malloc((size_t)n * sizeof(uint64_t));
        if (!fill) return ORC_NOMEM;
        memcpy(fill, nbr_begin, (size_t)n * sizeof(uint64_t));
    } else {
        memset(nbr_begin, 0, ((size_t)n + 1) * sizeof(uint64_t));
    }
    for (uint32_t i = 0; i < n; ++i)
        for (uint32_t j = i + 1; j < n; ++j)
            if (lifetimes_conflict(t_s[i], t_e[i], t_s[j], t_e[j])) {
                if (nbr) { nbr[fill[i]++] = j; nbr[fill[j]++] = i; }
                else     { nbr_begin[i + 1]++; nbr_begin[j + 1]++; }
            }
    if (!nbr)
        for (uint32_t i = 0; i < n; ++i) nbr_begin[i + 1] += nbr_begin[i];
    free(fill);
    return ORC_OK;
}

/* Same rule as oracle_plan_allpairs; candidates come from the conflict lists. */
int oracle_plan_lists(uint32_t n, const uint64_t *size, const uint64_t *nbr_begin,
                      const uint32_t *nbr, const uint32_t *order,
                      uint64_t *a, uint64_t *extent)
{
    if (n == 0 || !order || !a || !extent || !nbr_begin) return ORC_INVALID_ARG;
    uint64_t widest = 0;
    for (uint32_t i = 0; i < n; ++i)
        if (nbr_begin[i + 1] - nbr_begin[i] > widest) widest = nbr_begin[i + 1] - nbr_begin[i];
    span_t *spans = (span_t *)malloc((size_t)(widest + 1) * sizeof(span_t));
    uint8_t *placed = (uint8_t *)calloc(n, 1);
    if (!spans || !placed) { free(spans); free(placed); return ORC_NOMEM; }
    uint64_t top = 0;
    for (uint32_t k = 0; k < n; ++k) {
        uint32_t i = order[k];
        size_t m = 0;
        for (uint64_t e = nbr_begin[i]; e < nbr_begin[i + 1]; ++e) {
            uint32_t j = nbr[e];
            if (placed[j]) { spans[m].a = a[j]; spans[m].end = a[j] + size[j]; ++m; }
        }
        a[i] = lowest_free_address(spans, m, size[i]);
        placed[i] = 1;
        if (a[i] + size[i] > top) top = a[i] + size[i];
    }
    free(spans);
    free(placed);
    *extent = top;
    return ORC_OK;
}

/* Index of the smallest extent; the lowest index among equals. */
int oracle_best_plan(uint32_t P, const uint64_t *extent, uint32_t *best)
{
    if (P == 0 || !extent || !best) return ORC_INVALID_ARG;
    uint32_t b = 0;
    for (uint32_t p = 1; p < P; ++p)
        if (extent[p] < extent[b]) b = p;
    *best = b;
    return ORC_OK;
}

/*
 * Number of unordered pairs that conflict in lifespan and in address range,
 * and the lexicographically first such pair (i < j); {~0, ~0} if none.
 */
int oracle_validate(uint32_t n, const uint64_t *size, const uint32_t *t_s,
                    const uint32_t *t_e, const uint64_t *a,
                    uint64_t *conflicts, uint32_t *first_pair)
{
    if (n == 0 || !a || !conflicts || !first_pair) return ORC_INVALID_ARG;
    uint64_t cnt = 0;
    first_pair[0] = first_pair[1] = 0xFFFFFFFFu;
    for (uint32_t i = 0; i < n; ++i)
        for (uint32_t j = i + 1; j < n; ++j)
            if (lifetimes_conflict(t_s[i], t_e[i], t_s[j], t_e[j]) &&
                ranges_conflict(a[i], size[i], a[j], size[j])) {
                if (cnt == 0) { first_pair[0] = i; first_pair[1] = j; }
                ++cnt;
            }
    *conflicts = cnt;
    return ORC_OK;
}

/*
 * M_a of Eq. 1 by its definition: for every t in [0, t_end) add up the sizes of
 * the requests alive at t; keep the maximum and the earliest t reaching it.
 */
int oracle_lower_bound_definition(uint32_t n, uint32_t t_end, const uint64_t *size,
                                  const uint32_t *t_s, const uint32_t *t_e,
                                  uint64_t *max_live, uint32_t *t_at_max)
{
    if (n == 0 || !max_live) return ORC_INVALID_ARG;
    uint64_t best = 0; uint32_t best_t = 0;
    for (uint32_t t = 0; t < t_end; ++t) {
        uint64_t live = 0;
        for (uint32_t i = 0; i < n; ++i)
            if (t_s[i] <= t && t < t_e[i]) live += size[i];
        if (live > best) { best = live; best_t = t; }
    }
    *max_live = best;
    if (t_at_max) *t_at_max = best_t;
    return ORC_OK;
}

/* Same quantity from per-timestamp net changes and a running sum. */
int oracle_lower_bound_sweep(uint32_t n, uint32_t t_end, const uint64_t *size,
                             const uint32_t *t_s, const uint32_t *t_e,
                             uint64_t *max_live, uint32_t *t_at_max)
{
    if (n == 0 || !max_live) return ORC_INVALID_ARG;
    int64_t *net = (int64_t *)calloc((size_t)t_end + 1, sizeof(int64_t));
    if (!net) return ORC_NOMEM;
    for (uint32_t i = 0; i < n; ++i) {
        net[t_s[i]] += (int64_t)size[i];
        net[t_e[i]] -= (int64_t)size[i];
    }
    int64_t live = 0, best = 0; uint32_t best_t = 0;
    for (uint32_t t = 0; t < t_end; ++t) {
        live += net[t];
        if (live > best) { best = live; best_t = t; }
    }
    free(net);
    *max_live = (uint64_t)best;
    if (t_at_max) *t_at_max = best_t;
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Exhaustive searches for very small traces                                 */
/* ------------------------------------------------------------------------ */

/*
 * Smallest extent over all n! placement orders (n <= 9) and the first order,
 * in lexicographic enumeration, that reaches it.
 */
int oracle_best_over_all_orders(uint32_t n, const uint64_t *size, const uint32_t *t_s,
                                const uint32_t *t_e, uint64_t *best_extent,
                                uint32_t *best_order)
{
    if (n == 0 || n > 9 || !best_extent) return ORC_INVALID_ARG;
    uint32_t perm[9]; uint64_t a[9];
    for (uint32_t i = 0; i < n; ++i) perm[i] = i;
    uint64_t best = ~0ull;
    for (;;) {
        uint64_t ext = 0;
        int rc = oracle_plan_allpairs(n, size, t_s, t_e, perm, a, &ext);
        if (rc) return rc;
        if (ext < best) {
            best = ext;
            if (best_order) memcpy(best_order, perm, n * sizeof(uint32_t));
        }
        /* next permutation in lexicographic order */
        int k = (int)n - 2;
        while (k >= 0 && perm[k] > perm[k + 1]) --k;
        if (k < 0) break;
        int l = (int)n - 1;
        while (perm[l] < perm[k]) --l;
        uint32_t tmp = perm[k]; perm[k] = perm[l]; perm[l] = tmp;
        for (int lo = k + 1, hi = (int)n - 1; lo < hi; ++lo, --hi) {
            tmp = perm[lo]; perm[lo] = perm[hi]; perm[hi] = tmp;
        }
    }
    *best_extent = best;
    return ORC_OK;
}

/*
 * True optimum of the placement problem for n <= 6 without any placement order:
 * in some optimal plan every address is a sum of sizes of other requests (push
 * every block down until it rests on address 0 or on another block), so it is
 * enough to try, for each request, every subset sum of the other sizes.
 */
typedef struct {
    uint32_t n; const uint64_t *size; const uint32_t *t_s; const uint32_t *t_e;
    uint64_t a[6]; uint64_t best; uint64_t best_a[6];
} exact_search_t;

static void exact_search(exact_search_t *st, uint32_t i, uint64_t top)
{
    if (top >= st->best) return;
    if (i == st->n) {
        st->best = top;
        memcpy(st->best_a, st->a, sizeof(st->a));
        return;
    }
    uint32_t others = st->n - 1;
    for (uint32_t mask = 0; mask < (1u << others); ++mask) {
        uint64_t x = 0;
        for (uint32_t b = 0, j = 0; j < st->n; ++j) {
            if (j == i) continue;
            if (mask & (1u << b)) x += st->size[j];
            ++b;
        }
        int ok = 1;
        for (uint32_t j = 0; j < i && ok; ++j)
            if (lifetimes_conflict(st->t_s[i], st->t_e[i], st->t_s[j], st->t_e[j]) &&
                ranges_conflict(x, st->size[i], st->a[j], st->size[j])) ok = 0;
        if (!ok) continue;
        st->a[i] = x;
        uint64_t t2 = x + st->size[i] > top ? x + st->size[i] : top;
        exact_search(st, i + 1, t2);
    }
}

int oracle_exact_optimum(uint32_t n, const uint64_t *size, const uint32_t *t_s,
                         const uint32_t *t_e, uint64_t *opt_extent, uint64_t *opt_a)
{
    if (n == 0 || n > 6 || !opt_extent) return ORC_INVALID_ARG;
    exact_search_t st;
    st.n = n; st.size = size; st.t_s = t_s; st.t_e = t_e; st.best = ~0ull;
    memset(st.a, 0, sizeof(st.a));
    exact_search(&st, 0, 0);
    *opt_extent = st.best;
    if (opt_a) memcpy(opt_a, st.best_a, n * sizeof(uint64_t));
    return ORC_OK;
}

/*
 * Dynamic reusable space of a plan for one time window (Sec. 5.2).
 * The occupied addresses A_o of the window are the union of the address ranges
 * R_s(d) of the decisions whose lifespan R_t(d) meets the window; the pool A
 * runs from the lowest start address to the highest end address of the whole
 * plan; the reusable space A_i is A without A_o.  It is returned as its maximal
 * intervals [lo, hi) in ascending order: ranges[2c], ranges[2c+1] for the first
 * `cap` of them, *count = how many there are, *idle = their total length.
 * Readings: the window [w_lo, w_hi) is half-open like the lifespans (the paper
 * prints both closed), so a decision meets it iff t_s < w_hi and w_lo < t_e.
 */
int oracle_reusable_space(uint32_t n, const uint64_t *size, const uint32_t *t_s,
                          const uint32_t *t_e, const uint64_t *a, uint32_t w_lo, uint32_t w_hi,
                          uint64_t cap, uint64_t *ranges, uint64_t *count, uint64_t *idle)
{
    if (n == 0 || !size || !t_s || !t_e || !a || !count || !idle || (cap && !ranges)) return ORC_INVALID_ARG;
    if (w_lo >= w_hi) return ORC_INVALID_ARG;
    span_t *met = (span_t *)malloc((size_t)n * sizeof(span_t));
    if (!met) return ORC_NOMEM;
    uint64_t pool_lo = a[0], pool_hi = a[0] + size[0];
    size_t k = 0;
    for (uint32_t i = 0; i < n; ++i) {
        if (a[i] < pool_lo) pool_lo = a[i];
        if (a[i] + size[i] > pool_hi) pool_hi = a[i] + size[i];
        if (lifetimes_conflict(t_s[i], t_e[i], w_lo, w_hi)) {
            met[k].a = a[i];
            met[k].end = a[i] + size[i];
            ++k;
        }
    }
    qsort(met, k, sizeof(span_t), span_by_address);
    uint64_t found = 0, total = 0, reach = pool_lo;      /* everything below `reach` is accounted for */
    for (size_t c = 0; c <= k; ++c) {
        const uint64_t next = c < k ? met[c].a : pool_hi;
        if (next > reach) {                               /* [reach, next) is idle throughout the window */
            if (found < cap) { ranges[2 * found] = reach; ranges[2 * found + 1] = next; }
            ++found;
            total += next - reach;
        }
        if (c < k && met[c].end > reach) reach = met[c].end;
    }
    free(met);
    *count = found;
    *idle = total;
    return ORC_OK;
}

/*
 * Memory-layer construction for the HomoSize groups of a trace (Sec. 5.1,
 * HomoSize Group Planning, Algorithm 1).  A HomoSize group M_s holds the requests of
 * one size S; requests of a group whose lifetimes do not overlap can share one
 * range of S bytes, a memory-layer.  The rule of Algorithm 1: a group's requests are
 * taken by allocation time; each goes, among the layers that are free at its allocation
 * time, to the one that became free last, so that the layer idles least; if no layer is
 * free a new one is opened.
 *
 * Written here as a sweep over the group's events in time order instead of a search over
 * the layers per request: a layer becomes free when the request it holds is released, so
 * the free layers, kept in the order in which they became free, form a pile whose top is
 * "the free layer with the latest end"; a release puts its layer on the pile, an
 * allocation takes the top or opens a new layer when the pile is empty.
 *
 * Output: layer_of[i] = layer of request i.  Layers are numbered group by group in
 * descending size (the order in which the global plan takes the groups) and, inside
 * a group, in the order in which they were opened.  For every layer: its size, the
 * allocation time of its first request and the free time of its last one -- the
 * rectangle the layer occupies when it is planned as one request (as the local plan
 * of a group is, Sec. 5.1).  *n_layers = number of layers.
 *
 * Readings: lifetimes are half-open, so a layer whose request is released at t is free
 * for a request allocated at t (releases at t come before allocations at t; the listing
 * prints a strict comparison for closed lifetimes); requests with equal allocation times
 * are taken by request number; of layers that become free at the same time the one
 * opened first is taken first.
 */
typedef struct { uint64_t size; uint32_t id; } layer_member_t;
typedef struct { uint32_t t; uint32_t is_alloc; uint32_t id; } layer_event_t;

static int by_size_desc(const void *pa, const void *pb)
{
    const layer_member_t *x = (const layer_member_t *)pa, *y = (const layer_member_t *)pb;
    if (x->size != y->size) return x->size > y->size ? -1 : 1;
    return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);
}

static int by_time_release_first(const void *pa, const void *pb)
{
    const layer_event_t *x = (const layer_event_t *)pa, *y = (const layer_event_t *)pb;
    if (x->t != y->t) return x->t < y->t ? -1 : 1;
    if (x->is_alloc != y->is_alloc) return x->is_alloc < y->is_alloc ? -1 : 1;
    return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);
}

static int descending_u32(const void *pa, const void *pb)
{
    const uint32_t x = *(const uint32_t *)pa, y = *(const uint32_t *)pb;
    return (x < y) - (x > y);
}

int oracle_memory_layers(uint32_t n, const uint64_t *size, const uint32_t *t_s,
                         const uint32_t *t_e, uint32_t *layer_of, uint32_t *n_layers,
                         uint64_t *layer_size, uint32_t *layer_t_s, uint32_t *layer_t_e)
{
    if (n == 0 || !size || !t_s || !t_e || !layer_of || !n_layers || !layer_size || !layer_t_s || !layer_t_e)
        return ORC_INVALID_ARG;
    layer_member_t *m = (layer_member_t *)malloc((size_t)n * sizeof(layer_member_t));
    layer_event_t *ev = (layer_event_t *)malloc((size_t)n * 2 * sizeof(layer_event_t));
    uint32_t *pile = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));      /* free layers, freed last on top */
    uint32_t *freed = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));     /* layers freed at the current time */
    if (!m || !ev || !pile || !freed) { free(m); free(ev); free(pile); free(freed); return ORC_NOMEM; }
    for (uint32_t i = 0; i < n; ++i) { m[i].size = size[i]; m[i].id = i; }
    qsort(m, n, sizeof(layer_member_t), by_size_desc);
    uint32_t layers = 0;                       /* layers opened so far, over all groups */
    for (uint32_t g0 = 0; g0 < n; ) {
        uint32_t g1 = g0;                      /* the HomoSize group m[g0 .. g1) */
        while (g1 < n && m[g1].size == m[g0].size) ++g1;
        const uint32_t members = g1 - g0;
        for (uint32_t k = 0; k < members; ++k) {
            const uint32_t i = m[g0 + k].id;
            ev[2 * k].t = t_s[i]; ev[2 * k].is_alloc = 1; ev[2 * k].id = i;
            ev[2 * k + 1].t = t_e[i]; ev[2 * k + 1].is_alloc = 0; ev[2 * k + 1].id = i;
        }
        qsort(ev, 2 * (size_t)members, sizeof(layer_event_t), by_time_release_first);
        uint32_t on_pile = 0;                  /* every group starts with no layer */
        for (uint32_t e = 0; e < 2 * members; ) {
            /* the releases of this instant: their layers go on the pile, the one opened first on top */
            uint32_t k = 0;
            const uint32_t now = ev[e].t;
            while (e < 2 * members && ev[e].t == now && !ev[e].is_alloc) freed[k++] = layer_of[ev[e++].id];
            qsort(freed, k, sizeof(uint32_t), descending_u32);
            for (uint32_t q = 0; q < k; ++q) pile[on_pile++] = freed[q];
            /* the allocations of this instant, by request number */
            while (e < 2 * members && ev[e].t == now && ev[e].is_alloc) {
                const uint32_t i = ev[e++].id;
                uint32_t l;
                if (on_pile > 0) {
                    l = pile[--on_pile];
                } else {
                    l = layers++;
                    layer_size[l] = size[i];
                    layer_t_s[l] = t_s[i];
                }
                layer_of[i] = l;
                layer_t_e[l] = t_e[i];
            }
        }
        g0 = g1;
    }
    free(m); free(ev); free(pile); free(freed);
    *n_layers = layers;
    return ORC_OK;
}

/*
 * Candidate placement orders.  Row p is a permutation of the request numbers:
 *   p = 0          by size descending, then allocation time, then number -- large
 *                  requests first, so that smaller ones fill the intervals they leave
 *                  (Sec. 5.1, Global Planning);
 *   p = 1          by lifetime descending, then size descending, then number;
 *   p = 2          by allocation time, then number (the order Algorithm 1 takes);
 *   p >= 3, odd    by a 64-bit pseudo-random key k(p, i), then number: a uniform
 *                  random permutation;
 *   p >= 4, even   by (c(i) + 1) * 2^32 + (k(p, i) >> 31), then number, where c(i) is
 *                  the number of distinct sizes larger than request i's: size
 *                  descending, with a random order inside each size and a shift of up
 *                  to one size to either side.
 * k(p, i) = mix(i * 0xD1342543DE82EF95 + mix(seed + p)), all modulo 2^64, where mix(x)
 * is the output of the SplitMix64 generator (Steele, Lea, Flood: "Fast splittable
 * pseudorandom number generators", OOPSLA 2014; constants of Vigna's public-domain
 * splitmix64.c) whose state before the step is x: so any row, and any key, can be
 * produced on its own from (seed, p, i).
 * Writes rows first_plan .. first_plan + P - 1 to orders[P][n].
 */
uint64_t oracle_splitmix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

typedef struct { uint64_t k0, k1; uint32_t k2; uint32_t id; } order_key_t;

static int order_key_cmp(const void *pa, const void *pb)
{
    const order_key_t *x = (const order_key_t *)pa, *y = (const order_key_t *)pb;
    if (x->k0 != y->k0) return x->k0 < y->k0 ? -1 : 1;
    if (x->k1 != y->k1) return x->k1 < y->k1 ? -1 : 1;
    if (x->k2 != y->k2) return x->k2 < y->k2 ? -1 : 1;
    return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);
}

static int u64_desc(const void *pa, const void *pb)
{
    const uint64_t x = *(const uint64_t *)pa, y = *(const uint64_t *)pb;
    return x > y ? -1 : (x < y ? 1 : 0);
}

int oracle_make_orders(uint32_t n, const uint64_t *size, const uint32_t *t_s, const uint32_t *t_e,
                       uint32_t first_plan, uint32_t P, uint64_t seed, uint32_t *orders)
{
    if (n == 0 || P == 0 || !size || !t_s || !t_e || !orders) return ORC_INVALID_ARG;
    order_key_t *m = (order_key_t *)malloc((size_t)n * sizeof(order_key_t));
    uint64_t *distinct = (uint64_t *)malloc((size_t)n * sizeof(uint64_t));
    uint32_t *larger = (uint32_t *)malloc((size_t)n * sizeof(uint32_t));
    if (!m || !distinct || !larger) { free(m); free(distinct); free(larger); return ORC_NOMEM; }
    /* c(i): number of distinct sizes larger than size[i] */
    memcpy(distinct, size, (size_t)n * sizeof(uint64_t));
    qsort(distinct, n, sizeof(uint64_t), u64_desc);
    uint32_t d = 0;
    for (uint32_t k = 0; k < n; ++k)
        if (k == 0 || distinct[k] != distinct[k - 1]) distinct[d++] = distinct[k];
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t c = 0;
        while (distinct[c] != size[i]) ++c;
        larger[i] = c;
    }
    for (uint32_t r = 0; r < P; ++r) {
        const uint64_t p = (uint64_t)first_plan + r;
        const uint64_t stream = oracle_splitmix64(seed + p);
        for (uint32_t i = 0; i < n; ++i) {
            const uint64_t k = oracle_splitmix64((uint64_t)i * 0xD1342543DE82EF95ull + stream);
            m[i].id = i;
            m[i].k0 = 0; m[i].k1 = 0; m[i].k2 = 0;
            if (p == 0)          { m[i].k0 = ~size[i]; m[i].k2 = t_s[i]; }
            else if (p == 1)     { m[i].k0 = ~(uint64_t)(t_e[i] - t_s[i]); m[i].k1 = ~size[i]; }
            else if (p == 2)     { m[i].k2 = t_s[i]; }
            else if (p % 2 == 1) { m[i].k0 = k; }
            else                 { m[i].k0 = (((uint64_t)larger[i] + 1) << 32) + (k >> 31); }
        }
        qsort(m, n, sizeof(order_key_t), order_key_cmp);
        for (uint32_t q = 0; q < n; ++q) orders[(size_t)r * n + q] = m[q].id;
    }
    free(m); free(distinct); free(larger);
    return ORC_OK;
}


/* ---------------------------------------------------------------------------------------
 * Fusion of two HomoPhase groups (Sec. 5.1, HomoPhase Group Planning).
 *
 * A HomoPhase group holds the requests allocated in one computation phase and released in
 * one (other) phase; its local plan packs them contiguously, so its extent is the sum of
 * their sizes.  Two such plans are fused by inserting the smaller into the larger:
 *   - the larger plan's requests are packed from 0 in descending order of release time
 *     (request number among equals);
 *   - addr starts at the lowest start address of the larger plan; the requests of the smaller
 *     plan are tried in order of allocation time (request number among equals): the first
 *     one that conflicts with nothing placed so far when put at addr is placed there and
 *     addr moves up by its size; if none fits, addr moves to the next higher start address
 *     of the larger plan; when there is none, the requests still left are packed on top of
 *     everything placed, in the same order (the text does not say; they have to go somewhere);
 *   - the fusion is accepted only if its time-memory product (Eq. 2) exceeds the weighted
 *     average of the two plans' products, the weights being the memory-time each plan reserves
 *     (its extent times its span): the weighted average is then (used_1 + used_2) /
 *     (reserved_1 + reserved_2) and, the used memory-time being the same on both sides, the
 *     test is  reserved_fused < reserved_1 + reserved_2  in exact integers.
 *
 * members1 / members2: request numbers of the two groups.  order_out / addr_out [n1 + n2]: the
 * fused plan, the larger group's requests first (in packing order), then the smaller group's in
 * order of allocation time.  extent_out[3], span_out[3][2]: extent and (first allocation,
 * last release) of plan 1, plan 2 and the fused plan.  accepted_out[1].
 */
typedef struct { uint32_t id; uint32_t key; } fuse_key_t;

static int fuse_by_release_desc(const void *pa, const void *pb)
{
    const fuse_key_t *a = (const fuse_key_t *)pa, *b = (const fuse_key_t *)pb;
    if (a->key != b->key) return a->key > b->key ? -1 : 1;
    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

static int fuse_by_start_asc(const void *pa, const void *pb)
{
    const fuse_key_t *a = (const fuse_key_t *)pa, *b = (const fuse_key_t *)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);
}

int oracle_fuse_groups(uint32_t n, const uint64_t *size, const uint32_t *t_s, const uint32_t *t_e,
                       uint32_t n1, const uint32_t *members1, uint32_t n2, const uint32_t *members2,
                       uint32_t *order_out, uint64_t *addr_out, uint64_t *extent_out, uint32_t *span_out,
                       uint32_t *accepted_out)
{
    if (!size || !t_s || !t_e || !members1 || !members2 || n1 == 0 || n2 == 0 || !order_out || !addr_out ||
        !extent_out || !span_out || !accepted_out)
        return ORC_INVALID_ARG;
    for (uint32_t k = 0; k < n1; ++k) if (members1[k] >= n) return ORC_INVALID_ARG;
    for (uint32_t k = 0; k < n2; ++k) if (members2[k] >= n) return ORC_INVALID_ARG;
    /* the two local plans: extent = sum of sizes, span = first allocation .. last release */
    uint64_t ext[2] = {0, 0};
    uint32_t lo[2] = {0xffffffffu, 0xffffffffu}, hi[2] = {0, 0};
    for (uint32_t k = 0; k < n1; ++k) {
        uint32_t i = members1[k];
        ext[0] += size[i];
        if (t_s[i] < lo[0]) lo[0] = t_s[i];
        if (t_e[i] > hi[0]) hi[0] = t_e[i];
    }
    for (uint32_t k = 0; k < n2; ++k) {
        uint32_t i = members2[k];
        ext[1] += size[i];
        if (t_s[i] < lo[1]) lo[1] = t_s[i];
        if (t_e[i] > hi[1]) hi[1] = t_e[i];
    }
    const int first_is_larger = ext[0] >= ext[1];
    const uint32_t nl = first_is_larger ? n1 : n2, ns = first_is_larger ? n2 : n1;
    const uint32_t *larger = first_is_larger ? members1 : members2, *smaller = first_is_larger ? members2 : members1;
    fuse_key_t *kl = (fuse_key_t *)malloc(sizeof(fuse_key_t) * nl), *ks = (fuse_key_t *)malloc(sizeof(fuse_key_t) * ns);
    unsigned char *placed = (unsigned char *)calloc(ns, 1);
    if (!kl || !ks || !placed) { free(kl); free(ks); free(placed); return ORC_NOMEM; }
    for (uint32_t k = 0; k < nl; ++k) { kl[k].id = larger[k]; kl[k].key = t_e[larger[k]]; }
    for (uint32_t k = 0; k < ns; ++k) { ks[k].id = smaller[k]; ks[k].key = t_s[smaller[k]]; }
    qsort(kl, nl, sizeof(fuse_key_t), fuse_by_release_desc);
    qsort(ks, ns, sizeof(fuse_key_t), fuse_by_start_asc);
    /* the larger plan, packed from 0 */
    uint64_t top = 0;
    for (uint32_t k = 0; k < nl; ++k) {
        order_out[k] = kl[k].id;
        addr_out[k] = top;
        top += size[kl[k].id];
    }
    for (uint32_t k = 0; k < ns; ++k) order_out[nl + k] = ks[k].id;
    /* insertion of the smaller plan */
    uint64_t addr = addr_out[0];                 /* the lowest start address of the larger plan */
    uint32_t left = ns;
    for (;;) {
        if (left == 0) break;
        uint32_t fit = ns;
        for (uint32_t k = 0; k < ns && fit == ns; ++k) {
            if (placed[k]) continue;
            const uint32_t j = ks[k].id;
            int clash = 0;
            for (uint32_t q = 0; q < nl + ns && !clash; ++q) {
                if (q >= nl && !placed[q - nl]) continue;
                const uint32_t i = order_out[q];
                clash = lifetimes_conflict(t_s[i], t_e[i], t_s[j], t_e[j]) &&
                        ranges_conflict(addr_out[q], size[i], addr, size[j]);
            }
            if (!clash) fit = k;
        }
        if (fit < ns) {
            placed[fit] = 1;
            addr_out[nl + fit] = addr;
            addr += size[ks[fit].id];
            --left;
            continue;
        }
        /* nothing fits here: on to the next higher start address of the larger plan */
        uint64_t next = 0;
        int have = 0;
        for (uint32_t k = 0; k < nl; ++k)
            if (addr_out[k] > addr && (!have || addr_out[k] < next)) { next = addr_out[k]; have = 1; }
        if (!have) break;
        addr = next;
    }
    /* what is left goes on top of everything placed */
    for (uint32_t q = 0; q < nl + ns; ++q) {
        if (q >= nl && !placed[q - nl]) continue;
        const uint64_t end = addr_out[q] + size[order_out[q]];
        if (end > top) top = end;
    }
    for (uint32_t k = 0; k < ns; ++k) {
        if (placed[k]) continue;
        addr_out[nl + k] = top;
        top += size[ks[k].id];
    }
    extent_out[0] = ext[0];
    extent_out[1] = ext[1];
    extent_out[2] = top;
    span_out[0] = lo[0]; span_out[1] = hi[0];
    span_out[2] = lo[1]; span_out[3] = hi[1];
    span_out[4] = lo[0] < lo[1] ? lo[0] : lo[1];
    span_out[5] = hi[0] > hi[1] ? hi[0] : hi[1];
    const unsigned __int128 r1 = (unsigned __int128)ext[0] * (hi[0] - lo[0]);
    const unsigned __int128 r2 = (unsigned __int128)ext[1] * (hi[1] - lo[1]);
    const unsigned __int128 rf = (unsigned __int128)top * (span_out[5] - span_out[4]);
    *accepted_out = rf < r1 + r2 ? 1u : 0u;
    free(kl); free(ks); free(placed);
    return ORC_OK;
}
