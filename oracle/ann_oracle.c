/*
 * CPU oracle for batched top-k maximum-inner-product retrieval.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code, header, table or helper with
 * the HIP path and is never called by it; only the tests, the smoke check and
 * the benchmark's cpu_baseline leg load it.
 *
 * What it states (paper: Section 2.1 "Retrieval Mechanism", Section 3.3
 * "Non-Stall Retrieval", Appendix B.3 "Detailed Experimental Setup"):
 *
 *  - exact retrieval (ENN, "full recall"): score every corpus vector against the
 *    query, order all of them, keep the first k.  Written out literally:
 *    N dot products, one full sort.
 *  - graph retrieval (ANN): a best-first search over a fixed-degree proximity
 *    graph that keeps a candidate list of at most `ef` entries (the paper's
 *    "search range") with a best and a worst element, and refines it until no
 *    unexpanded candidate is left (the natural stop).
 *
 * Arithmetic: the stored values (fp16 / bf16 / fp32 bit patterns, exactly the
 * bits the GPU reads) are decoded exactly to double and every dot product is
 * accumulated in double, j = 0..d-1 in order.
 *
 * Order used everywhere: (s, id) precedes (s', id') iff s > s', or s == s' and
 * id < id'.  Larger inner product is better; ties go to the lower id.
 *
 * Threads: queries are independent; an OpenMP loop runs them on `threads`
 * host threads.  That is the only parallelism; nothing is blocked or fused.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_F32 = 2 };

/* IEEE binary16 -> double, exact. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* zero and subnormals: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m | 0x400), e - 25);    /* (1.m) * 2^(e-15) */
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* All 65536 binary16 values decoded once by the function above (a cache of a
 * pure function, so the scoring loops do not call ldexp per element). */
static double half_value[65536];
static int half_value_ready = 0;

static void prepare_tables(void)
{
    if (half_value_ready) return;
    for (uint32_t h = 0; h < 65536; ++h) half_value[h] = half_bits_to_double((uint16_t)h);
    half_value_ready = 1;
}

static double load_value(const void *base, int64_t index, int dtype)
{
    switch (dtype) {
    case ORACLE_F16:  return half_value[((const uint16_t *)base)[index]];
    case ORACLE_BF16: return bf16_bits_to_double(((const uint16_t *)base)[index]);
    default:          return (double)((const float *)base)[index];
    }
}

/* <q, x_n> with q already decoded to double. */
static double score_row(const void *corpus, int64_t n, int32_t d, int dtype, const double *q)
{
    double s = 0.0;
    for (int32_t j = 0; j < d; ++j)
        s += q[j] * load_value(corpus, n * (int64_t)d + j, dtype);
    return s;
}

typedef struct { double s; int32_t id; } scored_t;

static int precedes(double s, int32_t id, double s2, int32_t id2)
{
    return s > s2 || (s == s2 && id < id2);
}

static int by_order(const void *a, const void *b)
{
    const scored_t *x = a, *y = b;
    if (precedes(x->s, x->id, y->s, y->id)) return -1;
    if (precedes(y->s, y->id, x->s, x->id)) return 1;
    return 0;
}

static int use_threads(int threads)
{
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    return threads;
#else
    (void)threads;
    return 1;
#endif
}

/* Number of host threads a call with this `threads` argument will run on. */
int oracle_threads(int threads) { return use_threads(threads); }

/* Score of one (query, row) pair; lets a test look at any single entry of the
 * full score matrix. */
double oracle_score(const void *corpus, int32_t d, int dtype, int64_t row,
                    const void *queries, int32_t b)
{
    prepare_tables();
    double *q = malloc(sizeof(double) * (size_t)d);
    for (int32_t j = 0; j < d; ++j) q[j] = load_value(queries, (int64_t)b * d + j, dtype);
    double s = score_row(corpus, row, d, dtype, q);
    free(q);
    return s;
}

/*
 * Exact retrieval.  ids[B,k], scores[B,k] (fp32), scores64[B,k] optional.
 * A row whose score is NaN has no place in the order and is left out; should fewer than
 * k rows remain, the tail is (id -1, score -inf).
 *
 * Continuation ("the next k"): with after_scores / after_ids (both [B], or both NULL) only rows
 * that come strictly after the pair (after_scores[b], after_ids[b]) in the order are candidates
 * of query b, i.e. rows with a smaller score, or the same score and a larger id.  Feeding the
 * last pair of one answer (its binary64 score) into the next call enumerates the corpus in
 * order, k rows at a time.  A NaN after_score excludes nothing.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_flat_search(const void *corpus, int64_t N, int32_t d, int dtype,
                       const void *queries, int32_t B, int32_t k,
                       const double *after_scores, const int32_t *after_ids,
                       int32_t *ids, float *scores, double *scores64, int threads)
{
    if (!corpus || !queries || !ids || !scores || N < 1 || d < 1 || B < 1 || k < 1 || k > N)
        return -1;
    if ((after_scores == NULL) != (after_ids == NULL)) return -1;
    prepare_tables();
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(use_threads(threads))
    for (int32_t b = 0; b < B; ++b) {
        double *q = malloc(sizeof(double) * (size_t)d);
        scored_t *all = malloc(sizeof(scored_t) * (size_t)N);
        if (!q || !all) { failed = 1; free(q); free(all); continue; }
        for (int32_t j = 0; j < d; ++j) q[j] = load_value(queries, (int64_t)b * d + j, dtype);
        int64_t m = 0;                  /* rows with a score that can be ordered (not NaN) */
        for (int64_t n = 0; n < N; ++n) {
            const double s = score_row(corpus, n, d, dtype, q);
            if (s != s) continue;
            if (after_scores && after_scores[b] == after_scores[b] &&
                !precedes(after_scores[b], after_ids[b], s, (int32_t)n))
                continue;
            all[m].s = s;
            all[m].id = (int32_t)n;
            ++m;
        }
        qsort(all, (size_t)m, sizeof(scored_t), by_order);
        for (int32_t i = 0; i < k; ++i) {
            const int has = i < m;
            ids[(int64_t)b * k + i] = has ? all[i].id : -1;
            scores[(int64_t)b * k + i] = has ? (float)all[i].s : -INFINITY;
            if (scores64) scores64[(int64_t)b * k + i] = has ? all[i].s : -INFINITY;
        }
        free(q);
        free(all);
    }
    return failed ? -1 : 0;
}

/*
 * Graph retrieval: deterministic best-first search with a candidate list of at
 * most ef entries.
 *
 *   visited = {};  L = []
 *   for each entry node in the order given: skip ids outside [0, N) and ids already
 *           visited; otherwise mark visited, score it and put it into L by the rule below
 *   repeat: p = first unexpanded element of L (L is kept in order, so this is
 *           the best unexpanded candidate, ties to the lower id); stop if none
 *           mark p expanded
 *           for each slot of graph[p] in slot order: skip empty (-1),
 *           out-of-range and visited ids; otherwise mark visited, score it, and
 *           put it into L if L is not full or it precedes L's worst element;
 *           L is cut back to ef entries
 *   result: the first k elements of L, padded with (id -1, score -inf).
 *
 * Entry nodes: `entries` == NULL means every query starts from the one node `entry`
 * (E is ignored); otherwise query b starts from entries[b*E .. b*E + E), E >= 1 (a coarse
 * index in front of the graph, such as HNSW's upper layers named in Section 2.1, hands the
 * search one or several starting points; the paper does not say how many).
 * A node is marked visited when it is first scored, not when it is expanded.
 * A node whose score is NaN is scored, counted and marked visited like any other but never
 * enters L (no order relation holds for it).
 * n_dist[b] / n_expand[b] (optional) count scored nodes and expansions.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
typedef struct {
    scored_t *L;
    uint8_t *expanded;
    int32_t len, ef;
} list_t;

/* Put (s, v) into the ordered list unless it is NaN, or the list is full and (s, v) does not
 * precede its last element.  Returns 1 if it went in. */
static int list_offer(list_t *l, double s, int32_t v)
{
    if (s != s) return 0;
    if (l->len == l->ef && !precedes(s, v, l->L[l->len - 1].s, l->L[l->len - 1].id)) return 0;
    int32_t pos = l->len;               /* insertion point that keeps L in order */
    while (pos > 0 && precedes(s, v, l->L[pos - 1].s, l->L[pos - 1].id)) --pos;
    for (int32_t i = l->len; i > pos; --i) { l->L[i] = l->L[i - 1]; l->expanded[i] = l->expanded[i - 1]; }
    l->L[pos].s = s; l->L[pos].id = v; l->expanded[pos] = 0;
    if (l->len < l->ef) ++l->len;       /* otherwise the old worst fell off the end */
    return 1;
}

int oracle_graph_search(const void *corpus, int64_t N, int32_t d, int dtype,
                        const int32_t *graph, int32_t R, int32_t entry,
                        const int32_t *entries, int32_t E,
                        const void *queries, int32_t B, int32_t k, int32_t ef,
                        int32_t *ids, float *scores, double *scores64,
                        int64_t *n_dist, int64_t *n_expand, int threads)
{
    if (!corpus || !graph || !queries || !ids || !scores || N < 1 || d < 1 || R < 1 ||
        B < 1 || k < 1 || ef < k)
        return -1;
    if (entries ? E < 1 : (entry < 0 || entry >= N)) return -1;
    prepare_tables();
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(use_threads(threads))
    for (int32_t b = 0; b < B; ++b) {
        double *q = malloc(sizeof(double) * (size_t)d);
        uint8_t *visited = calloc((size_t)N, 1);
        list_t l = { malloc(sizeof(scored_t) * (size_t)(ef + 1)), malloc((size_t)(ef + 1)), 0, ef };
        if (!q || !visited || !l.L || !l.expanded) {
            failed = 1; free(q); free(visited); free(l.L); free(l.expanded); continue;
        }
        for (int32_t j = 0; j < d; ++j) q[j] = load_value(queries, (int64_t)b * d + j, dtype);

        int64_t dist_count = 0, expand_count = 0;
        const int32_t n_entries = entries ? E : 1;
        for (int32_t e = 0; e < n_entries; ++e) {
            const int32_t v = entries ? entries[(int64_t)b * E + e] : entry;
            if (v < 0 || v >= N || visited[v]) continue;
            visited[v] = 1;
            ++dist_count;
            list_offer(&l, score_row(corpus, v, d, dtype, q), v);
        }

        for (;;) {
            int32_t p = 0;
            while (p < l.len && l.expanded[p]) ++p;
            if (p == l.len) break;
            l.expanded[p] = 1;
            ++expand_count;
            int32_t node = l.L[p].id;     /* copy: L may shift below */
            for (int32_t slot = 0; slot < R; ++slot) {
                int32_t v = graph[(int64_t)node * R + slot];
                if (v < 0 || v >= N || visited[v]) continue;
                visited[v] = 1;
                ++dist_count;
                list_offer(&l, score_row(corpus, v, d, dtype, q), v);
            }
        }
        for (int32_t i = 0; i < k; ++i) {
            int has = i < l.len;
            ids[(int64_t)b * k + i] = has ? l.L[i].id : -1;
            scores[(int64_t)b * k + i] = has ? (float)l.L[i].s : -INFINITY;
            if (scores64) scores64[(int64_t)b * k + i] = has ? l.L[i].s : -INFINITY;
        }
        if (n_dist) n_dist[b] = dist_count;
        if (n_expand) n_expand[b] = expand_count;
        free(q); free(visited); free(l.L); free(l.expanded);
    }
    return failed ? -1 : 0;
}

/*
 * Graph retrieval with the non-stall (maturity) exit of Section 3.3 / Appendix B.2.
 *
 * The search is the one above.  In addition every node t scored during an expansion yields
 *     RQ_t = (d_t - d_best) / (d_worst - d_best),     d = -score (a distance),
 * where d_best / d_worst belong to the best and worst entries of the candidate list.
 * RQ is smoothed by an exponential moving average with window W ("window size of
 * 500"; read as alpha = 2 / (W + 1), EMA_0 = 0, EMA <- EMA + alpha (RQ - EMA)), and the
 * search stops as soon as EMA > tau (0.9 in the paper) AND the engine is ready; otherwise it
 * stops naturally.  A node whose RQ is undefined (fewer than two list entries, or
 * best == worst, or a NaN score) gives no sample; the entry nodes give none either (they are
 * handed to the search, not discovered by it); the exit test is made after each expansion.
 *
 * Section 3.3 takes best and worst from the list as it stands "currently", i.e. when node t
 * is scored.  Two forms of that are stated here, selected by `form`:
 *
 *   ORACLE_RQ_PER_NODE (0): the wording taken literally for a search that scores one node
 *     after the other: best / worst are those of the list at the moment t is scored, after
 *     the earlier neighbours of the same expansion have gone in.  All in binary64.
 *   ORACLE_RQ_PER_EXPANSION (1): the neighbours of one expansion are discovered together (one
 *     step of the search); "currently" is then the list as that step starts, the same for all
 *     of them, and the samples enter the average in slot order.  This is the form a search
 *     that scores all neighbours of a node at once can compute, and the one the GPU library
 *     is compared with.  Because the average decides an integer (the expansion at which the
 *     search leaves), this form takes the decision in the precision of the implementation
 *     under test, binary32: the score is rounded to binary32, RQ is one binary32 division,
 *     the update one fused multiply-add.
 *
 * The two forms differ only inside an expansion that changes the list's best or worst entry
 * while it is still being scored; tests/test_oracle_pins.py pins each by a hand trace and
 * measures how often they leave at different expansions.
 *
 * `ready_from` models the engine: it is ready from expansion count `ready_from` on
 * (0 = always, a huge value = never).  `max_expand` > 0 additionally stops the search
 * after that many expansions (used to check that an early exit returns exactly the
 * state the full search had at that point).
 * stats[b] = {early exit (0/1), scored nodes, expansions}.
 */
enum { ORACLE_RQ_PER_NODE = 0, ORACLE_RQ_PER_EXPANSION = 1 };

int oracle_graph_search_nonstall(const void *corpus, int64_t N, int32_t d, int dtype,
                                 const int32_t *graph, int32_t R, int32_t entry,
                                 const int32_t *entries, int32_t E,
                                 const void *queries, int32_t B, int32_t k, int32_t ef,
                                 float tau, int32_t window, int form, int64_t ready_from, int64_t max_expand,
                                 int32_t *ids, float *scores, double *scores64,
                                 int32_t *stats, float *ema_out, int threads)
{
    if (!corpus || !graph || !queries || !ids || !scores || N < 1 || d < 1 || R < 1 ||
        B < 1 || k < 1 || ef < k || window < 1)
        return -1;
    if (entries ? E < 1 : (entry < 0 || entry >= N)) return -1;
    if (form != ORACLE_RQ_PER_NODE && form != ORACLE_RQ_PER_EXPANSION) return -1;
    prepare_tables();
    const float alpha32 = 2.0f / ((float)window + 1.0f);
    const double alpha64 = 2.0 / ((double)window + 1.0);
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(use_threads(threads))
    for (int32_t b = 0; b < B; ++b) {
        double *q = malloc(sizeof(double) * (size_t)d);
        uint8_t *visited = calloc((size_t)N, 1);
        list_t l = { malloc(sizeof(scored_t) * (size_t)(ef + 1)), malloc((size_t)(ef + 1)), 0, ef };
        if (!q || !visited || !l.L || !l.expanded) {
            failed = 1; free(q); free(visited); free(l.L); free(l.expanded); continue;
        }
        for (int32_t j = 0; j < d; ++j) q[j] = load_value(queries, (int64_t)b * d + j, dtype);

        int32_t early = 0;
        int64_t dist_count = 0, expand_count = 0;
        float ema32 = 0.0f;             /* per-expansion form */
        double ema64 = 0.0;             /* per-node form */
        const int32_t n_entries = entries ? E : 1;
        for (int32_t e = 0; e < n_entries; ++e) {
            const int32_t v = entries ? entries[(int64_t)b * E + e] : entry;
            if (v < 0 || v >= N || visited[v]) continue;
            visited[v] = 1;
            ++dist_count;
            list_offer(&l, score_row(corpus, v, d, dtype, q), v);
        }

        for (;;) {
            int32_t p = 0;
            while (p < l.len && l.expanded[p]) ++p;
            if (p == l.len) break;
            if (max_expand > 0 && expand_count >= max_expand) break;
            l.expanded[p] = 1;
            ++expand_count;
            int32_t node = l.L[p].id;
            /* per-expansion form: best and worst of the list as this expansion starts */
            const int start_range = l.len >= 2;
            const float start_best = (float)l.L[0].s, start_worst = (float)l.L[l.len - 1].s;
            for (int32_t slot = 0; slot < R; ++slot) {
                int32_t v = graph[(int64_t)node * R + slot];
                if (v < 0 || v >= N || visited[v]) continue;
                visited[v] = 1;
                ++dist_count;
                double s = score_row(corpus, v, d, dtype, q);
                if (s == s) {
                    if (form == ORACLE_RQ_PER_EXPANSION) {
                        if (start_range && start_best != start_worst) {
                            /* (d_t - d_best) / (d_worst - d_best) with d = -score */
                            const float rq = (start_best - (float)s) / (start_best - start_worst);
                            ema32 = fmaf(alpha32, rq - ema32, ema32);
                        }
                    } else {
                        const double d_t = -s, d_best = -l.L[0].s, d_worst = -l.L[l.len - 1].s;
                        if (l.len >= 2 && d_worst != d_best) {
                            const double rq = (d_t - d_best) / (d_worst - d_best);
                            ema64 = ema64 + alpha64 * (rq - ema64);
                        }
                    }
                }
                list_offer(&l, s, v);
            }
            const int mature = form == ORACLE_RQ_PER_EXPANSION ? ema32 > tau : ema64 > (double)tau;
            if (mature && expand_count >= ready_from) { early = 1; break; }
        }
        for (int32_t i = 0; i < k; ++i) {
            int has = i < l.len;
            ids[(int64_t)b * k + i] = has ? l.L[i].id : -1;
            scores[(int64_t)b * k + i] = has ? (float)l.L[i].s : -INFINITY;
            if (scores64) scores64[(int64_t)b * k + i] = has ? l.L[i].s : -INFINITY;
        }
        if (stats) {
            stats[(int64_t)b * 3 + 0] = early;
            stats[(int64_t)b * 3 + 1] = (int32_t)dist_count;
            stats[(int64_t)b * 3 + 2] = (int32_t)expand_count;
        }
        if (ema_out) ema_out[b] = form == ORACLE_RQ_PER_EXPANSION ? ema32 : (float)ema64;
        free(q); free(visited); free(l.L); free(l.expanded);
    }
    return failed ? -1 : 0;
}

/*
 * Priority levels and execution order of the scheduler (Section 3.2, Eq. 1-2).
 *
 * Metrics of request i: R_i retrievals completed, W_i waiting time of the initial request,
 * C_i context length.  For each metric M and level j in [0, G): T_{M,j} = min(M) + j/G (max(M) - min(M)).
 * level_i = the largest j with R_i > T_{R,j} or W_i > T_{W,j} or C_i > T_{C,j}; 0 if there is none.
 * Execution order: levels from the highest down; inside a level by the current queueing time
 * Wcur_i, longest first (readings: equal times in index order; a time that is NaN counts as the
 * shortest possible wait, -inf, so that every request has exactly one place).
 * Arithmetic in binary64, the threshold exactly as Eq. 1-2 write it: min + (j/G) * (max - min),
 * every operation rounded once (this file is compiled without floating-point contraction).
 */
int oracle_priority_order(const int32_t *R, const double *W, const int32_t *C, const double *Wcur,
                          int32_t n, int32_t G, int32_t *level, int32_t *order)
{
    if (!R || !W || !C || !Wcur || !level || !order || n < 1 || G < 1) return -1;
    double mn[3], mx[3];
    for (int m = 0; m < 3; ++m) { mn[m] = INFINITY; mx[m] = -INFINITY; }
    for (int32_t i = 0; i < n; ++i) {
        const double v[3] = {(double)R[i], W[i], (double)C[i]};
        for (int m = 0; m < 3; ++m) { if (v[m] < mn[m]) mn[m] = v[m]; if (v[m] > mx[m]) mx[m] = v[m]; }
    }
    for (int32_t i = 0; i < n; ++i) {
        const double v[3] = {(double)R[i], W[i], (double)C[i]};
        int32_t best = 0;
        for (int32_t j = 0; j < G; ++j)
            for (int m = 0; m < 3; ++m)
                if (v[m] > mn[m] + ((double)j / (double)G) * (mx[m] - mn[m])) best = j;
        level[i] = best;
    }
    /* stable selection: position of i = number of requests that go before it */
    for (int32_t i = 0; i < n; ++i) {
        int32_t before = 0;
        const double wi = Wcur[i] == Wcur[i] ? Wcur[i] : -INFINITY;
        for (int32_t j = 0; j < n; ++j) {
            if (j == i) continue;
            const double wj = Wcur[j] == Wcur[j] ? Wcur[j] : -INFINITY;
            if (level[j] > level[i] || (level[j] == level[i] && (wj > wi || (wj == wi && j < i))))
                ++before;
        }
        order[before] = i;
    }
    return 0;
}
