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
 * Fewer than k rows cannot happen (k <= N is required).  Returns 0, or -1 on
 * bad arguments / allocation failure.
 */
int oracle_flat_search(const void *corpus, int64_t N, int32_t d, int dtype,
                       const void *queries, int32_t B, int32_t k,
                       int32_t *ids, float *scores, double *scores64, int threads)
{
    if (!corpus || !queries || !ids || !scores || N < 1 || d < 1 || B < 1 || k < 1 || k > N)
        return -1;
    prepare_tables();
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(use_threads(threads))
    for (int32_t b = 0; b < B; ++b) {
        double *q = malloc(sizeof(double) * (size_t)d);
        scored_t *all = malloc(sizeof(scored_t) * (size_t)N);
        if (!q || !all) { failed = 1; free(q); free(all); continue; }
        for (int32_t j = 0; j < d; ++j) q[j] = load_value(queries, (int64_t)b * d + j, dtype);
        for (int64_t n = 0; n < N; ++n) {
            all[n].s = score_row(corpus, n, d, dtype, q);
            all[n].id = (int32_t)n;
        }
        qsort(all, (size_t)N, sizeof(scored_t), by_order);
        for (int32_t i = 0; i < k; ++i) {
            ids[(int64_t)b * k + i] = all[i].id;
            scores[(int64_t)b * k + i] = (float)all[i].s;
            if (scores64) scores64[(int64_t)b * k + i] = all[i].s;
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
 *   visited = {entry};  L = [(score(entry), entry, unexpanded)]
 *   repeat: p = first unexpanded element of L (L is kept in order, so this is
 *           the best unexpanded candidate, ties to the lower id); stop if none
 *           mark p expanded
 *           for each slot of graph[p] in slot order: skip empty (-1),
 *           out-of-range and visited ids; otherwise mark visited, score it, and
 *           put it into L if L is not full or it precedes L's worst element;
 *           L is cut back to ef entries
 *   result: the first k elements of L, padded with (id -1, score -inf).
 *
 * A node is marked visited when it is first scored, not when it is expanded.
 * n_dist[b] / n_expand[b] (optional) count scored nodes and expansions.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_graph_search(const void *corpus, int64_t N, int32_t d, int dtype,
                        const int32_t *graph, int32_t R, int32_t entry,
                        const void *queries, int32_t B, int32_t k, int32_t ef,
                        int32_t *ids, float *scores, double *scores64,
                        int64_t *n_dist, int64_t *n_expand, int threads)
{
    if (!corpus || !graph || !queries || !ids || !scores || N < 1 || d < 1 || R < 1 ||
        B < 1 || k < 1 || ef < k || entry < 0 || entry >= N)
        return -1;
    prepare_tables();
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(use_threads(threads))
    for (int32_t b = 0; b < B; ++b) {
        double *q = malloc(sizeof(double) * (size_t)d);
        uint8_t *visited = calloc((size_t)N, 1);
        scored_t *L = malloc(sizeof(scored_t) * (size_t)(ef + 1));
        uint8_t *expanded = malloc((size_t)(ef + 1));
        if (!q || !visited || !L || !expanded) {
            failed = 1; free(q); free(visited); free(L); free(expanded); continue;
        }
        for (int32_t j = 0; j < d; ++j) q[j] = load_value(queries, (int64_t)b * d + j, dtype);

        int32_t len = 1;
        int64_t dist_count = 1, expand_count = 0;
        visited[entry] = 1;
        L[0].s = score_row(corpus, entry, d, dtype, q);
        L[0].id = entry;
        expanded[0] = 0;

        for (;;) {
            int32_t p = 0;
            while (p < len && expanded[p]) ++p;
            if (p == len) break;
            expanded[p] = 1;
            ++expand_count;
            int32_t node = L[p].id;     /* copy: L may shift below */
            for (int32_t slot = 0; slot < R; ++slot) {
                int32_t v = graph[(int64_t)node * R + slot];
                if (v < 0 || v >= N || visited[v]) continue;
                visited[v] = 1;
                ++dist_count;
                double s = score_row(corpus, v, d, dtype, q);
                if (len == ef && !precedes(s, v, L[len - 1].s, L[len - 1].id)) continue;
                int32_t pos = len;      /* insertion point that keeps L in order */
                while (pos > 0 && precedes(s, v, L[pos - 1].s, L[pos - 1].id)) --pos;
                for (int32_t i = len; i > pos; --i) { L[i] = L[i - 1]; expanded[i] = expanded[i - 1]; }
                L[pos].s = s; L[pos].id = v; expanded[pos] = 0;
                if (len < ef) ++len;    /* otherwise the old worst fell off the end */
            }
        }
        for (int32_t i = 0; i < k; ++i) {
            int has = i < len;
            ids[(int64_t)b * k + i] = has ? L[i].id : -1;
            scores[(int64_t)b * k + i] = has ? (float)L[i].s : -INFINITY;
            if (scores64) scores64[(int64_t)b * k + i] = has ? L[i].s : -INFINITY;
        }
        if (n_dist) n_dist[b] = dist_count;
        if (n_expand) n_expand[b] = expand_count;
        free(q); free(visited); free(L); free(expanded);
    }
    return failed ? -1 : 0;
}

/*
 * Graph retrieval with the non-stall (maturity) exit of Section 3.3 / Appendix B.2.
 *
 * The search is the one above.  In addition every newly scored node t yields
 *     RQ_t = (d_t - d_best) / (d_worst - d_best),     d = -score (a distance),
 * where d_best / d_worst belong to the best and worst entries of the candidate list.
 * RQ is smoothed by an exponential moving average with window W ("window size of
 * 500"; read as alpha = 2 / (W + 1), EMA_0 = 0), and the search stops as soon as
 * EMA > tau (0.9 in the paper) AND the engine is ready; otherwise it stops naturally.
 *
 * Readings: the neighbours of one expansion are handled as a batch, so best and worst
 * are those of the list as it stood when the expansion started; neighbours enter the
 * average in slot order; a node whose RQ is undefined (fewer than two list entries, or
 * best == worst) is skipped; the exit test is made after each expansion.
 * `ready_from` models the engine: it is ready from expansion count `ready_from` on
 * (0 = always, a huge value = never).  `max_expand` > 0 additionally stops the search
 * after that many expansions (used to check that an early exit returns exactly the
 * state the full search had at that point).
 *
 * Decision precision: RQ and the EMA are computed in binary32 with one fused
 * multiply-add per update, the same operations the GPU kernel uses, from the score
 * rounded to binary32.  stats[b] = {early exit (0/1), scored nodes, expansions}.
 */
int oracle_graph_search_nonstall(const void *corpus, int64_t N, int32_t d, int dtype,
                                 const int32_t *graph, int32_t R, int32_t entry,
                                 const void *queries, int32_t B, int32_t k, int32_t ef,
                                 float tau, int32_t window, int64_t ready_from, int64_t max_expand,
                                 int32_t *ids, float *scores, double *scores64,
                                 int32_t *stats, float *ema_out, int threads)
{
    if (!corpus || !graph || !queries || !ids || !scores || N < 1 || d < 1 || R < 1 ||
        B < 1 || k < 1 || ef < k || entry < 0 || entry >= N || window < 1)
        return -1;
    prepare_tables();
    const float alpha = 2.0f / ((float)window + 1.0f);
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(use_threads(threads))
    for (int32_t b = 0; b < B; ++b) {
        double *q = malloc(sizeof(double) * (size_t)d);
        uint8_t *visited = calloc((size_t)N, 1);
        scored_t *L = malloc(sizeof(scored_t) * (size_t)(ef + 1));
        uint8_t *expanded = malloc((size_t)(ef + 1));
        if (!q || !visited || !L || !expanded) {
            failed = 1; free(q); free(visited); free(L); free(expanded); continue;
        }
        for (int32_t j = 0; j < d; ++j) q[j] = load_value(queries, (int64_t)b * d + j, dtype);

        int32_t len = 1, early = 0;
        int64_t dist_count = 1, expand_count = 0;
        float ema = 0.0f;
        visited[entry] = 1;
        L[0].s = score_row(corpus, entry, d, dtype, q);
        L[0].id = entry;
        expanded[0] = 0;

        for (;;) {
            int32_t p = 0;
            while (p < len && expanded[p]) ++p;
            if (p == len) break;
            if (max_expand > 0 && expand_count >= max_expand) break;
            expanded[p] = 1;
            ++expand_count;
            int32_t node = L[p].id;
            /* best and worst of the list as this expansion starts */
            const int have_range = len >= 2;
            const float s_best = (float)L[0].s, s_worst = (float)L[len - 1].s;
            for (int32_t slot = 0; slot < R; ++slot) {
                int32_t v = graph[(int64_t)node * R + slot];
                if (v < 0 || v >= N || visited[v]) continue;
                visited[v] = 1;
                ++dist_count;
                double s = score_row(corpus, v, d, dtype, q);
                if (have_range && s_best != s_worst) {
                    /* (d_t - d_best) / (d_worst - d_best) with d = -score */
                    const float rq = (s_best - (float)s) / (s_best - s_worst);
                    ema = fmaf(alpha, rq - ema, ema);
                }
                if (len == ef && !precedes(s, v, L[len - 1].s, L[len - 1].id)) continue;
                int32_t pos = len;
                while (pos > 0 && precedes(s, v, L[pos - 1].s, L[pos - 1].id)) --pos;
                for (int32_t i = len; i > pos; --i) { L[i] = L[i - 1]; expanded[i] = expanded[i - 1]; }
                L[pos].s = s; L[pos].id = v; expanded[pos] = 0;
                if (len < ef) ++len;
            }
            if (ema > tau && expand_count >= ready_from) { early = 1; break; }
        }
        for (int32_t i = 0; i < k; ++i) {
            int has = i < len;
            ids[(int64_t)b * k + i] = has ? L[i].id : -1;
            scores[(int64_t)b * k + i] = has ? (float)L[i].s : -INFINITY;
            if (scores64) scores64[(int64_t)b * k + i] = has ? L[i].s : -INFINITY;
        }
        if (stats) {
            stats[(int64_t)b * 3 + 0] = early;
            stats[(int64_t)b * 3 + 1] = (int32_t)dist_count;
            stats[(int64_t)b * 3 + 2] = (int32_t)expand_count;
        }
        if (ema_out) ema_out[b] = ema;
        free(q); free(visited); free(L); free(expanded);
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
 * Wcur_i, longest first (reading: equal times in index order).
 * Arithmetic in binary64, the threshold as one fused multiply-add fma(j/G, max - min, min): the
 * GPU routine uses the same expression, so the integer decisions are taken in the same precision.
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
                if (v[m] > fma((double)j / (double)G, mx[m] - mn[m], mn[m])) best = j;
        level[i] = best;
    }
    /* stable selection: position of i = number of requests that go before it */
    for (int32_t i = 0; i < n; ++i) {
        int32_t before = 0;
        for (int32_t j = 0; j < n; ++j) {
            if (j == i) continue;
            if (level[j] > level[i] || (level[j] == level[i] && (Wcur[j] > Wcur[i] || (Wcur[j] == Wcur[i] && j < i))))
                ++before;
        }
        order[before] = i;
    }
    return 0;
}
