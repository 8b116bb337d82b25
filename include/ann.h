/*
 * ann.h — C ABI of the MI355X retrieval library (libann.so).
 *
 * The retrieval step a search agent calls between reasoning steps: batched
 * top-k maximum-inner-product search of query embeddings over a passage
 * embedding corpus, in the two forms the paper contrasts (Section 2.1,
 * "Retrieval Mechanism"; Section 2.2.1; Appendix B.3):
 *
 *   - exact retrieval ("ENN", full recall): every corpus vector is scored;
 *   - approximate graph retrieval ("ANN"): best-first search over a proximity
 *     graph with a candidate list whose size `ef` (the paper's "search range",
 *     efSearch) trades recall against cost (Section 2.2.1), refined until no
 *     unexpanded candidate is left (the natural stop of Section 3.3).
 *
 * Conventions common to every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; nothing is
 *     retained after a call returns except the record made by
 *     ann_register_corpus.  `stream` is a hipStream_t (NULL = default stream).
 *     Work is only enqueued: results are valid once the caller has
 *     synchronised `stream`.  No entry point synchronises the device except
 *     when the library-owned workspace has to grow (first call, or a larger
 *     B*k than any call before on this device).
 *   - One workspace per device: calls that use it (the flat search, the graph
 *     search with ef > 512, the non-stall graph search) are safe one after the
 *     other on one stream, or on several streams if the caller orders them; two
 *     of them running at once on one device race on the workspace.  The plain
 *     graph search with ef <= 512 uses no workspace and may overlap anything.
 *   - corpus  [N, d] row-major, contiguous, 16-byte aligned base.
 *     queries [B, d] row-major, same element type as the corpus.
 *     graph   [N, R] row-major int32; a slot < 0 or >= N is empty and skipped.
 *     ids     [B, k] int32 out; scores [B, k] float out.
 *   - Element types: ANN_F16 (IEEE binary16), ANN_BF16, ANN_F32.  d must be a
 *     multiple of 8 for the 16-bit types and of 4 for ANN_F32.
 *   - score(q, x) = sum_j q_j * x_j, accumulated in fp32 (products of two
 *     16-bit values are exact in fp32).  Larger is better.
 *   - Order: (s, id) precedes (s', id') iff s > s' or (s == s' and id < id').
 *     Row b of ids/scores holds the first k entries in that order.  When fewer
 *     than k entries exist (graph search that reaches fewer than k nodes) the
 *     tail is id = -1, score = -inf.  Same inputs give bitwise-same outputs.
 *   - Scores that are NaN are never returned: such a row never enters a top-k list or a
 *     candidate list (in the graph search it is scored and marked visited like any other,
 *     an entry node included, but is never listed or expanded).
 *   - Return value: ANN_OK, or a negative ANN_ERR_* code, in which case
 *     nothing was enqueued and no output was written.  ann_last_error() gives
 *     a message for the calling thread's last failure.
 */
#ifndef ANN_H
#define ANN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ANN_OK                  0
#define ANN_ERR_INVALID        -1   /* null pointer, size out of range, k > N, ef < k, ... */
#define ANN_ERR_ALIGNMENT      -2   /* d not a multiple of 8 (4 for fp32) or base not 16-B aligned */
#define ANN_ERR_UNKNOWN_CORPUS -3   /* ann_graph_search on a corpus pointer never registered */
#define ANN_ERR_LAUNCH         -4   /* HIP reported an error when a kernel was enqueued */
#define ANN_ERR_NOMEM          -5   /* the device workspace could not be allocated */

#define ANN_F16   0
#define ANN_BF16  1
#define ANN_F32   2

#define ANN_K_MAX    16      /* largest k of the flat search */
#define ANN_EF_MAX   16384   /* largest candidate list of the graph search (k <= ef) */
#define ANN_R_MAX    256     /* largest graph out-degree */
#define ANN_D_MAX    4096    /* largest embedding dimension */
#define ANN_ENTRIES_MAX 32   /* most entry nodes per query of the graph search */
#define ANN_REQUESTS_MAX 65536 /* largest request batch of ann_priority_order */

/* Library version as major*10000 + minor*100 + patch. */
int ann_version(void);

/* Message for the last error returned to the calling thread ("" if none). */
const char *ann_last_error(void);

/*
 * Exact top-k retrieval (Section 2.1: exact nearest neighbour search; the
 * "vLLM_ENN" configuration of Section 4.1 / Appendix B.3).
 *
 *   corpus  device, [N, d] of `dtype`      N >= 1, N < 2^31
 *   queries device, [B, d] of `dtype`      B >= 0 (an empty batch returns ANN_OK at once, here and
 *                                          in every other search entry point)
 *   k       1 <= k <= min(N, ANN_K_MAX)
 *   ids     device, [B, k] int32  (written)
 *   scores  device, [B, k] float  (written)
 *
 * Every corpus row is scored against every query; the score matrix is never
 * materialised.  Uses the library workspace of the current device: per query P
 * lists of 4 or 16 (score, id) pairs (P = number of corpus slabs, at most 2048) and,
 * for k > 4 on corpora of 128 Ki rows or more (at any corpus size when B > 64 and d is
 * a multiple of 32), a candidate array of 4096 pairs;
 * ann_flat_workspace_bytes gives the exact size.
 */
int ann_flat_search_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype,
                          const void *queries, int32_t B, int32_t k,
                          int32_t *ids, float *scores, void *stream);

/* Continuation of an exact retrieval (Section 2.1, exact search; the proximity graph of the
 * approximate retriever is built offline from the same embeddings, Appendix B.3), for callers that
 * need more than ANN_K_MAX rows per query, such as the k-NN rows of that graph: the k best rows
 * among those that come strictly after the pair (after_scores[b], after_ids[b]) in the order, i.e.
 * rows with a smaller score, or the same score and a larger id.  Feeding the last pair of one answer
 * into the next call enumerates the corpus in order, k rows at a time; when fewer than k rows are
 * left the tail is id -1, score -inf.  The boundary score is compared with the fp32 scores the
 * kernels compute, so pass the scores as they were returned, and use the same B, k and element type
 * for every page (each kernel variant sums in its own order; a row within one rounding of the
 * boundary could otherwise be seen on the other side of it).
 *   after_scores, after_ids   device [B] float / int32, both or neither; NULL = ann_flat_search_typed.
 *                             A NaN boundary score excludes nothing for that query. */
int ann_flat_search_after_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype,
                                const void *queries, int32_t B, int32_t k,
                                const float *after_scores, const int32_t *after_ids,
                                int32_t *ids, float *scores, void *stream);

/* Same, for a corpus of the default element type (ANN_F16 unless changed by
 * ann_set_default_dtype). */
int ann_flat_search(const void *corpus, int64_t N, int32_t d,
                    const void *queries, int32_t B, int32_t k,
                    int32_t *ids, float *scores, void *stream);

/* ann_flat_search_typed for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels,
 * same results, but the workspace is a fixed array of ANN_STATIC_WORKSPACE_BYTES that is part of
 * the library's code object (every device the library runs on holds it until the process ends),
 * and the call never allocates, frees or grows anything and records no timing events.
 *   - A search whose workspace (ann_flat_workspace_bytes) exceeds ANN_STATIC_WORKSPACE_BYTES is
 *     rejected with ANN_ERR_INVALID; nothing is enqueued.  8 MiB covers k <= 4 at any of the
 *     batch sizes used here (1 M x 768 fp16, B = 512, k = 3 needs 4.2 MB).
 *   - All calls on one device share that device's array: they are safe one after the other on
 *     one stream (or ordered by the caller across streams); calls that overlap on one device
 *     race.  It does not share anything with the workspace of the other entry points.
 *   - Nothing in the array has to survive between calls; each call writes what it reads. */
#define ANN_STATIC_WORKSPACE_BYTES (8 * 1024 * 1024)
int ann_flat_search_static(const void *corpus, int64_t N, int32_t d, int32_t dtype,
                           const void *queries, int32_t B, int32_t k,
                           int32_t *ids, float *scores, void *stream);

/*
 * Approximate retrieval by best-first search over a proximity graph (Section
 * 2.1: graph-based ANN; Section 3.3: a candidate list with a best and a worst
 * element that is refined iteratively; Appendix B.3: at most 32 neighbours per
 * node, search range efSearch).
 *
 * Per query: visited = {entry}; list L = [(score(entry), entry)].  Repeat:
 * take the first unexpanded element p of L (the best one, ties to the lower
 * id); stop when there is none; mark it expanded; for every slot of graph row
 * p in slot order, skip empty / out-of-range / already scored ids, score the
 * rest and put each into L when L has fewer than ef entries or it precedes
 * L's last element; L keeps its best ef entries.  Output: the first k of L.
 *
 *   corpus  device, [N, d] of `dtype`
 *   graph   device, [N, R] int32, 1 <= R <= ANN_R_MAX
 *   entry   node id in [0, N), by value, shared by all queries
 *   k, ef   1 <= k <= ef <= ANN_EF_MAX
 *
 * One workgroup serves one query; the candidate list lives in LDS.  Up to ef = 512
 * (2048 when R > 32) the visited filter does too and no workspace is used; longer lists
 * score so many nodes that an exact visited bitset in global memory is used instead (the
 * workspace of ann_graph_search_nonstall_typed, same size and rules).  d, R and ef together
 * must fit the 160 KB of LDS (ef = 16384 fits with d <= 1024 at 16 bits), else
 * ANN_ERR_INVALID.
 */
int ann_graph_search_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype,
                           const int32_t *graph, int32_t R, int32_t entry,
                           const void *queries, int32_t B, int32_t k, int32_t ef,
                           int32_t *ids, float *scores, void *stream);

/* Same with (N, d, dtype) looked up from a previous ann_register_corpus(corpus,...).
 * Returns ANN_ERR_UNKNOWN_CORPUS if `corpus` was never registered. */
int ann_graph_search(const void *corpus, const int32_t *graph, int32_t R, int32_t entry,
                     const void *queries, int32_t B, int32_t k, int32_t ef,
                     int32_t *ids, float *scores, void *stream);

/* ann_graph_search_typed with entry nodes of each query's own (Section 2.1: graph-based
 * approximate retrieval; the index the paper uses, HNSW, reaches the layer searched here
 * through coarser ones, i.e. every query starts from nodes chosen for it.  A caller with a
 * coarse index, e.g. an exact search over one representative per cluster by ann_flat_search
 * followed by ann_gather_ids, starts each query next to its answer).
 *
 *   entries    device, [B, n_entries] int32 node ids, 1 <= n_entries <= ANN_ENTRIES_MAX.
 *              The search starts with visited = the entries and the list = the entries in
 *              order, cut to ef.  Ids outside [0, N) and ids named earlier in the row are left
 *              out; a query with no usable entry gets k padding results (id -1, score -inf);
 *              neither is an error.
 */
int ann_graph_search_multi_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype,
                                 const int32_t *graph, int32_t R,
                                 const int32_t *entries, int32_t n_entries,
                                 const void *queries, int32_t B, int32_t k, int32_t ef,
                                 int32_t *ids, float *scores, void *stream);

/* The same with one entry node per query: entries is [B]. */
int ann_graph_search_entries_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype,
                                   const int32_t *graph, int32_t R, const int32_t *entries,
                                   const void *queries, int32_t B, int32_t k, int32_t ef,
                                   int32_t *ids, float *scores, void *stream);

/* out[i] = table[idx[i]] for i in [0, n), or -1 where idx[i] is not in [0, M): turns the
 * row numbers a search over a sub-matrix returns (representatives, a shard) into node ids,
 * e.g. into the `entries` above.  All three arrays device, int32; out may not alias idx
 * or table. */
int ann_gather_ids(const int32_t *table, int64_t M, const int32_t *idx, int64_t n,
                   int32_t *out, void *stream);

/* Approximate retrieval with the maturity (non-stall) exit (Section 3.3 "Non-Stall
 * Retrieval", Appendix B.2 "Retrieval Maturity Estimation").  The search of
 * ann_graph_search_typed, with one addition.  Every newly scored node t yields
 *     RQ_t = (d_t - d_best) / (d_worst - d_best),   d = -score,
 * against the best and worst entries of the candidate list; the values feed an
 * exponential moving average (EMA_0 = 0, alpha = 2 / (window + 1)); a query returns
 * its current list as soon as EMA > tau and the engine-ready word is non-zero, else
 * it stops naturally.  The neighbours of one expansion form a batch: best / worst are
 * those of the list as the expansion starts, samples are taken in slot order, nodes
 * with an undefined RQ (best == worst) are skipped, the test follows the expansion.
 * RQ and the average are binary32.
 *
 *   entries        NULL, or device [B, n_entries] per-query entry nodes used instead of `entry`
 *   n_entries      (as in ann_graph_search_multi_typed; ignored when entries is NULL).  Entry
 *                  nodes are given to the search, not discovered by it: they yield no RQ sample
 *   tau, window    threshold and EMA window (the paper uses 0.9 and 500); window >= 1
 *   engine_ready   device-visible int32 (device memory or pinned host memory) the host
 *                  may change while the call runs; read with system scope each time a
 *                  mature query tests it; NULL = always ready.  Not owned.
 *   stats          device, [B, 3] int32 = (1 if left early, nodes scored, expansions),
 *                  or NULL
 *   ema            device, [B] float, final value of the average, or NULL
 *
 * Uses a per-device workspace of B * 64 * ceil(N / 512) bytes (exact visited sets),
 * grown on demand and cleared by the call; calls on one device must not overlap.
 * Errors as ann_graph_search_typed, plus ANN_ERR_INVALID for window < 1 or a NaN tau
 * and ANN_ERR_NOMEM. */
int ann_graph_search_nonstall_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype,
                                    const int32_t *graph, int32_t R, int32_t entry,
                                    const void *queries, int32_t B, int32_t k, int32_t ef,
                                    const int32_t *entries, int32_t n_entries, float tau, int32_t window,
                                    const int32_t *engine_ready,
                                    int32_t *ids, float *scores, int32_t *stats, float *ema,
                                    void *stream);

/* Bytes of workspace ann_graph_search_nonstall_typed needs for (N, B). */
int64_t ann_graph_nonstall_workspace_bytes(int64_t N, int32_t B);

/* Remember the shape and element type of a corpus so that ann_graph_search can
 * be called with the short argument list.  Re-registering a pointer replaces
 * its record.  The library never dereferences or frees the pointer here. */
int ann_register_corpus(const void *corpus, int64_t N, int32_t d, int32_t dtype);

/* Forget a registered corpus (no error if it is unknown). */
int ann_unregister_corpus(const void *corpus);

/* Element type assumed by ann_flat_search (process-wide; default ANN_F16). */
int ann_set_default_dtype(int32_t dtype);

/* Bytes of device workspace a flat search of this shape needs. */
int64_t ann_flat_workspace_bytes(int64_t N, int32_t d, int32_t dtype, int32_t B, int32_t k);

/* Use a caller-owned device buffer as the workspace of the current device (so that, e.g., the
 * caller's allocator owns the memory and no entry point ever allocates): every call that needs
 * workspace (ann_flat_workspace_bytes, ann_graph_nonstall_workspace_bytes) then runs in it, and one
 * that needs more than `bytes` fails with ANN_ERR_NOMEM instead of growing anything.
 *   workspace  device pointer, 256-byte aligned, valid until it is replaced; NULL: back to the
 *              library-owned buffers.  Not freed by the library.  Calls that use it must not overlap. */
int ann_set_workspace(void *workspace, int64_t bytes);

/* Release the library-owned workspace of the current device (synchronises it). */
int ann_release_workspace(void);

/* Kernel timing for benchmarks (measurement support, no paper passage).  While it is on,
 * every launch of a main kernel is bracketed by a pair of HIP events recorded on the
 * call's own stream, so a benchmark can report a kernel's average duration without a
 * profiler and without synchronising between calls.  The small helper kernels of a call
 * (merges, the sampling pass, clearing) are not bracketed. */
#define ANN_KERNEL_FLAT_STREAM 0   /* flat search, streaming kernel (small batches) */
#define ANN_KERNEL_FLAT_WIDE   1   /* flat search, matrix-core kernel (main pass) */
#define ANN_KERNEL_FLAT_F32    2   /* flat search, fp32 corpus */
#define ANN_KERNEL_GRAPH       3   /* graph search, either variant */
#define ANN_KERNEL_COUNT       4

/* on != 0: drop earlier records and start recording; on == 0: stop (records are kept). */
int ann_timing_enable(int32_t on);

/* Waits for the recorded launches of `kernel` (an ANN_KERNEL_* code) and returns their
 * number and the sum of their durations in milliseconds.  Host pointers. */
int ann_timing_read(int32_t kernel, int32_t *launches, double *total_ms);

/* The same, launch by launch: ms[i] = duration of the i-th recorded launch of `kernel`, in the order
 * of the calls, for i < min(*launches, capacity); *launches = number recorded.  Host pointers. */
int ann_timing_read_each(int32_t kernel, int32_t capacity, int32_t *launches, float *ms);

/* Priority levels and execution order of the request scheduler (Section 3.2 "Priority
 * Scheduling", Eq. 1 and 2).  Metrics of request i: R[i] retrievals completed, W[i] waiting time
 * of the initial request, C[i] context length; for each metric M and level j in [0, G),
 * T_{M,j} = min(M) + j/G (max(M) - min(M)); level[i] = the largest j with R[i] > T_{R,j} or
 * W[i] > T_{W,j} or C[i] > T_{C,j}, 0 if there is none.  order[] lists the requests in execution
 * order: levels from the highest down, inside a level by the current queueing time Wcur[i],
 * longest first (equal times in index order; a NaN time counts as the shortest wait).  Thresholds are
 * evaluated in binary64 exactly as written, every operation rounded once.
 *
 *   R, C, level, order   device int32 [n];   W, Wcur   device double [n]
 *   1 <= n <= ANN_REQUESTS_MAX, 1 <= G <= 1024 (the paper uses G = 6)
 * Not part of the retrieval path; no workspace; errors as elsewhere. */
int ann_priority_order(const int32_t *R, const double *W, const int32_t *C, const double *Wcur,
                       int32_t n, int32_t G, int32_t *level, int32_t *order, void *stream);

/* Measurement support (no paper passage): the dense fp16 MFMA rate the current device sustains
 * on register-resident operands, in TFLOP/s, on the default stream (synchronises it).  With
 * random_operands != 0 the operands are random fp16 values that change from one MFMA to the
 * next, as in a real contraction; with 0 they are one constant.  On parts whose clocks follow
 * the switching activity of the data the two differ widely; the first is the ceiling a kernel
 * working on real data can be held against.  iters: MFMA groups per wave (100000 runs ~30 ms). */
int ann_measure_mfma_rate(int32_t random_operands, int32_t iters, double *tflops);

#ifdef __cplusplus
}
#endif
#endif /* ANN_H */
