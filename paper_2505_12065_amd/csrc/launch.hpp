// Host-side launchers of the kernels; one translation unit per kernel family so the
// library builds in parallel.  Each returns the HIP status of its launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace ann {

constexpr size_t LDS_MAX = 160 * 1024;   // LDS of one gfx950 compute unit
constexpr int STREAM_THREADS = 512;
// Wavefronts of a flat_stream_kernel workgroup: 8, or 16 when the queries' LDS leaves room for one
// workgroup per compute unit only (the corpus loads in flight are what keeps HBM busy); lists
// of 16 need too many registers for that.
int stream_waves(int nqg, int steps, int kp);

// A kernel that needs more than 64 KB of dynamic LDS has to be told so; `granted` holds
// the largest size already granted to that kernel.
inline hipError_t allow_big_lds(const void *kernel, size_t bytes, size_t *granted) {
    if (bytes <= 64 * 1024 || bytes <= *granted) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) *granted = bytes;
    return e;
}

size_t stream_lds_bytes(int nqg, int steps, int waves, int kp);
size_t f32_lds_bytes(int d, int waves, int kp);

// Optional behaviour of a flat_stream_kernel launch.
struct StreamOpts {
    const int *need = nullptr;   // [B]: a group of queries is skipped unless need[q] > need_above for
    int need_above = 0;          //      one of them (repair pass behind the candidate arrays)
    int passes = 1;              // consecutive groups of nqg * 16 queries served by the launch, from q0 on
    int row_stride = 1;          // S > 1: only rows 0, S, 2S, ... are scored (sampling pass)
    After after;                 // continuation: per-query boundary pairs, or null pointers
    const float *thr = nullptr;  // candidate-array mode: [B] lower bounds of the final k-th best score,
    int *count = nullptr;        //   [B] entry counters (zero on entry; a count past cap means overflow),
    int cap = 0;                 //   entries per query in the candidate array that `partial` then is
};
// nqg in 1..4 query groups of 16 starting at query q0.  kp 4 or 16: lists, partial[B, P, kp].
// kp 0: candidate-array mode, every (score, row) with score >= o.thr[q] is appended to
// partial[q o.cap ..) through o.count[q].
hipError_t launch_flat_stream_f16(int nqg, int kp, const void *X, int64_t N, int d, const void *Q, int B, int q0,
                                  Cand *partial, int P, const StreamOpts &o, hipStream_t stream);
hipError_t launch_flat_stream_bf16(int nqg, int kp, const void *X, int64_t N, int d, const void *Q, int B, int q0,
                                   Cand *partial, int P, const StreamOpts &o, hipStream_t stream);
// Large batches on the matrix cores (16-bit corpora, d % 32 == 0, lists of 4).
// Query tile is wide_query_tile(B) queries; gridDim = P slabs x NTG query-tile groups;
// rows [256 tile_begin, N) are scanned; results go to partial[(q pstride + pslot0 + slab) 4 ..).
// mode 0: list epilogue, thr_init = optional per-query lower bounds of the final k-th best score;
// mode 1: threshold-free selection epilogue (sampling pass), rows 0, row_stride, 2 row_stride, ... only;
// mode 2 (k > 4): every score >= thr_init[q] is appended to the candidate array
// partial[q pstride ..) through emit_count[q] (zero on entry; counts past pstride mean overflow).
int wide_query_tile(int B);
hipError_t launch_flat_wide(int dtype, int mode, const void *X, int64_t N, int d, const void *Q, int B,
                            Cand *partial, int P, int NTG, int64_t tile_begin, const float *thr_init, int pstride,
                            int pslot0, int *emit_count, int row_stride, After after, hipStream_t stream);
// thr[q] = k-th best score among the Ps sampled lists of 4 of query q (-inf if fewer), k <= 16;
// with dst, the 4 best of the sample also become slab pslot of dst[B, pstride, 4]; with count, count[q] = 0
hipError_t launch_flat_sample_kth(const Cand *src, int Ps, int B, int k, float *thr, Cand *dst, int pstride, int pslot,
                                  int *count, hipStream_t stream);
hipError_t launch_flat_f32(int kp, const float *X, int64_t N, int d, const float *Q, int B, Cand *partial, int P,
                           After after, hipStream_t stream);
// count == null: merge the P lists of every query.  count given: query q's input is its candidate
// array cand[q cap ..) of count[q] entries, or, when that overflowed, its P lists (repair pass).
hipError_t launch_flat_merge(int kp, const Cand *partial, int P, int B, int k, int32_t *ids, float *scores,
                             const int *count, const Cand *cand, int cap, hipStream_t stream);

constexpr int GRAPH_DENSE_MIN_B = 1280;   // batches beyond this run three graph-search workgroups per compute unit
constexpr int GRAPH_EF_DOUBLE = 2048;    // candidate lists up to this length are double-buffered in LDS
constexpr int GRAPH_EF_TWO_LEVEL = 512;  // beyond this, graphs of at most 32 slots per node use the two-level list
// cus workgroups of 8 waves, each wave iters x 8 MFMA 32x32x16 fp16 (32768 flop each) on register operands
hipError_t launch_mfma_rate(bool random_operands, int cus, int iters, float *sink, hipStream_t stream);

struct GraphLds {
    // byte offsets into dynamic LDS; all 16-byte aligned
    uint32_t q, ls0, ls1, li0, li1, cs, ci, cpos, cache, ctl, adj, um, rq, co, total;
    uint32_t cache_bits, rp;
    // two-level list (search ranges beyond GRAPH_EF_TWO_LEVEL on graphs of at most 32 slots per node):
    // ms / mi hold the large part of the list, ls0 .. li1 the small part (GRAPH_DELTA entries each)
    uint32_t two_level, ms, mi;
};
constexpr int GRAPH_DELTA = 256;
// The two-level layout keeps its small regions at fixed byte offsets at the start of LDS (the kernel
// then addresses them with immediates and needs no register per region); the large part of the
// list and the query, whose sizes depend on ef and d, follow.
constexpr uint32_t TL_LS0 = 0, TL_LI0 = 4 * GRAPH_DELTA, TL_LS1 = 8 * GRAPH_DELTA, TL_LI1 = 12 * GRAPH_DELTA;
constexpr uint32_t TL_CS = 16 * GRAPH_DELTA, TL_CI = TL_CS + 128, TL_CPOS = TL_CI + 128, TL_CTL = TL_CPOS + 128;
constexpr uint32_t TL_ADJ = TL_CTL + 32, TL_UM = TL_ADJ + 256;
constexpr uint32_t TL_MS = TL_UM + 8 * (16384 / 64) + 32;   // um: a bit per entry of the longest list, and 4 words
// Maturity exit of the graph search (Section 3.3, Appendix B.2): leave once the moving
// average of RQ exceeds tau and *ready != 0 (ready == nullptr: always ready).
struct NonStall {
    const int32_t *entries;   // [B, n_entries] per-query entry nodes replacing `entry`, or null (both kernel variants)
    int32_t n_entries;        // 1 .. 32 when entries is given
    float tau, alpha;
    const int32_t *ready;     // device-visible word the host may change while the kernel runs
    uint32_t *visited;        // [B][words] bitset, zero on entry
    int64_t words;            // words per query, a multiple of 4
    int32_t *stats;           // [B][3] = (early exit, scored nodes, expansions), may be null
    float *ema;               // [B] final moving average, may be null
};
GraphLds graph_lds_layout(int d, int elem_bytes, int R, int ef);
// dtype: ANN_F16 / ANN_BF16 / ANN_F32 codes 0 / 1 / 2
// entries: null, or device [B, n_entries] per-query entry nodes used instead of `entry`
hipError_t launch_graph_search(int dtype, const void *X, int64_t N, int d, const int32_t *graph, int R, int entry,
                               const int32_t *entries, int n_entries, const void *Q, int B, int k, int ef, int32_t *ids,
                               float *scores, const GraphLds &L, hipStream_t stream);
hipError_t launch_gather_ids(const int32_t *table, int64_t M, const int32_t *idx, int64_t n, int32_t *out,
                             hipStream_t stream);
// p[0 .. words) <- 0; words a multiple of 4, p 16-byte aligned
hipError_t launch_zero_words(uint32_t *p, size_t words, hipStream_t stream);
// Same with the maturity exit; ns.visited (B * ns.words words) must be zero.
hipError_t launch_graph_search_nonstall(int dtype, const void *X, int64_t N, int d, const int32_t *graph, int R,
                                        int entry, const void *Q, int B, int k, int ef, int32_t *ids, float *scores,
                                        const GraphLds &L, const NonStall &ns, hipStream_t stream);

// Scheduler priority levels (Section 3.2, Eq. 1-2) and execution order; all arrays device, length n.
hipError_t launch_priority(const int32_t *R, const double *W, const int32_t *C, const double *Wcur, int n, int G,
                           int32_t *level, int32_t *order, hipStream_t stream);

}  // namespace ann
