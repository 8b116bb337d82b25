// libann.so — host side of the C ABI declared in include/ann.h: argument checks,
// launch geometry, the per-device workspace and the corpus registry.  All compute
// runs in the kernels reached through launch.hpp.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/ann.h"
#include "launch.hpp"

using namespace ann;

namespace {

thread_local std::string g_last_error;

int fail(int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

constexpr int P_MAX = 2048;

}  // namespace

// Workspace of ann_flat_search_static: lives in the code object, so every device the library
// runs on holds one copy until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address is looked up once per device (device_state) and is
// what every launch and every offset computation uses.
static __device__ __align__(256) unsigned char scratch[ANN_STATIC_WORKSPACE_BYTES];

namespace {

struct DeviceState {
    int cus = 0;
    void *ws = nullptr;
    size_t ws_bytes = 0;
    void *vis = nullptr;          // visited bitsets of the non-stall graph search
    size_t vis_bytes = 0;
    void *scratch_ptr = nullptr;  // this device's address of `scratch`
    void *user_ws = nullptr;      // caller-owned workspace (ann_set_workspace), used instead of ws and vis
    size_t user_bytes = 0;
};

std::mutex g_mu;
std::unordered_map<int, DeviceState> g_dev;
struct CorpusInfo { int64_t N; int32_t d; int32_t dtype; };
std::unordered_map<const void *, CorpusInfo> g_corpora;
int g_default_dtype = ANN_F16;

int device_state(DeviceState **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(ANN_ERR_LAUNCH, "no HIP device is current");
    DeviceState &st = g_dev[dev];
    if (st.cus == 0) {
        if (hipDeviceGetAttribute(&st.cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || st.cus <= 0)
            return fail(ANN_ERR_LAUNCH, "cannot query the compute-unit count of device %d", dev);
    }
    if (!st.scratch_ptr) {                       // device `dev` is current here
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(ANN_ERR_LAUNCH, "cannot resolve the static workspace on device %d: %s", dev, hipGetErrorString(e));
        }
        st.scratch_ptr = p;
    }
    *out = &st;
    return ANN_OK;
}

int grow(void **buf, size_t *have, size_t bytes) {
    if (*have >= bytes) return ANN_OK;
    if (*buf) (void)hipFree(*buf);               // synchronises the device: no kernel still uses it
    *buf = nullptr;
    *have = 0;
    size_t want = bytes + bytes / 4;
    if (hipMalloc(buf, want) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ANN_ERR_NOMEM, "cannot allocate %zu bytes of device workspace", want);
    }
    *have = want;
    return ANN_OK;
}

// The device buffer a call may use as workspace: the caller's when one was set (never grown: a call
// that needs more fails), else the library's own, grown on demand.
int workspace_for(DeviceState *st, void **own, size_t *own_bytes, size_t bytes, void **out) {
    if (st->user_ws) {
        if (bytes > st->user_bytes)
            return fail(ANN_ERR_NOMEM, "this call needs %zu bytes of workspace, the buffer given to ann_set_workspace has %zu",
                        bytes, st->user_bytes);
        *out = st->user_ws;
        return ANN_OK;
    }
    if (int rc = grow(own, own_bytes, bytes)) return rc;
    *out = *own;
    return ANN_OK;
}

// words of one query's visited bitset: one bit per node, rounded to 16-byte units
int64_t visited_words(int64_t N) { return (N + 511) / 512 * 16; }

// ---- optional event timing of the main kernels -----------------------------------------------
struct TimedLaunch { hipEvent_t a, b; int kernel; };
bool g_timing = false;
bool g_timing_off = false;                 // set while an entry point that may not create events runs
std::vector<TimedLaunch> g_timed;          // records of the current session
std::vector<hipEvent_t> g_event_pool;      // events of earlier sessions, reused

hipEvent_t pooled_event() {
    if (!g_event_pool.empty()) {
        hipEvent_t e = g_event_pool.back();
        g_event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return e;
}

// Brackets a launch with events while timing is on (caller holds g_mu).
struct TimedScope {
    hipStream_t stream;
    int index = -1;
    TimedScope(int kernel, hipStream_t s) : stream(s) {     // kernel < 0: not recorded
        if (!g_timing || g_timing_off || kernel < 0) return;
        TimedLaunch t{pooled_event(), pooled_event(), kernel};
        if (!t.a || !t.b) return;
        if (hipEventRecord(t.a, stream) != hipSuccess) { (void)hipGetLastError(); return; }
        g_timed.push_back(t);
        index = (int)g_timed.size() - 1;
    }
    ~TimedScope() {
        if (index >= 0 && hipEventRecord(g_timed[index].b, stream) != hipSuccess) (void)hipGetLastError();
    }
};

int check_launch(const char *what, hipError_t e) {
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ANN_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
    }
    return ANN_OK;
}

int elem_bytes(int dtype) { return dtype == ANN_F32 ? 4 : 2; }

int check_common(const void *corpus, int64_t N, int32_t d, int32_t dtype, const void *queries, int32_t B,
                 int32_t k, const void *ids, const void *scores) {
    if (dtype != ANN_F16 && dtype != ANN_BF16 && dtype != ANN_F32)
        return fail(ANN_ERR_INVALID, "unknown element type %d", dtype);
    if (!corpus || !queries || !ids || !scores) return fail(ANN_ERR_INVALID, "null pointer argument");
    if (N < 1 || N > INT32_MAX) return fail(ANN_ERR_INVALID, "N = %lld out of range", (long long)N);
    if (B < 1) return fail(ANN_ERR_INVALID, "B = %d out of range", B);
    if (d < 1 || d > ANN_D_MAX) return fail(ANN_ERR_INVALID, "d = %d out of range [1, %d]", d, ANN_D_MAX);
    if (k < 1 || k > N) return fail(ANN_ERR_INVALID, "k = %d out of range [1, N]", k);
    if ((d * elem_bytes(dtype)) % 16 != 0)
        return fail(ANN_ERR_ALIGNMENT, "d = %d: a row must be a whole number of 16-byte chunks", d);
    if ((reinterpret_cast<uintptr_t>(corpus) | reinterpret_cast<uintptr_t>(queries)) & 15)
        return fail(ANN_ERR_ALIGNMENT, "corpus and queries must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(ids) | reinterpret_cast<uintptr_t>(scores)) & 3)
        return fail(ANN_ERR_ALIGNMENT, "ids and scores must be 4-byte aligned");
    return ANN_OK;
}

int kp_of(int k) { return k <= 4 ? 4 : 16; }

// ---- flat: launch geometry ---------------------------------------------------------------
struct FlatPlan {
    int kp, P, nqg_max;
    int wide_ntg;            // > 0: matrix-core path with this many query-tile groups
    int pstride;             // slabs per query in the partial array
    size_t sample_ofs, thr_ofs;   // byte offsets of the sample lists and thresholds in the workspace
    // k > 4 on the matrix-core path: candidate arrays instead of lists, streaming kernel as repair
    bool emit;
    int emit_cap;                 // entries of a query's candidate array
    int sample_P;                 // > 0: a sampling pass with this many slabs supplies thresholds
    int sample_skip;              // > 0: the sample is the first sample_skip tiles, which the main pass skips
    int st_P, st_nqg_max;         // geometry of the repair pass (streaming kernel, lists of 16)
    size_t cnt_ofs, cand_ofs;
    size_t ws_bytes;
};

constexpr int WIDE_MIN_B = 65;   // smallest batch sent to the matrix-core path
constexpr int EMIT_CAP = 4096;   // candidate-array entries per query (k > 4), a multiple of 16
constexpr int SAMPLE_STRIDE = 64; // a sampling pass scores every 64th row
constexpr int64_t SAMPLE_MIN_N = 64 * 1024;
constexpr int64_t EMIT_MIN_N = 128 * 1024;   // smallest corpus with candidate arrays when the batch streams

FlatPlan flat_plan(int cus, int64_t N, int d, int dtype, int B, int k, bool allow_emit = true) {
    FlatPlan pl;
    pl.kp = kp_of(k);
    pl.wide_ntg = 0;
    pl.emit = false;
    pl.emit_cap = 0;
    pl.sample_P = 0;
    pl.sample_skip = 0;
    // k > 4 on a large 16-bit corpus: lists of 16 per lane are slow to maintain (and do not fit the
    // matrix-core kernel's registers), so the main pass keeps no lists; it appends every score that
    // reaches a lower bound of the query's k-th best to a per-query candidate array.  The bound is
    // the k-th best of every 64th row (scored exactly by a short first pass), so about 64 k rows per
    // query pass it; an array that overflows all the same (heavily tied scores) is repaired by the
    // streaming kernel with lists of 16, which does no work otherwise.
    // A batch large enough for the matrix-core kernel, which keeps no lists of 16, takes this path at
    // any corpus size (a sample of fewer than k rows gives a bound of -inf: every row is a candidate);
    // a small batch streams, and lists of 16 are fine until the corpus is large.
    const bool wide_batch = B >= WIDE_MIN_B && d % 32 == 0;
    if (allow_emit && dtype != ANN_F32 && pl.kp == 16 && (wide_batch || N >= EMIT_MIN_N)) {
        const FlatPlan st = flat_plan(cus, N, d, dtype, B, k, false);     // repair pass
        const FlatPlan m4 = flat_plan(cus, N, d, dtype, B, 4, false);     // geometry of sampling and main pass
        pl.emit = true;
        pl.emit_cap = EMIT_CAP;
        pl.wide_ntg = m4.wide_ntg;
        pl.P = m4.P;
        pl.nqg_max = m4.nqg_max;
        pl.st_P = st.P;
        pl.st_nqg_max = st.nqg_max;
        pl.pstride = st.P;
        const int64_t nv = (N + SAMPLE_STRIDE - 1) / SAMPLE_STRIDE;
        if (pl.wide_ntg > 0) {
            const int64_t stiles = (nv + 255) / 256;
            pl.sample_P = (int)(stiles < pl.P ? stiles : pl.P);
        } else {
            const int64_t swaves = (nv + 15) / 16;                         // one 16-row tile per wave at least
            const int64_t sblocks = (swaves + 7) / 8;
            pl.sample_P = (int)(sblocks < pl.P ? sblocks : pl.P);
        }
        const size_t a16 = 15;
        pl.sample_ofs = ((size_t)B * st.P * pl.kp * sizeof(Cand) + a16) & ~a16;
        pl.thr_ofs = pl.sample_ofs + (size_t)B * pl.sample_P * 4 * sizeof(Cand);   // lists of 4 per sample slab
        pl.cnt_ofs = (pl.thr_ofs + (size_t)B * sizeof(float) + a16) & ~a16;
        pl.cand_ofs = (pl.cnt_ofs + (size_t)B * sizeof(int) + a16) & ~a16;
        pl.ws_bytes = pl.cand_ofs + (size_t)B * EMIT_CAP * sizeof(Cand);
        return pl;
    }
    if (dtype != ANN_F32 && B >= WIDE_MIN_B && pl.kp == 4 && d % 32 == 0) {
        const int nt = (B + wide_query_tile(B) - 1) / wide_query_tile(B);
        pl.wide_ntg = nt < 8 ? nt : 8;
        int P = cus / pl.wide_ntg;
        if (wide_query_tile(B) == 128) P *= 2;       // 4-wave workgroups, two per compute unit
        const int64_t mtiles = (N + 255) / 256;
        if (P > mtiles) P = (int)mtiles;
        pl.P = P < 1 ? 1 : P;
        pl.nqg_max = 4;
        // a corpus of some size: score a sample first, exactly, and start the main pass from the k-th
        // best scores of that sample (few rows then pass the threshold test at all).  Many tiles per
        // slab: the sample is the first tile of every slab-to-be, kept as one more slab and skipped by
        // the main pass; otherwise every 64th row, which the main pass scores again.
        if (mtiles >= 8 * (int64_t)pl.P) {
            pl.sample_P = pl.sample_skip = pl.P;
        } else if (N >= SAMPLE_MIN_N) {
            const int64_t stiles = ((N + SAMPLE_STRIDE - 1) / SAMPLE_STRIDE + 255) / 256;
            pl.sample_P = (int)(stiles < pl.P ? stiles : pl.P);
        }
    } else if (dtype == ANN_F32) {
        const int64_t groups = (N + 7) / 8;
        int64_t P = (groups + 3) / 4;
        const int64_t cap = (int64_t)cus * 4;
        pl.P = (int)(P < cap ? P : cap);
        pl.nqg_max = 0;
    } else {
        const int steps = (d + 31) / 32;
        int nqg_max = (int)((LDS_MAX - 16 * 1024) / ((size_t)steps * WAVE * 16));
        pl.nqg_max = nqg_max > 4 ? 4 : nqg_max;
        const int nqg = B > 16 * pl.nqg_max ? pl.nqg_max : (B + 15) / 16;
        const int wpb = stream_waves(nqg, steps, pl.kp);
        const size_t lds = stream_lds_bytes(nqg, steps, wpb, pl.kp);
        int occ = (int)(LDS_MAX / lds);
        occ = occ < 1 ? 1 : (occ > 2 ? 2 : occ);     // measured: more resident workgroups do not help
        const int64_t tiles = (N + 15) / 16;
        const int64_t cap = (int64_t)cus * occ;
        // every wave takes whole 16-row tiles in rounds; size the grid so that the last round
        // is as full as the others instead of leaving most of the chip idle
        const int64_t rounds = (tiles + cap * wpb - 1) / (cap * wpb);
        int64_t P = (tiles + rounds * wpb - 1) / (rounds * wpb);
        pl.P = (int)(P < cap ? P : cap);
    }
    if (pl.P > P_MAX) pl.P = P_MAX;
    if (pl.P < 1) pl.P = 1;
    pl.pstride = pl.P + (pl.sample_skip > 0 ? 1 : 0);
    pl.sample_ofs = (size_t)B * pl.pstride * pl.kp * sizeof(Cand);
    pl.thr_ofs = pl.sample_ofs + (size_t)B * pl.sample_P * 4 * sizeof(Cand);
    pl.ws_bytes = pl.thr_ofs + (pl.sample_P > 0 ? (size_t)B * sizeof(float) : 0);
    return pl;
}

// 16-bit corpus, streaming kernel over all B queries in one launch: groups of 16 nqg_max queries are
// served one after the other inside the kernel (kp 0: candidate-array mode)
int flat_stream_all(int kp, int nqg_max, int P, const void *X, int64_t N, int d, int dtype, const void *Q, int B,
                    Cand *partial, StreamOpts o, After after, bool timed_launch, hipStream_t stream) {
    o.after = after;
    const int group = 16 * nqg_max;
    const int nqg = B > group ? nqg_max : (B + 15) / 16;
    o.passes = B > group ? (B + group - 1) / group : 1;
    hipError_t e;
    {
        TimedScope timed(timed_launch ? ANN_KERNEL_FLAT_STREAM : -1, stream);
        e = dtype == ANN_F16 ? launch_flat_stream_f16(nqg, kp, X, N, d, Q, B, 0, partial, P, o, stream)
                             : launch_flat_stream_bf16(nqg, kp, X, N, d, Q, B, 0, partial, P, o, stream);
    }
    return check_launch("flat_stream_kernel", e);
}

int flat_search_emit(const FlatPlan &pl, const void *X, int64_t N, int d, int dtype, const void *Q, int B, int k,
                     int32_t *ids, float *scores, char *ws, After after, hipStream_t stream) {
    Cand *partial = reinterpret_cast<Cand *>(ws);
    Cand *sample = reinterpret_cast<Cand *>(ws + pl.sample_ofs);
    float *thr = reinterpret_cast<float *>(ws + pl.thr_ofs);
    int *cnt = reinterpret_cast<int *>(ws + pl.cnt_ofs);
    Cand *cand = reinterpret_cast<Cand *>(ws + pl.cand_ofs);
    // sampling pass: every 64th row, the best 4 per slab and query
    if (pl.wide_ntg > 0) {
        hipError_t e = launch_flat_wide(dtype, 1, X, N, d, Q, B, sample, pl.sample_P, pl.wide_ntg, 0, nullptr, pl.sample_P,
                                        0, nullptr, SAMPLE_STRIDE, after, stream);
        if (int rc = check_launch("flat_wide_kernel (sample)", e)) return rc;
    } else {
        StreamOpts o;
        o.row_stride = SAMPLE_STRIDE;
        if (int rc = flat_stream_all(4, pl.nqg_max, pl.sample_P, X, N, d, dtype, Q, B, sample, o, after, false, stream)) return rc;
    }
    if (int rc = check_launch("flat_sample_kth_kernel", launch_flat_sample_kth(sample, pl.sample_P, B, k, thr, nullptr, 0, 0, cnt, stream)))
        return rc;
    // main pass: candidates
    if (pl.wide_ntg > 0) {
        hipError_t e;
        {
            TimedScope timed(ANN_KERNEL_FLAT_WIDE, stream);
            e = launch_flat_wide(dtype, 2, X, N, d, Q, B, cand, pl.P, pl.wide_ntg, 0, thr, pl.emit_cap, 0, cnt, 1, after, stream);
        }
        if (int rc = check_launch("flat_wide_kernel (candidates)", e)) return rc;
    } else {
        StreamOpts o;
        o.thr = thr;
        o.count = cnt;
        o.cap = pl.emit_cap;
        if (int rc = flat_stream_all(0, pl.nqg_max, pl.P, X, N, d, dtype, Q, B, cand, o, after, true, stream)) return rc;
    }
    // repair pass: returns at once unless a candidate array overflowed
    StreamOpts o;
    o.need = cnt;
    o.need_above = pl.emit_cap;
    if (int rc = flat_stream_all(pl.kp, pl.st_nqg_max, pl.st_P, X, N, d, dtype, Q, B, partial, o, after, false, stream)) return rc;
    return check_launch("flat_merge_kernel",
                        launch_flat_merge(pl.kp, partial, pl.st_P, B, k, ids, scores, cnt, cand, pl.emit_cap, stream));
}

int flat_search_run(const FlatPlan &pl, const void *X, int64_t N, int d, int dtype, const void *Q, int B, int k,
                    int32_t *ids, float *scores, Cand *partial, After after, hipStream_t stream) {
    if (pl.emit) return flat_search_emit(pl, X, N, d, dtype, Q, B, k, ids, scores, reinterpret_cast<char *>(partial), after, stream);
    if (dtype == ANN_F32) {
        hipError_t e;
        {
            TimedScope timed(ANN_KERNEL_FLAT_F32, stream);
            e = launch_flat_f32(pl.kp, static_cast<const float *>(X), N, d, static_cast<const float *>(Q), B, partial,
                                pl.P, after, stream);
        }
        if (int rc = check_launch("flat_f32_kernel", e)) return rc;
    } else if (pl.wide_ntg > 0) {
        const float *thr0 = nullptr;
        if (pl.sample_P > 0) {
            Cand *sample = reinterpret_cast<Cand *>(reinterpret_cast<char *>(partial) + pl.sample_ofs);
            float *thr = reinterpret_cast<float *>(reinterpret_cast<char *>(partial) + pl.thr_ofs);
            const bool skip = pl.sample_skip > 0;
            hipError_t e = launch_flat_wide(dtype, 1, X, skip ? (int64_t)pl.sample_skip * 256 : N, d, Q, B, sample, pl.sample_P,
                                            pl.wide_ntg, 0, nullptr, pl.sample_P, 0, nullptr, skip ? 1 : SAMPLE_STRIDE, after, stream);
            if (int rc = check_launch("flat_wide_kernel (sample)", e)) return rc;
            e = launch_flat_sample_kth(sample, pl.sample_P, B, k, thr, skip ? partial : nullptr, pl.pstride, pl.P, nullptr,
                                       stream);
            if (int rc = check_launch("flat_sample_kth_kernel", e)) return rc;
            thr0 = thr;
        }
        hipError_t e;
        {
            TimedScope timed(ANN_KERNEL_FLAT_WIDE, stream);
            e = launch_flat_wide(dtype, 0, X, N, d, Q, B, partial, pl.P, pl.wide_ntg, pl.sample_skip, thr0, pl.pstride, 0,
                                 nullptr, 1, after, stream);
        }
        if (int rc = check_launch("flat_wide_kernel", e)) return rc;
    } else {
        if (int rc = flat_stream_all(pl.kp, pl.nqg_max, pl.P, X, N, d, dtype, Q, B, partial, StreamOpts(), after, true, stream)) return rc;
    }
    return check_launch("flat_merge_kernel", launch_flat_merge(pl.kp, partial, pl.pstride, B, k, ids, scores, nullptr, nullptr, 0, stream));
}

}  // namespace

extern "C" {

int ann_version(void) { return 100; }

const char *ann_last_error(void) { return g_last_error.c_str(); }

int ann_set_default_dtype(int32_t dtype) {
    if (dtype != ANN_F16 && dtype != ANN_BF16 && dtype != ANN_F32)
        return fail(ANN_ERR_INVALID, "unknown element type %d", dtype);
    std::lock_guard<std::mutex> lock(g_mu);
    g_default_dtype = dtype;
    return ANN_OK;
}

int ann_register_corpus(const void *corpus, int64_t N, int32_t d, int32_t dtype) {
    if (!corpus || N < 1 || N > INT32_MAX || d < 1 || d > ANN_D_MAX ||
        (dtype != ANN_F16 && dtype != ANN_BF16 && dtype != ANN_F32))
        return fail(ANN_ERR_INVALID, "ann_register_corpus: bad shape or element type");
    std::lock_guard<std::mutex> lock(g_mu);
    g_corpora[corpus] = CorpusInfo{N, d, dtype};
    return ANN_OK;
}

int ann_unregister_corpus(const void *corpus) {
    std::lock_guard<std::mutex> lock(g_mu);
    g_corpora.erase(corpus);
    return ANN_OK;
}

int64_t ann_flat_workspace_bytes(int64_t N, int32_t d, int32_t dtype, int32_t B, int32_t k) {
    if (N < 1 || N > INT32_MAX || d < 1 || d > ANN_D_MAX || B < 1 || k < 1 || k > ANN_K_MAX || k > N) return ANN_ERR_INVALID;
    if (dtype != ANN_F16 && dtype != ANN_BF16 && dtype != ANN_F32) return ANN_ERR_INVALID;
    if ((d * elem_bytes(dtype)) % 16 != 0) return ANN_ERR_ALIGNMENT;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *st = nullptr;
    int cus = 256;
    if (device_state(&st) == ANN_OK) cus = st->cus;
    return (int64_t)flat_plan(cus, N, d, dtype, B, k).ws_bytes;
}

int ann_timing_enable(int32_t on) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (on) {
        for (const TimedLaunch &t : g_timed) {
            g_event_pool.push_back(t.a);
            g_event_pool.push_back(t.b);
        }
        g_timed.clear();
    }
    g_timing = on != 0;
    return ANN_OK;
}

int ann_timing_read(int32_t kernel, int32_t *launches, double *total_ms) {
    if (!launches || !total_ms) return fail(ANN_ERR_INVALID, "null pointer argument");
    if (kernel < 0 || kernel >= ANN_KERNEL_COUNT) return fail(ANN_ERR_INVALID, "unknown kernel code %d", kernel);
    std::lock_guard<std::mutex> lock(g_mu);
    int n = 0;
    double sum = 0.0;
    for (const TimedLaunch &t : g_timed) {
        if (t.kernel != kernel) continue;
        float ms = 0.f;
        if (hipEventSynchronize(t.b) != hipSuccess || hipEventElapsedTime(&ms, t.a, t.b) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ANN_ERR_LAUNCH, "cannot read the events of a timed launch");
        }
        ++n;
        sum += ms;
    }
    *launches = n;
    *total_ms = sum;
    return ANN_OK;
}

int ann_timing_read_each(int32_t kernel, int32_t capacity, int32_t *launches, float *ms) {
    if (!launches || (capacity > 0 && !ms) || capacity < 0) return fail(ANN_ERR_INVALID, "bad arguments");
    if (kernel < 0 || kernel >= ANN_KERNEL_COUNT) return fail(ANN_ERR_INVALID, "unknown kernel code %d", kernel);
    std::lock_guard<std::mutex> lock(g_mu);
    int n = 0;
    for (const TimedLaunch &t : g_timed) {
        if (t.kernel != kernel) continue;
        float one = 0.f;
        if (hipEventSynchronize(t.b) != hipSuccess || hipEventElapsedTime(&one, t.a, t.b) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ANN_ERR_LAUNCH, "cannot read the events of a timed launch");
        }
        if (n < capacity) ms[n] = one;
        ++n;
    }
    *launches = n;
    return ANN_OK;
}

int ann_priority_order(const int32_t *R, const double *W, const int32_t *C, const double *Wcur, int32_t n, int32_t G,
                       int32_t *level, int32_t *order, void *stream) {
    if (n == 0) return ANN_OK;
    if (!R || !W || !C || !Wcur || !level || !order) return fail(ANN_ERR_INVALID, "null pointer argument");
    if (n < 1 || n > ANN_REQUESTS_MAX) return fail(ANN_ERR_INVALID, "n = %d out of range [1, %d]", n, ANN_REQUESTS_MAX);
    if (G < 1 || G > 1024) return fail(ANN_ERR_INVALID, "G = %d out of range [1, 1024]", G);
    if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(Wcur)) & 7)
        return fail(ANN_ERR_ALIGNMENT, "W and Wcur must be 8-byte aligned");
    if ((reinterpret_cast<uintptr_t>(R) | reinterpret_cast<uintptr_t>(C) | reinterpret_cast<uintptr_t>(level) |
         reinterpret_cast<uintptr_t>(order)) & 3)
        return fail(ANN_ERR_ALIGNMENT, "R, C, level and order must be 4-byte aligned");
    return check_launch("priority kernels",
                        launch_priority(R, W, C, Wcur, n, G, level, order, static_cast<hipStream_t>(stream)));
}

int ann_measure_mfma_rate(int32_t random_operands, int32_t iters, double *tflops) {
    if (!tflops || iters < 1) return fail(ANN_ERR_INVALID, "ann_measure_mfma_rate: bad arguments");
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *st = nullptr;
    if (int rc = device_state(&st)) return rc;
    if (int rc = grow(&st->ws, &st->ws_bytes, 256)) return rc;
    hipEvent_t a = pooled_event(), b = pooled_event();
    if (!a || !b) return fail(ANN_ERR_LAUNCH, "cannot create events");
    float ms = 0.f;
    hipError_t e = launch_mfma_rate(random_operands != 0, st->cus, iters, static_cast<float *>(st->ws), nullptr);   // warm-up
    if (e == hipSuccess) e = hipEventRecord(a, nullptr);
    if (e == hipSuccess) e = launch_mfma_rate(random_operands != 0, st->cus, iters, static_cast<float *>(st->ws), nullptr);
    if (e == hipSuccess) e = hipEventRecord(b, nullptr);
    if (e == hipSuccess) e = hipEventSynchronize(b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
    g_event_pool.push_back(a);
    g_event_pool.push_back(b);
    if (int rc = check_launch("mfma_rate_kernel", e)) return rc;
    *tflops = (double)st->cus * 8.0 * iters * 8.0 * 32768.0 / ((double)ms * 1e9);
    return ANN_OK;
}

int ann_set_workspace(void *workspace, int64_t bytes) {
    if (workspace && bytes < 1) return fail(ANN_ERR_INVALID, "ann_set_workspace: bytes = %lld", (long long)bytes);
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(ANN_ERR_ALIGNMENT, "the workspace must be 256-byte aligned");
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *st = nullptr;
    if (int rc = device_state(&st)) return rc;
    st->user_ws = workspace;
    st->user_bytes = workspace ? (size_t)bytes : 0;
    return ANN_OK;
}

int ann_release_workspace(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *st = nullptr;
    if (int rc = device_state(&st)) return rc;
    if (st->ws) (void)hipFree(st->ws);
    st->ws = nullptr;
    st->ws_bytes = 0;
    if (st->vis) (void)hipFree(st->vis);
    st->vis = nullptr;
    st->vis_bytes = 0;
    return ANN_OK;
}

int ann_flat_search_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype, const void *queries,
                          int32_t B, int32_t k, int32_t *ids, float *scores, void *stream) {
    return ann_flat_search_after_typed(corpus, N, d, dtype, queries, B, k, nullptr, nullptr, ids, scores, stream);
}

int ann_flat_search_after_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype, const void *queries,
                                int32_t B, int32_t k, const float *after_scores, const int32_t *after_ids,
                                int32_t *ids, float *scores, void *stream) {
    if (B == 0) return ANN_OK;                            // an empty batch: nothing to do
    if (int rc = check_common(corpus, N, d, dtype, queries, B, k, ids, scores)) return rc;
    if (k > ANN_K_MAX) return fail(ANN_ERR_INVALID, "k = %d exceeds ANN_K_MAX = %d", k, ANN_K_MAX);
    if ((after_scores == nullptr) != (after_ids == nullptr))
        return fail(ANN_ERR_INVALID, "after_scores and after_ids must be given together");
    if ((reinterpret_cast<uintptr_t>(after_scores) | reinterpret_cast<uintptr_t>(after_ids)) & 3)
        return fail(ANN_ERR_ALIGNMENT, "after_scores and after_ids must be 4-byte aligned");
    After after;
    after.s = after_scores;
    after.id = after_ids;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *st = nullptr;
    if (int rc = device_state(&st)) return rc;
    const FlatPlan pl = flat_plan(st->cus, N, d, dtype, B, k);
    if (dtype != ANN_F32 && pl.nqg_max < 1) return fail(ANN_ERR_INVALID, "d = %d too large for LDS", d);
    void *ws = nullptr;
    if (int rc = workspace_for(st, &st->ws, &st->ws_bytes, pl.ws_bytes, &ws)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return flat_search_run(pl, corpus, N, d, dtype, queries, B, k, ids, scores, static_cast<Cand *>(ws), after, s);
}

int ann_flat_search(const void *corpus, int64_t N, int32_t d, const void *queries, int32_t B, int32_t k,
                    int32_t *ids, float *scores, void *stream) {
    int dtype;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        dtype = g_default_dtype;
    }
    return ann_flat_search_typed(corpus, N, d, dtype, queries, B, k, ids, scores, stream);
}

int ann_flat_search_static(const void *corpus, int64_t N, int32_t d, int32_t dtype, const void *queries,
                           int32_t B, int32_t k, int32_t *ids, float *scores, void *stream) {
    if (B == 0) return ANN_OK;
    if (int rc = check_common(corpus, N, d, dtype, queries, B, k, ids, scores)) return rc;
    if (k > ANN_K_MAX) return fail(ANN_ERR_INVALID, "k = %d exceeds ANN_K_MAX = %d", k, ANN_K_MAX);
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *st = nullptr;
    if (int rc = device_state(&st)) return rc;
    const FlatPlan pl = flat_plan(st->cus, N, d, dtype, B, k);
    if (dtype != ANN_F32 && pl.nqg_max < 1) return fail(ANN_ERR_INVALID, "d = %d too large for LDS", d);
    if (pl.ws_bytes > (size_t)ANN_STATIC_WORKSPACE_BYTES)
        return fail(ANN_ERR_INVALID, "this search needs %zu bytes of workspace, the static one holds %d",
                    pl.ws_bytes, ANN_STATIC_WORKSPACE_BYTES);
    g_timing_off = true;                                  // event pairs would have to be created
    const int rc = flat_search_run(pl, corpus, N, d, dtype, queries, B, k, ids, scores,
                                   static_cast<Cand *>(st->scratch_ptr), After(), static_cast<hipStream_t>(stream));
    g_timing_off = false;
    return rc;
}

static int check_graph(const void *corpus, int64_t N, int32_t d, int32_t dtype, const int32_t *graph, int32_t R,
                       int32_t entry, const void *queries, int32_t B, int32_t k, int32_t ef, const int32_t *ids,
                       const float *scores, GraphLds *L) {
    if (!graph) return fail(ANN_ERR_INVALID, "null graph pointer");
    if (R < 1 || R > ANN_R_MAX) return fail(ANN_ERR_INVALID, "R = %d out of range [1, %d]", R, ANN_R_MAX);
    if (ef < 1 || ef > ANN_EF_MAX) return fail(ANN_ERR_INVALID, "ef = %d out of range [1, %d]", ef, ANN_EF_MAX);
    if (int rc = check_common(corpus, N, d, dtype, queries, B, k, ids, scores)) return rc;
    if (k > ef) return fail(ANN_ERR_INVALID, "ef = %d is smaller than k = %d", ef, k);
    if (entry < 0 || entry >= N) return fail(ANN_ERR_INVALID, "entry = %d is not a node id", entry);
    if (reinterpret_cast<uintptr_t>(graph) & 3) return fail(ANN_ERR_ALIGNMENT, "graph must be 4-byte aligned");
    *L = graph_lds_layout(d, elem_bytes(dtype), R, ef);
    if (L->total > LDS_MAX) return fail(ANN_ERR_INVALID, "d = %d, ef = %d need %u bytes of LDS", d, ef, L->total);
    return ANN_OK;
}

int64_t ann_graph_nonstall_workspace_bytes(int64_t N, int32_t B) {
    if (N < 1 || N > INT32_MAX || B < 1) return ANN_ERR_INVALID;
    return (int64_t)B * visited_words(N) * 4;
}

int ann_graph_search_nonstall_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype, const int32_t *graph,
                                    int32_t R, int32_t entry, const void *queries, int32_t B, int32_t k, int32_t ef,
                                    const int32_t *entries, int32_t n_entries, float tau, int32_t window,
                                    const int32_t *engine_ready, int32_t *ids, float *scores, int32_t *stats,
                                    float *ema, void *stream) {
    if (B == 0) return ANN_OK;                            // an empty batch: nothing to do
    GraphLds L;
    if (int rc = check_graph(corpus, N, d, dtype, graph, R, entries ? 0 : entry, queries, B, k, ef, ids, scores, &L))
        return rc;
    if (reinterpret_cast<uintptr_t>(entries) & 3) return fail(ANN_ERR_ALIGNMENT, "entries must be 4-byte aligned");
    if (entries && (n_entries < 1 || n_entries > ANN_ENTRIES_MAX))
        return fail(ANN_ERR_INVALID, "n_entries = %d out of range [1, %d]", n_entries, ANN_ENTRIES_MAX);
    if (window < 1) return fail(ANN_ERR_INVALID, "window = %d must be at least 1", window);
    if (tau != tau) return fail(ANN_ERR_INVALID, "tau is not a number");
    if ((reinterpret_cast<uintptr_t>(engine_ready) | reinterpret_cast<uintptr_t>(stats) |
         reinterpret_cast<uintptr_t>(ema)) & 3)
        return fail(ANN_ERR_ALIGNMENT, "engine_ready, stats and ema must be 4-byte aligned");
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState *st = nullptr;
    if (int rc = device_state(&st)) return rc;
    NonStall ns;
    ns.entries = entries;
    ns.n_entries = n_entries;
    ns.tau = tau;
    ns.alpha = 2.0f / ((float)window + 1.0f);
    ns.ready = engine_ready;
    ns.words = visited_words(N);
    ns.stats = stats;
    ns.ema = ema;
    void *vis = nullptr;
    if (int rc = workspace_for(st, &st->vis, &st->vis_bytes, (size_t)B * (size_t)ns.words * 4, &vis)) return rc;
    ns.visited = static_cast<uint32_t *>(vis);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (int rc = check_launch("zero_words_kernel", launch_zero_words(ns.visited, (size_t)B * (size_t)ns.words, s)))
        return rc;
    TimedScope timed(ANN_KERNEL_GRAPH, s);
    return check_launch("graph_search_kernel (non-stall)",
                        launch_graph_search_nonstall(dtype, corpus, N, d, graph, R, entry, queries, B, k, ef, ids,
                                                     scores, L, ns, s));
}

// Plain search.  Long lists (the two-level list, or more than GRAPH_EF_DOUBLE entries) score far
// more nodes than an id cache in LDS remembers, so they run on the kernel variant with the exact
// visited bitset, with an exit threshold no average can exceed.
static int graph_search_any(const void *corpus, int64_t N, int32_t d, int32_t dtype, const int32_t *graph, int32_t R,
                            int32_t entry, const int32_t *entries, int32_t n_entries, const void *queries, int32_t B, int32_t k,
                            int32_t ef, int32_t *ids, float *scores, const GraphLds &L, hipStream_t s) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (ef <= GRAPH_EF_DOUBLE && !L.two_level) {
        TimedScope timed(ANN_KERNEL_GRAPH, s);
        return check_launch("graph_search_kernel", launch_graph_search(dtype, corpus, N, d, graph, R, entry, entries, n_entries,
                                                                       queries, B, k, ef, ids, scores, L, s));
    }
    DeviceState *st = nullptr;
    if (int rc = device_state(&st)) return rc;
    NonStall ns{};
    ns.entries = entries;
    ns.n_entries = n_entries;
    ns.tau = INFINITY;
    ns.alpha = 0.f;
    ns.words = visited_words(N);
    void *vis = nullptr;
    if (int rc = workspace_for(st, &st->vis, &st->vis_bytes, (size_t)B * (size_t)ns.words * 4, &vis)) return rc;
    ns.visited = static_cast<uint32_t *>(vis);
    if (int rc = check_launch("zero_words_kernel", launch_zero_words(ns.visited, (size_t)B * (size_t)ns.words, s)))
        return rc;
    TimedScope timed(ANN_KERNEL_GRAPH, s);
    return check_launch("graph_search_kernel (long list)",
                        launch_graph_search_nonstall(dtype, corpus, N, d, graph, R, entry, queries, B, k, ef, ids,
                                                     scores, L, ns, s));
}

int ann_graph_search_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype, const int32_t *graph,
                           int32_t R, int32_t entry, const void *queries, int32_t B, int32_t k, int32_t ef,
                           int32_t *ids, float *scores, void *stream) {
    if (B == 0) return ANN_OK;                            // an empty batch: nothing to do
    GraphLds L;
    if (int rc = check_graph(corpus, N, d, dtype, graph, R, entry, queries, B, k, ef, ids, scores, &L)) return rc;
    return graph_search_any(corpus, N, d, dtype, graph, R, entry, nullptr, 0, queries, B, k, ef, ids, scores, L,
                            static_cast<hipStream_t>(stream));
}

int ann_graph_search_multi_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype, const int32_t *graph,
                                 int32_t R, const int32_t *entries, int32_t n_entries, const void *queries, int32_t B,
                                 int32_t k, int32_t ef, int32_t *ids, float *scores, void *stream) {
    if (B == 0) return ANN_OK;                            // an empty batch: nothing to do
    if (!entries) return fail(ANN_ERR_INVALID, "null entries pointer");
    if (reinterpret_cast<uintptr_t>(entries) & 3) return fail(ANN_ERR_ALIGNMENT, "entries must be 4-byte aligned");
    if (n_entries < 1 || n_entries > ANN_ENTRIES_MAX)
        return fail(ANN_ERR_INVALID, "n_entries = %d out of range [1, %d]", n_entries, ANN_ENTRIES_MAX);
    GraphLds L;
    if (int rc = check_graph(corpus, N, d, dtype, graph, R, 0, queries, B, k, ef, ids, scores, &L)) return rc;
    return graph_search_any(corpus, N, d, dtype, graph, R, 0, entries, n_entries, queries, B, k, ef, ids, scores, L,
                            static_cast<hipStream_t>(stream));
}

int ann_graph_search_entries_typed(const void *corpus, int64_t N, int32_t d, int32_t dtype, const int32_t *graph,
                                   int32_t R, const int32_t *entries, const void *queries, int32_t B, int32_t k,
                                   int32_t ef, int32_t *ids, float *scores, void *stream) {
    return ann_graph_search_multi_typed(corpus, N, d, dtype, graph, R, entries, 1, queries, B, k, ef, ids, scores, stream);
}

int ann_gather_ids(const int32_t *table, int64_t M, const int32_t *idx, int64_t n, int32_t *out, void *stream) {
    if (n == 0) return ANN_OK;
    if (!table || !idx || !out) return fail(ANN_ERR_INVALID, "null pointer argument");
    if (M < 1 || n < 1) return fail(ANN_ERR_INVALID, "M = %lld, n = %lld out of range", (long long)M, (long long)n);
    if ((reinterpret_cast<uintptr_t>(table) | reinterpret_cast<uintptr_t>(idx) | reinterpret_cast<uintptr_t>(out)) & 3)
        return fail(ANN_ERR_ALIGNMENT, "table, idx and out must be 4-byte aligned");
    return check_launch("gather_ids_kernel",
                        launch_gather_ids(table, M, idx, n, out, static_cast<hipStream_t>(stream)));
}

int ann_graph_search(const void *corpus, const int32_t *graph, int32_t R, int32_t entry, const void *queries,
                     int32_t B, int32_t k, int32_t ef, int32_t *ids, float *scores, void *stream) {
    CorpusInfo info;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        auto it = g_corpora.find(corpus);
        if (it == g_corpora.end())
            return fail(ANN_ERR_UNKNOWN_CORPUS, "corpus %p was never passed to ann_register_corpus", corpus);
        info = it->second;
    }
    return ann_graph_search_typed(corpus, info.N, info.d, info.dtype, graph, R, entry, queries, B, k, ef, ids,
                                  scores, stream);
}

}  // extern "C"
