// Approximate retrieval: best-first search over a fixed-degree proximity graph with
// a candidate list of at most ef entries (Sections 2.1 and 3.3, Appendix B.3 of the
// paper: graph-based ANN whose "search range" is the candidate-list size; the list
// has a best and a worst element and is refined until nothing is left to expand).
//
// One workgroup (4 wavefronts) serves one query.  In LDS: the query, the candidate
// list (score-ordered, double-buffered), the scored neighbours of the current
// expansion, and a direct-mapped cache of recently scored ids.
//
// Visited filter.  The reference semantics score every node at most once.  Scoring
// a node again can never change the list: it is either still in the list (found
// as a duplicate during the merge) or it was rejected/evicted before, and since
// the list's worst entry only improves it is rejected again.  So a filter that
// never claims an unseen node as seen (no false positives) gives identical
// results whatever it forgets.  The id cache is such a filter; it fits LDS at any
// corpus size, where an exact bitset (N/8 bytes per query) does not.
#pragma once

#include "common.hpp"
#include "launch.hpp"

namespace ann {

constexpr int GRAPH_THREADS = 256;
constexpr int GRAPH_WAVES = GRAPH_THREADS / WAVE;
constexpr int LANES_PER_ROW = 8;
constexpr int ROWS_PER_PASS = GRAPH_THREADS / LANES_PER_ROW;   // 32 neighbours scored at once
constexpr uint32_t EXPANDED = 0x80000000u;

// number of entries of the ordered list (s[0..len), id[0..len)) that precede (v, vid)
__device__ __forceinline__ int list_lower_bound(const float *s, const uint32_t *id, int len, float v, int vid) {
    int lo = 0, hi = len;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (precedes(s[mid], (int)(id[mid] & ~EXPANDED), v, vid)) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

template <class T>
__global__ __launch_bounds__(GRAPH_THREADS) void graph_search_kernel(
    const void *__restrict__ X, int64_t N, int d, const int32_t *__restrict__ graph, int R, int entry,
    const void *__restrict__ Q, int k, int ef, int32_t *__restrict__ ids, float *__restrict__ scores,
    GraphLds L) {
    extern __shared__ __align__(16) unsigned char smem[];
    u4 *qs = reinterpret_cast<u4 *>(smem + L.q);
    float *ls[2] = {reinterpret_cast<float *>(smem + L.ls0), reinterpret_cast<float *>(smem + L.ls1)};
    uint32_t *li[2] = {reinterpret_cast<uint32_t *>(smem + L.li0), reinterpret_cast<uint32_t *>(smem + L.li1)};
    float *cs = reinterpret_cast<float *>(smem + L.cs);
    int *ci = reinterpret_cast<int *>(smem + L.ci);
    int *cpos = reinterpret_cast<int *>(smem + L.cpos);
    int *cache = reinterpret_cast<int *>(smem + L.cache);
    int *ctl = reinterpret_cast<int *>(smem + L.ctl);     // [0], [1]: first unexpanded index, by parity

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    const int nch = d * T::bytes / 16;                    // 16-byte chunks per row
    const int RP = (int)L.rp;
    const uint32_t cache_shift = 32u - L.cache_bits;

    for (int c = tid; c < nch; c += GRAPH_THREADS)
        qs[c] = load_chunk(static_cast<const char *>(Q) + ((size_t)b * nch + c) * 16);
    for (int i = tid; i < (1 << L.cache_bits); i += GRAPH_THREADS) cache[i] = -1;
    __syncthreads();

    const int sub = lane & (LANES_PER_ROW - 1);           // lane's position inside its row group
    const int grp = wave * (WAVE / LANES_PER_ROW) + lane / LANES_PER_ROW;   // 0..31

    // <q, x_v> by the 8 lanes of a row group; every lane of the group gets the sum
    auto score_row = [&](int v) -> float {
        const char *rp = static_cast<const char *>(X) + (size_t)v * nch * 16;
        float acc = 0.f;
        int c = sub;
        for (; c + 3 * LANES_PER_ROW < nch; c += 4 * LANES_PER_ROW) {
            const u4 x0 = load_chunk(rp + (size_t)c * 16);
            const u4 x1 = load_chunk(rp + (size_t)(c + LANES_PER_ROW) * 16);
            const u4 x2 = load_chunk(rp + (size_t)(c + 2 * LANES_PER_ROW) * 16);
            const u4 x3 = load_chunk(rp + (size_t)(c + 3 * LANES_PER_ROW) * 16);
            acc = dot_chunk<T>(x0, qs[c], acc);
            acc = dot_chunk<T>(x1, qs[c + LANES_PER_ROW], acc);
            acc = dot_chunk<T>(x2, qs[c + 2 * LANES_PER_ROW], acc);
            acc = dot_chunk<T>(x3, qs[c + 3 * LANES_PER_ROW], acc);
        }
        for (; c < nch; c += LANES_PER_ROW) acc = dot_chunk<T>(load_chunk(rp + (size_t)c * 16), qs[c], acc);
        acc += __shfl_xor(acc, 1);
        acc += __shfl_xor(acc, 2);
        acc += __shfl_xor(acc, 4);
        return acc;
    };

    // list <- [(score(entry), entry)]
    if (grp == 0) {
        const float s = score_row(entry);
        if (sub == 0) {
            ls[0][0] = s;
            li[0][0] = (uint32_t)entry;
            cache[((uint32_t)entry * 2654435761u) >> cache_shift] = entry;
            ctl[0] = 0;
        }
    }
    __syncthreads();

    int cur = 0, len = 1, par = 0;
    for (;;) {
        const int p = ctl[par];
        if (p == INT_MAX) break;                          // nothing left to expand: natural stop
        const int node = (int)(li[cur][p] & ~EXPANDED);
        __syncthreads();                                  // all have read p and node
        if (tid == 0) { li[cur][p] |= EXPANDED; ctl[par ^ 1] = INT_MAX; }

        // score the unseen neighbours of `node`, 32 graph slots per pass
        for (int base = 0; base < RP; base += ROWS_PER_PASS) {
            const int slot = base + grp;
            int v = -1;
            if (slot < R) v = graph[(size_t)node * R + slot];
            int fresh = 0;
            if ((unsigned)v < (unsigned)N) {
                if (sub == 0) {
                    const int old = atomicExch(&cache[((uint32_t)v * 2654435761u) >> cache_shift], v);
                    fresh = old != v;
                }
                fresh = __shfl(fresh, lane & ~(LANES_PER_ROW - 1));
            }
            float s = 0.f;
            if (fresh) s = score_row(v);
            if (sub == 0) { cs[slot] = s; ci[slot] = fresh ? v : -1; }
        }
        __syncthreads();

        // where would each scored neighbour go?  cpos = entries of the list that precede it,
        // or -1 when it is a duplicate or does not make it into the best ef
        for (int i = tid; i < RP; i += GRAPH_THREADS) {
            const int v = ci[i];
            int pos = -1;
            if (v >= 0) {
                const float s = cs[i];
                bool dup = false;
                for (int j = 0; j < i; ++j) dup |= (ci[j] == v);
                if (!dup && s == s) {                      // a NaN score is never listed
                    pos = list_lower_bound(ls[cur], li[cur], len, s, v);
                    if (pos >= ef || (pos < len && (int)(li[cur][pos] & ~EXPANDED) == v)) pos = -1;
                }
            }
            cpos[i] = pos;
        }
        __syncthreads();

        // merge into the other buffer: new entries at pos + (rank among new entries),
        // old entry j moves down by the number of new entries that precede it
        const int nxt = cur ^ 1;
        int n_new = 0;
        for (int i = 0; i < RP; ++i) n_new += (cpos[i] >= 0);
        for (int i = tid; i < RP; i += GRAPH_THREADS) {
            const int pos = cpos[i];
            if (pos >= 0) {
                const float s = cs[i];
                const int v = ci[i];
                int r = 0;
                for (int j = 0; j < RP; ++j) r += (cpos[j] >= 0 && precedes(cs[j], ci[j], s, v));
                if (pos + r < ef) { ls[nxt][pos + r] = s; li[nxt][pos + r] = (uint32_t)v; }
            }
        }
        for (int j = tid; j < len; j += GRAPH_THREADS) {
            int shift = 0;
            if (n_new)
                for (int i = 0; i < RP; ++i) shift += (cpos[i] >= 0 && cpos[i] <= j);
            if (j + shift < ef) { ls[nxt][j + shift] = ls[cur][j]; li[nxt][j + shift] = li[cur][j]; }
        }
        len = min(ef, len + n_new);
        cur = nxt;
        par ^= 1;
        __syncthreads();

        // first unexpanded entry of the new list
        int first = INT_MAX;
        for (int j = tid; j < len; j += GRAPH_THREADS)
            if (!(li[cur][j] & EXPANDED)) { first = j; break; }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) first = min(first, __shfl_xor(first, m));
        if (lane == 0 && first != INT_MAX) atomicMin(&ctl[par], first);
        __syncthreads();
    }

    for (int j = tid; j < k; j += GRAPH_THREADS) {
        const bool has = j < len;
        ids[(size_t)b * k + j] = has ? (int)(li[cur][j] & ~EXPANDED) : -1;
        scores[(size_t)b * k + j] = has ? ls[cur][j] : -INFINITY;
    }
}

}  // namespace ann
