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
//
// Maturity (non-stall) exit, Section 3.3 and Appendix B.2: every newly scored node t gives
// RQ_t = (d_t - d_best) / (d_worst - d_best) against the best and worst list entries, the
// values are smoothed by an exponential moving average, and the search returns its current
// list once the average exceeds tau and the engine-ready word is non-zero.  Here the
// neighbours of one expansion form a batch: best and worst are those of the list as the
// expansion starts, samples enter the average in slot order, the test follows the merge.
// The sample stream must not contain re-scored nodes, so this variant backs the id cache
// with an exact per-query bitset in global memory (its word is read together with the row,
// so it adds no round trip of its own, and set afterwards by an atomic without return).
#pragma once

#include "common.hpp"
#include "launch.hpp"

namespace ann {

constexpr int GRAPH_THREADS = 256;
constexpr int GRAPH_WAVES = GRAPH_THREADS / WAVE;
constexpr int LANES_PER_ROW = 8;
constexpr int ROWS_PER_PASS = GRAPH_THREADS / LANES_PER_ROW;   // 32 neighbours scored at once
constexpr uint32_t EXPANDED = 0x80000000u;
constexpr int RMAX_LDS = 256;                                  // row stride of the read-ahead buffers (>= R)

// Number of entries of the ordered list (s[0..len), id[0..len)) that precede (v, vid), found by
// the 8 lanes of a row group together: every round each lane probes one entry, which
// cuts the range to a ninth, so a list of 512 entries takes 3 LDS round trips and a last one over
// at most 8 neighbouring entries, where a binary search takes 9 or 10.  All lanes of the group must
// call it with the same arguments; all get the result.
__device__ __forceinline__ int group_lower_bound(const float *s, const uint32_t *id, int len, float v, int vid,
                                                 int sub, int lane) {
    const int gshift = lane & ~(LANES_PER_ROW - 1);
    int lo = 0, hi = len;                                 // the answer lies in [lo, hi]
    while (hi - lo > LANES_PER_ROW) {
        const int w = hi - lo;                            // >= 9: the probes are distinct and inside (lo, hi)
        const int m = lo + ((sub + 1) * w) / (LANES_PER_ROW + 1);
        const bool pr = precedes(s[m], (int)(id[m] & ~EXPANDED), v, vid);
        const int c = __builtin_popcount((unsigned)(__builtin_amdgcn_ballot_w64(pr) >> gshift) & 0xffu);
        // entries are ordered, so exactly the first c probes precede (v, vid)
        const int nlo = c > 0 ? lo + (c * w) / (LANES_PER_ROW + 1) + 1 : lo;
        const int nhi = c < LANES_PER_ROW ? lo + ((c + 1) * w) / (LANES_PER_ROW + 1) : hi;
        lo = nlo;
        hi = nhi;
    }
    const int m = lo + sub;
    const bool pr = m < hi && precedes(s[m], (int)(id[m] & ~EXPANDED), v, vid);
    return lo + __builtin_popcount((unsigned)(__builtin_amdgcn_ballot_w64(pr) >> gshift) & 0xffu);
}

// precedes() as 0 / 1 without short-circuit evaluation (no branches in unrolled loops)
__device__ __forceinline__ int precedes01(float s, int id, float s2, int id2) {
    return (int)(s > s2) | ((int)(s == s2) & (int)(id < id2));
}

// Sum over the 8 lanes of a row group, every lane gets it.  Three data-parallel-primitive moves
// (swap with the neighbour, swap the pairs of a quad, mirror the group of 8) in place of three
// trips through the LDS crossbar.  After the first two steps the four lanes of a quad hold the
// same bits (a + b and b + a are the same number), so the mirror step adds the same two quad
// sums in every lane: the result is bit for bit that of a butterfly over lanes ^1, ^2, ^4.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int x) {
    return __builtin_amdgcn_update_dpp(x, x, CTRL, 0xf, 0xf, false);
}
constexpr int DPP_SWAP1 = 0xB1;                           // quad_perm [1,0,3,2]
constexpr int DPP_SWAP2 = 0x4E;                           // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;                    // lane i of each 8 <- lane 7 - i
constexpr int DPP_MIRROR = 0x140;                         // lane i of each 16 <- lane 15 - i
__device__ __forceinline__ float group_sum(float x) {
    x += __int_as_float(dpp_move<DPP_SWAP1>(__float_as_int(x)));
    x += __int_as_float(dpp_move<DPP_SWAP2>(__float_as_int(x)));
    x += __int_as_float(dpp_move<DPP_HALF_MIRROR>(__float_as_int(x)));
    return x;
}
__device__ __forceinline__ int group_sum(int x) {
    x += dpp_move<DPP_SWAP1>(x);
    x += dpp_move<DPP_SWAP2>(x);
    x += dpp_move<DPP_HALF_MIRROR>(x);
    return x;
}

// The same count for lists of up to 64 NBLK entries (512, or 256 for NBLK = 4), in at most two LDS round trips.  First the 8
// lanes probe the last entries of the 8 blocks of 64 (skipped for lists of up to 64), which
// names the block the answer lies in; then every lane reads 8 neighbouring entries of that
// block with wide loads and counts.  *listed is set when the block holds `vid` itself: the node
// is in the list already (then it sits exactly at the returned position).  Reads may run up to
// 63 entries past `len` (never past the end of LDS: the list buffers are not the last region);
// what they return is masked out.
template <int NBLK = LANES_PER_ROW>
__device__ __forceinline__ int group_lower_bound_512(const float *s, const uint32_t *id, int len, float v, int vid,
                                                     int sub, int lane, bool *listed) {
    const int gshift = lane & ~(LANES_PER_ROW - 1);
    int blk = 0;
    if (len > 64) {
        const int m = 64 * min(sub, NBLK - 1) + 63;
        const bool pr = sub < NBLK && m < len && precedes(s[m], (int)(id[m] & ~EXPANDED), v, vid);
        blk = __builtin_popcount((unsigned)(__builtin_amdgcn_ballot_w64(pr) >> gshift) & 0xffu);
        if (blk == NBLK) { *listed = false; return 64 * NBLK; }
    }
    const int j0 = 64 * blk + 8 * sub;
    const f4 sa = *reinterpret_cast<const f4 *>(s + j0), sb = *reinterpret_cast<const f4 *>(s + j0 + 4);
    const int4 ia = *reinterpret_cast<const int4 *>(id + j0), ib = *reinterpret_cast<const int4 *>(id + j0 + 4);
    int cnt = 0, same = 0;
    auto one = [&](float es, int e, int j) {
        const int eid = e & (int)~EXPANDED;
        cnt += (int)(j < len) & precedes01(es, eid, v, vid);
        same |= (int)(j < len) & (int)(eid == vid);
    };
    one(sa[0], ia.x, j0 + 0); one(sa[1], ia.y, j0 + 1); one(sa[2], ia.z, j0 + 2); one(sa[3], ia.w, j0 + 3);
    one(sb[0], ib.x, j0 + 4); one(sb[1], ib.y, j0 + 5); one(sb[2], ib.z, j0 + 6); one(sb[3], ib.w, j0 + 7);
    *listed = ((unsigned)(__builtin_amdgcn_ballot_w64(same != 0) >> gshift) & 0xffu) != 0;
    return 64 * blk + group_sum(cnt);
}

// The same again, for the common case that no probed entry has exactly the score v: then ids
// play no part, and because list positions from `len` up to the next multiple of 64 hold -inf
// (set when the kernel starts, never written afterwards) the length does not either: two
// comparisons and two carries per entry.  Any lane that meets the score v itself sends its
// whole group to the general routine.
template <int NBLK = LANES_PER_ROW>
__device__ __forceinline__ int group_lower_bound_fast(const float *s, const uint32_t *id, int len, float v, int vid,
                                                      int sub, int lane, bool *listed) {
    const int gshift = lane & ~(LANES_PER_ROW - 1);
    int blk = 0;
    bool tie = false;
    if (len > 64) {
        const int m = 64 * min(sub, NBLK - 1) + 63;
        const float es = s[m];
        const bool in = sub < NBLK && m < len;
        tie = in && es == v;
        blk = __builtin_popcount((unsigned)(__builtin_amdgcn_ballot_w64(in && es > v) >> gshift) & 0xffu);
    }
    int gt = 0, ge = 0;
    if (blk < NBLK) {
        const int j0 = 64 * blk + 8 * sub;
        const f4 sa = *reinterpret_cast<const f4 *>(s + j0), sb = *reinterpret_cast<const f4 *>(s + j0 + 4);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            gt += (int)(sa[t] > v) + (int)(sb[t] > v);
            ge += (int)(sa[t] >= v) + (int)(sb[t] >= v);
        }
    }
    tie |= gt != ge;
    if (((unsigned)(__builtin_amdgcn_ballot_w64(tie) >> gshift) & 0xffu) != 0)
        return group_lower_bound_512<NBLK>(s, id, len, v, vid, sub, lane, listed);
    *listed = false;
    return 64 * blk + group_sum(gt);
}

// RPT: 32 for graphs with R <= 32 slots per node (one scoring pass per expansion, loops over the
// scored neighbours fully unrolled: the software-pipelined loop), 0 for wider graphs (the number
// of slots, rounded up to 32, comes from the layout at run time: the plain loop).
// NS: with the maturity exit (parameters in `ns`, ignored otherwise).
// QREG: the lane's share of the query stays in registers (fastest for one resident round of
// queries: two workgroups per compute unit).  Without it the products read the query from LDS and
// the kernel fits three workgroups per compute unit: more queries in flight, for batches larger
// than the chip holds at once, where throughput and not the latency of one query counts.
// LONG: the two-level candidate list for search ranges beyond GRAPH_EF_TWO_LEVEL (R <= 32, exact visited
// set, i.e. NS): see "two-level list" below.
template <class T, int RPT, bool NS, bool QREG = true, bool LONG = false>
__global__ __launch_bounds__(GRAPH_THREADS, QREG ? 2 : 3) void graph_search_kernel(
    const void *__restrict__ X, int64_t N, int d, const int32_t *__restrict__ graph, int R, int entry,
    const void *__restrict__ Q, int k, int ef, int32_t *__restrict__ ids, float *__restrict__ scores,
    GraphLds L, NonStall ns) {
    extern __shared__ __align__(16) unsigned char smem[];
    u4 *qs = reinterpret_cast<u4 *>(smem + L.q);
    // the two list buffers, selected by offset arithmetic on the LDS base (an array of pointers
    // indexed at run time would turn every list access into a generic-address load)
    // (LONG: the small regions sit at fixed offsets, see TL_LS0 ..)
    auto ls = [&](int which) {
        return reinterpret_cast<float *>(smem + (LONG ? (which ? TL_LS1 : TL_LS0) : (which ? L.ls1 : L.ls0)));
    };
    auto li = [&](int which) {
        return reinterpret_cast<uint32_t *>(smem + (LONG ? (which ? TL_LI1 : TL_LI0) : (which ? L.li1 : L.li0)));
    };
    float *cs = reinterpret_cast<float *>(smem + (LONG ? TL_CS : L.cs));
    int *ci = reinterpret_cast<int *>(smem + (LONG ? TL_CI : L.ci));
    int *cpos = reinterpret_cast<int *>(smem + (LONG ? TL_CPOS : L.cpos));
    int *cache = reinterpret_cast<int *>(smem + L.cache);
    static_assert(!LONG || (NS && RPT == 32 && QREG), "the two-level list needs the exact visited set and R <= 32");
    constexpr int ADJ = LONG ? 32 : RMAX_LDS;             // row stride of the adjacency rows read ahead
    int *adj = reinterpret_cast<int *>(smem + (LONG ? TL_ADJ : L.adj));     // [2][ADJ] adjacency rows read ahead
    int *adj_id = reinterpret_cast<int *>(smem + (LONG ? TL_CTL : L.ctl));  // [2] whose rows they are
    uint64_t *um = reinterpret_cast<uint64_t *>(smem + (LONG ? TL_UM : L.um));   // [ef/64] "unexpanded" bit masks
    float *rq = reinterpret_cast<float *>(smem + L.rq);   // RQ of each scored neighbour, NaN = no sample
    int *co = reinterpret_cast<int *>(smem + L.co);       // the valid ids of the adjacency row as read

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    // entry nodes of this query: ns.n_entries of its own, or the one shared `entry`
    const int32_t *my_entries = ns.entries ? ns.entries + (size_t)b * ns.n_entries : nullptr;
    const int E = ns.entries ? ns.n_entries : 1;
    const int nch = d * T::bytes / 16;                    // 16-byte chunks per row
    const int RP = RPT ? RPT : (int)L.rp;
    constexpr bool PIPELINED = RPT == 32;                 // R <= 32: the software-pipelined loop
    const uint32_t cache_shift = 32u - L.cache_bits;
    uint32_t *seen_bits = NS ? ns.visited + (size_t)b * ns.words : nullptr;   // zero on entry

    for (int c = tid; c < nch; c += GRAPH_THREADS)
        qs[c] = load_chunk(static_cast<const char *>(Q) + ((size_t)b * nch + c) * 16);
    if constexpr (!LONG)
        for (int i = tid; i < (1 << L.cache_bits); i += GRAPH_THREADS) cache[i] = -1;
    // list scores start as -inf up to the next multiple of 64 entries (see group_lower_bound_fast)
    constexpr int DCAP = GRAPH_DELTA;                     // LONG: entries of the small part of the list
    for (int i = tid; i < (LONG ? DCAP : ((ef + 63) & ~63)); i += GRAPH_THREADS) { ls(0)[i] = -INFINITY; ls(1)[i] = -INFINITY; }
    __syncthreads();

    const int sub = lane & (LANES_PER_ROW - 1);           // lane's position inside its row group
    const int grp = wave * (WAVE / LANES_PER_ROW) + lane / LANES_PER_ROW;   // 0..31

    // The lane's share of the first 128 chunks of the query (chunks sub, sub + 8, ...) stays in
    // registers for the whole search: up to 1024 16-bit dimensions are scored without reading
    // the query from LDS at all.
    constexpr int NX = QREG ? 16 : 8;                     // 16-byte loads of a row a lane keeps in flight
    constexpr int BLK = NX * LANES_PER_ROW;               // chunks of a row covered by those loads
    constexpr int TAIL = 8 * LANES_PER_ROW;               // chunks per round of the loop over the rest of a row
    u4 qr[QREG ? 16 : 1];
    if constexpr (QREG) {
#pragma unroll
        for (int u = 0; u < 16; ++u) qr[u] = qs[min(sub + u * LANES_PER_ROW, nch - 1)];
    }
    auto q_chunk = [&](int u) -> u4 {
        if constexpr (QREG) return qr[u];
        else return qs[min(sub + u * LANES_PER_ROW, nch - 1)];
    };

    // <q, x_v> by the 8 lanes of a row group; every lane of the group gets the sum.  All
    // of a lane's 16-byte loads of the row are issued before the first one is used, so a
    // whole expansion costs one memory latency, not one per batch of loads.  Loads and
    // products come in runs of four with one scalar test each (is any of the run's 32
    // chunks inside the row?); a lane whose chunk lies past the end of the row loads the
    // row's last chunk instead and leaves the product out of the sum (`lim` is re-derived
    // per call on purpose: sixteen loop-invariant lane masks would not fit the scalar registers).
    // (in two halves, so that other work can be put between the loads and their use)
    auto row_issue = [&](int v, u4 (&x)[NX]) {
        const char *rp = static_cast<const char *>(X) + (size_t)v * nch * 16;
        int lim = nch - sub;                              // chunk sub + 8u is in the row iff 8u < lim
        asm volatile("" : "+v"(lim));
        const char *rl = rp + sub * 16;
#pragma unroll
        for (int g = 0; g < NX / 4; ++g)
            if ((g + 1) * 4 * LANES_PER_ROW <= nch) {      // the whole run is inside: constant offsets
#pragma unroll
                for (int u = 4 * g; u < 4 * g + 4; ++u) x[u] = load_chunk(rl + u * LANES_PER_ROW * 16);
            } else if (g * 4 * LANES_PER_ROW < nch) {
#pragma unroll
                for (int u = 4 * g; u < 4 * g + 4; ++u)
                    x[u] = load_chunk(rp + (size_t)(sub + min(u * LANES_PER_ROW, lim - 1)) * 16);
            }
    };
    auto row_dots = [&](int v, u4 (&x)[NX]) -> float {
        const char *rp = static_cast<const char *>(X) + (size_t)v * nch * 16;
        f4 acc = {0.f, 0.f, 0.f, 0.f};                    // four independent chains, added at the end
        int lim = nch - sub;
        asm volatile("" : "+v"(lim));
#pragma unroll
        for (int g = 0; g < NX / 4; ++g)
            if ((g + 1) * 4 * LANES_PER_ROW <= nch) {      // the whole run is inside the row
#pragma unroll
                for (int u = 4 * g; u < 4 * g + 4; ++u) dot_chunk4<T>(x[u], q_chunk(u), acc);
            } else if (g * 4 * LANES_PER_ROW < nch) {
#pragma unroll
                for (int u = 4 * g; u < 4 * g + 4; ++u) {
                    f4 t = acc;
                    dot_chunk4<T>(x[u], q_chunk(u), t);
                    acc = u * LANES_PER_ROW < lim ? t : acc;
                }
            }
        for (int cb = BLK; cb < nch; cb += TAIL) {        // longer rows: the query comes from LDS
            u4 qv[8];
            lim -= cb == BLK ? BLK : TAIL;
#pragma unroll
            for (int g = 0; g < 2; ++g)
                if (cb + g * 4 * LANES_PER_ROW < nch) {
#pragma unroll
                    for (int u = 4 * g; u < 4 * g + 4; ++u) {
                        const int c = cb + sub + min(u * LANES_PER_ROW, lim - 1);
                        x[u] = load_chunk(rp + (size_t)c * 16);
                        qv[u] = qs[c];
                    }
                }
#pragma unroll
            for (int g = 0; g < 2; ++g)
                if (cb + g * 4 * LANES_PER_ROW < nch) {
#pragma unroll
                    for (int u = 4 * g; u < 4 * g + 4; ++u) {
                        f4 t = acc;
                        dot_chunk4<T>(x[u], qv[u], t);
                        acc = u * LANES_PER_ROW < lim ? t : acc;
                    }
                }
        }
        return group_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    };
    auto score_row = [&](int v) -> float {
        u4 x[NX];
        row_issue(v, x);
        return row_dots(v, x);
    };

    // list <- the entry nodes (at most 32, one row group each), scored and put in order; ids that
    // are no nodes and ids named by an earlier slot are left out, a NaN score is never listed
    int len = 0, n_dist = 0;                              // n_dist: scored nodes (used by the last wave)
    {
        int v0 = -1;
        if (grp < E) {
            v0 = my_entries ? my_entries[grp] : entry;
            if ((unsigned)v0 >= (unsigned)N) v0 = -1;
            for (int j = 0; j < grp && v0 >= 0; ++j)
                if (my_entries[j] == v0) v0 = -1;
        }
        float s0 = 0.f;
        if (v0 >= 0) s0 = score_row(v0);
        if (sub == 0) { cs[grp] = s0; ci[grp] = v0; }
        __syncthreads();
        const int cl = lane & 31;
        const float c_s = cs[cl];
        const int c_v = ci[cl];
        const bool c_valid = lane < 32 && c_v >= 0, c_ok = c_valid && c_s == c_s;
        const uint32_t ok_mask = (uint32_t)__builtin_amdgcn_ballot_w64(c_ok);
        n_dist = __builtin_popcountll(__builtin_amdgcn_ballot_w64(c_valid));
        len = min(ef, __builtin_popcount(ok_mask));
        int r = 0;                                        // listed entries that precede this lane's
        for (uint32_t m = ok_mask; m != 0; m &= m - 1) {
            const int l = __builtin_ctz(m);
            r += precedes01(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(c_s), l)),
                            __builtin_amdgcn_readlane(c_v, l), c_s, c_v);
        }
        if (wave == 0 && c_valid) {
            if (c_ok && r < ef) { ls(0)[r] = c_s; li(0)[r] = (uint32_t)c_v; }
            if constexpr (!LONG) cache[((uint32_t)c_v * 2654435761u) >> cache_shift] = c_v;
            if (NS) atomicOr(&seen_bits[c_v >> 5], 1u << (c_v & 31));
        }
        if (tid < 2) adj_id[tid] = -1;                    // adj[s] may hold the adjacency row of node adj_id[s]
        __syncthreads();
    }
    if (len == 0) {                                       // no entry that is a node with a score: padding only
        for (int j = tid; j < k; j += GRAPH_THREADS) {
            ids[(size_t)b * k + j] = -1;
            scores[(size_t)b * k + j] = -INFINITY;
        }
        if (NS && tid == 0) {
            if (ns.stats) { ns.stats[(size_t)b * 3] = 0; ns.stats[(size_t)b * 3 + 1] = n_dist; ns.stats[(size_t)b * 3 + 2] = 0; }
            if (ns.ema) ns.ema[b] = 0.f;
        }
        return;
    }
    // the best entry node is expanded first (masked: thread 0 may already have set the entry's
    // "expanded" bit below when a slower wave gets here; the id bits do not change)
    entry = (int)(li(0)[0] & ~EXPANDED);

    int cur = 0;
    float ema = 0.f;                                      // kept by the last wave, copied to the others
    int n_expand = 0, early = 0;
    // LONG: the large part M of the list (the small part D is the list ls / li / len of the code below)
    float *Ms = reinterpret_cast<float *>(smem + (LONG ? TL_MS : L.ls0));
    uint32_t *Mi = reinterpret_cast<uint32_t *>(smem + (LONG ? L.mi : L.li0));
    int mlen = 0;
    if constexpr (PIPELINED) {
    // ---- R <= 32: a software-pipelined loop -------------------------------------------------------
    // As soon as the neighbours of one expansion are scored, the next node to expand is known: the
    // better of the best unexpanded list entry and the best newly scored neighbour.  Its rows are
    // requested at once, and the merge of the current neighbours into the list and the scan for the
    // following runner-up then run while those rows are on their way.  The order of expansions and
    // merges, and so the result, is that of the plain loop below.
    //   per iteration:  scan (runner-up) | products, list positions | barrier | next node, its
    //                   neighbours filtered, rows requested | merge | barrier
    // The second barrier waits for LDS traffic only: __syncthreads() would also wait for the rows.
    auto lds_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    const int gbase = lane & ~(LANES_PER_ROW - 1);
    int aid0 = -1, aid1 = -1, tog = 0;                    // whose adjacency rows adj[0], adj[1] hold
    int node = entry, p = 0;                              // the node being expanded and its list index
    if (tid == 0) li(0)[0] = (uint32_t)entry | EXPANDED;  // (scans leave entry p out by index as well)
    u4 x[NX];
    int v = -1, fresh = 0;                                // this group's neighbour of `node`; to be scored?
    uint32_t seen = 0;                                    // NS: the word of the exact visited set that holds v
    float *ema_s = reinterpret_cast<float *>(adj_id + 3);
    // the samples are followed only when they can end the search or the caller wants the counters
    // (a plain search with a long list runs here with tau = inf and no counters)
    const bool track = NS && (ns.tau < INFINITY || ns.stats != nullptr || ns.ema != nullptr);
    if (NS && tid == 0) ema_s[0] = 0.f;

    // neighbour `grp` of node nd: duplicates within the row and ids the cache knows are dropped,
    // the row of a remaining one is requested
    // (in two steps, so that the merge can be put between them when the row has to come from the graph)
    int o4[4];                                            // 4 of the row's ids per lane, for the duplicate test
    auto request_row = [&](int nd) {
        const int have = aid0 == nd ? 0 : (aid1 == nd ? 1 : -1);
        const int slot = grp;
        const int vslot = min(slot, R - 1);
        if (have >= 0) {
            // (through a pointer that names the LDS address space: with plain pointers the compiler
            // folds the two cases into loads through a generic address, which are much slower;
            // one wide read: slots past R are masked below)
            typedef __attribute__((address_space(3))) const int lds_int;
            typedef int int4v __attribute__((ext_vector_type(4)));
            typedef __attribute__((address_space(3))) const int4v lds_int4;
            lds_int *row = (lds_int *)(adj + have * ADJ);
            v = row[vslot];
            const int4v o = *(lds_int4 *)(row + sub * 4);
            o4[0] = o[0]; o4[1] = o[1]; o4[2] = o[2]; o4[3] = o[3];
        } else {
            const int32_t *row = graph + (size_t)nd * R;
            v = row[vslot];
#pragma unroll
            for (int t = 0; t < 4; ++t) o4[t] = row[min(sub * 4 + t, R - 1)];
        }
    };
    auto request_rest = [&] {
        const int slot = grp;
        if (slot >= R) v = -1;
        int dup = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) dup |= (int)(sub * 4 + t < min(slot, R)) & (int)(o4[t] == v);
        if (((unsigned)(__builtin_amdgcn_ballot_w64(dup != 0) >> gbase) & 0xffu) != 0) v = -1;
        if constexpr (LONG) {
            // Long lists score tens of thousands of nodes, far more than an id cache in LDS remembers,
            // and a row fetched for a node that turns out to be scored already is wasted traffic.  Here
            // only the word of the exact visited set is requested; the rows of the nodes it shows as
            // new are requested when it has arrived (issue_rows, after the merge and its barrier,
            // which take about as long as the round trip), and arrive under the list work that
            // precedes the products.
            // (When the adjacency row itself had to come from the graph, requesting the rows of all
            // neighbours together with the word was measured as well: not faster, and it brings back
            // the wasted rows.)
            fresh = (int)((unsigned)v < (unsigned)N);
            if (fresh && sub == 0)
                seen = __hip_atomic_load(&seen_bits[v >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        bool first_time = false;
        if ((unsigned)v < (unsigned)N && sub == 0)
            first_time = atomicExch(&cache[((uint32_t)v * 2654435761u) >> cache_shift], v) != v;
        fresh = (int)((__builtin_amdgcn_ballot_w64(first_time) >> gbase) & 1u);
        // NS: the exact visited bit is read with the row (one round trip for both; the read
        // bypasses the vector L1, the atomics of earlier expansions completed before the barrier
        // after their scoring) and set after scoring by an atomic that returns nothing
        if (NS && fresh && sub == 0)
            seen = __hip_atomic_load(&seen_bits[v >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (fresh) row_issue(v, x);
    };
    request_row(node);
    request_rest();
    // LONG: rows of the neighbours the visited set shows as new (the marks of every earlier expansion
    // were complete before the barrier that preceded the request of the word)
    auto issue_rows = [&] {
        const bool unseen = sub == 0 && fresh && !((seen >> (v & 31)) & 1u);
        fresh = (int)((__builtin_amdgcn_ballot_w64(unseen) >> gbase) & 1u);
        if (fresh) row_issue(v, x);
    };

    // ---- LONG: the two-level list ------------------------------------------------------------------
    // A list of thousands of entries is not moved for every insertion.  It is kept as a large part M
    // (ordered, rewritten only by a rebuild) and a small part D (ordered, at most DCAP entries: the
    // double-buffered list ls / li / len of the code below); the candidate list of the method is the
    // merge of the two, cut at ef entries.  New entries go into D; when D is nearly full, it is
    // merged into M in one pass over M (once in some tens of expansions).
    //   * the worst entry of the list is the worse of the two tails.  A merge of new entries into D
    //     that takes the total past ef is followed, before the next expansion looks at the list, by
    //     dropping that many entries from the two tails, worst first (`pend`, `trim_tails`);
    //   * the best unexpanded entry is the better of D's (the scan below) and M's first unexpanded
    //     one, found through one bit per entry of M (um) and held in registers until it is
    //     expanded itself;
    //   * the exact visited set scores no node twice, so M is never searched for an id, and a new
    //     score is only compared with the worst entry and placed in D.
    // Order of expansions, contents of the list and counters are those of the single list.
    int pend = 0;                                         // entries still to be dropped from the tails
    bool stale_worst = true;                              // w_s, w_v are to be read again
    int m1 = -1, m1_v = -1;                               // M's first unexpanded entry (position, node), -1: none
    float m1_s = 0.f;
    float w_s = 0.f;                                      // the worst entry of the list (w_v < 0: the list is empty)
    int w_v = -1;
    // m1 <- first position >= from whose bit is set
    // (Lane and thread numbers go through an empty asm in these routines, so that nothing computed
    // from them is kept in a register across the whole search loop, where registers are short.)
    auto opaque = [](int x) { asm volatile("" : "+v"(x)); return x; };
    auto m_find = [&](int from) {
        m1 = -1;
        const int nw = (mlen + 63) >> 6;
        // (as a rule the next one is a few entries further on, in the word that holds `from`:
        // that word alone is read first, by all lanes at once)
        if ((from >> 6) < nw) {
            uint64_t word = um[from >> 6] & (~0ull << (from & 63));
            if ((from >> 6) == nw - 1 && (mlen & 63) != 0) word &= (1ull << (mlen & 63)) - 1ull;
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)word);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(word >> 32));
            const uint64_t wu = ((uint64_t)hi << 32) | lo;
            if (wu != 0) m1 = (from & ~63) + __builtin_ctzll(wu);
            else from = (from | 63) + 1;
        }
        if (m1 >= 0) {
            m1_s = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(Ms[m1])));
            m1_v = __builtin_amdgcn_readfirstlane((int)(Mi[m1] & ~EXPANDED));
            return;
        }
        const int lane_ = opaque(lane);
        for (int w0 = from >> 6; w0 < nw; w0 += WAVE) {
            const int w = w0 + lane_;
            uint64_t word = w < nw ? um[w] : 0ull;
            if (w == (from >> 6)) word &= ~0ull << (from & 63);
            if (w == nw - 1 && (mlen & 63) != 0) word &= (1ull << (mlen & 63)) - 1ull;
            const uint64_t any = __builtin_amdgcn_ballot_w64(word != 0);
            if (any != 0) {
                const int l = __builtin_ctzll(any);
                const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)word, l);
                const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(word >> 32), l);
                m1 = (w0 + l) * 64 + __builtin_ctzll(((uint64_t)hi << 32) | lo);
                break;
            }
        }
        if (m1 >= 0) {
            m1_s = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(Ms[m1])));
            m1_v = __builtin_amdgcn_readfirstlane((int)(Mi[m1] & ~EXPANDED));
        }
    };
    // After a merge into D: the `pend` worst entries of M and D together leave, and the worst entry
    // that remains is read again, in one round trip.  Lane j reads M's and D's j-th entries from the
    // end; lane j < pend asks whether M's is among the pend worst, i.e. whether fewer than pend - j
    // entries of D are worse than it (it reads that entry of D as well); the count of such lanes is
    // what M loses, D loses the rest, and the new worst is the worse of the first entries that stay.
    auto trim_tails = [&] {
        const int lane_ = opaque(lane);
        const float *dsc = ls(cur);
        const uint32_t *did = li(cur);
        const int ia = mlen - 1 - lane_, it = len - 1 - lane_, ix = len - pend + lane_;
        const float a_s = Ms[max(ia, 0)];
        const int a_v = (int)(Mi[max(ia, 0)] & ~EXPANDED);
        const float t_s = dsc[max(it, 0)];
        const int t_v = (int)(did[max(it, 0)] & ~EXPANDED);
        const int ixc = min(max(ix, 0), DCAP - 1);
        const float x_s = dsc[ixc];
        const int x_v = (int)(did[ixc] & ~EXPANDED);
        const bool c = lane_ < pend && ia >= 0 && (ix < 0 || precedes(x_s, x_v, a_s, a_v));
        const int tm = __builtin_popcountll(__builtin_amdgcn_ballot_w64(c)), td = pend - tm;
        mlen -= tm;
        len -= td;
        pend = 0;
        if (m1 >= mlen) m1 = -1;
        const float wa_s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a_s), tm));
        const int wa_v = __builtin_amdgcn_readlane(a_v, tm);
        const float wt_s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t_s), td));
        const int wt_v = __builtin_amdgcn_readlane(t_v, td);
        const bool take_d = len > 0 && (mlen <= 0 || precedes(wa_s, wa_v, wt_s, wt_v));
        w_s = take_d ? wt_s : wa_s;
        w_v = take_d ? wt_v : (mlen > 0 ? wa_v : -1);
    };
    // M <- merge of M and D, in place; D <- empty.  Thread t places D's entry t: its final position
    // is (entries of M that precede it) + t.  Those positions are marked in a bit per final position
    // (the words of um from the lowest marked position's block of 1024 on: um is rewritten there
    // anyway), with the number of marks before every word beside it; then every final position,
    // 1024 at a time from the top down, takes D's entry (rank) if marked and M's entry
    // (position - rank) if not.  Its sources lie at most DCAP below it, so one barrier between the
    // reads and the writes of a block suffices.  The expanded flags travel with the ids and give
    // the new bits of um.
    auto rebuild = [&] {
        constexpr int BLOCK = 4 * GRAPH_THREADS;
        const int tid_ = opaque(tid), lane_ = tid_ & (WAVE - 1), wave_ = tid_ >> 6;
        const int dn = len, total = mlen + dn;            // total <= ef: the tails have been cut
        int f = -1;
        if (tid_ < dn) {
            const float ds = ls(cur)[tid_];
            const int dv = (int)(li(cur)[tid_] & ~EXPANDED);
            int lo = 0, hi = mlen;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (precedes(Ms[mid], (int)(Mi[mid] & ~EXPANDED), ds, dv)) lo = mid + 1; else hi = mid;
            }
            f = lo + tid_;
        }
        if (tid_ == 0) adj_id[2] = f;
        lds_barrier();
        const int f0 = adj_id[2];                         // lowest position that changes
        const int lo_b = f0 & ~(BLOCK - 1);
        const int w_lo = lo_b >> 6, w_hi = (total + 63) >> 6;
        for (int w = w_lo + tid_; w < w_hi; w += GRAPH_THREADS) um[w] = 0ull;
        lds_barrier();
        if (f >= 0) atomicOr(reinterpret_cast<uint32_t *>(um) + (f >> 5), 1u << (f & 31));
        lds_barrier();
        int *rk = reinterpret_cast<int *>(ls(cur ^ 1));   // marks before word w_lo + t (D's other buffer is free)
        int *wt = reinterpret_cast<int *>(li(cur ^ 1));
        {
            const int w = w_lo + tid_;                     // w_hi - w_lo <= ef / 64 <= GRAPH_THREADS
            const int c = w < w_hi ? __builtin_popcountll(um[w]) : 0;
            int incl = c;
            for (int o = 1; o < WAVE; o <<= 1) {
                const int t = __shfl_up(incl, o);
                if (lane_ >= o) incl += t;
            }
            if (lane_ == WAVE - 1) wt[wave_] = incl;
            lds_barrier();
            int off = 0;
            for (int ww = 0; ww < wave_; ++ww) off += wt[ww];
            rk[tid_] = off + incl - c;
        }
        lds_barrier();
        for (int base = (total - 1) & ~(BLOCK - 1); base >= lo_b; base -= BLOCK) {
            float vs[4];
            uint32_t ve[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = base + u * GRAPH_THREADS + tid_;
                vs[u] = 0.f;
                ve[u] = EXPANDED;
                if (g < total) {
                    const uint64_t word = um[g >> 6];
                    const int bit = g & 63;
                    const int r = rk[(g >> 6) - w_lo] + __builtin_popcountll(word & ((1ull << bit) - 1ull));
                    if ((word >> bit) & 1ull) { vs[u] = ls(cur)[r]; ve[u] = li(cur)[r]; }
                    else { vs[u] = Ms[g - r]; ve[u] = Mi[g - r]; }
                }
            }
            lds_barrier();
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = base + u * GRAPH_THREADS + tid_;
                if (g < total) { Ms[g] = vs[u]; Mi[g] = ve[u]; }
                const uint64_t un = __builtin_amdgcn_ballot_w64(g < total && !(ve[u] & EXPANDED));
                const int w = (base + u * GRAPH_THREADS + wave_ * WAVE) >> 6;
                if (lane_ == 0 && w < w_hi) um[w] = un;
            }
        }
        lds_barrier();                                    // D and its other buffer have been read
        for (int i = tid_; i < DCAP; i += GRAPH_THREADS) { ls(0)[i] = -INFINITY; ls(1)[i] = -INFINITY; }
        const int from = min(m1 >= 0 ? m1 : total, f0);   // nothing unexpanded lies below either
        mlen = total;
        len = 0;
        cur = 0;
        lds_barrier();
        m_find(from);
    };

    for (;;) {
        if constexpr (LONG) {
            issue_rows();
            if (stale_worst) trim_tails();                // (the tails change only when entries go in)
            stale_worst = false;
        }
        // the runner-up: first unexpanded entry other than p (everything before p is expanded)
        int p2 = -1, node2 = -1;
        float s2 = 0.f;
        if (LONG || ef <= DCAP) {
            // A list of at most 256 entries (D always is one) in buffers that hold 256: every wave reads
            // all four blocks of 64 without conditions, takes one ballot per block, picks the first
            // block with a candidate by scalar selects and reads the pair out of one lane.
            const float *dsc = ls(cur);
            const uint32_t *did = li(cur);
            const uint32_t e0 = did[lane], e1 = did[lane + 64], e2 = did[lane + 128], e3 = did[lane + 192];
            const float f0 = dsc[lane], f1 = dsc[lane + 64], f2 = dsc[lane + 128], f3 = dsc[lane + 192];
            const uint64_t m0 = __builtin_amdgcn_ballot_w64(lane < len && lane != p && !(e0 & EXPANDED));
            const uint64_t m1 = __builtin_amdgcn_ballot_w64(lane + 64 < len && lane + 64 != p && !(e1 & EXPANDED));
            const uint64_t m2 = __builtin_amdgcn_ballot_w64(lane + 128 < len && lane + 128 != p && !(e2 & EXPANDED));
            const uint64_t m3 = __builtin_amdgcn_ballot_w64(lane + 192 < len && lane + 192 != p && !(e3 & EXPANDED));
            const int blk = m0 ? 0 : (m1 ? 1 : (m2 ? 2 : 3));
            const uint64_t mb = m0 ? m0 : (m1 ? m1 : (m2 ? m2 : m3));
            if (mb != 0) {
                const int l = __builtin_ctzll(mb);
                const uint32_t eb = blk == 0 ? e0 : (blk == 1 ? e1 : (blk == 2 ? e2 : e3));
                const float fb = blk == 0 ? f0 : (blk == 1 ? f1 : (blk == 2 ? f2 : f3));
                p2 = blk * 64 + l;
                node2 = __builtin_amdgcn_readlane((int)eb, l);
                s2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fb), l));
            }
        } else {
            // Every wave looks itself at the 256 entries from the block of 64 that holds p + 1 on:
            // ids and scores in one round trip, the runner-up's own pair then comes out of a lane.
            // No exchange between the waves and no barrier, whatever the length of the list.
            const int base0 = (p + 1) & ~63;
            uint32_t e4[GRAPH_WAVES];
            float s4[GRAPH_WAVES];
#pragma unroll
            for (int w = 0; w < GRAPH_WAVES; ++w) {
                e4[w] = EXPANDED;
                s4[w] = 0.f;
                if (base0 + w * 64 < len) {
                    const int j = min(base0 + w * 64 + lane, len - 1);
                    e4[w] = li(cur)[j];
                    s4[w] = ls(cur)[j];
                }
            }
#pragma unroll
            for (int w = 0; w < GRAPH_WAVES; ++w) {
                const int j = base0 + w * 64 + lane;
                const uint64_t mw = __builtin_amdgcn_ballot_w64(j < len && j != p && !(e4[w] & EXPANDED));
                if (mw != 0 && p2 < 0) {
                    const int l = __builtin_ctzll(mw);
                    p2 = base0 + w * 64 + l;
                    node2 = __builtin_amdgcn_readlane((int)e4[w], l);
                    s2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s4[w]), l));
                }
            }
            // nothing unexpanded among those 256 (rare): the rest, 256 entries per round, one ballot per
            // wave handed round through LDS
            if (!LONG && p2 < 0 && base0 + GRAPH_THREADS < len) {
                for (int base = base0 + GRAPH_THREADS; base < len; base += GRAPH_THREADS) {
                    const int j = base + tid;
                    const uint64_t m = __builtin_amdgcn_ballot_w64(j < len && !(li(cur)[j] & EXPANDED));
                    if (lane == 0) um[wave] = m;
                    lds_barrier();
#pragma unroll
                    for (int w = 0; w < GRAPH_WAVES; ++w) {
                        const uint64_t mw = um[w];
                        if (mw != 0 && p2 < 0) p2 = base + w * 64 + __builtin_ctzll(mw);
                    }
                    if (p2 >= 0) break;
                    lds_barrier();                        // um is rewritten in the next round
                }
                if (p2 >= 0) {
                    node2 = __builtin_amdgcn_readfirstlane((int)(li(cur)[p2] & ~EXPANDED));
                    s2 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(ls(cur)[p2])));
                }
            }
        }
        bool from_m = false;                              // LONG: the runner-up is M's first unexpanded entry
        if constexpr (LONG) {
            if (m1 >= 0 && (p2 < 0 || precedes(m1_s, m1_v, s2, node2))) {
                from_m = true;
                p2 = -1;
                node2 = m1_v;
                s2 = m1_s;
            }
        }
        // Read-ahead: the runner-up is the most likely next expansion, so its adjacency row is
        // fetched now, behind the rows already requested; it is stored once those are used.
        const bool have2 = (LONG ? (unsigned)node2 >= (unsigned)N : node2 < 0) || aid0 == node2 || aid1 == node2;
        int ahead = -1;
        if (!have2 && tid < R) ahead = graph[(size_t)node2 * R + tid];

        // products and list positions of the neighbours of `node`
        ++n_expand;
        float s = 0.f;
        if (fresh) s = row_dots(v, x);
        if (NS) {                                         // the cache may have forgotten v: the bitset has not
            if constexpr (!LONG) {                        // (LONG: only unseen nodes were requested)
                const bool was_seen = sub == 0 && fresh && ((seen >> (v & 31)) & 1u);
                if ((__builtin_amdgcn_ballot_w64(was_seen) >> gbase) & 1u) fresh = 0;
            }
            if (fresh && sub == 0) atomicOr(&seen_bits[v >> 5], 1u << (v & 31));
        }
        int pos = -1;
        if (fresh && s == s) {                             // a NaN score is never listed
            if constexpr (LONG) {
                // a full list takes what beats its worst entry; the position is the one in D
                if (mlen + len < ef || precedes(s, v, w_s, w_v)) {
                    bool listed;
                    pos = group_lower_bound_fast<DCAP / 64>(ls(cur), li(cur), len, s, v, sub, lane, &listed);
                    if (listed) pos = -1;
                }
            } else if (len <= 512) {
                bool listed;
                pos = group_lower_bound_fast(ls(cur), li(cur), len, s, v, sub, lane, &listed);
                if (pos >= ef || listed) pos = -1;
            } else {
                pos = group_lower_bound(ls(cur), li(cur), len, s, v, sub, lane);
                if (pos >= ef || (pos < len && (int)(li(cur)[pos] & ~EXPANDED) == v)) pos = -1;
            }
        }
        if (sub == 0) {
            cs[grp] = s;
            ci[grp] = fresh ? v : -1;
            cpos[grp] = pos;
        }
        if (!have2) {
            const int into = aid0 == node ? 0 : (aid1 == node ? 1 : (tog ^= 1));
            if (tid < R) adj[into * ADJ + tid] = ahead;
            if (into == 0) aid0 = node2; else aid1 = node2;
        }
        __syncthreads();                                  // (also waits for the marks set above)

        // LONG: D needs room for the entries of one expansion.  The rebuild runs here, where no rows
        // are in flight (their registers are free); it leaves D empty, so the position in D of every
        // new entry becomes 0, and the runner-up, the same entry as before, is now M's first
        // unexpanded one.
        bool rebuilt = false;
        if constexpr (LONG) {
            if (len > DCAP - ROWS_PER_PASS) {
                rebuild();
                rebuilt = true;
                p = -1;
                p2 = -1;
                from_m = m1 >= 0;
            }
        }

        // NS: the relative quality of every newly scored node against the best and worst entries of
        // the list as it stands before they go in, into the moving average in slot order (a slot
        // holds a sample exactly when it scored a node: later slots that name the same id were
        // dropped with the row).  Kept by the last wave, handed to the others through LDS.
        if (NS && track && wave == GRAPH_WAVES - 1) {
            float s_best, s_worst;
            if constexpr (LONG) {
                s_best = len > 0 ? ls(cur)[0] : -INFINITY;
                if (mlen > 0) s_best = fmaxf(s_best, Ms[0]);
                s_worst = w_s;
            } else {
                s_best = ls(cur)[0];
                s_worst = ls(cur)[len - 1];
            }
            float r = NAN;                                // NaN: no sample; -inf: one, but best == worst
            if (lane < 32 && ci[lane] >= 0) r = s_best != s_worst ? (s_best - cs[lane]) / (s_best - s_worst) : -INFINITY;
            const uint32_t mag = __float_as_uint(r) & 0x7fffffffu;
            n_dist += __builtin_popcountll(__builtin_amdgcn_ballot_w64(mag <= 0x7f800000u));
            for (uint64_t defined = __builtin_amdgcn_ballot_w64(mag < 0x7f800000u); defined != 0; defined &= defined - 1) {
                const float ri = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(r), __builtin_ctzll(defined)));
                ema = fmaf(ns.alpha, ri - ema, ema);
            }
            if (lane == 0) ema_s[0] = ema;
        }

        // what is inserted (lane i < 32 of every wave looks at neighbour i) and which node is next
        const int cl = lane & 31;
        const float c_s = cs[cl];
        const int c_v = ci[cl];
        int c_p = cpos[cl];
        asm volatile("" ::"v"(c_s), "v"(c_v));            // all three reads now, in one round trip
        if (LONG && rebuilt) c_p = min(c_p, 0);
        const bool c_ok = lane < 32 && c_p >= 0;
        const uint32_t new_mask = (uint32_t)__builtin_amdgcn_ballot_w64(c_ok);
        const int n_new = __builtin_popcount(new_mask);
        // The best new entry: scores as integers that order the other way round (0.0f is added so
        // that -0 and +0 get the same one), their minimum over lanes 0 .. 31 by data-parallel moves
        // inside the rows of 16 lanes and two lane reads; equal scores (rare) are settled by id.
        int best_v = node2, best_l = -1;
        if (n_new != 0) {
            const uint32_t c_u = (uint32_t)__float_as_int(c_s + 0.0f);
            const uint32_t c_k = c_ok ? ~(c_u ^ ((uint32_t)((int32_t)c_u >> 31) | 0x80000000u)) : 0xffffffffu;
            uint32_t mk = c_k;
            mk = min(mk, (uint32_t)dpp_move<DPP_SWAP1>((int)mk));
            mk = min(mk, (uint32_t)dpp_move<DPP_SWAP2>((int)mk));
            mk = min(mk, (uint32_t)dpp_move<DPP_HALF_MIRROR>((int)mk));
            mk = min(mk, (uint32_t)dpp_move<DPP_MIRROR>((int)mk));
            const uint32_t kmin = min((uint32_t)__builtin_amdgcn_readlane((int)mk, 0), (uint32_t)__builtin_amdgcn_readlane((int)mk, 16));
            uint64_t m = __builtin_amdgcn_ballot_w64(c_ok && c_k == kmin);
            int l = __builtin_ctzll(m);
            int lv = __builtin_amdgcn_readlane(c_v, l);
            for (m &= m - 1; m != 0; m &= m - 1) {        // several with the best score: lowest id
                const int l2 = __builtin_ctzll(m), v2 = __builtin_amdgcn_readlane(c_v, l2);
                if (v2 < lv) { l = l2; lv = v2; }
            }
            const float lsc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c_s), l));
            if (node2 < 0 || precedes(lsc, lv, s2, node2)) { best_l = l; best_v = lv; }
        }
        // nothing left to expand: natural stop (LONG: an id that is no node, or more expansions than
        // there are nodes, neither of which a sound list ever shows, end the search as well instead
        // of being followed into the graph or spinning)
        const bool last = LONG ? ((unsigned)best_v >= (unsigned)N || (int64_t)n_expand > N + ROWS_PER_PASS) : best_v < 0;
        if (!NS && last) break;                           // (NS: after the maturity test below)

        // New entries at or before list position j.  A few insertions (the rule once the list has
        // settled): their positions are read out of lanes one by one; many: the 32 positions are
        // read from LDS (as broadcasts) and compared in one unrolled run.  (Holding the positions
        // in registers across the merge, next to the rows in flight, would not fit the register file.)
        constexpr int FEW = 6;
        const bool few = n_new <= FEW;
        auto shift_of = [&](int j) {
            int shift = 0;
            if (few) {
                for (uint32_t m = new_mask; m != 0; m &= m - 1)
                    shift += (int)((unsigned)__builtin_amdgcn_readlane(c_p, __builtin_ctz(m)) <= (unsigned)j);
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int4 q4 = reinterpret_cast<const int4 *>(cpos)[u];
                    shift += (int)((unsigned)q4.x <= (unsigned)j) + (int)((unsigned)q4.y <= (unsigned)j) +
                             (int)((unsigned)q4.z <= (unsigned)j) + (int)((unsigned)q4.w <= (unsigned)j);
                }
            }
            return shift;
        };
        // where the next node will be in the merged list: the best new entry goes to its position
        // as it is (no new entry precedes it), an old one moves up like every old entry
        // (when an old entry stays the best, every new entry comes after it)
        const int next_p = best_l >= 0 ? __builtin_amdgcn_readlane(c_p, best_l) : p2;

        // Its adjacency row is held in LDS when it was the runner-up; a new entry's row has to come
        // from the graph, a global round trip, and then the merge goes first, under that load.
        const bool held = aid0 == best_v || aid1 == best_v;
        if (!last) {
            request_row(best_v);
            if (held) request_rest();
        }

        // merge, as in the plain loop; the entry of the next node is marked as expanded on its way
        if (n_new != 0) {
            int new_at = -1;
            float new_s = 0.f;
            uint32_t new_e = 0;
            int gpos = cpos[grp];
            if (LONG && rebuilt) gpos = min(gpos, 0);
            if (gpos >= 0) {
                new_s = cs[grp];
                const int new_v = ci[grp];
                const f4 sq = reinterpret_cast<const f4 *>(cs)[sub];
                const int4 cq = reinterpret_cast<const int4 *>(ci)[sub];
                const int4 pq = reinterpret_cast<const int4 *>(cpos)[sub];
                int r = ((int)(pq.x >= 0) & precedes01(sq[0], cq.x, new_s, new_v)) +
                        ((int)(pq.y >= 0) & precedes01(sq[1], cq.y, new_s, new_v)) +
                        ((int)(pq.z >= 0) & precedes01(sq[2], cq.z, new_s, new_v)) +
                        ((int)(pq.w >= 0) & precedes01(sq[3], cq.w, new_s, new_v));
                r = group_sum(r);
                if (sub == 0 && gpos + r < ef) new_at = gpos + r;
                new_e = (uint32_t)new_v | (grp == best_l ? EXPANDED : 0u);
            }
            const int old_next = best_l < 0 ? p2 : -1;   // an old entry that becomes the next node
            {   // (this loop serves lists of at most 512 entries, and D: always double-buffered)
                const int nxt = cur ^ 1;
                if (new_at >= 0) { ls(nxt)[new_at] = new_s; li(nxt)[new_at] = new_e; }
                for (int j = tid; j < len; j += GRAPH_THREADS) {
                    const int to = j + shift_of(j);
                    if (to < ef) { ls(nxt)[to] = ls(cur)[j]; li(nxt)[to] = li(cur)[j] | (j == old_next ? EXPANDED : 0u); }
                }
                cur = nxt;
            }
            if constexpr (LONG) {
                len += n_new;                             // at most DCAP; what exceeds ef in all leaves next
                pend = max(0, mlen + len - ef);
                stale_worst = true;
            } else {
                len = min(ef, len + n_new);
            }
        } else if (tid == 0 && !last && p2 >= 0) {
            atomicOr(&li(cur)[p2], EXPANDED);             // the list stays as it is (no return value to wait for)
        }
        if constexpr (LONG) {
            if (!last && best_l < 0 && from_m) {          // the next node is M's first unexpanded entry
                if (tid == 0) {                             // (LDS atomics without return: nothing to wait for)
                    atomicOr(&Mi[m1], EXPANDED);
                    atomicAnd(reinterpret_cast<unsigned long long *>(&um[m1 >> 6]), ~(1ull << (m1 & 63)));
                }
                m_find(m1 + 1);                           // (looks only at bits above the one just cleared)
            }
        }
        if (!last && !held) request_rest();
        lds_barrier();
        if (NS) {
            ema = ema_s[0];
            if (ema > ns.tau) {                           // mature: leave as soon as the engine is ready
                int ready = 1;
                if (ns.ready) {
                    if (tid == 0) adj_id[2] = __hip_atomic_load(ns.ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    __syncthreads();
                    ready = adj_id[2];
                }
                if (ready) { early = 1; break; }
            }
            if (last) break;
        }
        node = best_v;
        p = next_p;
    }
    if constexpr (LONG) {                                 // (both exits follow the barrier that ends a merge)
        if (pend > 0) trim_tails();
        if (len > 0) rebuild();
    }
    } else {
    // ---- R > 32: the plain loop, 32 graph slots per scoring pass -----------------------------------
    // read the list top, score, barrier, sort out ids named twice, barrier, merge, barrier, scan
    int p = 0, p2 = -1;                                   // best and second-best unexpanded entries
    float *ema_s = reinterpret_cast<float *>(adj_id + 3);
    for (;;) {
        if (p < 0) break;                                 // nothing left to expand: natural stop
        ++n_expand;
        const int node = (int)(li(cur)[p] & ~EXPANDED);
        const int node2 = p2 >= 0 ? (int)(li(cur)[p2] & ~EXPANDED) : -1;
        const int have = adj_id[0] == node ? 0 : (adj_id[1] == node ? 1 : -1);
        const int have_u = __builtin_amdgcn_readfirstlane(have);   // the same in all lanes
        const bool have2 = node2 < 0 || adj_id[0] == node2 || adj_id[1] == node2;
        __syncthreads();                                  // all have read the list and adj_id
        if (tid == 0) li(cur)[p] |= EXPANDED;

        // Read-ahead: the second-best unexpanded entry is the most likely next expansion, so
        // its adjacency row is fetched now, under the gathers of this expansion.  It only
        // saves a dependent memory round trip later; nothing is decided from it here.
        int ahead = -1;
        if (!have2 && tid < R) ahead = graph[(size_t)node2 * R + tid];

        // score the unseen neighbours of `node`, 32 graph slots per pass
        for (int base = 0; base < RP; base += ROWS_PER_PASS) {
            const int slot = base + grp;
            // the row comes from LDS if it was read ahead, else from the graph
            int v = -1;
            if (slot < R) {
                if (have_u >= 0) v = adj[have_u * RMAX_LDS + slot];
                else v = graph[(size_t)node * R + slot];
            }
            // the group's first lane asks the cache; its answer reaches the others as a lane mask
            bool first_time = false;
            if ((unsigned)v < (unsigned)N && sub == 0)
                first_time = atomicExch(&cache[((uint32_t)v * 2654435761u) >> cache_shift], v) != v;
            int fresh = (int)((__builtin_amdgcn_ballot_w64(first_time) >> (lane & ~(LANES_PER_ROW - 1))) & 1u);
            // The exact visited bit is read with the row (one round trip for both) and set
            // afterwards by an atomic that returns nothing.  The read bypasses the vector L1;
            // the atomics of earlier expansions completed before the barriers in between.
            uint32_t seen = 0;
            if (NS && fresh && sub == 0)
                seen = __hip_atomic_load(&seen_bits[v >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            float s = 0.f;
            if (fresh) s = score_row(v);
            if (NS) {                                     // the cache may have forgotten v: the bitset has not
                const bool was_seen = sub == 0 && fresh && ((seen >> (v & 31)) & 1u);
                if ((__builtin_amdgcn_ballot_w64(was_seen) >> (lane & ~(LANES_PER_ROW - 1))) & 1u) fresh = 0;
                if (fresh && sub == 0) atomicOr(&seen_bits[v >> 5], 1u << (v & 31));
            }
            // Where would it go?  pos = entries of the list that precede it, or -1 when it does not
            // make it into the best ef or is in the list already (the cache may have forgotten it).
            // Found here, by the row group that scored it, while the list is at rest; ids named by
            // two slots are sorted out after the barrier.
            int pos = -1;
            if (fresh && s == s) {                         // a NaN score is never listed
                if (len <= 512) {
                    bool listed;
                    pos = group_lower_bound_fast(ls(cur), li(cur), len, s, v, sub, lane, &listed);
                    if (pos >= ef || listed) pos = -1;
                } else {
                    pos = group_lower_bound(ls(cur), li(cur), len, s, v, sub, lane);
                    if (pos >= ef || (pos < len && (int)(li(cur)[pos] & ~EXPANDED) == v)) pos = -1;
                }
            }
            if (sub == 0) {
                cs[slot] = s;
                ci[slot] = fresh ? v : -1;
                cpos[slot] = pos;
                if (NS) co[slot] = (unsigned)v < (unsigned)N ? v : -1;
            }
        }
        if (!have2) {                                     // keep the row of `node` if it is in a slot
            const int into = have == 0 ? 1 : 0;
            if (tid < R) adj[into * RMAX_LDS + tid] = ahead;
            if (tid == 0) adj_id[into] = node2;
        }
        __syncthreads();

        // an id named by an earlier slot as well is taken once: cpos = -1 for the later slot
        for (int i = tid; i < RP; i += GRAPH_THREADS) {
            const int v = ci[i];
            if (v >= 0) {
                int dup = 0;
                for (int j = 0; j < i; ++j) dup |= (int)(ci[j] == v);
                if (dup) cpos[i] = -1;
            }
        }
        // The moving average is kept by the last wave alone, beside the list work of the
        // others (for short rows and lists that is all on wave 0), and handed over in LDS.
        if (NS && wave == GRAPH_WAVES - 1) {
            // best / worst of the list as it stands before this expansion's entries go in
            const float s_best = ls(cur)[0], s_worst = ls(cur)[len - 1];
            // RQ of slot i, or NaN: no newly scored node there, or -inf: one, but best == worst.
            // An id named more than once in the row is scored by whichever slot won the race
            // for the cache entry (rarely by two); its one sample belongs to the first slot
            // that names it.
            auto rq_of = [&](int i, int me, bool first, bool scored, float sv) -> float {
                (void)i; (void)me;
                return !(first && scored) ? NAN : s_best != s_worst ? (s_best - sv) / (s_best - s_worst) : -INFINITY;
            };
            auto take = [&](float r) {
                if (r == r) {
                    ++n_dist;
                    if (r != -INFINITY) ema = fmaf(ns.alpha, r - ema, ema);
                }
            };
            for (int i = lane; i < RP; i += WAVE) {
                const int me = co[i];
                bool first = me >= 0, scored = false;
                float sv = 0.f;
                for (int j = 0; j < RP; ++j) {
                    if (j < i && co[j] == me) first = false;
                    if (ci[j] == me) { scored = true; sv = cs[j]; }
                }
                rq[i] = rq_of(i, me, first, scored, sv);
            }
            // rq[] is written and read by this wave only, in program order
            for (int i = 0; i < RP; ++i) take(rq[i]);
            if (lane == 0) ema_s[0] = ema;
        }
        __syncthreads();

        // merge: new entries go to pos + (rank among the new entries), old entry j moves up by the
        // number of new entries that precede it.  Lists of up to 2048 entries are double-buffered
        // (merged into the other buffer); longer ones have one buffer and are merged in place.
        const bool inplace = L.ls1 == L.ls0;
        int n_new = 0;
        unsigned jmin = 0xffffffffu;                      // lowest position a new entry takes
        for (int i = 0; i < RP; ++i) {
            n_new += (cpos[i] >= 0);
            jmin = min(jmin, (unsigned)cpos[i]);
        }
        // nothing to insert (most expansions once the list has settled): the list stays where it is
        const int nxt = inplace || n_new == 0 ? cur : cur ^ 1;
        // number of new entries at or before list position j (a position is in 0 .. j exactly
        // when, as an unsigned number, it is <= j; -1 is not)
        auto shift_of = [&](int j) {
            int shift = 0;
            for (int i = 0; i < RP; ++i) shift += (int)((unsigned)cpos[i] <= (unsigned)j);
            return shift;
        };
        // the new entry of this thread: final position or -1
        int new_at = -1;
        float new_s = 0.f;
        int new_v = 0;
        if (n_new != 0 && tid < RP) {                     // slot tid, RP <= GRAPH_THREADS
            const int pos = cpos[tid];
            if (pos >= 0) {
                new_s = cs[tid];
                new_v = ci[tid];
                int r = 0;
                for (int j = 0; j < RP; ++j) r += (int)(cpos[j] >= 0) & precedes01(cs[j], ci[j], new_s, new_v);
                if (pos + r < ef) new_at = pos + r;
            }
        }
        if (!inplace && n_new != 0) {
            if (new_at >= 0) { ls(nxt)[new_at] = new_s; li(nxt)[new_at] = (uint32_t)new_v; }
            for (int j = tid; j < len; j += GRAPH_THREADS) {
                const int shift = shift_of(j);
                if (j + shift < ef) { ls(nxt)[j + shift] = ls(cur)[j]; li(nxt)[j + shift] = li(cur)[j]; }
            }
        } else if (n_new) {
            // Entries below jmin stay.  The others move up by at most RP: chunks of MOVE entries
            // are taken from the top down; a chunk is read by everyone before anyone writes it
            // (its targets lie in itself and in the chunk above, which has already moved).
            constexpr int PER = 4, MOVE = PER * GRAPH_THREADS;
            const int lowest = (int)jmin & ~(MOVE - 1);
            for (int base = (len - 1) & ~(MOVE - 1); base >= lowest; base -= MOVE) {
                float ms[PER];
                uint32_t mi[PER];
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    const int j = base + u * GRAPH_THREADS + tid;
                    if (j < len && j >= (int)jmin) { ms[u] = ls(cur)[j]; mi[u] = li(cur)[j]; }
                }
                __syncthreads();
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    const int j = base + u * GRAPH_THREADS + tid;
                    if (j < len && j >= (int)jmin) {
                        const int to = j + shift_of(j);
                        if (to < ef) { ls(cur)[to] = ms[u]; li(cur)[to] = mi[u]; }
                    }
                }
            }
            __syncthreads();                              // every old entry is out of the way
            if (new_at >= 0) { ls(cur)[new_at] = new_s; li(cur)[new_at] = (uint32_t)new_v; }
        }
        len = min(ef, len + n_new);
        cur = nxt;
        if (NS || n_new != 0) __syncthreads();            // an untouched list needs no barrier (n_new is uniform)

        // Best and second-best unexpanded entries of the new list: one ballot per 64 entries.
        // Everything before the entry just expanded was expanded already, and the merge has not
        // touched the list before its lowest insertion, so the scan starts at the lower of the
        // two and goes on, 256 entries per round, only until two are found (one round as a rule,
        // whatever the length of the list).
        if (len <= GRAPH_THREADS) {
            // short list: every wave looks at all of it itself (up to four entries per lane, read
            // together), so no exchange between the waves and no second barrier is needed
            p = -1;
            p2 = -1;
            uint32_t e4[GRAPH_WAVES];
#pragma unroll
            for (int w = 0; w < GRAPH_WAVES; ++w) e4[w] = w * 64 < len ? li(cur)[min(w * 64 + lane, len - 1)] : EXPANDED;
#pragma unroll
            for (int w = 0; w < GRAPH_WAVES; ++w) {
                uint64_t mw = __builtin_amdgcn_ballot_w64(w * 64 + lane < len && !(e4[w] & EXPANDED));
                while (mw != 0 && p2 < 0) {
                    const int jj = w * 64 + __builtin_ctzll(mw);
                    mw &= mw - 1;
                    if (p < 0) p = jj; else p2 = jj;
                }
            }
        } else {
            const unsigned first = min((unsigned)p, jmin);
            p = -1;
            p2 = -1;
            for (int base = (int)first & ~(GRAPH_THREADS - 1); base < len; base += GRAPH_THREADS) {
                const int j = base + tid;
                const uint64_t m = __builtin_amdgcn_ballot_w64(j < len && !(li(cur)[j] & EXPANDED));
                if (lane == 0) um[wave] = m;
                __syncthreads();
#pragma unroll
                for (int w = 0; w < GRAPH_WAVES; ++w) {
                    uint64_t mw = um[w];
                    while (mw != 0 && p2 < 0) {
                        const int jj = base + w * 64 + __builtin_ctzll(mw);
                        mw &= mw - 1;
                        if (p < 0) p = jj; else p2 = jj;
                    }
                }
                if (p2 >= 0) break;
                __syncthreads();                          // um is rewritten in the next round
            }
        }
        if (NS) ema = ema_s[0];                           // written before the last two barriers
        if (NS && ema > ns.tau) {                         // mature: leave as soon as the engine is ready
            int ready = 1;
            if (ns.ready) {
                if (tid == 0) adj_id[2] = __hip_atomic_load(ns.ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                __syncthreads();
                ready = adj_id[2];
            }
            if (ready) { early = 1; break; }
        }
    }

    }   // plain loop

    for (int j = tid; j < k; j += GRAPH_THREADS) {
        if constexpr (LONG) {                             // (everything is in M by now)
            const bool has = j < mlen;
            ids[(size_t)b * k + j] = has ? (int)(Mi[j] & ~EXPANDED) : -1;
            scores[(size_t)b * k + j] = has ? Ms[j] : -INFINITY;
        } else {
            const bool has = j < len;
            ids[(size_t)b * k + j] = has ? (int)(li(cur)[j] & ~EXPANDED) : -1;
            scores[(size_t)b * k + j] = has ? ls(cur)[j] : -INFINITY;
        }
    }
    if (NS && tid == GRAPH_THREADS - WAVE) {
        if (ns.stats) {
            ns.stats[(size_t)b * 3 + 0] = early;
            ns.stats[(size_t)b * 3 + 1] = n_dist;
            ns.stats[(size_t)b * 3 + 2] = n_expand;
        }
        if (ns.ema) ns.ema[b] = ema;
    }
}

// out[i] <- table[idx[i]], or -1 where idx[i] is not in [0, M)
__global__ __launch_bounds__(256) void gather_ids_kernel(const int32_t *__restrict__ table, int64_t M,
                                                         const int32_t *__restrict__ idx, int64_t n,
                                                         int32_t *__restrict__ out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t j = idx[i];
        out[i] = (j >= 0 && j < M) ? table[j] : -1;
    }
}

// words[0 .. n) <- 0, 16 bytes per store (n a multiple of 4)
__global__ __launch_bounds__(256) void zero_words_kernel(u4 *__restrict__ p, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = zero_chunk();
}

}  // namespace ann
