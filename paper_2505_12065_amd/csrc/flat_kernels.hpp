// Exact (flat) retrieval kernels: every corpus row is scored against every query
// and the k best per query are kept (Section 2.1 of the paper: exact nearest
// neighbour retrieval; the score matrix is never written to memory).
//
//   flat_stream_kernel  16-bit corpora, up to 64 queries per pass: the corpus is
//                       streamed from HBM exactly once straight into MFMA operand
//                       registers; queries sit in LDS in MFMA fragment order.
//   flat_f32_kernel     fp32 corpora: vector FMA, 8 lanes per row.
//   flat_merge_kernel   per query: the k best of all slabs' partial lists.
//
// Every kernel keeps, per lane, a sorted register list of the KP >= k best
// pairs it has seen; lists are merged lane -> wave -> workgroup -> grid under
// the same total order, so the result does not depend on how rows were split.
#pragma once

#include "common.hpp"
#include "launch.hpp"

namespace ann {

constexpr int STREAM_UNROLL = 8;   // 16-byte loads a lane keeps in flight (6..24 measured alike)

// Corpus rows are the M side of a 16x16x32 MFMA, queries the N side: a lane ends
// up with one query (lane % 16) and four rows (4*(lane/16) + i) per tile of 16 rows.
//   X        [N, d] 16-bit           Q  [B, d] 16-bit (queries q0 .. q0+NQG*16 are used)
//   partial  [B, P, KP] pairs, P = gridDim.x
//   o        see StreamOpts: row stride of a sampling pass, and (EMIT, for k > 4) no lists at all:
//            every (score, row) with score >= o.thr[q] is appended to the candidate array
//            partial[q * o.cap ..) through o.count[q]
// One pass of the whole workgroup (NWV wavefronts) over its share of the corpus for NQG*16 queries.
template <class T, int NQG, int KP, bool DFULL, bool EMIT, int NWV>
__device__ __forceinline__ void flat_stream_pass(const void *__restrict__ X, int64_t N, int d,
                                                 const void *__restrict__ Q, int B, int q0,
                                                 Cand *__restrict__ partial, const StreamOpts &o,
                                                 unsigned char *smem) {
    const int S = o.row_stride;
    const int64_t NV = (N + S - 1) / S;               // rows 0, S, 2S, ... are "virtual" rows 0 .. NV-1
    u4 *qf = reinterpret_cast<u4 *>(smem);            // [NQG][steps][64]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int steps = (d + 31) >> 5;
    const int P = gridDim.x;

    // queries -> LDS, already in B-operand order: fragment (g, s) holds for lane l
    // the 8 values k = 32 s + 8 (l / 16) .. of query q0 + 16 g + l % 16
    for (int idx = tid; idx < NQG * steps * WAVE; idx += blockDim.x) {
        const int l = idx & 63, s = (idx >> 6) % steps, g = (idx >> 6) / steps;
        const int q = q0 + g * 16 + (l & 15), kb = s * 32 + (l >> 4) * 8;
        u4 v = zero_chunk();
        if (q < B && kb < d) v = load_chunk(static_cast<const char *>(Q) + ((size_t)q * d + kb) * 2);
        qf[idx] = v;
    }
    __syncthreads();

    TopList<KP> best[NQG];
    float thr[NQG];
    float bnd_s[NQG];                                 // continuation: this lane's queries' boundary pairs
    int bnd_id[NQG];
    const bool bounded = o.after.s != nullptr;
#pragma unroll
    for (int g = 0; g < NQG; ++g) {
        const int qb = min(q0 + g * 16 + (lane & 15), B - 1);
        bnd_s[g] = bounded ? o.after.s[qb] : 0.f;
        bnd_id[g] = bounded ? o.after.id[qb] : 0;
    }
#pragma unroll
    for (int g = 0; g < NQG; ++g) {
        best[g].init();
        thr[g] = -INFINITY;
        if constexpr (EMIT) {                         // fixed thresholds; queries past B never emit
            const int q = q0 + g * 16 + (lane & 15);
            thr[g] = q < B ? o.thr[q] : INFINITY;
        }
    }

    const int64_t ntiles = (NV + 15) >> 4;
    const int kofs = (lane >> 4) * 8;                 // this lane's k offset inside a 32-wide step
    for (int64_t tile = (int64_t)blockIdx.x * nwaves + wave; tile < ntiles; tile += (int64_t)P * nwaves) {
        int64_t row = tile * 16 + (lane & 15);
        if (row >= NV) row = NV - 1;                  // tail tile: re-read the last row, masked below
        const char *rp = static_cast<const char *>(X) + ((size_t)row * S * d + kofs) * 2;
        f4 acc[NQG];
#pragma unroll
        for (int g = 0; g < NQG; ++g) acc[g] = f4{0.f, 0.f, 0.f, 0.f};

        int s = 0;
        for (; s + STREAM_UNROLL <= steps; s += STREAM_UNROLL) {
            u4 a[STREAM_UNROLL];
#pragma unroll
            for (int u = 0; u < STREAM_UNROLL; ++u) {
                if (DFULL || (s + u) * 32 + kofs < d) a[u] = load_chunk(rp + (size_t)(s + u) * 64);
                else a[u] = zero_chunk();
            }
#pragma unroll
            for (int u = 0; u < STREAM_UNROLL; ++u)
#pragma unroll
                for (int g = 0; g < NQG; ++g)
                    acc[g] = mfma16<T>(a[u], qf[(g * steps + s + u) * WAVE + lane], acc[g]);
        }
        for (; s < steps; ++s) {
            u4 a = zero_chunk();
            if (DFULL || s * 32 + kofs < d) a = load_chunk(rp + (size_t)s * 64);
#pragma unroll
            for (int g = 0; g < NQG; ++g)
                acc[g] = mfma16<T>(a, qf[(g * steps + s) * WAVE + lane], acc[g]);
        }

        const int64_t rbase = tile * 16 + (lane >> 4) * 4;
        if (bounded) {                                // rows at or before a query's boundary do not take part
#pragma unroll
            for (int g = 0; g < NQG; ++g)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[g][i] = after_boundary(acc[g][i], (int)((rbase + i) * S), bnd_s[g], bnd_id[g]);
        }
        static_for<NQG>([&](auto gc) {
            constexpr int g = decltype(gc)::value;
            const f4 a = acc[g];
            const float m = fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3]));
            if (__builtin_amdgcn_ballot_w64(m >= thr[g]) != 0) {        // rare after warm-up
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t r = rbase + i;
                    if constexpr (EMIT) {
                        if (r < NV && a[i] >= thr[g]) {
                            const int q = q0 + g * 16 + (lane & 15);
                            const int slot = atomicAdd(&o.count[q], 1);
                            if (slot < o.cap) partial[(size_t)q * o.cap + slot] = Cand{a[i], (int)(r * S)};
                        }
                    } else {
                        const int id = (int)(r * S);
                        if (r < NV && a[i] >= thr[g] && best[g].admits(a[i], id)) best[g].insert(a[i], id);
                    }
                }
                if constexpr (!EMIT) {
                    // the KP-th best of any lane that serves the same query bounds the final
                    // KP-th best from below, so it is a safe rejection threshold for all four
                    float t = best[g].s[KP - 1];
                    t = fmaxf(t, __shfl_xor(t, 16));
                    t = fmaxf(t, __shfl_xor(t, 32));
                    thr[g] = fmaxf(thr[g], t);
                }
            }
        });
    }

    if constexpr (EMIT) return;
    // the four lanes that share a query -> one list per wave and query
    __syncthreads();                                   // query fragments are dead from here
    Cand *wl = reinterpret_cast<Cand *>(smem);         // [nwaves][NQG*16][KP]
    static_for<NQG>([&](auto gc) {
        constexpr int g = decltype(gc)::value;
        TopList<KP> wbest;
        group_top<KP, KP, 16, 64>(best[g], wbest);
        if (lane < 16) {
#pragma unroll
            for (int j = 0; j < KP; ++j)
                wl[((size_t)wave * NQG * 16 + g * 16 + lane) * KP + j] = Cand{wbest.s[j], wbest.id[j]};
        }
    });
    __syncthreads();
    // the block's list of a query: its NWV wave lists spread over 4 NWV lanes (4 lanes per wave
    // list, KP/4 consecutive entries each), 16 queries per pass of the workgroup
    constexpr int LP = KP / 4, LG = 4 * NWV;
    static_assert((NWV == 8 || NWV == 16) && KP % 4 == 0, "the final selection splits every wave list four ways");
    const int sub = tid & (LG - 1), w = sub >> 2, part = sub & 3;
#pragma unroll
    for (int pass = 0; pass < NQG; ++pass) {
        const int qi = pass * 16 + tid / LG;
        TopList<LP> mine;
#pragma unroll
        for (int j = 0; j < LP; ++j) {
            const Cand c = wl[((size_t)w * NQG * 16 + qi) * KP + part * LP + j];
            mine.s[j] = c.s;
            mine.id[j] = c.id;
        }
        TopList<KP> fin;
        group_top<KP, LP, 1, LG>(mine, fin);
        if (sub == 0 && q0 + qi < B) {
            Cand *out = partial + ((size_t)(q0 + qi) * P + blockIdx.x) * KP;
#pragma unroll
            for (int j = 0; j < KP; ++j) out[j] = Cand{fin.s[j], fin.id[j]};
        }
    }
}

// o.passes consecutive groups of NQG*16 queries starting at q0, one after the other in one launch.
// With o.need, a group is skipped unless need[q] > need_above for one of its queries (the repair
// pass behind the candidate arrays: usually every group is skipped).
template <class T, int NQG, int KP, bool DFULL, bool EMIT, int NWV>
__global__ __launch_bounds__(NWV * 64) void flat_stream_kernel(const void *__restrict__ X, int64_t N, int d,
                                                          const void *__restrict__ Q, int B, int q0,
                                                          Cand *__restrict__ partial, StreamOpts o) {
    extern __shared__ __align__(16) unsigned char smem[];
    for (int pass = 0; pass < o.passes; ++pass, q0 += NQG * 16) {
        if (o.need) {
            const int q = q0 + (int)threadIdx.x;
            const int mine = threadIdx.x < NQG * 16 && q < B && o.need[q] > o.need_above;
            if (!__syncthreads_or(mine)) continue;
        }
        if (pass) __syncthreads();                    // the previous pass is done with the LDS
        flat_stream_pass<T, NQG, KP, DFULL, EMIT, NWV>(X, N, d, Q, B, q0, partial, o, smem);
    }
}

// fp32 corpora.  8 lanes share a row (float4 chunks c, c+8, ...), a wave covers 8
// rows per step, 8 queries per pass live in LDS; lane c of a row group keeps the
// list of query q0 + c.  gridDim = (P slabs, ceil(B / 8)).
//   partial [B, P, KP]
template <int KP>
__global__ __launch_bounds__(256) void flat_f32_kernel(const float *__restrict__ X, int64_t N, int d,
                                                       const float *__restrict__ Q, int B,
                                                       Cand *__restrict__ partial, After after) {
    extern __shared__ __align__(16) unsigned char smem[];
    u4 *qs = reinterpret_cast<u4 *>(smem);            // [8][d/4]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int nch = d >> 2;
    const int q0 = blockIdx.y * 8;
    const int P = gridDim.x;
    for (int idx = tid; idx < 8 * nch; idx += blockDim.x) {
        const int q = q0 + idx / nch, c = idx % nch;
        qs[idx] = q < B ? load_chunk(Q + (size_t)q * d + c * 4) : zero_chunk();
    }
    __syncthreads();

    TopList<KP> best;
    best.init();
    const int r8 = lane >> 3, c8 = lane & 7;
    const int qb = min(q0 + c8, B - 1);               // continuation: the boundary pair of this lane's query
    const float bnd_s = after.s ? after.s[qb] : 0.f;
    const int bnd_id = after.s ? after.id[qb] : 0;
    const int64_t ngroups = (N + 7) >> 3;
    for (int64_t grp = (int64_t)blockIdx.x * nwaves + wave; grp < ngroups; grp += (int64_t)P * nwaves) {
        const int64_t row = grp * 8 + r8;
        const int64_t rowc = row < N ? row : N - 1;
        const float *rp = X + (size_t)rowc * d;
        float acc[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = 0.f;
        for (int c = c8; c < nch; c += 8) {
            const u4 x = load_chunk(rp + c * 4);
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = dot_chunk<F32>(x, qs[q * nch + c], acc[q]);
        }
        float mine = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float v = acc[q];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            if (q == c8) mine = v;
        }
        if (after.s) mine = after_boundary(mine, (int)row, bnd_s, bnd_id);
        if (row < N && best.admits(mine, (int)row)) best.insert(mine, (int)row);
    }
    best.merge_xor(8);
    best.merge_xor(16);
    best.merge_xor(32);

    __syncthreads();
    Cand *wl = reinterpret_cast<Cand *>(smem);         // [nwaves][8][KP]
    if (lane < 8) {
#pragma unroll
        for (int j = 0; j < KP; ++j) wl[((size_t)wave * 8 + lane) * KP + j] = Cand{best.s[j], best.id[j]};
    }
    __syncthreads();
    if (tid < 8 && q0 + tid < B) {
        TopList<KP> fin;
        fin.init();
        for (int w = 0; w < nwaves; ++w)
            for (int j = 0; j < KP; ++j) {
                const Cand c = wl[((size_t)w * 8 + tid) * KP + j];
                if (fin.admits(c.s, c.id)) fin.insert(c.s, c.id);
            }
        Cand *out = partial + ((size_t)(q0 + tid) * P + blockIdx.x) * KP;
#pragma unroll
        for (int j = 0; j < KP; ++j) out[j] = Cand{fin.s[j], fin.id[j]};
    }
}

// One workgroup (1 to 4 wavefronts, by the amount of work) per query: the k best of its
// P*KP partial pairs, written in order; unused tail slots become id -1 / score -inf.
// best <- best of itself and in[first], in[first + stride], ...: eight loads in flight per
// thread, so a short list costs one memory latency instead of one per element
template <int KP>
__device__ __forceinline__ void gather_best(const Cand *__restrict__ in, int total, int first, int stride,
                                            TopList<KP> &best) {
    for (int e0 = first; e0 < total; e0 += 8 * stride) {
        Cand c[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int e = e0 + u * stride;
            c[u] = e < total ? in[e] : Cand{-INFINITY, EMPTY_ID};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (best.admits(c[u].s, c[u].id)) best.insert(c[u].s, c[u].id);
    }
}

// count == null: query q's input is its P lists of KP at partial[q * P * KP ..).  count given: the
// input is the candidate array of count[q] entries at cand[q * cap ..), unless it overflowed
// (count[q] > cap): then the P lists, which the repair pass has filled for exactly those queries.
template <int KP>
__global__ __launch_bounds__(256) void flat_merge_kernel(const Cand *__restrict__ partial, int P, int k,
                                                         int32_t *__restrict__ ids, float *__restrict__ scores,
                                                         const int *__restrict__ count, const Cand *__restrict__ cand,
                                                         int cap) {
    __shared__ Cand wl[4 * KP];
    const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwaves = blockDim.x >> 6;
    int total = P * KP;
    const Cand *in = partial + (size_t)q * P * KP;
    if (count) {
        const int n = count[q];                           // uniform for the workgroup
        if (n <= cap) {
            total = n;
            in = cand + (size_t)q * cap;
        }
    }
    TopList<KP> best;
    best.init();
    gather_best<KP>(in, total, tid, blockDim.x, best);
    TopList<KP> wbest;
    group_top<KP, KP, 1, 64>(best, wbest);
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < KP; ++j) wl[wave * KP + j] = Cand{wbest.s[j], wbest.id[j]};
    }
    __syncthreads();
    if (wave == 0) {                                  // one entry per lane, at most 4 waves x KP <= 64
        TopList<1> one;
        one.init();
        if (lane < nwaves * KP) { one.s[0] = wl[lane].s; one.id[0] = wl[lane].id; }
        TopList<KP> fin;
        group_top<KP, 1, 1, 64>(one, fin);
        if (lane == 0) {
#pragma unroll
            for (int j = 0; j < KP; ++j)
                if (j < k) {
                    const bool has = fin.id[j] != EMPTY_ID;
                    ids[(size_t)q * k + j] = has ? fin.id[j] : -1;
                    scores[(size_t)q * k + j] = has ? fin.s[j] : -INFINITY;
                }
        }
    }
}

// One wavefront per query: the k-th best score among Ps sampled lists of KS entries (src[(q Ps + s) KS ..)),
// -inf when the sample holds fewer than k rows.  The lists come from disjoint rows, so this is the
// k-th best of a subset of the corpus: a lower bound of the final k-th best score.  With dst, the
// sample's KS best are also kept, as slab pslot of the query's lists dst[(q pstride + pslot) KS ..)
// (for a sample whose rows the main pass then skips).  With count, count[q] is set to 0.
template <int KS, int KO>
__global__ __launch_bounds__(64) void flat_sample_kth_kernel(const Cand *__restrict__ src, int Ps, int k,
                                                             float *__restrict__ thr, Cand *__restrict__ dst,
                                                             int pstride, int pslot, int *__restrict__ count) {
    const int q = blockIdx.x, lane = threadIdx.x;
    TopList<KO> best;
    best.init();
    gather_best<KO>(src + (size_t)q * Ps * KS, Ps * KS, lane, 64, best);
    TopList<KO> top;
    group_top<KO, KO, 1, 64>(best, top);
    if (lane == 0) {
        float t = -INFINITY;
#pragma unroll
        for (int j = 0; j < KO; ++j)
            if (j == k - 1 && top.id[j] != EMPTY_ID) t = top.s[j];
        thr[q] = t;
        if (count) count[q] = 0;                      // the query's candidate array starts empty
        if (dst) {
#pragma unroll
            for (int j = 0; j < KS; ++j) dst[((size_t)q * pstride + pslot) * KS + j] = Cand{top.s[j], top.id[j]};
        }
    }
}

}  // namespace ann
