// Exact (flat) retrieval for large query batches (Section 2.1 of the paper: exact
// retrieval; the batch stands for the agent's concurrent requests).  The score
// matrix S = X Q^T is a dense contraction, so it runs on the matrix cores:
//
//   workgroup tile  256 corpus rows x BN queries, 2 x NWN wavefronts
//   wavefront tile  128 rows x 32 WNF queries = 4 x WNF MFMA 32x32x16 accumulators
//                   (BN = 32 WNF NWN: 128 = 2x2 waves of 128x64, 256 = 2x4 waves of 128x64)
//   K loop          32 columns of d (64 bytes of a row) per stage, 4 LDS stages; every
//                   stage is filled by direct global->LDS loads issued three stages
//                   ahead.  One load instruction brings 16 rows x 64 B (4 lanes per row,
//                   whole half cache lines) and lands as a 1 KB block of 16 rows; inside
//                   a row the four 16-byte chunks sit in slots XOR-swizzled by the row
//                   number, so the MFMA operand reads (32 rows x one chunk) hit all banks
//   epilogue        each lane owns WNF queries (the MFMA column) and 64 rows per tile;
//                   scores below the query's running threshold (the workgroup's k-th
//                   best so far, shared through LDS) are dropped with one compare; the
//                   rest pass through a per-wave LDS queue into the owning lane's sorted
//                   register list
//
// S is never written.  A workgroup walks a slab of corpus tiles for one query tile and
// leaves its k best per query in partial[B, P, KP].
#pragma once

#include "common.hpp"

namespace ann {

constexpr int WIDE_BM = 256;          // corpus rows per workgroup tile
constexpr int WIDE_STAGES = 4;
constexpr int WIDE_KP = 4;            // list length (k <= 4 on this path)
constexpr int WIDE_QCAP = 128;        // entries of a wave's pass queue (drained when > 64 are queued)

template <int WNF, int NWN>
struct WideCfg {
    static constexpr int WAVES = 2 * NWN;
    static constexpr int THREADS = WAVES * WAVE;
    static constexpr int BN = 32 * WNF * NWN;           // queries per workgroup tile
    static constexpr int A_FRAGS = 16;                  // 8 row blocks x 2 k-halves
    static constexpr int B_FRAGS = 2 * WNF * NWN;       // BN/32 column blocks x 2 k-halves
    static constexpr int FRAGS = A_FRAGS + B_FRAGS;     // 1 KB each
    static constexpr int LPW = FRAGS / WAVES;           // fragments loaded per wave and stage
    static_assert(FRAGS % WAVES == 0, "fragments must divide evenly over the waves");
    static constexpr int STAGE_BYTES = FRAGS * 1024;
    // The 128-query tile has 4 waves only: three stages of 24 KB (and the exchange buffer inside
    // them) let two such workgroups share a compute unit, so every SIMD still holds two waves.
    static constexpr int STAGES = NWN == 2 ? 3 : WIDE_STAGES;
    static constexpr int XCH_BYTES = 2 * BN * WIDE_KP * (int)sizeof(Cand);
    static_assert(XCH_BYTES <= STAGES * STAGE_BYTES, "the exchange buffer lives in the stage buffers");
    static constexpr int DYN_LDS_BYTES = STAGES * STAGE_BYTES;
};

// order-preserving map float -> int (for atomicMax on thresholds)
__device__ __forceinline__ int float_key(float f) {
    const int b = __float_as_int(f);
    return b >= 0 ? b : b ^ 0x7fffffff;
}
__device__ __forceinline__ float key_float(int k) { return __int_as_float(k >= 0 ? k : k ^ 0x7fffffff); }

#define ANN_GLOBAL_TO_LDS_16(gptr, lptr)                                                          \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gptr),      \
                                     (__attribute__((address_space(3))) void *)(lptr), 16, 0, 0)

// wait until at most `n` of this wave's vector-memory operations are outstanding
template <int n>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(n >= 0 && n < 64, "vmcnt is a 6-bit field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (n & 15) | ((n >> 4) << 14));
}

// LDS atomic max without a return value.  Written as an instruction because the
// compiler, seeing an LDS store while direct global->LDS loads are in flight, would
// first wait for every one of those loads (it cannot tell the targets apart); the
// threshold words never overlap a stage buffer.
__device__ __forceinline__ void lds_atomic_max(int *p, int v) {
    const uint32_t a = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) int *)p);
    asm volatile("ds_max_i32 %0, %1" ::"v"(a), "v"(v) : "memory");
}

__device__ __forceinline__ void lds_store(void *p, int v) {   // same reason as lds_atomic_max
    const uint32_t a = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) void *)p);
    asm volatile("ds_write_b32 %0, %1" ::"v"(a), "v"(v) : "memory");
}

__device__ __forceinline__ void lds_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

//   X [N, d], Q [B, d] 16-bit, d a multiple of 32.   partial [B, P, WIDE_KP]
//   gridDim.x = P * NTG; block -> (slab, query-tile group), same-slab blocks on one XCD
//   rows [256 tile_begin, N) are scanned, split into P slabs of whole tiles.
//   thr_init (optional, [B]): per query a lower bound of its final k-th best score (the k-th best
//   of a sample of the corpus); rows scoring below it are dropped at once.
//   Slab s of query q is written to partial[(q * pstride + pslot0 + s) * KP ..).
//   MODE WIDE_LISTS: the epilogue described above.
//   MODE WIDE_SELECT: threshold-free epilogue (per lane the KP best of its 64 scores by repeated
//   maximum), constant cost; meant for the short sampling pass that produces thr_init.  Only in
//   this mode, row_stride > 1 scans rows 0, S, 2S, ... instead of every row (tile_begin and the
//   slabs then count tiles of 256 such rows).
//   MODE WIDE_EMIT (k > 4): no lists at all.  thr_init[q] must be a lower bound of query q's final
//   k-th best score (the k-th best of a sample); every (score, row) with score >= thr_init[q] is
//   appended to the query's candidate array partial[q * pstride ..) through the counter
//   emit_count[q] (entries beyond pstride are counted but not stored: the caller then knows that
//   the array overflowed and recomputes that query another way).
constexpr int WIDE_LISTS = 0, WIDE_SELECT = 1, WIDE_EMIT = 2;
template <class T, int WNF, int NWN, int MODE>
__global__ __launch_bounds__(128 * NWN, 2) void flat_wide_kernel(const void *__restrict__ X, int64_t N, int d,
                                                                    const void *__restrict__ Q, int B,
                                                                    Cand *__restrict__ partial, int P, int NTG,
                                                                    int64_t tile_begin,
                                                                    const float *__restrict__ thr_init,
                                                                    int pstride, int pslot0,
                                                                    int *__restrict__ emit_count, int row_stride,
                                                                    After after) {
    constexpr bool SELECT = MODE == WIDE_SELECT;
    // WIDE_SELECT may scan every row_stride-th row only (rows 0, S, 2S, ...): all the tiling below
    // then runs over these NV "virtual" rows, and only addresses and reported ids use S
    const int S = SELECT ? row_stride : 1;
    const int64_t NV = SELECT ? (N + S - 1) / S : N;
    using C = WideCfg<WNF, NWN>;
    constexpr int KP = WIDE_KP, NST = C::STAGES, LPW = C::LPW;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *stage_mem = smem;                  // dynamic LDS: the stage buffers ...
    Cand *xch = reinterpret_cast<Cand *>(smem);       // ... reused as [2][BN][KP] once a slab is done
    // separate LDS objects, so that stores to them are known not to touch a stage buffer
    // a direct global->LDS load may still be writing (no wait on those loads is needed)
    __shared__ int thr_l[C::BN];
    __shared__ float wq_s[C::WAVES * WIDE_QCAP];      // per-wave queue of passing scores:
    __shared__ int wq_r[C::WAVES * WIDE_QCAP];        //   score, row id, owning lane
    __shared__ int wq_l[C::WAVES * WIDE_QCAP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int ksteps = d >> 5;

    // blocks are dealt to the 8 XCDs round-robin; make the blocks that share a corpus
    // slab neighbours on one XCD so the slab is fetched from HBM once into that L2
    int lb = blockIdx.x;
    const int G = gridDim.x;
    if ((G & 7) == 0) lb = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);
    const int ntg = lb % NTG, slab = lb / NTG;
    const int NT = (B + C::BN - 1) / C::BN;
    const int64_t mtiles = (NV + WIDE_BM - 1) / WIDE_BM - tile_begin;
    const int64_t t0 = tile_begin + mtiles * slab / P, t1 = tile_begin + mtiles * (slab + 1) / P;
    const int total = (int)(t1 - t0) * ksteps;

    for (int nt = ntg; nt < NT; nt += NTG) {
        const int n0 = nt * C::BN;
        TopList<KP> best[WNF];
        float thr[WNF];
        static_for<WNF>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            best[j].init();
            thr[j] = -INFINITY;
            const int q = n0 + (wn * WNF + j) * 32 + l32;
            if constexpr (MODE == WIDE_EMIT) {               // fixed thresholds; queries past B never emit
                thr[j] = q < B ? thr_init[q] : INFINITY;
            } else if (thr_init) {
                thr[j] = thr_init[q < B ? q : B - 1];
            }
        });
        if (tid < C::BN) {
            const int q = n0 + tid < B ? n0 + tid : B - 1;
            thr_l[tid] = float_key(thr_init ? thr_init[q] : -INFINITY);
        }
        // continuation: the boundary pairs of this lane's WNF queries
        float bnd_s[WNF];
        int bnd_id[WNF];
        static_for<WNF>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int q = min(n0 + (wn * WNF + j) * 32 + l32, B - 1);
            bnd_s[j] = after.s ? after.s[q] : 0.f;
            bnd_id[j] = after.s ? after.id[q] : 0;
        });

        // Block e of a stage (1 KB = 16 rows x 64 B): blocks 0..15 corpus rows, the rest
        // queries.  Lane l fetches row l/4 of the block; LDS slot l%4 of that row receives
        // chunk (l%4) ^ ((row/4)%4) of the stage's 64 bytes.
        const int my_chunk = (lane & 3) ^ ((lane >> 4) & 3);
        // Address of a load = uniform base (corpus: start of the tile, advanced per k step;
        // queries: start of the query tile) + a 32-bit per-lane offset that does not change
        // from tile to tile, except in the ragged last tile where rows are clamped to N-1.
        uint32_t loff[LPW];
        auto lane_offsets = [&](int64_t tile) {
#pragma unroll
            for (int e = 0; e < LPW; ++e) {
                const int blk = wave * LPW + e;
                if (blk < C::A_FRAGS) {
                    int64_t row = tile * WIDE_BM + blk * 16 + (lane >> 2);
                    row = row < NV ? row : NV - 1;
                    loff[e] = (uint32_t)(row - tile * WIDE_BM) * (uint32_t)(d * 2 * S) + my_chunk * 16;
                } else {
                    int q = n0 + (blk - C::A_FRAGS) * 16 + (lane >> 2);
                    q = q < B ? q : B - 1;
                    loff[e] = (uint32_t)(q - n0) * (uint32_t)(d * 2) + my_chunk * 16;
                }
            }
        };
        lane_offsets(t0);
        const char *xbase = static_cast<const char *>(X) + (size_t)t0 * WIDE_BM * d * 2 * S;   // tile start + k step
        const char *qbase = static_cast<const char *>(Q) + (size_t)n0 * d * 2;
        int iks = 0;                                         // k step of the next stage to issue
        int64_t itile = t0;
        auto issue = [&](int it) {
            unsigned char *sbase = stage_mem + (it % NST) * C::STAGE_BYTES;
#pragma unroll
            for (int e = 0; e < LPW; ++e) {
                const int blk = wave * LPW + e;
                const char *base = blk < C::A_FRAGS ? xbase : qbase;
                ANN_GLOBAL_TO_LDS_16(base + iks * 64 + loff[e], sbase + blk * 1024);
            }
            if (++iks == ksteps) {
                iks = 0;
                ++itile;
                xbase += (size_t)WIDE_BM * d * 2 * S;
                if ((itile + 1) * WIDE_BM > NV && itile < t1) lane_offsets(itile);   // ragged last tile
            }
        };

        f16v acc[4][WNF];
        auto clear_acc = [&]() {
            static_for<4>([&](auto ic) {
                static_for<WNF>([&](auto jc) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[decltype(ic)::value][decltype(jc)::value][r] = 0.f;
                });
            });
        };
        clear_acc();

        __syncthreads();                                     // thr_l initialised; stage buffers idle
        for (int it = 0; it < NST - 1 && it < total; ++it) issue(it);

        int cks = 0;                                         // k step being computed
        int64_t ctile = t0;                                  // tile being computed
        for (int it = 0; it < total; ++it) {
            // stage `it` has landed once only the newer stages' loads are outstanding
            if (NST >= 4 && it + 2 < total) wait_vmcnt<2 * LPW>();
            else if (it + 1 < total) wait_vmcnt<LPW>();
            else wait_vmcnt<0>();
            lds_barrier();                                   // ... for every wave; buffer (it-1)%NST is free
            if (it + NST - 1 < total) issue(it + NST - 1);

            const unsigned char *sb = stage_mem + (it % NST) * C::STAGE_BYTES;
            {
                // operand row r = lane % 32 of a 32-row block pair, chunk 2 kh + lane / 32.
                // All operand reads of the stage are issued before the first MFMA, so the
                // LDS pipeline always has a dozen 1 KB reads of this wave in flight.
                const int r = l32;
                u4 a[2][4], b[2][WNF];
#pragma unroll
                for (int kh = 0; kh < 2; ++kh) {
                    const int lofs = (r >> 4) * 1024 + (r & 15) * 64 + (((2 * kh + lhi) ^ ((r >> 2) & 3)) * 16);
#pragma unroll
                    for (int j = 0; j < WNF; ++j)
                        b[kh][j] = *reinterpret_cast<const u4 *>(sb + (C::A_FRAGS + (wn * WNF + j) * 2) * 1024 + lofs);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        a[kh][i] = *reinterpret_cast<const u4 *>(sb + (wm * 8 + i * 2) * 1024 + lofs);
                }
                __builtin_amdgcn_sched_barrier(0);           // keep the reads ahead of the MFMAs
                static_for<2>([&](auto kc) {
                    constexpr int kh = decltype(kc)::value;
                    static_for<4>([&](auto ic) {
                        static_for<WNF>([&](auto jc) {
                            constexpr int i = decltype(ic)::value, j = decltype(jc)::value;
                            acc[i][j] = mfma32<T>(a[kh][i], b[kh][j], acc[i][j]);
                        });
                    });
                });
            }

            if (++cks == ksteps) {                           // a tile of scores is complete
                cks = 0;
                const int64_t tile = ctile++;
                const int rbase = (int)(tile * WIDE_BM) + wm * 128 + 4 * lhi;    // N < 2^31
                const int nrows = (int)NV;
                if ((tile + 1) * WIDE_BM > NV) {               // ragged last tile: rows >= N never score
                    // (NaN, not -inf: a NaN passes no threshold and enters no list, whereas -inf would
                    // pass a threshold of -inf, which is what a sample with fewer than k rows gives)
                    static_for<4>([&](auto ic) {
                        constexpr int i = decltype(ic)::value;
                        static_for<WNF>([&](auto jc) {
                            constexpr int j = decltype(jc)::value;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (rbase + (i * 32 + 8 * (r / 4) + (r % 4)) >= nrows) acc[i][j][r] = __builtin_nanf("");
                        });
                    });
                }
                if (after.s) {                                 // rows at or before a query's boundary do not take part
                    static_for<4>([&](auto ic) {
                        constexpr int i = decltype(ic)::value;
                        static_for<WNF>([&](auto jc) {
                            constexpr int j = decltype(jc)::value;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                acc[i][j][r] = after_boundary(acc[i][j][r], (rbase + (i * 32 + 8 * (r / 4) + (r % 4))) * S,
                                                              bnd_s[j], bnd_id[j]);
                        });
                    });
                }
                if constexpr (MODE == WIDE_EMIT) {
                    static_for<WNF>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        const float t = thr[j];
                        float m = acc[0][j][0];
                        static_for<4>([&](auto ic) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) m = fmaxf(m, acc[decltype(ic)::value][j][r]);
                        });
                        if (__builtin_amdgcn_ballot_w64(m >= t) != 0) {      // rare: some hundred rows per query in all
                            const int q = n0 + (wn * WNF + j) * 32 + l32;
                            uint32_t mask[2] = {0u, 0u};                      // accumulator e passes: bit e
                            static_for<4>([&](auto ic) {
                                constexpr int i = decltype(ic)::value;
#pragma unroll
                                for (int r = 0; r < 16; ++r) mask[i / 2] |= acc[i][j][r] >= t ? 1u << ((i & 1) * 16 + r) : 0u;
                            });
                            uint64_t left = ((uint64_t)mask[1] << 32) | mask[0];
                            while (left != 0) {
                                const int e = __builtin_ctzll(left);
                                left &= left - 1;
                                float s = 0.f;
                                static_for<4>([&](auto ic) {
                                    constexpr int i = decltype(ic)::value;
#pragma unroll
                                    for (int r = 0; r < 16; ++r) s = (e == i * 16 + r) ? acc[i][j][r] : s;
                                });
                                const int slot = atomicAdd(&emit_count[q], 1);
                                const int r = e & 15;
                                if (slot < pstride)
                                    partial[(size_t)q * pstride + slot] = Cand{s, rbase + (e >> 4) * 32 + 8 * (r >> 2) + (r & 3)};
                            }
                        }
                    });
                } else if constexpr (SELECT) {
                    static_for<WNF>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
#pragma unroll
                        for (int round = 0; round < KP; ++round) {
                            float m = -INFINITY;
                            static_for<4>([&](auto ic) {
#pragma unroll
                                for (int r = 0; r < 16; ++r) m = fmaxf(m, acc[decltype(ic)::value][j][r]);
                            });
                            int idx = 64;                          // first accumulator holding the maximum
                            static_for<4>([&](auto ic) {
                                constexpr int i = decltype(ic)::value;
#pragma unroll
                                for (int r = 0; r < 16; ++r) idx = min(idx, acc[i][j][r] == m ? i * 16 + r : 64);
                            });
                            static_for<4>([&](auto ic) {
                                constexpr int i = decltype(ic)::value;
#pragma unroll
                                for (int r = 0; r < 16; ++r) acc[i][j][r] = (i * 16 + r == idx) ? -INFINITY : acc[i][j][r];
                            });
                            // accumulator e = 16 i + r holds tile row 32 i + 8 (r / 4) + r % 4 (+ 4 lhi), so
                            // the first maximum in accumulator order is also the one with the lowest row id
                            const int r = idx & 15;
                            const int row = rbase + (idx >> 4) * 32 + 8 * (r >> 2) + (r & 3);
                            if (m > -INFINITY && best[j].admits(m, row * S)) best[j].insert(m, row * S);
                        }
                    });
                } else {
                static_for<WNF>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    const int ql = (wn * WNF + j) * 32 + l32;
                    // with a sampled threshold the workgroup's own running k-th best (a bound from
                    // 1/P of the corpus) never overtakes it: the shared word is left alone
                    float t = thr[j];
                    if (!thr_init) t = fmaxf(t, key_float(thr_l[ql]));
                    float gm[4];                             // best score of each 32-row block
                    static_for<4>([&](auto ic) {
                        constexpr int i = decltype(ic)::value;
                        gm[i] = acc[i][j][0];
#pragma unroll
                        for (int r = 1; r < 16; ++r) gm[i] = fmaxf(gm[i], acc[i][j][r]);
                    });
                    if (t == -INFINITY) {
                        // no threshold yet: the 8 block maxima of this lane pair come from 8
                        // distinct rows, so their KP-th largest bounds the final KP-th best
                        TopList<KP> w;
                        w.init();
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float mine = gm[i], other = __shfl_xor(gm[i], 32);
                            if (w.admits(mine, 2 * i)) w.insert(mine, 2 * i);
                            if (w.admits(other, 2 * i + 1)) w.insert(other, 2 * i + 1);
                        }
                        t = w.s[KP - 1];
                    }
                    const float m = fmaxf(fmaxf(gm[0], gm[1]), fmaxf(gm[2], gm[3]));
                    if (__builtin_amdgcn_ballot_w64(m >= t) != 0) {
                        // Scores that pass go through a small per-wave LDS queue and are then
                        // inserted one by one by the lane that owns them, so there is one
                        // insert body per query fragment, not one per accumulator.  If the
                        // queue fills up, the pass stops there, the queue is drained (which
                        // tightens the threshold) and the pass resumes at that accumulator.
                        int start = 0;
                        do {
                            int cnt = 0, stop = 64;
                            static_for<4>([&](auto ic) {
                                constexpr int i = decltype(ic)::value;
                                // only 32-row blocks whose maximum passes are looked at; their 16
                                // compare masks are formed first, then walked by scalar code
                                if (__builtin_amdgcn_ballot_w64(gm[i] >= t) != 0 && i * 16 + 15 >= start && stop == 64) {
                                    uint64_t masks[16];
#pragma unroll
                                    for (int r = 0; r < 16; ++r) masks[r] = __builtin_amdgcn_ballot_w64(acc[i][j][r] >= t);
                                    static_for<16>([&](auto rc) {
                                        constexpr int r = decltype(rc)::value;
                                        constexpr int idx = i * 16 + r;
                                        const uint64_t mask = masks[r];
                                        if (mask != 0 && idx >= start && stop == 64) {
                                            const int n = __builtin_popcountll(mask);
                                            if (cnt + n > WIDE_QCAP) {
                                                stop = idx;
                                            } else {
                                                if ((mask >> lane) & 1) {
                                                    const int pos = wave * WIDE_QCAP + cnt +
                                                                    __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                        __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
                                                    lds_store(&wq_s[pos], __float_as_int(acc[i][j][r]));
                                                    lds_store(&wq_r[pos], rbase + (i * 32 + 8 * (r / 4) + (r % 4)));
                                                    lds_store(&wq_l[pos], lane);
                                                }
                                                cnt += n;
                                            }
                                        }
                                    });
                                }
                            });
                            for (int e = 0; e < cnt; ++e) {
                                const float s = wq_s[wave * WIDE_QCAP + e];
                                const int row = wq_r[wave * WIDE_QCAP + e];
                                if (wq_l[wave * WIDE_QCAP + e] == lane && best[j].admits(s, row)) best[j].insert(s, row);
                            }
                            // a lane's KP-th best bounds the final KP-th best from below: publish it
                            float mine = best[j].s[KP - 1];
                            mine = fmaxf(mine, __shfl_xor(mine, 32));
                            if (mine > t) {
                                if (!thr_init) lds_atomic_max(&thr_l[ql], float_key(mine));
                                t = mine;
                            }
                            start = stop;
                        } while (start < 64);
                    }
                    thr[j] = t;
                });
                }
                clear_acc();
            }
        }

        if constexpr (MODE == WIDE_EMIT) {
            __syncthreads();                                 // thr_l is reused by the next query tile
            continue;
        }
        // lanes l and l^32 hold the same queries; then the two wm-waves meet in LDS
        static_for<WNF>([&](auto jc) { best[decltype(jc)::value].merge_xor(32); });
        __syncthreads();                                     // every wave is done with the stage buffers
        if (lhi == 0) {
            static_for<WNF>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                const int ql = (wn * WNF + j) * 32 + l32;
#pragma unroll
                for (int e = 0; e < KP; ++e) xch[(wm * C::BN + ql) * KP + e] = Cand{best[j].s[e], best[j].id[e]};
            });
        }
        __syncthreads();
        if (tid < C::BN && n0 + tid < B) {
            TopList<KP> fin;
            fin.init();
            for (int w = 0; w < 2; ++w)
                for (int e = 0; e < KP; ++e) {
                    const Cand c = xch[(w * C::BN + tid) * KP + e];
                    if (fin.admits(c.s, c.id)) fin.insert(c.s, c.id);
                }
            Cand *out = partial + ((size_t)(n0 + tid) * pstride + pslot0 + slab) * KP;
#pragma unroll
            for (int e = 0; e < KP; ++e) out[e] = Cand{fin.s[e], fin.id[e]};
        }
        __syncthreads();                                     // xch and thr_l are reused by the next query tile
    }
}

}  // namespace ann
