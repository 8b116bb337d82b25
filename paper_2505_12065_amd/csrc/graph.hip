// graph_search_kernel instantiations, LDS layout and launcher.
#include "graph_kernel.hpp"

namespace ann {

GraphLds graph_lds_layout(int d, int elem_bytes, int R, int ef) {
    auto up = [](uint32_t x) { return (x + 15u) & ~15u; };
    const bool inplace = ef > GRAPH_EF_DOUBLE;           // long lists: one buffer, merged in place
    auto lay = [&](uint32_t bits) {
        GraphLds L{};
        uint32_t off = 0;
        L.rp = (uint32_t)((R + ROWS_PER_PASS - 1) / ROWS_PER_PASS * ROWS_PER_PASS);
        L.cache_bits = bits;
        L.q = off; off = up(off + (uint32_t)d * elem_bytes);
        // score lists are padded to 64 entries; lists of up to 256 entries get buffers of 256, which
        // the scan for the next unexpanded entry then reads without conditions
        const uint32_t ef64 = ef <= GRAPH_DELTA ? (uint32_t)GRAPH_DELTA : ((uint32_t)ef + 63u) & ~63u;
        const uint32_t efi = ef <= GRAPH_DELTA ? (uint32_t)GRAPH_DELTA : (uint32_t)ef;
        L.ls0 = off; off = up(off + 4u * ef64);
        if (inplace) L.ls1 = L.ls0; else { L.ls1 = off; off = up(off + 4u * ef64); }
        L.li0 = off; off = up(off + 4u * efi);
        if (inplace) L.li1 = L.li0; else { L.li1 = off; off = up(off + 4u * efi); }
        L.cs = off; off = up(off + 4u * L.rp);
        L.ci = off; off = up(off + 4u * L.rp);
        L.cpos = off; off = up(off + 4u * L.rp);
        L.cache = off; off = up(off + (4u << bits));
        L.ctl = off; off = up(off + 16u);
        L.adj = off; off = up(off + 2u * 4u * RMAX_LDS);
        L.um = off; off = up(off + 8u * (((uint32_t)ef + 63u) / 64u) + 32u);   // the scans use um[0 .. 3] at any ef
        L.rq = off; off = up(off + 4u * L.rp);
        L.co = off; off = up(off + 4u * L.rp);
        L.total = off;
        return L;
    };
    // Long lists on graphs of at most 32 slots per node: the two-level list.  The large part has one
    // buffer of ef entries, the small part two of GRAPH_DELTA; the adjacency rows read ahead take 32
    // slots each; the words of um double as the position marks of a rebuild; there is no id cache.
    auto lay2 = [&] {
        GraphLds L{};
        L.rp = ROWS_PER_PASS;
        L.cache_bits = 0;                                  // no id cache: the visited set is asked first
        L.two_level = 1;
        L.ls0 = TL_LS0; L.li0 = TL_LI0; L.ls1 = TL_LS1; L.li1 = TL_LI1;
        L.cs = TL_CS; L.ci = TL_CI; L.cpos = TL_CPOS;
        L.ctl = L.cache = TL_CTL;
        L.adj = TL_ADJ;
        L.um = L.rq = L.co = TL_UM;                        // (rq, co: used by the plain loop only)
        L.ms = TL_MS;
        L.mi = up(L.ms + 4u * (uint32_t)ef);
        L.q = up(L.mi + 4u * (uint32_t)ef);
        L.total = up(L.q + (uint32_t)d * elem_bytes);
        return L;
    };
    // (it is the only layout of such lists on such graphs: the software-pipelined loop has no code for
    // a single list of more than 512 entries; with d <= ANN_D_MAX it always fits)
    if (ef > GRAPH_EF_TWO_LEVEL && R <= ROWS_PER_PASS) return lay2();
    // cache slots: a few times the number of nodes a search scores (about 10 ef), at most 2^14;
    // fewer when that lets two workgroups share a compute unit, or when the list needs the room
    uint32_t want = 10;
    while ((1u << want) < 32u * (uint32_t)ef && want < 14) ++want;
    uint32_t bits = want;
    if (lay(11).total <= LDS_MAX / 2)
        while (bits > 11 && lay(bits).total > LDS_MAX / 2) --bits;
    while (bits > 10 && lay(bits).total > LDS_MAX) --bits;
    return lay(bits);
}

namespace {
template <class T, int RPT, bool NS, bool QREG = true, bool LONG = false>
hipError_t launch_rp(const void *X, int64_t N, int d, const int32_t *graph, int R, int entry, const void *Q, int B,
                     int k, int ef, int32_t *ids, float *scores, const GraphLds &L, const NonStall &ns,
                     hipStream_t stream) {
    static size_t big = 0;
    if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&graph_search_kernel<T, RPT, NS, QREG, LONG>), L.total, &big))
        return e;
    hipLaunchKernelGGL((graph_search_kernel<T, RPT, NS, QREG, LONG>), dim3(B), dim3(GRAPH_THREADS), L.total, stream, X, N, d,
                       graph, R, entry, Q, k, ef, ids, scores, L, ns);
    return hipGetLastError();
}

template <class T, bool NS>
hipError_t launch(const void *X, int64_t N, int d, const int32_t *graph, int R, int entry, const void *Q, int B,
                  int k, int ef, int32_t *ids, float *scores, const GraphLds &L, const NonStall &ns,
                  hipStream_t stream) {
    // More queries than two workgroups per compute unit hold at once, and a layout small enough for
    // three: the variant that reads the query from LDS and runs three per compute unit.
    if constexpr (!NS) {
        if (L.rp == 32 && B > GRAPH_DENSE_MIN_B && 3 * (size_t)L.total + 3 * 1024 <= LDS_MAX)
            return launch_rp<T, 32, false, false>(X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream);
    }
    if constexpr (NS) {
        if (L.two_level)
            return launch_rp<T, 32, true, true, true>(X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream);
    } else if (L.two_level) {
        return hipErrorInvalidValue;                      // long lists run with the exact visited set
    }
    return L.rp == 32 ? launch_rp<T, 32, NS>(X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream)
                      : launch_rp<T, 0, NS>(X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream);
}

template <bool NS>
hipError_t launch_dtype(int dtype, const void *X, int64_t N, int d, const int32_t *graph, int R, int entry,
                        const void *Q, int B, int k, int ef, int32_t *ids, float *scores, const GraphLds &L,
                        const NonStall &ns, hipStream_t stream) {
    switch (dtype) {
    case 0: return launch<F16, NS>(X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream);
    case 1: return launch<BF16, NS>(X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream);
    default: return launch<F32, NS>(X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream);
    }
}
}  // namespace

hipError_t launch_graph_search(int dtype, const void *X, int64_t N, int d, const int32_t *graph, int R, int entry,
                               const int32_t *entries, int n_entries, const void *Q, int B, int k, int ef, int32_t *ids,
                               float *scores, const GraphLds &L, hipStream_t stream) {
    NonStall ns{};
    ns.entries = entries;
    ns.n_entries = n_entries;
    return launch_dtype<false>(dtype, X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream);
}

hipError_t launch_zero_words(uint32_t *p, size_t words, hipStream_t stream) {
    const size_t n16 = words / 4;
    const size_t blocks = (n16 + 255) / 256;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, stream,
                       reinterpret_cast<u4 *>(p), n16);
    return hipGetLastError();
}

hipError_t launch_gather_ids(const int32_t *table, int64_t M, const int32_t *idx, int64_t n, int32_t *out,
                             hipStream_t stream) {
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(gather_ids_kernel, dim3((unsigned)(blocks < 1024 ? blocks : 1024)), dim3(256), 0, stream, table,
                       M, idx, n, out);
    return hipGetLastError();
}

hipError_t launch_graph_search_nonstall(int dtype, const void *X, int64_t N, int d, const int32_t *graph, int R,
                                        int entry, const void *Q, int B, int k, int ef, int32_t *ids, float *scores,
                                        const GraphLds &L, const NonStall &ns, hipStream_t stream) {
    return launch_dtype<true>(dtype, X, N, d, graph, R, entry, Q, B, k, ef, ids, scores, L, ns, stream);
}

}  // namespace ann
