// flat_wide_kernel instantiations and launcher.
#include "flat_wide_kernel.hpp"
#include "launch.hpp"

namespace ann {
namespace {
template <class T, int WNF, int NWN, bool SELECT>
hipError_t launch(const void *X, int64_t N, int d, const void *Q, int B, Cand *partial, int P, int NTG,
                  int64_t tile_begin, const float *thr_init, int pstride, int pslot0, hipStream_t stream) {
    static size_t big = 0;
    using C = WideCfg<WNF, NWN>;
    const size_t lds = C::DYN_LDS_BYTES;
    if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&flat_wide_kernel<T, WNF, NWN, SELECT>), lds, &big))
        return e;
    hipLaunchKernelGGL((flat_wide_kernel<T, WNF, NWN, SELECT>), dim3(P * NTG), dim3(C::THREADS), lds, stream, X, N, d,
                       Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0);
    return hipGetLastError();
}

template <class T, bool SELECT>
hipError_t launch_tile(const void *X, int64_t N, int d, const void *Q, int B, Cand *partial, int P, int NTG,
                       int64_t tile_begin, const float *thr_init, int pstride, int pslot0, hipStream_t stream) {
    return wide_query_tile(B) == 128
               ? launch<T, 2, 2, SELECT>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, stream)
               : launch<T, 2, 4, SELECT>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, stream);
}
}  // namespace

int wide_query_tile(int B) { return B <= 128 ? 128 : 256; }

hipError_t launch_flat_wide(int dtype, bool select, const void *X, int64_t N, int d, const void *Q, int B,
                            Cand *partial, int P, int NTG, int64_t tile_begin, const float *thr_init, int pstride,
                            int pslot0, hipStream_t stream) {
    if (dtype == 0)
        return select ? launch_tile<F16, true>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, stream)
                      : launch_tile<F16, false>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, stream);
    return select ? launch_tile<BF16, true>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, stream)
                  : launch_tile<BF16, false>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, stream);
}

}  // namespace ann
