// flat_wide_kernel instantiations and launcher.
#include "flat_wide_kernel.hpp"
#include "launch.hpp"

namespace ann {
namespace {
template <class T, int WNF, int NWN, int MODE>
hipError_t launch(const void *X, int64_t N, int d, const void *Q, int B, Cand *partial, int P, int NTG,
                  int64_t tile_begin, const float *thr_init, int pstride, int pslot0, int *emit_count, int row_stride,
                  After after, hipStream_t stream) {
    static size_t big = 0;
    using C = WideCfg<WNF, NWN>;
    const size_t lds = C::DYN_LDS_BYTES;
    if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&flat_wide_kernel<T, WNF, NWN, MODE>), lds, &big))
        return e;
    hipLaunchKernelGGL((flat_wide_kernel<T, WNF, NWN, MODE>), dim3(P * NTG), dim3(C::THREADS), lds, stream, X, N, d,
                       Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, emit_count, row_stride, after);
    return hipGetLastError();
}

template <class T, int MODE>
hipError_t launch_tile(const void *X, int64_t N, int d, const void *Q, int B, Cand *partial, int P, int NTG,
                       int64_t tile_begin, const float *thr_init, int pstride, int pslot0, int *emit_count, int row_stride,
                  After after, hipStream_t stream) {
    return wide_query_tile(B) == 128
               ? launch<T, 2, 2, MODE>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, emit_count, row_stride, after, stream)
               : launch<T, 2, 4, MODE>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, emit_count, row_stride, after, stream);
}
}  // namespace

int wide_query_tile(int B) { return B <= 128 ? 128 : 256; }

hipError_t launch_flat_wide(int dtype, int mode, const void *X, int64_t N, int d, const void *Q, int B,
                            Cand *partial, int P, int NTG, int64_t tile_begin, const float *thr_init, int pstride,
                            int pslot0, int *emit_count, int row_stride, After after, hipStream_t stream) {
#define ANN_WIDE_CASE(TYPE, MODE)                                                                                    \
    return launch_tile<TYPE, MODE>(X, N, d, Q, B, partial, P, NTG, tile_begin, thr_init, pstride, pslot0, emit_count, \
                                   row_stride, after, stream)
    if (dtype == 0) {
        if (mode == WIDE_SELECT) ANN_WIDE_CASE(F16, WIDE_SELECT);
        if (mode == WIDE_EMIT) ANN_WIDE_CASE(F16, WIDE_EMIT);
        ANN_WIDE_CASE(F16, WIDE_LISTS);
    }
    if (mode == WIDE_SELECT) ANN_WIDE_CASE(BF16, WIDE_SELECT);
    if (mode == WIDE_EMIT) ANN_WIDE_CASE(BF16, WIDE_EMIT);
    ANN_WIDE_CASE(BF16, WIDE_LISTS);
#undef ANN_WIDE_CASE
}

}  // namespace ann
