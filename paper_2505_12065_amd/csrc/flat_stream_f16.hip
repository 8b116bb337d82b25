// flat_stream_kernel instantiations for f16 corpora.
#include "flat_kernels.hpp"
#include "launch.hpp"

namespace ann {
namespace {

template <int NQG, int KP>
hipError_t launch(const void *X, int64_t N, int d, const void *Q, int B, int q0, Cand *partial, int P,
                  hipStream_t stream) {
    static size_t big[2] = {0, 0};
    const int steps = (d + 31) / 32;
    const size_t lds = stream_lds_bytes(NQG, steps, STREAM_THREADS / WAVE, KP);
    if ((d % 32) == 0) {
        if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&flat_stream_kernel<F16, NQG, KP, true>), lds, &big[0])) return e;
        hipLaunchKernelGGL((flat_stream_kernel<F16, NQG, KP, true>), dim3(P), dim3(STREAM_THREADS), lds, stream,
                           X, N, d, Q, B, q0, partial);
    } else {
        if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&flat_stream_kernel<F16, NQG, KP, false>), lds, &big[1])) return e;
        hipLaunchKernelGGL((flat_stream_kernel<F16, NQG, KP, false>), dim3(P), dim3(STREAM_THREADS), lds, stream,
                           X, N, d, Q, B, q0, partial);
    }
    return hipGetLastError();
}

template <int KP>
hipError_t launch_nqg(int nqg, const void *X, int64_t N, int d, const void *Q, int B, int q0, Cand *partial, int P,
                      hipStream_t stream) {
    switch (nqg) {
    case 1: return launch<1, KP>(X, N, d, Q, B, q0, partial, P, stream);
    case 2: return launch<2, KP>(X, N, d, Q, B, q0, partial, P, stream);
    case 3: return launch<3, KP>(X, N, d, Q, B, q0, partial, P, stream);
    default: return launch<4, KP>(X, N, d, Q, B, q0, partial, P, stream);
    }
}

}  // namespace

hipError_t launch_flat_stream_f16(int nqg, int kp, const void *X, int64_t N, int d, const void *Q, int B, int q0,
                                  Cand *partial, int P, hipStream_t stream) {
    return kp == 4 ? launch_nqg<4>(nqg, X, N, d, Q, B, q0, partial, P, stream)
                   : launch_nqg<16>(nqg, X, N, d, Q, B, q0, partial, P, stream);
}

}  // namespace ann
