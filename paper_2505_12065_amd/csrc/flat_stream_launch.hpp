// Launcher of flat_stream_kernel for one element type; included by one translation unit per type
// so that the instantiations compile in parallel.
#pragma once

#include "flat_kernels.hpp"
#include "launch.hpp"

namespace ann {

template <class T, int NQG, int KP, bool EMIT, int NWV>
hipError_t launch_stream_waves(const void *X, int64_t N, int d, const void *Q, int B, int q0, Cand *partial, int P,
                               const StreamOpts &o, hipStream_t stream) {
    static size_t big[2] = {0, 0};
    const int steps = (d + 31) / 32;
    const size_t lds = stream_lds_bytes(NQG, steps, NWV, KP);
    if ((d % 32) == 0) {
        if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&flat_stream_kernel<T, NQG, KP, true, EMIT, NWV>), lds, &big[0]))
            return e;
        hipLaunchKernelGGL((flat_stream_kernel<T, NQG, KP, true, EMIT, NWV>), dim3(P), dim3(NWV * WAVE), lds, stream, X, N, d,
                           Q, B, q0, partial, o);
    } else {
        if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&flat_stream_kernel<T, NQG, KP, false, EMIT, NWV>), lds, &big[1]))
            return e;
        hipLaunchKernelGGL((flat_stream_kernel<T, NQG, KP, false, EMIT, NWV>), dim3(P), dim3(NWV * WAVE), lds, stream, X, N, d,
                           Q, B, q0, partial, o);
    }
    return hipGetLastError();
}

template <class T, int NQG, int KP, bool EMIT>
hipError_t launch_stream(const void *X, int64_t N, int d, const void *Q, int B, int q0, Cand *partial, int P,
                         const StreamOpts &o, hipStream_t stream) {
    if constexpr (KP != 16 && NQG >= 2) {            // one query group never fills half the LDS (d <= 4096)
        if (stream_waves(NQG, (d + 31) / 32, KP) == 16)
            return launch_stream_waves<T, NQG, KP, EMIT, 16>(X, N, d, Q, B, q0, partial, P, o, stream);
    }
    return launch_stream_waves<T, NQG, KP, EMIT, 8>(X, N, d, Q, B, q0, partial, P, o, stream);
}

template <class T, int KP, bool EMIT>
hipError_t launch_stream_nqg(int nqg, const void *X, int64_t N, int d, const void *Q, int B, int q0, Cand *partial,
                             int P, const StreamOpts &o, hipStream_t stream) {
    switch (nqg) {
    case 1: return launch_stream<T, 1, KP, EMIT>(X, N, d, Q, B, q0, partial, P, o, stream);
    case 2: return launch_stream<T, 2, KP, EMIT>(X, N, d, Q, B, q0, partial, P, o, stream);
    case 3: return launch_stream<T, 3, KP, EMIT>(X, N, d, Q, B, q0, partial, P, o, stream);
    default: return launch_stream<T, 4, KP, EMIT>(X, N, d, Q, B, q0, partial, P, o, stream);
    }
}

// kp: 4 or 16 = list length; 0 = candidate-array mode (o.thr, o.count, o.cap)
template <class T>
hipError_t launch_stream_any(int nqg, int kp, const void *X, int64_t N, int d, const void *Q, int B, int q0,
                             Cand *partial, int P, const StreamOpts &o, hipStream_t stream) {
    if (kp == 0) return launch_stream_nqg<T, 4, true>(nqg, X, N, d, Q, B, q0, partial, P, o, stream);
    return kp == 4 ? launch_stream_nqg<T, 4, false>(nqg, X, N, d, Q, B, q0, partial, P, o, stream)
                   : launch_stream_nqg<T, 16, false>(nqg, X, N, d, Q, B, q0, partial, P, o, stream);
}

}  // namespace ann
