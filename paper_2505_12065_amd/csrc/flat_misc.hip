// fp32 flat kernel, the per-query merge kernel, and the LDS sizing helpers.
#include "flat_kernels.hpp"
#include "launch.hpp"

namespace ann {

size_t stream_lds_bytes(int nqg, int steps, int waves, int kp) {
    size_t q = (size_t)nqg * steps * WAVE * 16;
    size_t m = (size_t)waves * nqg * 16 * kp * sizeof(Cand);
    return q > m ? q : m;
}

size_t f32_lds_bytes(int d, int waves, int kp) {
    size_t q = (size_t)8 * d * 4;
    size_t m = (size_t)waves * 8 * kp * sizeof(Cand);
    return q > m ? q : m;
}

namespace {
template <int KP>
hipError_t launch_f32(const float *X, int64_t N, int d, const float *Q, int B, Cand *partial, int P,
                      hipStream_t stream) {
    static size_t big = 0;
    const size_t lds = f32_lds_bytes(d, 4, KP);
    if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&flat_f32_kernel<KP>), lds, &big)) return e;
    hipLaunchKernelGGL((flat_f32_kernel<KP>), dim3(P, (B + 7) / 8), dim3(256), lds, stream, X, N, d, Q, B, partial);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_flat_f32(int kp, const float *X, int64_t N, int d, const float *Q, int B, Cand *partial, int P,
                           hipStream_t stream) {
    return kp == 4 ? launch_f32<4>(X, N, d, Q, B, partial, P, stream) : launch_f32<16>(X, N, d, Q, B, partial, P, stream);
}

hipError_t launch_flat_merge(int kp, const Cand *partial, int P, int B, int k, int32_t *ids, float *scores,
                             hipStream_t stream) {
    const int threads = P * kp <= 512 ? 64 : 256;       // one batch of loads per lane where possible
    if (kp == 4)
        hipLaunchKernelGGL((flat_merge_kernel<4>), dim3(B), dim3(threads), 0, stream, partial, P, k, ids, scores);
    else
        hipLaunchKernelGGL((flat_merge_kernel<16>), dim3(B), dim3(threads), 0, stream, partial, P, k, ids, scores);
    return hipGetLastError();
}

hipError_t launch_flat_sample_merge(int kp, const Cand *src, int Ps, int B, Cand *dst, int pstride, int pslot,
                                    float *thr, hipStream_t stream) {
    if (kp == 4)
        hipLaunchKernelGGL((flat_sample_merge_kernel<4>), dim3(B), dim3(64), 0, stream, src, Ps, dst, pstride, pslot, thr);
    else
        hipLaunchKernelGGL((flat_sample_merge_kernel<16>), dim3(B), dim3(64), 0, stream, src, Ps, dst, pstride, pslot, thr);
    return hipGetLastError();
}

}  // namespace ann
