// fp32 flat kernel, the per-query merge kernel, and the LDS sizing helpers.
#include "flat_kernels.hpp"
#include "launch.hpp"

namespace ann {

size_t stream_lds_bytes(int nqg, int steps, int waves, int kp) {
    size_t q = (size_t)nqg * steps * WAVE * 16;
    size_t m = (size_t)waves * nqg * 16 * kp * sizeof(Cand);
    return q > m ? q : m;
}

int stream_waves(int nqg, int steps, int kp) {
    return kp != 16 && stream_lds_bytes(nqg, steps, STREAM_THREADS / WAVE, kp) > LDS_MAX / 2 ? 16 : 8;
}

size_t f32_lds_bytes(int d, int waves, int kp) {
    size_t q = (size_t)8 * d * 4;
    size_t m = (size_t)waves * 8 * kp * sizeof(Cand);
    return q > m ? q : m;
}

namespace {
template <int KP>
hipError_t launch_f32(const float *X, int64_t N, int d, const float *Q, int B, Cand *partial, int P, After after,
                      hipStream_t stream) {
    static size_t big = 0;
    const size_t lds = f32_lds_bytes(d, 4, KP);
    if (hipError_t e = allow_big_lds(reinterpret_cast<const void *>(&flat_f32_kernel<KP>), lds, &big)) return e;
    hipLaunchKernelGGL((flat_f32_kernel<KP>), dim3(P, (B + 7) / 8), dim3(256), lds, stream, X, N, d, Q, B, partial, after);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_flat_f32(int kp, const float *X, int64_t N, int d, const float *Q, int B, Cand *partial, int P,
                           After after, hipStream_t stream) {
    return kp == 4 ? launch_f32<4>(X, N, d, Q, B, partial, P, after, stream) : launch_f32<16>(X, N, d, Q, B, partial, P, after, stream);
}

hipError_t launch_flat_merge(int kp, const Cand *partial, int P, int B, int k, int32_t *ids, float *scores,
                             const int *count, const Cand *cand, int cap, hipStream_t stream) {
    const int threads = !count && P * kp <= 512 ? 64 : 256;       // one batch of loads per lane where possible
    if (kp == 4)
        hipLaunchKernelGGL((flat_merge_kernel<4>), dim3(B), dim3(threads), 0, stream, partial, P, k, ids, scores, count,
                           cand, cap);
    else
        hipLaunchKernelGGL((flat_merge_kernel<16>), dim3(B), dim3(threads), 0, stream, partial, P, k, ids, scores, count,
                           cand, cap);
    return hipGetLastError();
}

hipError_t launch_flat_sample_kth(const Cand *src, int Ps, int B, int k, float *thr, Cand *dst, int pstride, int pslot,
                                  int *count, hipStream_t stream) {
    if (k <= 4)   // short lists: a fraction of the selection work
        hipLaunchKernelGGL((flat_sample_kth_kernel<4, 4>), dim3(B), dim3(64), 0, stream, src, Ps, k, thr, dst, pstride, pslot, count);
    else
        hipLaunchKernelGGL((flat_sample_kth_kernel<4, 16>), dim3(B), dim3(64), 0, stream, src, Ps, k, thr, dst, pstride, pslot,
                           count);
    return hipGetLastError();
}

// ---- measurement support: what the matrix cores of this device sustain --------------------------
// Eight independent 32x32x16 fp16 accumulators per wave, 8 waves per workgroup, one workgroup per
// compute unit, operands held in registers (no LDS or memory traffic).  With RANDOM the operand
// registers hold random fp16 values and differ from one MFMA to the next, as in a real contraction;
// without, one constant: the difference is what data-dependent power management costs.
template <bool RANDOM>
__global__ __launch_bounds__(512) void mfma_rate_kernel(float *out, int iters) {
    u4 ra[4], rb[2];
    uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    auto next = [&]() {
        h ^= h << 13; h ^= h >> 17; h ^= h << 5;
        return RANDOM ? ((h & 0x83ff83ffu) | 0x2c002c00u) : 0x211f211fu;   // fp16 pairs of magnitude 1/16 .. 1/8
    };
    for (int i = 0; i < 4; ++i) for (int c = 0; c < 4; ++c) ra[i][c] = next();
    for (int i = 0; i < 2; ++i) for (int c = 0; c < 4; ++c) rb[i][c] = next();
    f16v acc[8];
    for (int j = 0; j < 8; ++j) for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i * 2 + j] = mfma32<F16>(ra[i], rb[j], acc[i * 2 + j]);
    }
    float s = 0.f;
    for (int j = 0; j < 8; ++j) for (int r = 0; r < 16; ++r) s += acc[j][r];
    if (s == 12345.678f) out[0] = s;                   // keeps the loop alive, never true in practice
}

hipError_t launch_mfma_rate(bool random_operands, int cus, int iters, float *sink, hipStream_t stream) {
    if (random_operands) hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(cus), dim3(512), 0, stream, sink, iters);
    else hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(cus), dim3(512), 0, stream, sink, iters);
    return hipGetLastError();
}

}  // namespace ann
