// Priority levels and execution order of the request scheduler (Section 3.2, Eq. 1-2 of the
// paper): a small batched routine beside the retrieval kernels, O(n) + O(n^2 / threads) work for
// the n requests of a serving batch.
#include "launch.hpp"

namespace ann {

constexpr int PRIO_THREADS = 256;

// Block-wide minimum and maximum of v over the threads' values (LDS scratch of 2 x 4 doubles).
__device__ __forceinline__ void block_min_max(double lo, double hi, double *scratch, double &mn, double &mx) {
    for (int m = 1; m < WAVE; m <<= 1) {
        lo = fmin(lo, __shfl_xor(lo, m));
        hi = fmax(hi, __shfl_xor(hi, m));
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { scratch[wave] = lo; scratch[4 + wave] = hi; }
    __syncthreads();
    mn = fmin(fmin(scratch[0], scratch[1]), fmin(scratch[2], scratch[3]));
    mx = fmax(fmax(scratch[4], scratch[5]), fmax(scratch[6], scratch[7]));
    __syncthreads();
}

// One workgroup: extremes of the three metrics, then
//   level_i = largest j in [0, G) with R_i > T_{R,j} or W_i > T_{W,j} or C_i > T_{C,j}, else 0,
//   T_{M,j} = min(M) + j/G (max(M) - min(M)), evaluated in binary64 exactly as written: the quotient,
//   the difference, their product and the sum are each rounded once (no fused multiply-add).
__global__ __launch_bounds__(PRIO_THREADS) void priority_level_kernel(const int32_t *__restrict__ R,
                                                                      const double *__restrict__ W,
                                                                      const int32_t *__restrict__ C, int n, int G,
                                                                      int32_t *__restrict__ level) {
    __shared__ double scratch[8];
    double lo[3] = {INFINITY, INFINITY, INFINITY}, hi[3] = {-INFINITY, -INFINITY, -INFINITY};
    for (int i = threadIdx.x; i < n; i += PRIO_THREADS) {
        const double v[3] = {(double)R[i], W[i], (double)C[i]};
#pragma unroll
        for (int m = 0; m < 3; ++m) { lo[m] = fmin(lo[m], v[m]); hi[m] = fmax(hi[m], v[m]); }
    }
    double mn[3], mx[3];
#pragma unroll
    for (int m = 0; m < 3; ++m) block_min_max(lo[m], hi[m], scratch, mn[m], mx[m]);
    for (int i = threadIdx.x; i < n; i += PRIO_THREADS) {
        const double v[3] = {(double)R[i], W[i], (double)C[i]};
        int best = 0;
        for (int j = 0; j < G; ++j) {
            const double f = (double)j / (double)G;
#pragma unroll
            for (int m = 0; m < 3; ++m)
                if (v[m] > __dadd_rn(mn[m], __dmul_rn(f, mx[m] - mn[m]))) best = j;
        }
        level[i] = best;
    }
}

// order[position of i] = i, position = number of requests that run before i: higher level first,
// inside a level longer current queueing time first, equal times in index order; a queueing time
// that is NaN counts as the shortest possible wait (-inf), so every request gets exactly one place.
__global__ __launch_bounds__(PRIO_THREADS) void priority_order_kernel(const int32_t *__restrict__ level,
                                                                      const double *__restrict__ Wcur, int n,
                                                                      int32_t *__restrict__ order) {
    const int i = blockIdx.x * PRIO_THREADS + threadIdx.x;
    if (i >= n) return;
    const int li = level[i];
    double wi = Wcur[i];
    wi = wi == wi ? wi : -INFINITY;
    int before = 0;
    for (int j = 0; j < n; ++j) {
        const int lj = level[j];
        double wj = Wcur[j];
        wj = wj == wj ? wj : -INFINITY;
        before += (int)(lj > li) | ((int)(lj == li) & ((int)(wj > wi) | ((int)(wj == wi) & (int)(j < i))));
    }
    order[before] = i;
}

hipError_t launch_priority(const int32_t *R, const double *W, const int32_t *C, const double *Wcur, int n, int G,
                           int32_t *level, int32_t *order, hipStream_t stream) {
    hipLaunchKernelGGL(priority_level_kernel, dim3(1), dim3(PRIO_THREADS), 0, stream, R, W, C, n, G, level);
    if (hipError_t e = hipGetLastError()) return e;
    hipLaunchKernelGGL(priority_order_kernel, dim3((n + PRIO_THREADS - 1) / PRIO_THREADS), dim3(PRIO_THREADS), 0, stream,
                       level, Wcur, n, order);
    return hipGetLastError();
}

}  // namespace ann
