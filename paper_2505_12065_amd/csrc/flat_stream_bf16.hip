// flat_stream_kernel instantiations for bf16 corpora.
#include "flat_stream_launch.hpp"

namespace ann {

hipError_t launch_flat_stream_bf16(int nqg, int kp, const void *X, int64_t N, int d, const void *Q, int B, int q0,
                                  Cand *partial, int P, const StreamOpts &o, hipStream_t stream) {
    return launch_stream_any<BF16>(nqg, kp, X, N, d, Q, B, q0, partial, P, o, stream);
}

}  // namespace ann
