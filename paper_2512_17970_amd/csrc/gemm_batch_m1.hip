// Batched gather kernels for m = 1 codebook (see gemm_batch_impl.h).
#include "gemm_batch_impl.h"

namespace cg {
int launch_gemm_batch_m1(const Geometry& g, const GemmParams& p, hipStream_t stream) { return launch_gemm_batch_m<1, false>(g, p, stream); }
}  // namespace cg
