// Batched gather kernels for m = 3 codebooks (see gemm_batch_impl.h).
#include "gemm_batch_impl.h"

namespace cg {
int launch_gemm_batch_m3(const Geometry& g, const GemmParams& p, hipStream_t stream) { return launch_gemm_batch_m<3, false>(g, p, stream); }
}  // namespace cg
