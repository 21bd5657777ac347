// Batched gather kernels with group scales for m = 2 codebooks (see gemm_batch_impl.h).
#include "gemm_batch_impl.h"

namespace cg {
int launch_gemm_batch_gs_m2(const Geometry& g, const GemmParams& p, hipStream_t stream) { return launch_gemm_batch_m<2, true>(g, p, stream); }
}  // namespace cg
