// Gather kernels with an fp16 Psumbook for m = 4 codebooks (see gemm_impl.h).
#include "gemm_impl.h"

namespace cg {
int launch_gemm_h_m4(const Geometry& g, const GemmParams& p, hipStream_t stream) { return launch_gemm_h_m<4, false>(g, p, stream); }
}  // namespace cg
