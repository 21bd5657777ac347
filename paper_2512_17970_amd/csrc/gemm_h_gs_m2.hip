// Gather kernels with an fp16 Psumbook and group scales for m = 2 codebooks (see gemm_impl.h).
#include "gemm_impl.h"

namespace cg {
int launch_gemm_h_gs_m2(const Geometry& g, const GemmParams& p, hipStream_t stream) { return launch_gemm_h_m<2, true>(g, p, stream); }
}  // namespace cg
