// Gather kernels with an fp16 Psumbook and group scales for m = 1 codebook (see gemm_impl.h).
#include "gemm_impl.h"

namespace cg {
int launch_gemm_h_gs_m1(const Geometry& g, const GemmParams& p, hipStream_t stream) { return launch_gemm_h_m<1, true>(g, p, stream); }
}  // namespace cg
