// Diagnostic build only (libcodegemm_trace.so): a probe of how many vector loads a compute
// unit keeps outstanding, the machine fact the depth of the code ring in the gather kernels
// is chosen by.  Compiles to nothing in the production library.
#ifdef CODEGEMM_TRACE
#include "cg_common.h"
#include "codegemm_trace.h"

namespace cg {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Every lane of every wavefront issues NL coalesced 16-byte loads (the gather kernels' code
// loads: bounds-checked buffer loads with the nt hint) from its workgroup's own stretch of
// `src`, then waits for the first and for all of them.  Per wavefront, shader-clock counts
// since its own start: [0] all loads issued, [1] first datum there, [2] all data there;
// [3] that span on the constant 100 MHz clock.
template <int NL>
__global__ void __launch_bounds__(1024) probe_kernel(const uint8_t* src, unsigned bytes_per_wg, uint64_t* out, uint32_t* sink)
{
    const uint64_t c0 = clock64(), w0 = wall_clock64();
    const int tid = threadIdx.x, nt = blockDim.x;
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(src) + (size_t)blockIdx.x * bytes_per_wg, 0, bytes_per_wg, 0x00020000u);
    u32x4_t v[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b128(r, (i * nt + tid) * 16, 0, 2);
    __builtin_amdgcn_sched_barrier(0);
    const uint64_t c1 = clock64();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" : "+v"(v[0]));
    __builtin_amdgcn_sched_barrier(0);
    const uint64_t c2 = clock64();
    __builtin_amdgcn_sched_barrier(0);
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < NL; ++i) s += v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
    asm volatile("" : "+v"(s));
    const uint64_t c3 = clock64(), w3 = wall_clock64();
    if ((tid & 63) == 0) {
        uint64_t* o = out + ((size_t)blockIdx.x * (nt / 64) + tid / 64) * 4;
        o[0] = c1 - c0;
        o[1] = c2 - c0;
        o[2] = c3 - c0;
        o[3] = w3 - w0;
    }
    if (s == 0x9e3779b9u) *sink = s;   // keeps the loads alive; practically never taken
}

}  // namespace cg

using namespace cg;

extern "C" int codegemm_probe_load_issue(const void* src, size_t src_bytes, int workgroups, int waves,
                                         int loads_per_lane, uint64_t* out, void* stream)
{
    if (!src || !out || misaligned(src) || workgroups < 1 || workgroups > 4096 || waves < 1 || waves > 16)
        return CODEGEMM_INVALID_ARG;
    const size_t per = (size_t)loads_per_lane * waves * 64 * 16;
    if (loads_per_lane < 1 || src_bytes < per * workgroups + 16) return CODEGEMM_INVALID_ARG;
    // out: [workgroups][waves][4] stamps followed by one 32-bit sink word
    uint32_t* sink = reinterpret_cast<uint32_t*>(out + (size_t)workgroups * waves * 4);
    const dim3 grid(workgroups), block(waves * 64);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (loads_per_lane) {
        case 1: hipLaunchKernelGGL(probe_kernel<1>, grid, block, 0, s, static_cast<const uint8_t*>(src), (unsigned)per, out, sink); break;
        case 2: hipLaunchKernelGGL(probe_kernel<2>, grid, block, 0, s, static_cast<const uint8_t*>(src), (unsigned)per, out, sink); break;
        case 4: hipLaunchKernelGGL(probe_kernel<4>, grid, block, 0, s, static_cast<const uint8_t*>(src), (unsigned)per, out, sink); break;
        case 8: hipLaunchKernelGGL(probe_kernel<8>, grid, block, 0, s, static_cast<const uint8_t*>(src), (unsigned)per, out, sink); break;
        default: return CODEGEMM_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}
#endif
