// C entry point of the hot path: validation, plan -> kernel instance, launch.
#include <mutex>
#include <utility>
#include <vector>

#include "gemm_batch_impl.h"

namespace cg {

// The dynamic-LDS limit of a kernel has to be raised above the 64 KB default once per
// (kernel, device); remember which pairs are done so the hot call does not repeat it.
int set_max_lds(const void* fn, size_t bytes)
{
    if (bytes <= 64 * 1024) return CODEGEMM_OK;
    static std::mutex mu;
    static std::vector<std::pair<const void*, int>> done;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return CODEGEMM_LAUNCH_FAILED;
    std::lock_guard<std::mutex> lock(mu);
    for (const auto& e : done)
        if (e.first == fn && e.second == dev) return CODEGEMM_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess)
        return CODEGEMM_LAUNCH_FAILED;
    done.emplace_back(fn, dev);
    return CODEGEMM_OK;
}

}  // namespace cg

using namespace cg;

#ifdef CODEGEMM_TRACE
#include "codegemm_trace.h"
static uint64_t* g_trace = nullptr;
extern "C" void codegemm_set_trace(uint64_t* stamps) { g_trace = stamps; }
#endif

extern "C" int codegemm_gemm(const codegemm_desc* desc, const codegemm_plan* plan, const void* x,
                             const uint8_t* packed_codes, const void* codebooks, const void* scales,
                             void* y, void* workspace, size_t workspace_bytes, void* stream)
{
    Geometry g;
    int st = make_geometry(desc, plan, &g);
    if (st) return st;
    if (!x || !packed_codes || !codebooks || !scales || !y || !workspace) return CODEGEMM_INVALID_ARG;
    if (misaligned(x) || misaligned(packed_codes) || misaligned(codebooks) || misaligned(scales) ||
        misaligned(y) || misaligned(workspace))
        return CODEGEMM_INVALID_ARG;
    const size_t cbytes = workspace_counter_bytes(g);
    const size_t need = cbytes + (size_t)g.B * g.NKS * g.Npad * sizeof(float);
    if (workspace_bytes < need) return CODEGEMM_WORKSPACE_TOO_SMALL;

    GemmParams p;
    p.x = static_cast<const _Float16*>(x);
    p.packed = packed_codes;
    p.codebooks = static_cast<const _Float16*>(codebooks);
    p.scales = g.g > 0 ? nullptr : static_cast<const _Float16*>(scales);
    p.gscales = g.g > 0 ? static_cast<const uint8_t*>(scales) : nullptr;
    p.GPU = g.GPU;
    p.gshift = g.gshift;
    p.y = y;
    p.counters = static_cast<uint32_t*>(workspace);
    p.cstride = counter_stride(g);
    p.partials = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + cbytes);
    p.B = g.B; p.K = g.K; p.N = g.N;
    p.NGR = g.NGR; p.NKT = g.NKT; p.NKS = g.NKS; p.KPW = g.KPW; p.Npad = g.Npad;
    p.y_fp32 = g.y_fp32 ? 1 : 0;
    p.trace = nullptr;
#ifdef CODEGEMM_TRACE
    p.trace = reinterpret_cast<unsigned long long*>(g_trace);
#endif
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (g.BG == 4) {
        switch (g.m) {
            case 1: return g.g > 0 ? launch_gemm_batch_gs_m1(g, p, s) : launch_gemm_batch_m1(g, p, s);
            case 2: return g.g > 0 ? launch_gemm_batch_gs_m2(g, p, s) : launch_gemm_batch_m2(g, p, s);
            case 3: return g.g > 0 ? launch_gemm_batch_gs_m3(g, p, s) : launch_gemm_batch_m3(g, p, s);
            case 4: return g.g > 0 ? launch_gemm_batch_gs_m4(g, p, s) : launch_gemm_batch_m4(g, p, s);
        }
        return CODEGEMM_UNSUPPORTED;
    }
    if (g.g > 0) {
        switch (g.m) {
            case 1: return launch_gemm_gs_m1(g, p, s);
            case 2: return launch_gemm_gs_m2(g, p, s);
            case 3: return launch_gemm_gs_m3(g, p, s);
            case 4: return launch_gemm_gs_m4(g, p, s);
        }
        return CODEGEMM_UNSUPPORTED;
    }
    switch (g.m) {
        case 1: return launch_gemm_m1(g, p, s);
        case 2: return launch_gemm_m2(g, p, s);
        case 3: return launch_gemm_m3(g, p, s);
        case 4: return launch_gemm_m4(g, p, s);
    }
    return CODEGEMM_UNSUPPORTED;
}
