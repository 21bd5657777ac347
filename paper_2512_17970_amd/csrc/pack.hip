// Code re-ordering between the canonical [m][N][K/v] array and the packed
// streaming layout of the gather kernel, and the workspace fill.
#include "cg_common.h"

namespace cg {

// One thread per (codebook, padded row, padded sub-vector): every packed byte is
// written exactly once, positions outside the matrix get code 0.
__global__ void __launch_bounds__(256)
pack_kernel(const uint8_t* __restrict__ codes, uint8_t* __restrict__ packed,
            int N, int J, int m, int NKT, int Npad, int Jpad)
{
    const size_t total = (size_t)m * Npad * Jpad;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(idx % Jpad);
        const int n = (int)((idx / Jpad) % Npad);
        const int c = (int)(idx / ((size_t)Jpad * Npad));
        uint8_t code = 0;
        if (n < N && j < J) code = codes[((size_t)c * N + n) * J + j];
        packed[packed_offset(c, n, j, m, NKT)] = code;
    }
}

__global__ void __launch_bounds__(256)
unpack_kernel(const uint8_t* __restrict__ packed, uint8_t* __restrict__ codes,
              int N, int J, int m, int NKT)
{
    const size_t total = (size_t)m * N * J;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(idx % J);
        const int n = (int)((idx / J) % N);
        const int c = (int)(idx / ((size_t)J * N));
        codes[idx] = packed[packed_offset(c, n, j, m, NKT)];
    }
}

// One thread per packed scale: entry (granule, K tile, group of the tile, octet, row).
__global__ void __launch_bounds__(256)
pack_scales_kernel(const _Float16* __restrict__ scales, _Float16* __restrict__ packed,
                   int N, int K, int v, int g, int NKT, int GPU, size_t total)
{
    const int groups = K / g;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (size_t)gridDim.x * blockDim.x) {
        const int r = (int)(idx % 8);
        const int o = (int)((idx / 8) % 16);
        const int q = (int)((idx / 128) % GPU);
        const int kt = (int)((idx / ((size_t)128 * GPU)) % NKT);
        const int rg = (int)(idx / ((size_t)128 * GPU * NKT));
        const int n = rg * kGranuleRows + o * kRowsPerLane + r;
        const long long first_weight = ((long long)kt * kSlots) * v + (long long)q * g;   // of the group's part in this tile
        const int grp = (int)(first_weight / g);
        _Float16 val = (_Float16)0.0f;
        if (n < N && first_weight < K && grp < groups) val = scales[(size_t)n * groups + grp];
        packed[idx] = val;
    }
}

// A plain fill kernel rather than a memset node, so the call can be captured
// in a HIP graph.
__global__ void __launch_bounds__(256) zero_kernel(uint32_t* p, size_t words)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

static int grid_for(size_t total)
{
    size_t blocks = (total + 255) / 256;
    return (int)(blocks > 8192 ? 8192 : (blocks ? blocks : 1));
}

}  // namespace cg

using namespace cg;

extern "C" int codegemm_pack_codes(const codegemm_desc* desc, const codegemm_plan* plan,
                                   const uint8_t* codes, uint8_t* packed, void* stream)
{
    Geometry g;
    int st = make_geometry(desc, plan, &g);
    if (st) return st;
    if (!codes || !packed || misaligned(codes) || misaligned(packed)) return CODEGEMM_INVALID_ARG;
    const int Jpad = g.NKT * kSlots;
    const size_t total = (size_t)g.m * g.Npad * Jpad;
    hipLaunchKernelGGL(pack_kernel, dim3(grid_for(total)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       codes, packed, g.N, g.J, g.m, g.NKT, g.Npad, Jpad);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}

extern "C" int codegemm_unpack_codes(const codegemm_desc* desc, const codegemm_plan* plan,
                                     const uint8_t* packed, uint8_t* codes, void* stream)
{
    Geometry g;
    int st = make_geometry(desc, plan, &g);
    if (st) return st;
    if (!codes || !packed || misaligned(codes) || misaligned(packed)) return CODEGEMM_INVALID_ARG;
    const size_t total = (size_t)g.m * g.N * g.J;
    hipLaunchKernelGGL(unpack_kernel, dim3(grid_for(total)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       packed, codes, g.N, g.J, g.m, g.NKT);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}

// Host versions: plain loops over the same offset function the kernels use (host pointers, synchronous).
extern "C" int codegemm_pack_codes_host(const codegemm_desc* desc, const uint8_t* codes, uint8_t* packed)
{
    Geometry g;
    int st = make_geometry(desc, nullptr, &g);
    if (st) return st;
    if (!codes || !packed) return CODEGEMM_INVALID_ARG;
    const int Jpad = g.NKT * kSlots;
    for (int c = 0; c < g.m; ++c)
        for (int n = 0; n < g.Npad; ++n)
            for (int j = 0; j < Jpad; ++j)
                packed[packed_offset(c, n, j, g.m, g.NKT)] =
                    (n < g.N && j < g.J) ? codes[((size_t)c * g.N + n) * g.J + j] : (uint8_t)0;
    return CODEGEMM_OK;
}

extern "C" int codegemm_unpack_codes_host(const codegemm_desc* desc, const uint8_t* packed, uint8_t* codes)
{
    Geometry g;
    int st = make_geometry(desc, nullptr, &g);
    if (st) return st;
    if (!codes || !packed) return CODEGEMM_INVALID_ARG;
    for (int c = 0; c < g.m; ++c)
        for (int n = 0; n < g.N; ++n)
            for (int j = 0; j < g.J; ++j)
                codes[((size_t)c * g.N + n) * g.J + j] = packed[packed_offset(c, n, j, g.m, g.NKT)];
    return CODEGEMM_OK;
}

extern "C" int codegemm_pack_scales(const codegemm_desc* desc, const void* scales, void* packed, void* stream)
{
    Geometry g;
    int st = make_geometry(desc, nullptr, &g);
    if (st) return st;
    if (g.g <= 0) return CODEGEMM_INVALID_ARG;       // row-wise scales are used as they are
    if (!scales || !packed || misaligned(scales) || misaligned(packed)) return CODEGEMM_INVALID_ARG;
    const size_t total = (size_t)g.NGR * g.NKT * g.GPU * 128;
    hipLaunchKernelGGL(pack_scales_kernel, dim3(grid_for(total)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const _Float16*>(scales), static_cast<_Float16*>(packed), g.N, g.K, g.v, g.g,
                       g.NKT, g.GPU, total);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}

extern "C" int codegemm_workspace_init(void* workspace, size_t workspace_bytes, void* stream)
{
    if (!workspace || workspace_bytes == 0 || (workspace_bytes & 3) || misaligned(workspace))
        return CODEGEMM_INVALID_ARG;
    const size_t words = workspace_bytes / 4;
    hipLaunchKernelGGL(zero_kernel, dim3(grid_for(words)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint32_t*>(workspace), words);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}
