// Dequantization-based comparator kernel (Section 2.3): the codebooks live in LDS,
// every code fetches its centroid vector from there, and the vector is multiplied
// with the matching activations.  O(N*B*K) multiply-adds; same inputs and outputs as
// the Psumbook kernel, canonical code layout, no workspace.
//
// One wavefront owns a whole output row at a time: lane l takes sub-vectors
// 16*l .. 16*l+15 of each 1024-sub-vector chunk (one 16-byte code load per codebook),
// keeps one fp32 accumulator, and the 64 lanes are summed with DPP shuffles at the
// end of the row.  x is staged in LDS once per workgroup in the order the lanes read
// it, so those reads are conflict-free; the centroid reads are data-dependent.
#include "cg_common.h"

namespace cg {

constexpr int kDqWaves = 4;
constexpr int kDqChunk = 1024;   // sub-vectors per chunk: 64 lanes x 16 codes

struct DequantParams {
    const _Float16* x;
    const uint8_t* codes;
    const _Float16* codebooks;
    const _Float16* scales;
    void* y;
    int K, N, J, m, nchunks;
    int y_fp32;
    int groups;     // scales per row: 1 (one per output row) or K / g
    int gshift;     // sub-vector j belongs to group j >> gshift
};

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

template <int V>
__global__ void __launch_bounds__(kDqWaves * kWave) dequant_kernel(const DequantParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    _Float16* cbs = reinterpret_cast<_Float16*>(smem);                         // [m*256][V]
    _Float16* xs = cbs + (size_t)p.m * kCentroids * V;                         // [nchunks][16][64][V]
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int b = blockIdx.y;

    {
        const int chunks = p.m * kCentroids * V / 8;
        const uint4* src = reinterpret_cast<const uint4*>(p.codebooks);
        uint4* dst = reinterpret_cast<uint4*>(cbs);
        for (int i = tid; i < chunks; i += blockDim.x) dst[i] = src[i];
    }
    {
        // sub-vector j = 1024*ch + 16*l + jj is stored at index (ch*16 + jj)*64 + l
        const _Float16* xrow = p.x + (size_t)b * p.K;
        const int total = p.nchunks * kDqChunk * V;
        for (int i = tid; i < total; i += blockDim.x) {
            const int k = i % V;
            const int sv = i / V;
            const int l = sv % kWave;
            const int jj = (sv / kWave) % 16;
            const int ch = sv / (kWave * 16);
            const int j = ch * kDqChunk + 16 * l + jj;
            xs[i] = (j < p.J) ? xrow[(size_t)j * V + k] : (_Float16)0.0f;
        }
    }
    __syncthreads();

    const bool vec_ok = (p.J % 16) == 0;
    for (int n = blockIdx.x * kDqWaves + wave; n < p.N; n += gridDim.x * kDqWaves) {
        float acc = 0.0f;
        const _Float16* srow = p.scales + (size_t)n * p.groups;
        for (int ch = 0; ch < p.nchunks; ++ch) {
            const int j0 = ch * kDqChunk + 16 * lane;
            for (int c = 0; c < p.m; ++c) {
                const uint8_t* crow = p.codes + ((size_t)c * p.N + n) * p.J;
                uint32_t cw[4] = {0u, 0u, 0u, 0u};
                if (vec_ok) {
                    if (j0 < p.J) {
                        const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(crow + j0));
                        cw[0] = t.x; cw[1] = t.y; cw[2] = t.z; cw[3] = t.w;
                    }
                } else {
                    for (int jj = 0; jj < 16; ++jj)
                        if (j0 + jj < p.J) cw[jj >> 2] |= (uint32_t)crow[j0 + jj] << (8 * (jj & 3));
                }
                const _Float16* cb = cbs + (size_t)c * kCentroids * V;
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    const uint32_t code = (cw[jj >> 2] >> (8 * (jj & 3))) & 0xffu;
                    const _Float16* cen = cb + code * V;
                    const _Float16* xv = xs + ((size_t)(ch * 16 + jj) * kWave + lane) * V;
                    if (p.groups == 1) {
#pragma unroll
                        for (int h = 0; h < V / 2; ++h)
                            acc = __builtin_amdgcn_fdot2(*reinterpret_cast<const half2_t*>(cen + 2 * h),
                                                         *reinterpret_cast<const half2_t*>(xv + 2 * h), acc, false);
                    } else if (j0 + jj < p.J) {
                        // group scales: the sub-vector's dot product is scaled by its group's factor
                        float dot = 0.0f;
#pragma unroll
                        for (int h = 0; h < V / 2; ++h)
                            dot = __builtin_amdgcn_fdot2(*reinterpret_cast<const half2_t*>(cen + 2 * h),
                                                         *reinterpret_cast<const half2_t*>(xv + 2 * h), dot, false);
                        acc = __builtin_fmaf((float)srow[(j0 + jj) >> p.gshift], dot, acc);
                    }
                }
            }
        }
        acc = wave_sum(acc);
        if (lane == 0) {
            const float val = p.groups == 1 ? acc * (float)p.scales[n] : acc;
            if (p.y_fp32) static_cast<float*>(p.y)[(size_t)b * p.N + n] = val;
            else static_cast<_Float16*>(p.y)[(size_t)b * p.N + n] = (_Float16)val;
        }
    }
}

int set_max_lds(const void* fn, size_t bytes);   // gemm.hip

}  // namespace cg

using namespace cg;

extern "C" int codegemm_dequant_gemm(const codegemm_desc* desc, const void* x, const uint8_t* codes,
                                     const void* codebooks, const void* scales, void* y, void* stream)
{
    Geometry g;
    int st = make_geometry(desc, nullptr, &g);
    if (st) return st;
    if (!x || !codes || !codebooks || !scales || !y) return CODEGEMM_INVALID_ARG;
    if (misaligned(x) || misaligned(codes) || misaligned(codebooks) || misaligned(scales) || misaligned(y))
        return CODEGEMM_INVALID_ARG;
    DequantParams p;
    p.x = static_cast<const _Float16*>(x);
    p.codes = codes;
    p.codebooks = static_cast<const _Float16*>(codebooks);
    p.scales = static_cast<const _Float16*>(scales);
    p.y = y;
    p.K = g.K; p.N = g.N; p.J = g.J; p.m = g.m;
    p.nchunks = ceil_div(g.J, kDqChunk);
    p.y_fp32 = g.y_fp32 ? 1 : 0;
    p.groups = g.g > 0 ? g.K / g.g : 1;
    p.gshift = 0;
    if (g.g > 0)
        while ((g.v << p.gshift) < g.g) ++p.gshift;
    const size_t lds = (size_t)g.m * kCentroids * g.v * 2 + (size_t)p.nchunks * kDqChunk * g.v * 2;
    if (lds > (size_t)kMaxLds) return CODEGEMM_UNSUPPORTED;   // x does not fit in LDS (K > ~70k)
    const void* fn = (g.v == 16) ? reinterpret_cast<const void*>(dequant_kernel<16>)
                     : (g.v == 8) ? reinterpret_cast<const void*>(dequant_kernel<8>)
                                  : reinterpret_cast<const void*>(dequant_kernel<4>);
    if ((st = set_max_lds(fn, lds)) != CODEGEMM_OK) return st;
    int gx = ceil_div(g.N, kDqWaves);
    if (gx > 2048) gx = 2048;
    const dim3 grid((unsigned)gx, (unsigned)desc->batch);
    if (g.v == 16)
        hipLaunchKernelGGL(dequant_kernel<16>, grid, dim3(kDqWaves * kWave), lds, static_cast<hipStream_t>(stream), p);
    else if (g.v == 8)
        hipLaunchKernelGGL(dequant_kernel<8>, grid, dim3(kDqWaves * kWave), lds, static_cast<hipStream_t>(stream), p);
    else
        hipLaunchKernelGGL(dequant_kernel<4>, grid, dim3(kDqWaves * kWave), lds, static_cast<hipStream_t>(stream), p);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}
