// Dequantization-based comparator kernel (Section 2.3): the codebooks live in LDS,
// every code fetches its centroid vector from there, and the vector is multiplied
// with the matching activations.  O(N*B*K) multiply-adds; same inputs and outputs as
// the Psumbook kernel, canonical code layout, no workspace.
//
// One wavefront owns two whole output rows at a time: lane l takes sub-vectors
// 16*l .. 16*l+15 of each 1024-sub-vector chunk (one 16-byte code load per row and
// codebook), keeps one fp32 accumulator per row, and the 64 lanes are summed with
// shuffles at the end of the rows.  x is staged in LDS once per workgroup in the order
// the lanes read it, so those reads are conflict-free; the centroid reads are
// data-dependent.
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

// Codes of one row and one codebook for this lane's 16 sub-vectors of chunk ch: one 16-byte
// load when the row's code run is 16-byte aligned, bytes otherwise; zeros past the end.
__device__ __forceinline__ void load_code_words(uint32_t (&cw)[4], const uint8_t* crow, int j0, int J, bool vec_ok)
{
    cw[0] = cw[1] = cw[2] = cw[3] = 0u;
    if (vec_ok) {
        if (j0 < J) {
            const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(crow + j0));
            cw[0] = t.x; cw[1] = t.y; cw[2] = t.z; cw[3] = t.w;
        }
    } else {
        for (int jj = 0; jj < 16; ++jj)
            if (j0 + jj < J) cw[jj >> 2] |= (uint32_t)crow[j0 + jj] << (8 * (jj & 3));
    }
}

// The workgroups form a persistent grid (a few per compute unit): each stages the codebooks
// and one batch row of x in LDS once, with 16-byte (8-byte for v = 4) loads, and then walks
// over its share of the output rows, two rows per wavefront at a time so that the code
// loads of one row are in flight while the other is multiplied.
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
        // sub-vector j = 1024*ch + 16*l + jj is stored at index (ch*16 + jj)*64 + l; moved in pieces
        // of PIECE halves (a whole sub-vector for v = 4 and 8, half of one for v = 16)
        constexpr int PIECE = V == 4 ? 4 : 8;
        typedef _Float16 piece_t __attribute__((ext_vector_type(PIECE)));
        const _Float16* xrow = p.x + (size_t)b * p.K;
        const int pieces = p.nchunks * kDqChunk * V / PIECE;
        for (int i = tid; i < pieces; i += blockDim.x) {
            const int h0 = i * PIECE;                  // first half of the piece in row order
            const int j = h0 / V;
            const int l = (j % kDqChunk) / 16;
            const int jj = j % 16;
            const int ch = j / kDqChunk;
            piece_t val = {};
            if (j < p.J) val = *reinterpret_cast<const piece_t*>(xrow + h0);
            *reinterpret_cast<piece_t*>(xs + ((size_t)(ch * 16 + jj) * kWave + l) * V + h0 % V) = val;
        }
    }
    __syncthreads();

    const bool vec_ok = (p.J % 16) == 0;
    const int stride = gridDim.x * kDqWaves;
    for (int n0 = blockIdx.x * kDqWaves + wave; n0 < p.N; n0 += 2 * stride) {
        const int n1 = n0 + stride;                    // second row of the pair (may lie past the end)
        const bool two = n1 < p.N;
        float acc0 = 0.0f, acc1 = 0.0f;
        const _Float16* srow0 = p.scales + (size_t)n0 * p.groups;
        const _Float16* srow1 = p.scales + (size_t)(two ? n1 : n0) * p.groups;
        for (int ch = 0; ch < p.nchunks; ++ch) {
            const int j0 = ch * kDqChunk + 16 * lane;
            for (int c = 0; c < p.m; ++c) {
                uint32_t cw0[4], cw1[4];
                load_code_words(cw0, p.codes + ((size_t)c * p.N + n0) * p.J, j0, p.J, vec_ok);
                load_code_words(cw1, p.codes + ((size_t)c * p.N + (two ? n1 : n0)) * p.J, j0, two ? p.J : 0, vec_ok);
                const _Float16* cb = cbs + (size_t)c * kCentroids * V;
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    const _Float16* xv = xs + ((size_t)(ch * 16 + jj) * kWave + lane) * V;
                    const _Float16* cen0 = cb + ((cw0[jj >> 2] >> (8 * (jj & 3))) & 0xffu) * V;
                    const _Float16* cen1 = cb + ((cw1[jj >> 2] >> (8 * (jj & 3))) & 0xffu) * V;
                    if (p.groups == 1) {
#pragma unroll
                        for (int h = 0; h < V / 2; ++h) {
                            const half2_t xh = *reinterpret_cast<const half2_t*>(xv + 2 * h);
                            acc0 = __builtin_amdgcn_fdot2(*reinterpret_cast<const half2_t*>(cen0 + 2 * h), xh, acc0, false);
                            acc1 = __builtin_amdgcn_fdot2(*reinterpret_cast<const half2_t*>(cen1 + 2 * h), xh, acc1, false);
                        }
                    } else if (j0 + jj < p.J) {
                        // group scales: the sub-vector's dot product is scaled by its group's factor
                        float dot0 = 0.0f, dot1 = 0.0f;
#pragma unroll
                        for (int h = 0; h < V / 2; ++h) {
                            const half2_t xh = *reinterpret_cast<const half2_t*>(xv + 2 * h);
                            dot0 = __builtin_amdgcn_fdot2(*reinterpret_cast<const half2_t*>(cen0 + 2 * h), xh, dot0, false);
                            dot1 = __builtin_amdgcn_fdot2(*reinterpret_cast<const half2_t*>(cen1 + 2 * h), xh, dot1, false);
                        }
                        acc0 = __builtin_fmaf((float)srow0[(j0 + jj) >> p.gshift], dot0, acc0);
                        acc1 = __builtin_fmaf((float)srow1[(j0 + jj) >> p.gshift], dot1, acc1);
                    }
                }
            }
        }
        acc0 = wave_sum(acc0);
        acc1 = wave_sum(acc1);
        if (lane == 0) {
            const float val0 = p.groups == 1 ? acc0 * (float)p.scales[n0] : acc0;
            if (p.y_fp32) static_cast<float*>(p.y)[(size_t)b * p.N + n0] = val0;
            else static_cast<_Float16*>(p.y)[(size_t)b * p.N + n0] = (_Float16)val0;
            if (two) {
                const float val1 = p.groups == 1 ? acc1 * (float)p.scales[n1] : acc1;
                if (p.y_fp32) static_cast<float*>(p.y)[(size_t)b * p.N + n1] = val1;
                else static_cast<_Float16*>(p.y)[(size_t)b * p.N + n1] = (_Float16)val1;
            }
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
    // A persistent grid: as many workgroups per compute unit as their LDS allows (at most 4), every one
    // staging x once and then looping over rows; fewer when there are not that many rows or batch rows
    // already multiply the grid.
    int cus = 256;
    {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
    }
    int per_cu = (int)((size_t)kMaxLds / lds);
    if (per_cu > 4) per_cu = 4;
    if (per_cu < 1) per_cu = 1;
    int gx = ceil_div(cus * per_cu, desc->batch);
    if (gx < 1) gx = 1;
    const int max_gx = ceil_div(g.N, kDqWaves);
    if (gx > max_gx) gx = max_gx;
    const dim3 grid((unsigned)gx, (unsigned)desc->batch);
    if (g.v == 16)
        hipLaunchKernelGGL(dequant_kernel<16>, grid, dim3(kDqWaves * kWave), lds, static_cast<hipStream_t>(stream), p);
    else if (g.v == 8)
        hipLaunchKernelGGL(dequant_kernel<8>, grid, dim3(kDqWaves * kWave), lds, static_cast<hipStream_t>(stream), p);
    else
        hipLaunchKernelGGL(dequant_kernel<4>, grid, dim3(kDqWaves * kWave), lds, static_cast<hipStream_t>(stream), p);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}
