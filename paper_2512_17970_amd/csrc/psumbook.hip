// Stand-alone Psumbook build (Section 3, Eq. 2) for the whole of K, written to HBM:
//     psumbook[b][c][j][i] = sum_{k<v} C[c][i][k] * x[b][v*j + k]        (fp32)
// The fused kernel never materialises this table; the entry point exists so Eq. 2 can
// be checked and profiled on its own.  Two implementations:
//   * vector ALU: one thread per (b, j, c, i), packed fp16 dot products;
//   * MFMA: the table is the dense product of the (B*J) x v matrix of sub-vectors
//     with the v x 256 matrix of centroids, one 32x32x8 fp16 tile per wavefront
//     (for v = 4 the upper half of the contraction is fed zeros; v = 16 takes two passes).
#include "cg_common.h"

namespace cg {

template <int V>
__global__ void __launch_bounds__(256)
psumbook_valu_kernel(const _Float16* __restrict__ x, const _Float16* __restrict__ codebooks,
                     float* __restrict__ P, int m, long rows /* B*J */, int J)
{
    // blockIdx.x walks (row, c); the 256 threads are the 256 centroids.
    const int i = threadIdx.x;
    for (long rc = blockIdx.x; rc < rows * m; rc += gridDim.x) {
        const long row = rc / m;          // b*J + j  (x is [B*J][v] contiguous)
        const int c = (int)(rc % m);
        const int b = (int)(row / J);
        const int j = (int)(row % J);
        const _Float16* xv = x + row * V;
        const _Float16* cen = codebooks + ((size_t)c * kCentroids + i) * V;
        float a = 0.0f;
#pragma unroll
        for (int h = 0; h < V / 2; ++h) {
            half2_t cv = {cen[2 * h], cen[2 * h + 1]};
            half2_t xx = {xv[2 * h], xv[2 * h + 1]};
            a = __builtin_amdgcn_fdot2(cv, xx, a, false);
        }
        P[(((size_t)b * m + c) * J + j) * kCentroids + i] = a;
    }
}

// One wavefront per (32 sub-vector rows, codebook, 32 centroids) tile:
//   A[r][k] = x[row0 + r][k],  Bm[k][q] = C[c][i0 + q][k],  D = A Bm  (32 x 32, fp32)
// Lane l feeds A row l%32 and B column l%32 with k = 4*(l/32) .. +3, and receives
// D[8*blk + 4*(l/32) + e][l%32] in accumulator 4*blk + e.
template <int V>
__global__ void __launch_bounds__(256)
psumbook_mfma_kernel(const _Float16* __restrict__ x, const _Float16* __restrict__ codebooks,
                     float* __restrict__ P, int m, long rows, int J)
{
    const int lane = threadIdx.x & (kWave - 1);
    const long wave_global = (long)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x >> 6);
    const long nwaves = (long)gridDim.x * (blockDim.x / kWave);
    const long row_tiles = (rows + 31) / 32;
    const long total = row_tiles * m * 8;
    const int col = lane & 31;
    const int khalf = lane >> 5;
    for (long t = wave_global; t < total; t += nwaves) {
        const int iblk = (int)(t % 8);
        const int c = (int)((t / 8) % m);
        const long row0 = (t / (8 * m)) * 32;
        const long ar = row0 + col;
        float16_t d = {0};
#pragma unroll
        for (int pass = 0; pass < (V + 7) / 8; ++pass) {         // 8 elements of the contraction per pass
            half4_t a = {0, 0, 0, 0}, bm = {0, 0, 0, 0};
            const int k0 = 8 * pass + 4 * khalf;
            if (k0 < V) {
                if (ar < rows) {
                    const _Float16* xv = x + ar * V + k0;
                    a = half4_t{xv[0], xv[1], xv[2], xv[3]};
                }
                const _Float16* cen = codebooks + ((size_t)c * kCentroids + iblk * 32 + col) * V + k0;
                bm = half4_t{cen[0], cen[1], cen[2], cen[3]};
            }
            d = __builtin_amdgcn_mfma_f32_32x32x8f16(a, bm, d, 0, 0, 0);
        }
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const long row = row0 + 8 * blk + 4 * khalf + e;
                if (row < rows) {
                    const int b = (int)(row / J);
                    const int j = (int)(row % J);
                    P[(((size_t)b * m + c) * J + j) * kCentroids + iblk * 32 + col] = d[4 * blk + e];
                }
            }
        }
    }
}

}  // namespace cg

using namespace cg;

extern "C" int codegemm_psumbook_build(const codegemm_desc* desc, const void* x, const void* codebooks,
                                       float* psumbook, int use_mfma, void* stream)
{
    Geometry g;
    int st = make_geometry(desc, nullptr, &g);
    if (st) return st;
    if (!x || !codebooks || !psumbook) return CODEGEMM_INVALID_ARG;
    if (misaligned(x) || misaligned(codebooks) || misaligned(psumbook)) return CODEGEMM_INVALID_ARG;
    const _Float16* xh = static_cast<const _Float16*>(x);
    const _Float16* cb = static_cast<const _Float16*>(codebooks);
    const long rows = (long)desc->batch * g.J;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (use_mfma) {
        const long tiles = ((rows + 31) / 32) * g.m * 8;
        long blocks = (tiles + 3) / 4;
        if (blocks > 16384) blocks = 16384;
        if (g.v == 16)
            hipLaunchKernelGGL(psumbook_mfma_kernel<16>, dim3((unsigned)blocks), dim3(256), 0, s, xh, cb, psumbook, g.m, rows, g.J);
        else if (g.v == 8)
            hipLaunchKernelGGL(psumbook_mfma_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, s, xh, cb, psumbook, g.m, rows, g.J);
        else
            hipLaunchKernelGGL(psumbook_mfma_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, s, xh, cb, psumbook, g.m, rows, g.J);
    } else {
        long blocks = rows * g.m;
        if (blocks > 65536) blocks = 65536;
        if (g.v == 16)
            hipLaunchKernelGGL(psumbook_valu_kernel<16>, dim3((unsigned)blocks), dim3(256), 0, s, xh, cb, psumbook, g.m, rows, g.J);
        else if (g.v == 8)
            hipLaunchKernelGGL(psumbook_valu_kernel<8>, dim3((unsigned)blocks), dim3(256), 0, s, xh, cb, psumbook, g.m, rows, g.J);
        else
            hipLaunchKernelGGL(psumbook_valu_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, s, xh, cb, psumbook, g.m, rows, g.J);
    }
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}
