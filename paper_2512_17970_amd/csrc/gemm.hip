// The hot path: fused Psumbook build + gather-by-code GEMV/GEMM (Section 3, Steps 1-3)
// followed by the row scale, for gfx950.
//
// Work decomposition.  The weight matrix is cut into tiles of (512 * RW) rows by S
// sub-vectors (S * v weights along K).  One workgroup of RW * JW wavefronts owns one
// tile:
//   1. every lane first issues ALL global loads of the tile's packed codes it will
//      consume (at most 16 steps of 8*m bytes), so HBM is streaming while
//   2. the workgroup stages the codebooks and the x slice in LDS and builds the
//      tile's Psumbook P[c][i][slot] (fp32, slot fastest) from them (Eq. 2);
//   3. after one barrier each lane gathers P by code for its 8 rows.  In step t lane l
//      works on slot (t + l) mod S, so the 64 lanes of a wavefront always address 64
//      different slots = different LDS banks, whatever the code values are;
//   4. the JW wavefronts that share rows add their accumulators through LDS, the
//      workgroup writes one fp32 partial per row to the workspace, and the last
//      workgroup to finish a row tile (atomic ticket) adds the K tiles' partials in
//      tile order, multiplies by the row scale and stores y.
// For B > 1 steps 2-4 repeat per batch row with the codes kept in registers, so the
// compressed weights are read from HBM once per call whatever the batch.
#include <mutex>
#include <utility>
#include <vector>

#include "cg_common.h"

namespace cg {

struct GemmParams {
    const _Float16* x;
    const uint8_t* packed;
    const _Float16* codebooks;
    const _Float16* scales;
    void* y;
    float* partials;
    uint32_t* counters;
    int B, K, N, J;
    int RW, JW, log2JW;
    int NRB, NKT, Npad;
    int y_fp32;
};

// Psumbook build on the vector ALU: each thread owns 4 consecutive slots and walks
// over (codebook, centroid) rows; fp16 x fp16 products are exact in fp32 and are
// accumulated in fp32 by the packed dot-product instruction.
template <int M, int V, int S>
__device__ __forceinline__ void build_valu(float* planes, const _Float16* cbs, const _Float16* xs,
                                           int tid, int nthreads)
{
    constexpr int Q = S / 4;
    const int q = tid % Q;
    const int cg0 = tid / Q;
    const int ncg = nthreads / Q;
    half2_t xq[4][V / 2];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int h = 0; h < V / 2; ++h)
            xq[s][h] = *reinterpret_cast<const half2_t*>(xs + (4 * q + s) * V + 2 * h);
    for (int row = cg0; row < M * kCentroids; row += ncg) {
        half2_t cv[V / 2];
#pragma unroll
        for (int h = 0; h < V / 2; ++h) cv[h] = *reinterpret_cast<const half2_t*>(cbs + row * V + 2 * h);
        float4_t out;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            float a = 0.0f;
#pragma unroll
            for (int h = 0; h < V / 2; ++h) a = __builtin_amdgcn_fdot2(cv[h], xq[s][h], a, false);
            out[s] = a;
        }
        *reinterpret_cast<float4_t*>(planes + row * S + 4 * q) = out;
    }
}

template <int S>
__device__ __forceinline__ float psum_at(const unsigned char* plane_bytes, uint32_t word, int byte, uint32_t slot_off)
{
    const uint32_t code = (word >> (8 * byte)) & 0xffu;
    return *reinterpret_cast<const float*>(plane_bytes + code * (S * 4) + slot_off);
}

template <int M, int V, int S, int NSTEP, int BUILD>
__global__ void __launch_bounds__(1024) gemm_kernel(const GemmParams p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float* planes = reinterpret_cast<float*>(smem);                               // [M][256][S]
    _Float16* cbs = reinterpret_cast<_Float16*>(smem + (size_t)M * kCentroids * S * 4);   // [M*256][V]
    _Float16* xs = cbs + M * kCentroids * V;                                      // [S][V]
    uint32_t* flag = reinterpret_cast<uint32_t*>(xs + S * V);

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int kt = blockIdx.x % p.NKT;
    const int rt = blockIdx.x / p.NKT;
    const int rw = wave >> p.log2JW;
    const int jw = wave & (p.JW - 1);
    const int rb = rt * p.RW + rw;
    const bool active = rb < p.NRB;
    const int t0 = jw * NSTEP;

    // 1. All code loads of this lane, issued before anything else.
    uint32_t w[NSTEP][2 * M];
    if (active) {
        const uint8_t* base = p.packed + (((size_t)rb * p.NKT + kt) * S + t0) * (size_t)step_bytes(M);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            const uint8_t* sb = base + (size_t)st * step_bytes(M);
#pragma unroll
            for (int part = 0; part < (M + 1) / 2; ++part) {
                if (2 * part + 1 == M) {
                    const u32x2_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(sb + part * 16 * kWave) + lane);
                    w[st][4 * part + 0] = t.x;
                    w[st][4 * part + 1] = t.y;
                } else {
                    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(sb + part * 16 * kWave) + lane);
                    w[st][4 * part + 0] = t.x;
                    w[st][4 * part + 1] = t.y;
                    w[st][4 * part + 2] = t.z;
                    w[st][4 * part + 3] = t.w;
                }
            }
        }
    } else {
#pragma unroll
        for (int st = 0; st < NSTEP; ++st)
#pragma unroll
            for (int i = 0; i < 2 * M; ++i) w[st][i] = 0u;
    }

    // 2a. Codebooks -> LDS (16-byte chunks; the buffer is a whole number of them).
    {
        constexpr int chunks = M * kCentroids * V / 8;
        const uint4* src = reinterpret_cast<const uint4*>(p.codebooks);
        uint4* dst = reinterpret_cast<uint4*>(cbs);
        for (int i = tid; i < chunks; i += nthreads) dst[i] = src[i];
    }

    const int tile_rows = p.RW * kBlockRows;
    const int n_base = rt * tile_rows;

    for (int b = 0; b < p.B; ++b) {
        // 2b. x slice of this tile (Step 1: x^j_k = x[v*j + k]); zero beyond K.
        {
            const int e0 = kt * S * V;
            const _Float16* xrow = p.x + (size_t)b * p.K;
            for (int i = tid; i < S * V; i += nthreads) {
                const int e = e0 + i;
                xs[i] = (e < p.K) ? xrow[e] : (_Float16)0.0f;
            }
        }
        __syncthreads();

        // 2c. Psumbook of the tile (Eq. 2).
        build_valu<M, V, S>(planes, cbs, xs, tid, nthreads);
        __syncthreads();

        // 3. Gather by code and accumulate (Step 3).
        float acc[kRowsPerLane];
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) acc[r] = 0.0f;
        if (active) {
            const unsigned char* pb = reinterpret_cast<const unsigned char*>(planes);
#pragma unroll
            for (int st = 0; st < NSTEP; ++st) {
                const uint32_t slot_off = (uint32_t)((t0 + st + lane) & (S - 1)) * 4u;
#pragma unroll
                for (int c = 0; c < M; ++c) {
                    const unsigned char* plane = pb + (size_t)c * kCentroids * S * 4;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        acc[r] += psum_at<S>(plane, w[st][2 * c], r, slot_off);
                        acc[4 + r] += psum_at<S>(plane, w[st][2 * c + 1], r, slot_off);
                    }
                }
            }
        }
        __syncthreads();   // every wavefront is done reading the planes

        // 4a. Add the accumulators of the JW wavefronts that share rows (through LDS).
        float* red = planes;
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) red[wave * kBlockRows + r * kWave + lane] = acc[r];
        __syncthreads();
        for (int o = tid; o < tile_rows; o += nthreads) {
            const int rwo = o / kBlockRows;
            const int idx = o % kBlockRows;
            float sum = 0.0f;
            for (int q = 0; q < p.JW; ++q) sum += red[(rwo * p.JW + q) * kBlockRows + idx];
            const int n = n_base + o;
            if (p.NKT == 1) {
                if (n < p.N) {
                    const float val = sum * (float)p.scales[n];
                    if (p.y_fp32) static_cast<float*>(p.y)[(size_t)b * p.N + n] = val;
                    else static_cast<_Float16*>(p.y)[(size_t)b * p.N + n] = (_Float16)val;
                }
            } else if (n < p.Npad) {
                p.partials[((size_t)b * p.NKT + kt) * p.Npad + n] = sum;
            }
        }
        __syncthreads();   // red / xs are rewritten by the next batch row
    }

    if (p.NKT == 1) return;

    // 4b. Ticket: the last workgroup of this row tile combines the K tiles' partials.
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t old = atomicAdd(&p.counters[rt], 1u);
        *flag = (old == (uint32_t)(p.NKT - 1)) ? 1u : 0u;
    }
    __syncthreads();
    if (*flag == 0u) return;
    __threadfence();
    for (int b = 0; b < p.B; ++b) {
        for (int o = tid; o < tile_rows; o += nthreads) {
            const int n = n_base + o;
            if (n >= p.N) continue;
            const float* src = p.partials + (size_t)b * p.NKT * p.Npad + n;
            float sum = 0.0f;
            for (int k2 = 0; k2 < p.NKT; ++k2)
                sum += __hip_atomic_load(src + (size_t)k2 * p.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const float val = sum * (float)p.scales[n];
            if (p.y_fp32) static_cast<float*>(p.y)[(size_t)b * p.N + n] = val;
            else static_cast<_Float16*>(p.y)[(size_t)b * p.N + n] = (_Float16)val;
        }
    }
    if (tid == 0) __hip_atomic_store(&p.counters[rt], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

typedef void (*gemm_fn)(const GemmParams);

template <int M, int V, int S, int NSTEP>
static gemm_fn pick_build(int build)
{
    (void)build;
    return gemm_kernel<M, V, S, NSTEP, 0>;
}

template <int M, int V, int S>
static gemm_fn pick_nstep(int nstep, int build)
{
    switch (nstep) {
        case 4: return pick_build<M, V, S, 4>(build);
        case 8: return pick_build<M, V, S, 8>(build);
        case 16: return pick_build<M, V, S, 16>(build);
    }
    return nullptr;
}

template <int M, int V>
static gemm_fn pick_slots(int S, int nstep, int build)
{
    if (S == 32) return pick_nstep<M, V, 32>(nstep, build);
    if constexpr (M <= 2) {
        if (S == 64) return pick_nstep<M, V, 64>(nstep, build);
    }
    return nullptr;
}

template <int V>
static gemm_fn pick_m(int m, int S, int nstep, int build)
{
    switch (m) {
        case 1: return pick_slots<1, V>(S, nstep, build);
        case 2: return pick_slots<2, V>(S, nstep, build);
        case 3: return pick_slots<3, V>(S, nstep, build);
        case 4: return pick_slots<4, V>(S, nstep, build);
    }
    return nullptr;
}

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

static int log2i(int x)
{
    int l = 0;
    while ((1 << l) < x) ++l;
    return l;
}

}  // namespace cg

using namespace cg;

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
    const size_t need = cbytes + (size_t)g.B * g.NKT * g.Npad * sizeof(float);
    if (workspace_bytes < need) return CODEGEMM_WORKSPACE_TOO_SMALL;

    gemm_fn fn = (g.v == 8) ? pick_m<8>(g.m, g.S, g.NSTEP, g.build) : pick_m<4>(g.m, g.S, g.NSTEP, g.build);
    if (!fn) return CODEGEMM_UNSUPPORTED;

    GemmParams p;
    p.x = static_cast<const _Float16*>(x);
    p.packed = packed_codes;
    p.codebooks = static_cast<const _Float16*>(codebooks);
    p.scales = static_cast<const _Float16*>(scales);
    p.y = y;
    p.counters = static_cast<uint32_t*>(workspace);
    p.partials = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + cbytes);
    p.B = g.B; p.K = g.K; p.N = g.N; p.J = g.J;
    p.RW = g.RW; p.JW = g.JW; p.log2JW = log2i(g.JW);
    p.NRB = g.NRB; p.NKT = g.NKT; p.Npad = g.Npad;
    p.y_fp32 = g.y_fp32 ? 1 : 0;

    const size_t lds = lds_bytes_gemm(g);
    if ((st = set_max_lds(reinterpret_cast<const void*>(fn), lds)) != CODEGEMM_OK) return st;
    const dim3 grid((unsigned)((size_t)g.NRT * g.NKT));
    const dim3 block((unsigned)(g.RW * g.JW * kWave));
    hipLaunchKernelGGL(fn, grid, block, lds, static_cast<hipStream_t>(stream), p);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}
