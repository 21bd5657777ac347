// The hot path: fused Psumbook build + gather-by-code GEMV/GEMM (Section 3, Steps 1-3)
// followed by the row scale, for gfx950.  Included by one translation unit per number
// of codebooks (gemm_m1.hip .. gemm_m4.hip), which instantiate the kernels they need.
//
// Work decomposition.  The weight matrix is cut into "units" of 512 rows by S
// sub-vectors (S * v weights along K); the packed codes of a unit are contiguous in
// HBM, and so are the units of consecutive K tiles of one row block.  One workgroup of
// NW wavefronts owns one row block (512 rows) and a contiguous range of K tiles, and
// streams through its units:
//   * lane l of every wavefront owns rows 64*r + l (r = 0..7) of the block and keeps
//     their 8 accumulators in registers for the whole range; the NW wavefronts split
//     the S slots of a tile (NSTEP = S / NW steps each);
//   * the codes of the next D units are always in flight (a register ring of
//     16-byte loads), so HBM streams continuously with a bounded queue;
//   * while the lanes gather unit u from one Psumbook buffer in LDS, the matrix cores
//     build the Psumbook of unit u+1 (Eq. 2) into the other buffer: 32x32x8 fp16 MFMA
//     blocks, one or two per wavefront, whose centroid operands stay in registers for
//     the whole kernel and whose activation operand is 8 bytes per lane per unit.
//     One barrier per unit separates the two;
//   * in step t lane l works on slot (t + l) mod S, so the 64 lanes of a wavefront
//     always address 64 (at S = 32: 2 x 32) different slots = different LDS banks,
//     whatever the code values are;
//   * at the end of the range the NW wavefronts add their accumulators through LDS,
//     the workgroup writes one fp32 partial per row to the workspace, and the last
//     workgroup to finish a row block (atomic ticket) adds the K ranges' partials in
//     range order, multiplies by the row scale and stores y.
// Batch rows are processed in groups of BG (1, 2 or 4) per pass over the codes: the
// code words in registers are reused for the BG Psumbooks of a unit; groups are
// separate workgroups (grid.y).
//
// LDS layout of the Psumbook.  Rows of 256 bytes, one per centroid index, grouped in
// "superplanes" of 256 rows (64 KB).  With S = 64 a row holds the 64 slots of one
// codebook (codebook c = superplane c).  With S = 32 a row holds 32 slots of two
// codebooks (codebook c = superplane c/2, byte offset 128*(c%2)).  The byte address
//     (superplane << 16) | (code << 8) | (sub-offset + 4*slot)
// is then assembled from a code byte by a single byte-permute instruction.
#pragma once

#include "cg_common.h"

namespace cg {

struct GemmParams {
    const _Float16* x;
    const uint8_t* packed;
    const _Float16* codebooks;
    const _Float16* scales;
    void* y;
    float* partials;             // [B][NKS][Npad]
    uint32_t* counters;          // [groups][NRB]
    int B, K, N;
    int NRB, NKT, NKS, KPW, Npad;
    int y_fp32;
    unsigned long long* trace;   // [grid][16] timestamps (100 MHz) when built with CODEGEMM_TRACE, else unused
};

#ifdef CODEGEMM_TRACE
#define CG_STAMP(k) do { if (p.trace && threadIdx.x == 0 && blockIdx.y == 0) p.trace[(size_t)blockIdx.x * 16 + (k)] = wall_clock64(); } while (0)
#else
#define CG_STAMP(k) do { } while (0)
#endif

template <int M, int S>
struct PsumLayout {
    static constexpr int kSuperplanes = (S == 64) ? M : (M + 1) / 2;
    static constexpr int kBytes = kSuperplanes * 65536;                 // one buffer
    static constexpr int kBuffers = (2 * kBytes <= 131072) ? 2 : 1;     // double-buffer when it fits
    __host__ __device__ static constexpr int superplane(int c) { return (S == 64) ? c : c / 2; }
    __host__ __device__ static constexpr int sub_bytes(int c) { return (S == 64) ? 0 : 128 * (c % 2); }
};

// One 32x32 block of the Psumbook on the matrix cores:
//   D[i][slot] = sum_k C[c][32*iblk + i][k] * x[32*sblk + slot][k]
// Lane l supplies row / column l%32 with k = 4*(l/32)..+3 (for v = 4 the upper half of
// the contraction is fed zeros) and receives D[8*blk + 4*(l/32) + e][l%32] in
// accumulator 4*blk + e; for fixed (blk, e) the 32 lanes of a half-wavefront write 32
// consecutive slots of one row.
template <int M, int S>
__device__ __forceinline__ void mfma_block_to_lds(float* buf, int c, int iblk, int sblk, int lane,
                                                  half4_t cfrag, half4_t xfrag)
{
    float16_t d = {0};
    d = __builtin_amdgcn_mfma_f32_32x32x8f16(cfrag, xfrag, d, 0, 0, 0);
    float* dst = buf + PsumLayout<M, S>::superplane(c) * 16384 + PsumLayout<M, S>::sub_bytes(c) / 4 +
                 (iblk * 32 + 4 * (lane >> 5)) * 64 + sblk * 32 + (lane & 31);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[(8 * blk + e) * 64] = d[4 * blk + e];
}

// LDS byte address of a Psum: byte 0 <- low byte of `off` (sub-offset + 4*slot), byte 1 <-
// code byte `k` of `word`, byte 2 <- byte 2 of `off` (buffer and superplane), byte 3 <- 0.
template <int k>
__device__ __forceinline__ uint32_t psum_addr(uint32_t word, uint32_t off)
{
    return __builtin_amdgcn_perm(word, off, 0x0c020000u | ((4u + k) << 8));
}

template <int M, int V, int S, int NW, int BG>
__global__ void __launch_bounds__(NW * 64) gemm_kernel(const GemmParams p)
{
    constexpr int NSTEP = S / NW;                      // gather steps per wavefront per unit
    constexpr int NT = NW * kWave;
    constexpr int SB = S / 32;
    constexpr int NTILES = 8 * M * SB;                 // 32x32 MFMA blocks in one Psumbook
    constexpr int TPW = (NTILES + NW - 1) / NW;        // blocks per wavefront
    constexpr int D = 4;                               // units of codes in flight per lane
    typedef PsumLayout<M, S> L;
    constexpr int NBUF = L::kBuffers;
    static_assert(NSTEP >= 1 && NSTEP * NW == S, "slots must split evenly over the wavefronts");
    static_assert((D & 1) == 0, "ring depth must be even (buffer parity is compile-time)");

    extern __shared__ __align__(16) unsigned char smem[];
    float* planes = reinterpret_cast<float*>(smem);                     // NBUF buffers of L::kBytes
    uint32_t* flag = reinterpret_cast<uint32_t*>(smem + NBUF * L::kBytes);

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int ks = blockIdx.x % p.NKS;
    const int rb = blockIdx.x / p.NKS;
    const int b0 = blockIdx.y * BG;
    const int kt0 = ks * p.KPW;
    const int nq = min(p.KPW, p.NKT - kt0);            // units of this workgroup (>= 1 by construction)
    const int khalf = lane >> 5;
    const bool kvalid = 4 * khalf < V;
    const half4_t zero4 = {0, 0, 0, 0};

    CG_STAMP(0);
    // Every global load below is unconditional (out-of-range units read a small, cache-
    // resident dummy address and out-of-range lanes are zeroed only where the value is
    // used): the hardware returns loads in issue order and the compiler can count
    // outstanding loads exactly only along branch-free code.
    //
    // Centroid operands of this wavefront's MFMA blocks: fixed for the whole kernel.
    half4_t cfrag[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        int tile = wave + i * NW;
        if (tile >= NTILES) tile = NTILES - 1;
        const int ci = tile / SB;                      // c*8 + iblk
        cfrag[i] = *reinterpret_cast<const half4_t*>(p.codebooks + (size_t)(ci * 32 + (lane & 31)) * V + (kvalid ? 4 * khalf : 0));
    }
    // Activation operand: sub-vector (kt*S + 32*sblk + l%32), elements 4*(l/32)..+3 (Step 1).
    const int xe0 = ((wave % SB) * 32 + (lane & 31)) * V + (kvalid ? 4 * khalf : 0);
    auto x_valid = [&](int u) -> bool { return kvalid && u < nq && (kt0 + u) * S * V + xe0 < p.K; };
    auto load_x = [&](int u, int bb) -> half4_t {
        const int e = (kt0 + u) * S * V + xe0;
        const int row = min(b0 + bb, p.B - 1);
        return *reinterpret_cast<const half4_t*>(p.x + (size_t)row * p.K + ((u < nq && e < p.K) ? e : 0));
    };
    // Codes of unit u for this lane: NSTEP steps of 8*M bytes.
    const uint8_t* code_base = p.packed + (((size_t)rb * p.NKT + kt0) * S + wave * NSTEP) * (size_t)step_bytes(M) + (size_t)lane * 16;
    const uint8_t* dummy_base = reinterpret_cast<const uint8_t*>(p.codebooks) + (size_t)lane * 16;
    auto load_codes = [&](uint32_t (&dst)[NSTEP][2 * M], int u) {
        // units past the end of the range re-read the first 1 KB of the codebooks (L2 hits)
        const bool real = u < nq;
        const uint8_t* ub = real ? code_base + (size_t)u * S * step_bytes(M) : dummy_base;
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            const uint8_t* sb = ub + (real ? (size_t)st * step_bytes(M) : 0);
#pragma unroll
            for (int part = 0; part < (M + 1) / 2; ++part) {
                if (2 * part + 1 == M) {
                    // 8-byte part: lane offset is 8, not 16
                    const u32x2_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(sb + (real ? part * 16 * kWave : 0) - (size_t)lane * 8));
                    dst[st][4 * part + 0] = t.x;
                    dst[st][4 * part + 1] = t.y;
                } else {
                    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(sb + (real ? part * 16 * kWave : 0)));
                    dst[st][4 * part + 0] = t.x;
                    dst[st][4 * part + 1] = t.y;
                    dst[st][4 * part + 2] = t.z;
                    dst[st][4 * part + 3] = t.w;
                }
            }
        }
    };
    auto build = [&](float* buf, half4_t xraw, bool xok) {
        const half4_t xf = xok ? xraw : zero4;
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int tile = wave + i * NW;
            if (NTILES % NW == 0 || tile < NTILES) {
                const int ci = tile / SB;
                mfma_block_to_lds<M, S>(buf, ci / 8, ci % 8, tile % SB, lane, kvalid ? cfrag[i] : zero4, xf);
            }
        }
    };

    // Prologue: activations of the first D units, then codes of the first D units.
    half4_t xr[D][BG];
    uint32_t w[D][NSTEP][2 * M];
#pragma unroll
    for (int d = 0; d < D; ++d)
#pragma unroll
        for (int bb = 0; bb < BG; ++bb) xr[d][bb] = load_x(d, bb);
    __builtin_amdgcn_sched_barrier(0);
    // The compute unit serves vector loads in issue order across its wavefronts: the
    // barrier puts every wavefront's (small, L2-resident) build inputs ahead of all code
    // loads of the workgroup, so the first Psumbook does not wait behind 100+ KB of codes.
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int d = 0; d < D; ++d) load_codes(w[d], d);
    __builtin_amdgcn_sched_barrier(0);

    float acc[BG][kRowsPerLane];
#pragma unroll
    for (int bb = 0; bb < BG; ++bb)
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) acc[bb][r] = 0.0f;

    // Slot of this lane in step st: (wave*NSTEP + st + lane) mod S; constant for the kernel.
    uint32_t slot4[NSTEP];
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) slot4[st] = (uint32_t)((wave * NSTEP + st + lane) & (S - 1)) * 4u;

    // Psumbook of (unit 0, batch row 0).
    CG_STAMP(2);
    build(planes, xr[0][0], x_valid(0));
    if (BG == 1) xr[0][0] = load_x(D, 0);
    __syncthreads();
    CG_STAMP(1);

    // Main loop over the sequence (unit u, batch row bb).  In every iteration the matrix
    // cores build the next Psumbook of the sequence while the lanes gather the current one.
    // Builds and loads run unconditionally (past the end they work on dummy data nobody
    // reads); only the gather is skipped for units past the end.
    for (int u0 = 0; u0 < nq; u0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int u = u0 + d;
#pragma unroll
            for (int bb = 0; bb < BG; ++bb) {
                const int par = (NBUF == 2) ? ((BG == 1) ? (d & 1) : (bb & 1)) : 0;   // buffer of the current Psumbook
                float* nxt = planes + (NBUF == 2 ? (par ^ 1) : 0) * (L::kBytes / 4);
                const bool last_bb = (bb == BG - 1);
                const bool has_next = !last_bb || u + 1 < nq;
                if (NBUF == 2) {
                    // build the next Psumbook of the sequence into the other buffer
                    if (has_next) {
                        if (last_bb) build(nxt, xr[(d + 1) % D][0], x_valid(u + 1));
                        else build(nxt, xr[d][(bb + 1) % BG], x_valid(u));
                    }
                    if (BG == 1) xr[(d + 1) % D][0] = load_x(u + 1 + D, 0);   // its slot is free again
                }
                // gather the current one (Step 3)
                if (u < nq) {
                    const unsigned char* pb = reinterpret_cast<const unsigned char*>(planes);
#pragma unroll
                    for (int st = 0; st < NSTEP; ++st) {
                        // Opaque to the optimiser: keeps the address arithmetic on the codes
                        // here instead of hoisting it out of the loops into registers.
#pragma unroll
                        for (int i = 0; i < 2 * M; ++i) asm volatile("" : "+v"(w[d][st][i]));
#pragma unroll
                        for (int c = 0; c < M; ++c) {
                            const uint32_t off = slot4[st] + (uint32_t)L::sub_bytes(c) +
                                                 ((uint32_t)(L::superplane(c) + par * L::kSuperplanes) << 16);
                            const uint32_t lo = w[d][st][2 * c], hi = w[d][st][2 * c + 1];
                            acc[bb][0] += *reinterpret_cast<const float*>(pb + psum_addr<0>(lo, off));
                            acc[bb][1] += *reinterpret_cast<const float*>(pb + psum_addr<1>(lo, off));
                            acc[bb][2] += *reinterpret_cast<const float*>(pb + psum_addr<2>(lo, off));
                            acc[bb][3] += *reinterpret_cast<const float*>(pb + psum_addr<3>(lo, off));
                            acc[bb][4] += *reinterpret_cast<const float*>(pb + psum_addr<0>(hi, off));
                            acc[bb][5] += *reinterpret_cast<const float*>(pb + psum_addr<1>(hi, off));
                            acc[bb][6] += *reinterpret_cast<const float*>(pb + psum_addr<2>(hi, off));
                            acc[bb][7] += *reinterpret_cast<const float*>(pb + psum_addr<3>(hi, off));
                        }
                    }
                }
                if (NBUF == 1) {
                    // single buffer: everyone must be done reading before it is rebuilt
                    __syncthreads();
                    if (has_next) {
                        if (last_bb) build(nxt, xr[(d + 1) % D][0], x_valid(u + 1));
                        else build(nxt, xr[d][(bb + 1) % BG], x_valid(u));
                    }
                    if (BG == 1) xr[(d + 1) % D][0] = load_x(u + 1 + D, 0);
                }
                if (last_bb) load_codes(w[d], u + D);                       // refill the code ring
                __syncthreads();
            }
            CG_STAMP(8 + (u < 7 ? u : 7));
            if (BG > 1) {
                // activations of unit u+D for all rows of the group (ring slot d is free now)
#pragma unroll
                for (int bb = 0; bb < BG; ++bb) xr[d][bb] = load_x(u + D, bb);
            }
        }
    }
    CG_STAMP(4);

    // Add the accumulators of the NW wavefronts (all hold the same 512 rows) through LDS.
    float* red = planes;                                // BG * NW * 512 floats <= 128 KB
#pragma unroll
    for (int bb = 0; bb < BG; ++bb)
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r) red[(bb * NW + wave) * kBlockRows + r * kWave + lane] = acc[bb][r];
    __syncthreads();
    const int n_base = rb * kBlockRows;
    for (int o = tid; o < BG * kBlockRows; o += NT) {
        const int bb = o / kBlockRows;
        const int idx = o % kBlockRows;
        float sum = 0.0f;
#pragma unroll
        for (int q = 0; q < NW; ++q) sum += red[(bb * NW + q) * kBlockRows + idx];
        const int n = n_base + idx;
        const int row = b0 + bb;
        if (row >= p.B) continue;
        if (p.NKS == 1) {
            if (n < p.N) {
                const float val = sum * (float)p.scales[n];
                if (p.y_fp32) static_cast<float*>(p.y)[(size_t)row * p.N + n] = val;
                else static_cast<_Float16*>(p.y)[(size_t)row * p.N + n] = (_Float16)val;
            }
        } else {
            // write-through store, visible device-wide once acknowledged
            __hip_atomic_store(p.partials + ((size_t)row * p.NKS + ks) * p.Npad + n, sum,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    CG_STAMP(5);
    if (p.NKS == 1) return;

    // Ticket: the last workgroup of this row block combines the K ranges' partials.
    // Every datum that crosses workgroups is moved by device-scope atomic accesses
    // (write-through stores, cache-bypassing loads, one RMW on the counter), so no
    // L2 write-back / invalidate is needed: each thread waits for its own partial
    // stores to be acknowledged, the barrier collects that for the workgroup, and only
    // then is the ticket taken.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    CG_STAMP(6);
    // the scale of this thread's row(s), requested before the ticket round trip
    const int n_mine = n_base + tid % kBlockRows;
    const _Float16 scale_mine = p.scales[n_mine < p.N ? n_mine : 0];
    if (tid == 0) {
        uint32_t* ctr = p.counters + (size_t)blockIdx.y * p.NRB + rb;
        const uint32_t old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = old == (uint32_t)(p.NKS - 1);
        if (last) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
        *flag = last ? 1u : 0u;
    }
    __syncthreads();
    CG_STAMP(7);
    if (*flag == 0u) return;
    for (int o = tid; o < BG * kBlockRows; o += NT) {
        const int bb = o / kBlockRows;
        const int n = n_base + o % kBlockRows;
        const int row = b0 + bb;
        if (row >= p.B || n >= p.N) continue;
        const float* src = p.partials + (size_t)row * p.NKS * p.Npad + n;
        float sum = 0.0f;
        int k2 = 0;
        for (; k2 + 8 <= p.NKS; k2 += 8) {              // 8 loads in flight, added in range order
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                v[i] = __hip_atomic_load(src + (size_t)(k2 + i) * p.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += v[i];
        }
        for (; k2 < p.NKS; ++k2)
            sum += __hip_atomic_load(src + (size_t)k2 * p.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float val = sum * (float)((NT % kBlockRows == 0 || kBlockRows % NT == 0) ? scale_mine : p.scales[n]);
        if (p.y_fp32) static_cast<float*>(p.y)[(size_t)row * p.N + n] = val;
        else static_cast<_Float16*>(p.y)[(size_t)row * p.N + n] = (_Float16)val;
    }
    CG_STAMP(3);
}

int set_max_lds(const void* fn, size_t bytes);

template <int M, int V, int S, int NW, int BG>
int launch_gemm_one(const GemmParams& p, int groups, hipStream_t stream)
{
    auto fn = gemm_kernel<M, V, S, NW, BG>;
    typedef PsumLayout<M, S> L;
    size_t lds = (size_t)L::kBuffers * L::kBytes;
    const size_t red = (size_t)BG * NW * kBlockRows * sizeof(float);
    if (red > lds) lds = red;
    lds += 64;
    if (lds > (size_t)kMaxLds) return CODEGEMM_UNSUPPORTED;
    int st = set_max_lds(reinterpret_cast<const void*>(fn), lds);
    if (st != CODEGEMM_OK) return st;
    hipLaunchKernelGGL(fn, dim3((unsigned)((size_t)p.NRB * p.NKS), (unsigned)groups), dim3(NW * kWave), lds, stream, p);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}

template <int M, int V, int BG>
int launch_gemm_mvb(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    const int groups = ceil_div(g.B, BG);
#define CG_CASE(S_, NW_)                                                                    \
    if (g.S == S_ && g.NW == NW_) {                                                         \
        if constexpr ((S_ == 32 || M <= 2) && (S_ / NW_) * M <= 8)                          \
            return launch_gemm_one<M, V, S_, NW_, BG>(p, groups, stream);                   \
        else                                                                                \
            return CODEGEMM_UNSUPPORTED;                                                    \
    }
    CG_CASE(32, 16) CG_CASE(64, 16) CG_CASE(32, 8) CG_CASE(64, 8)
#undef CG_CASE
    return CODEGEMM_UNSUPPORTED;
}

template <int M>
int launch_gemm_m(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    if (g.v == 8) {
        switch (g.BG) {
            case 1: return launch_gemm_mvb<M, 8, 1>(g, p, stream);
            case 2: return launch_gemm_mvb<M, 8, 2>(g, p, stream);
            case 4: return launch_gemm_mvb<M, 8, 4>(g, p, stream);
        }
    } else {
        switch (g.BG) {
            case 1: return launch_gemm_mvb<M, 4, 1>(g, p, stream);
            case 2: return launch_gemm_mvb<M, 4, 2>(g, p, stream);
            case 4: return launch_gemm_mvb<M, 4, 4>(g, p, stream);
        }
    }
    return CODEGEMM_UNSUPPORTED;
}

int launch_gemm_m1(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_m2(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_m3(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_m4(const Geometry& g, const GemmParams& p, hipStream_t stream);

}  // namespace cg
