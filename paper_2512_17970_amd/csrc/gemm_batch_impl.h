// The hot path for batches (Section 3, Steps 1-3 with a batch axis on the Psumbook): four
// batch rows per pass over the codes.  Included by gemm_batch_m1.hip .. gemm_batch_m4.hip.
//
// With B > 1 the HBM bytes stay what they are while the gathers grow B-fold, so the bound
// moves from HBM to LDS and the vector ALU.  The batch axis is therefore made the
// innermost axis of the Psumbook: an entry is the 16-byte vector of the 4 batch rows'
// partial sums, one 128-bit LDS read fetches it, and the address arithmetic on a code is
// shared by the 4 rows.
//
// A "tile" is TS sub-vectors (8, or 16 when there is one codebook) of one 128-row unit.
// LDS layout of a tile's Psumbook: rows of 256 bytes, one per centroid index, holding 16
// columns of 16 bytes; column = (codebook parity, slot) for two or more codebooks,
// column = slot for one.  Pairs of codebooks form 64 KB "superplanes", as in the batch-1
// kernel, so the byte address (superplane << 16) | (code << 8) | (16 * column) is again
// assembled by one byte-permute.  The 16 lanes of a DPP row own the 16 columns: they read
// 16 different columns of (in general) 16 different rows, which covers every LDS bank
// exactly once whatever the codes are.  A lane therefore gathers for ONE codebook parity
// at ONE slot, for 8 rows x 4 batch rows (32 accumulators per row word), and the row
// totals are the sums over the 16 lanes of a DPP row.
//
// The build is the same MFMA contraction as in the batch-1 kernel with the 32 columns of
// a block re-read as (slot, batch row) pairs, batch row fastest: the accumulators of the
// 32 lanes of a half-wavefront are again 32 consecutive floats of one Psumbook row.
#pragma once

#include "gemm_impl.h"

namespace cg {

typedef __attribute__((address_space(3))) float4_t lds_float4;

// Sums 32 per-lane values over the 16 lanes of each DPP row.  On return lane l holds, in
// v[0] and v[1], the totals of values number i0 and i0 + 1 with
//   i0 = 16 * bit3(l) + 8 * bit2(l) + 4 * bit1(l) + 2 * bit0(l).
__device__ __forceinline__ void row16_transpose_sum(float (&v)[32], int lane)
{
    halve<0x128, 32>(v, (lane & 8) != 0);                  // row_ror:8
    float (&v16)[16] = reinterpret_cast<float (&)[16]>(v);
    halve<0x141, 16>(v16, (lane & 4) != 0);                // row_half_mirror: l <-> l ^ 7
    float (&v8)[8] = reinterpret_cast<float (&)[8]>(v);
    halve<0x4e, 8>(v8, (lane & 2) != 0);                   // quad_perm [2,3,0,1]: l <-> l ^ 2
    float (&v4)[4] = reinterpret_cast<float (&)[4]>(v);
    halve<0xb1, 4>(v4, (lane & 1) != 0);                   // quad_perm [1,0,3,2]: l <-> l ^ 1
}

// Psum lookup for 4 batch rows: same address assembly as psum_at, 128-bit read.
template <int k>
__device__ __forceinline__ float4_t psum4_at(uint32_t word, uint32_t off)
{
    const uint32_t addr = __builtin_amdgcn_perm(word, off, 0x0c020000u | ((4u + k) << 8));
    return *reinterpret_cast<const lds_float4*>(static_cast<uintptr_t>(addr));
}

template <int M, int V, int NW, int RPL, int D, bool GS, int NB = 0>
__global__ void __launch_bounds__(NW * 64) gemm_batch_kernel(CG_HEAD_PARAMS, const GemmParams pk)
{
    const GemmParams p = with_head(pk, hx, hpacked, hcodebooks, hgscales, hK, hNKT, hKPW, hB, hNGR, hmisc);
    constexpr int BG = 4;                              // batch rows per pass
    constexpr int TS = (M == 1) ? 16 : 8;              // sub-vectors per tile
    constexpr int TPU = kSlots / TS;                   // tiles per 32-slot unit
    constexpr int NBLOCKS = (M == 1) ? 16 : 8 * M;     // 32x32 MFMA blocks in one tile's Psumbook
    constexpr int TPW = (NBLOCKS + NW - 1) / NW;       // blocks per wavefront
    constexpr int XN = (M == 1) ? TPW : 1;             // distinct activation operands per wavefront and tile
    constexpr int SP = (M + 1) / 2;                    // superplanes
    // NB > 0: the last NB wavefronts build every Psumbook and nothing else, one tile ahead; the
    // first NG stream, gather and own the rows (see the batch-1 kernel).
    constexpr int NG = NW - NB;                        // wavefronts that own rows
    constexpr int PIECES = RPL * NG;                   // 32-row pieces (one row word of one wavefront) per workgroup
    typedef PsumLayout<M> L;
    constexpr int NBUF = L::kBuffers;
    static_assert(NW == 8 || NW == 16, "8 or 16 wavefronts");
    static_assert(NB == 0 || (NBUF == 2 && NBLOCKS % NB == 0 && 8 % NB == 0), "build-only wavefronts: a double-buffered Psumbook");
    static_assert((D & 1) == 0, "ring depth must be even (buffer parity is compile-time)");

    extern __shared__ __align__(16) unsigned char smem[];
    float* planes = reinterpret_cast<float*>(smem);                     // NBUF buffers of L::kBytes
    uint32_t* flag = reinterpret_cast<uint32_t*>(smem + NBUF * L::kBytes);

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be: keeps buffer descriptors in scalar registers
    const int ks = blockIdx.x;
    const Member mm = member_of(p, blockIdx.y);        // the layer this workgroup works for
    const int blk = blockIdx.y - mm.blk0;              // its row block of PIECES x 32 rows
    const int b0 = blockIdx.z * BG;
    const int kt0 = ks * p.KPW;
    const int nq = min(p.KPW, p.NKT - kt0);            // units of this workgroup (>= 1 by construction)
    const int ntiles = nq * TPU;
    const int J = p.K / V;
    // gather roles
    const int col = lane & 15;                         // Psumbook column of this lane
    const int oct = lane >> 4;                         // which of the wavefront's 4 row octets
    const int slot = (M == 1) ? col : (col & 7);
    const int par_cb = (M == 1) ? 0 : (col >> 3);      // codebook parity
    // build roles
    const int khalf = lane >> 5;
    const bool kvalid = 4 * khalf < V;
    typedef typename Frag<V>::type frag_t;
    constexpr int FE = frag_elems<V>();                // operand elements per lane
    const frag_t zero4 = {};

    CG_STAMP(0);
    constexpr uint32_t kRsrcFlags = 0x00020000u;       // raw 32-bit buffer, gfx9 family
    constexpr int kOutOfRange = 0x7ffffff0;            // beyond every descriptor: the load returns zeros

    // A codebook of odd M in the last superplane leaves the other half of its rows unused;
    // lanes of that parity read it with all-zero codes (row 0), so it must hold zeros.
    if (M >= 3 && (M & 1)) {
        for (int i = tid; i < NBUF * 256 * 32; i += NW * kWave)
            planes[(i / 8192) * (L::kBytes / 4) + (SP - 1) * 16384 + ((i % 8192) / 32) * 64 + 32 + (i % 32)] = 0.0f;
    }

    // Centroid operands of this wavefront's MFMA blocks: fixed for the whole kernel.
    // Block t: for M >= 2 codebook t / 8, centroids 32 * (t % 8)..+31, all TS = 8 slots;
    //          for M == 1 centroids 32 * (t % 8)..+31, slots 8 * (t / 8)..+7.
    frag_t cfrag[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        int t = wave + i * NW;
        if (t >= NBLOCKS) t = NBLOCKS - 1;
        const int cb = (M == 1) ? 0 : t / 8;
        if constexpr (NB > 0) cfrag[i] = zero4;        // the builders keep their own (below)
        else cfrag[i] = *reinterpret_cast<const frag_t*>(mm.codebooks + (size_t)((cb * 8 + t % 8) * 32 + (lane & 31)) * V + (kvalid ? FE * khalf : 0));
    }
    // Activation operand (Step 1): column n = lane % 32 of a block is (slot n / 4, batch row
    // n % 4); the lane supplies elements 4 * (lane / 32)..+3 of that sub-vector.  One
    // descriptor covers all of x; lanes whose batch row or sub-vector lies outside get an
    // out-of-range offset, i.e. zeros.
    const __amdgpu_buffer_rsrc_t x_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(p.x), 0, p.B * p.K * 2, kRsrcFlags);
    const int x_row = b0 + (lane & 3);
    int x_j0[XN], x_off0[XN];
#pragma unroll
    for (int i = 0; i < XN; ++i) {
        const int half_slots = (M == 1) ? ((wave + i * NW) / 8) * 8 : 0;
        x_j0[i] = kt0 * kSlots + half_slots + ((lane & 31) >> 2);
        x_off0[i] = (x_row * p.K + x_j0[i] * V + FE * khalf) * 2;
        if (!(kvalid && x_row < p.B)) x_j0[i] = J;                    // never valid
    }
    auto load_x = [&](int t, int i) -> frag_t {
        if constexpr (NB > 0) return zero4;            // a gathering wavefront loads no activations
        const bool ok = x_j0[i] + t * TS < J;
        const int off = ok ? x_off0[i] + t * (TS * V * 2) : kOutOfRange;
        if constexpr (V == 16) {
            return __builtin_bit_cast(frag_t, __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, off, 0, 0));
        } else {
            return __builtin_bit_cast(frag_t, __builtin_amdgcn_raw_buffer_load_b64(x_rsrc, off, 0, 0));
        }
    };
    // Codes of tile t for this lane: per row word q and superplane, the 8 bytes (8 rows) of
    // its codebook at its slot.  Word q of this wavefront is piece blk * PIECES + q * NG + wave of
    // the matrix: rows 32 * piece .. +31, i.e. row octets 4 * (piece % 4) + oct of granule piece / 4
    // (piece % 4 = wave % 4 for every q unless 14 wavefronts own the rows).
    constexpr int kUnitBytes = 128 * 32 * M;
    auto piece_of = [&](int q) -> int { return blk * PIECES + q * NG + wave; };
    int g16[RPL];
#pragma unroll
    for (int q = 0; q < RPL; ++q) g16[q] = (piece_of(q) & 3) * 4 + oct;
    __amdgpu_buffer_rsrc_t c_rsrc[RPL];
#pragma unroll
    for (int q = 0; q < RPL; ++q) {
        const int gr = piece_of(q) >> 2;
        const uint8_t* base = mm.packed + ((size_t)min(gr, mm.NGR - 1) * p.NKT + kt0) * kUnitBytes;
        c_rsrc[q] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, gr < mm.NGR ? nq * kUnitBytes : 0, kRsrcFlags);
    }
    int c_off[RPL][SP];
#pragma unroll
    for (int q = 0; q < RPL; ++q)
#pragma unroll
        for (int sp = 0; sp < SP; ++sp) {
            const bool single = (2 * sp + 1 == M);         // last part of an odd M: 8 bytes per entry, one codebook
            if (single) c_off[q][sp] = (par_cb == 0) ? sp * 8192 + (g16[q] * kSlots + slot) * 8 : kOutOfRange;
            else c_off[q][sp] = sp * 8192 + (g16[q] * kSlots + slot) * 16 + 8 * par_cb;
        }
    auto load_codes = [&](uint32_t (&dst)[RPL][SP][2], int t) {
        const int toff = (t / TPU) * kUnitBytes + (t % TPU) * TS * 16;
#pragma unroll
        for (int q = 0; q < RPL; ++q) {
#pragma unroll
            for (int sp = 0; sp < SP; ++sp) {
                const bool single = (2 * sp + 1 == M);
                const int o = c_off[q][sp] + (single ? (t / TPU) * kUnitBytes + (t % TPU) * TS * 8 : toff);
                const u32x2_t r = __builtin_amdgcn_raw_buffer_load_b64(c_rsrc[q], o, 0, 2);
                dst[q][sp][0] = r.x;
                dst[q][sp][1] = r.y;
            }
        }
    };
    // Group scales (Section 2.2, Step 1) of tile t for this lane: per row word, the 8 fp16
    // scales of its 8 rows for the group its slot belongs to in that tile, one 16-byte load;
    // a ring of their own, DS tiles deep.
    constexpr int DS = (D < 4) ? D : 4;
    __amdgpu_buffer_rsrc_t s_rsrc[GS ? RPL : 1];
    if constexpr (GS) {
#pragma unroll
        for (int q = 0; q < RPL; ++q) {
            const int gr = piece_of(q) >> 2;
            const uint8_t* base = mm.gscales + ((size_t)min(gr, mm.NGR - 1) * p.NKT + kt0) * p.GPU * 256;
            s_rsrc[q] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, gr < mm.NGR ? nq * p.GPU * 256 : 0, kRsrcFlags);
        }
    }
    auto load_scales = [&](half8_t (&dst)[RPL], int t) {
        const int group = ((t % TPU) * TS + slot) >> p.gshift;       // of the tile's unit
        const int o = ((t / TPU) * p.GPU + group) * 256;
#pragma unroll
        for (int q = 0; q < RPL; ++q)
            dst[q] = __builtin_bit_cast(half8_t, __builtin_amdgcn_raw_buffer_load_b128(s_rsrc[GS ? q : 0], o + g16[q] * 16, 0, 0));
    };
    auto build = [&](float* buf, const frag_t (&xf)[XN]) {
        if constexpr (NB > 0) return;                  // not this wavefront's job
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int t = wave + i * NW;
            // t / 8 selects superplane and row half: the codebook, or for M == 1 the slot half
            if (NBLOCKS % NW == 0 || t < NBLOCKS)
                mfma_block_to_lds<(M == 1) ? 2 : M, V>(buf, t / 8, t % 8, lane, kvalid ? cfrag[i] : zero4, xf[(M == 1) ? i : 0]);
        }
    };

    if constexpr (NB > 0) {
        if (wave >= NG) {
            // A builder: blocks (wave - NG) + i * NB of every tile's Psumbook, one tile ahead of the
            // gatherers, through the same barriers (one after the first table, one per tile).
            constexpr int TB = NBLOCKS / NB;
            constexpr int XB = (M == 1) ? 2 : 1;       // one codebook: the two slot halves have their own operands
            frag_t cb[TB];
#pragma unroll
            for (int i = 0; i < TB; ++i) {
                const int t = (wave - NG) + i * NB;
                const int c = (M == 1) ? 0 : t / 8;
                cb[i] = *reinterpret_cast<const frag_t*>(mm.codebooks + (size_t)((c * 8 + t % 8) * 32 + (lane & 31)) * V + (kvalid ? FE * khalf : 0));
                if (!kvalid) cb[i] = zero4;
            }
            int xb_j0[XB], xb_off0[XB];
#pragma unroll
            for (int h = 0; h < XB; ++h) {
                xb_j0[h] = kt0 * kSlots + h * 8 + ((lane & 31) >> 2);
                xb_off0[h] = (x_row * p.K + xb_j0[h] * V + FE * khalf) * 2;
                if (!(kvalid && x_row < p.B)) xb_j0[h] = J;                   // never valid
            }
            auto load_xb = [&](frag_t (&dst)[XB], int t) {
#pragma unroll
                for (int h = 0; h < XB; ++h) {
                    const bool ok = xb_j0[h] + t * TS < J;
                    const int off = ok ? xb_off0[h] + t * (TS * V * 2) : kOutOfRange;
                    if constexpr (V == 16) dst[h] = __builtin_bit_cast(frag_t, __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, off, 0, 0));
                    else dst[h] = __builtin_bit_cast(frag_t, __builtin_amdgcn_raw_buffer_load_b64(x_rsrc, off, 0, 0));
                }
            };
            // software pipeline: the product of the next block is issued before the stores of the current one
            auto build_all = [&](float* buf, const frag_t (&xf)[XB]) {
                float16_t cur = mfma_block<V>(cb[0], xf[0]);
#pragma unroll
                for (int i = 0; i < TB; ++i) {
                    float16_t nxt = cur;
                    // (block t belongs to slot half t / 8 = i * NB / 8: NB divides 8, so the wavefront's own
                    // offset never carries into it and the operand index is a compile-time constant)
                    if (i + 1 < TB) nxt = mfma_block<V>(cb[i + 1], xf[(M == 1) ? ((i + 1) * NB) / 8 : 0]);
                    __builtin_amdgcn_sched_barrier(0);
                    const int t = (wave - NG) + i * NB;
                    block_to_lds<(M == 1) ? 2 : M>(buf, t / 8, t % 8, lane, cur);
                    __builtin_amdgcn_sched_barrier(0);
                    cur = nxt;
                }
            };
            frag_t xs[2][XB];
            load_xb(xs[0], 0);
            load_xb(xs[1], 1);
            build_all(planes, xs[0]);
            load_xb(xs[0], 2);
            __syncthreads();
            for (int t0 = 0; t0 < ntiles; t0 += D) {
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const int t = t0 + d;
                    if (t + 1 < ntiles) build_all(planes + ((d + 1) & 1) * (L::kBytes / 4), xs[(d + 1) & 1]);
                    load_xb(xs[(d + 1) & 1], t + 3);
                    __syncthreads();
                }
            }
            finish_block<NW * kWave, BG, PIECES * 32>(p, mm, planes, flag, tid, blk, ks, b0);
            return;
        }
    }

    // Prologue: activations of the first D tiles and codes of the first; the rest of the code
    // ring is requested after the first Psumbook has been written (as in the batch-1 kernel).
    frag_t xr[D][XN];
    uint32_t w[D][RPL][SP][2];
#pragma unroll
    for (int d = 0; d < D; ++d)
#pragma unroll
        for (int i = 0; i < XN; ++i) xr[d][i] = load_x(d, i);
    __builtin_amdgcn_sched_barrier(0);
    load_codes(w[0], 0);
    half8_t sc[GS ? DS : 1][RPL];
    if constexpr (GS) {
#pragma unroll
        for (int d = 0; d < DS; ++d) load_scales(sc[d], d);
    }
    __builtin_amdgcn_sched_barrier(0);

    float acc[RPL][kRowsPerLane][BG];
#pragma unroll
    for (int q = 0; q < RPL; ++q)
#pragma unroll
        for (int r = 0; r < kRowsPerLane; ++r)
#pragma unroll
            for (int bb = 0; bb < BG; ++bb) acc[q][r][bb] = 0.0f;

    const uint32_t col16 = (uint32_t)reinterpret_cast<uintptr_t>((lds_float*)planes) + (uint32_t)col * 16u;

    CG_STAMP(2);
    build(planes, xr[0]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int d = 1; d < D; ++d) load_codes(w[d], d);
#pragma unroll
    for (int i = 0; i < XN; ++i) xr[0][i] = load_x(D, i);
    __syncthreads();
    CG_STAMP(1);

    // Main loop over the tiles.  In every iteration the matrix cores build the next tile's
    // Psumbook while the lanes gather the current one (one buffer and two barriers per tile
    // when only one buffer fits).  Loads run unconditionally; past the end they return zeros
    // without memory traffic.
    for (int t0 = 0; t0 < ntiles; t0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int t = t0 + d;
            const int par = (NBUF == 2) ? (d & 1) : 0;
            float* nxt = planes + (NBUF == 2 ? (par ^ 1) : 0) * (L::kBytes / 4);
            auto gather = [&]() {
#pragma unroll
                for (int q = 0; q < RPL; ++q) {
#pragma unroll
                    for (int sp = 0; sp < SP; ++sp) {
                        asm volatile("" : "+v"(w[d][q][sp][0]));
                        asm volatile("" : "+v"(w[d][q][sp][1]));
                        const uint32_t off = col16 + ((uint32_t)(sp + par * SP) << 16);
                        const uint32_t lo = w[d][q][sp][0], hi = w[d][q][sp][1];
                        float4_t f[8];
                        f[0] = psum4_at<0>(lo, off);
                        f[1] = psum4_at<1>(lo, off);
                        f[2] = psum4_at<2>(lo, off);
                        f[3] = psum4_at<3>(lo, off);
                        f[4] = psum4_at<0>(hi, off);
                        f[5] = psum4_at<1>(hi, off);
                        f[6] = psum4_at<2>(hi, off);
                        f[7] = psum4_at<3>(hi, off);
                        const half8_t sv = sc[GS ? d % DS : 0][q];
#pragma unroll
                        for (int r = 0; r < 8; ++r) {
                            acc[q][r][0] = accumulate<GS>(acc[q][r][0], f[r].x, sv[r]);
                            acc[q][r][1] = accumulate<GS>(acc[q][r][1], f[r].y, sv[r]);
                            acc[q][r][2] = accumulate<GS>(acc[q][r][2], f[r].z, sv[r]);
                            acc[q][r][3] = accumulate<GS>(acc[q][r][3], f[r].w, sv[r]);
                        }
                    }
                }
            };
            if (t < ntiles) gather();
            if (NBUF == 1) __syncthreads();                // single buffer: everyone is done reading before it is rebuilt
            if (t + 1 < ntiles) build(nxt, xr[(d + 1) % D]);
#pragma unroll
            for (int i = 0; i < XN; ++i) xr[(d + 1) % D][i] = load_x(t + 1 + D, i);   // its ring slot is free again
            load_codes(w[d], t + D);
            if constexpr (GS) load_scales(sc[d % DS], t + DS);
            __syncthreads();
            CG_STAMP(8 + (t < 7 ? t : 7));
        }
    }
    CG_STAMP(4);

    // Row totals = sums over the 16 lanes of a DPP row; parked in LDS (the Psumbook is no
    // longer needed) as [batch row][row of the block].
    constexpr int ROWS = PIECES * 32;
    float* stage = planes;
    {
        const int l = lane & 15;
        const int i0 = ((l >> 3) & 1) * 16 + ((l >> 2) & 1) * 8 + ((l >> 1) & 1) * 4 + (l & 1) * 2;
        const int r = i0 >> 2, bb = i0 & 3;            // i = 4 * row + batch row
#pragma unroll
        for (int q = 0; q < RPL; ++q) {
            float v[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) v[i] = acc[q][i >> 2][i & 3];
            row16_transpose_sum(v, lane);
            const int local = (q * NG + wave) * 32 + oct * kRowsPerLane + r;      // piece, row octet, row
            stage[bb * ROWS + local] = v[0];
            stage[(bb + 1) * ROWS + local] = v[1];
        }
    }
    finish_block<NW * kWave, BG, ROWS>(p, mm, stage, flag, tid, blk, ks, b0);
}

template <int M, int V, int NW, int RPL, int D, bool GS, int NB = 0>
int launch_gemm_batch_one(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    auto fn = gemm_batch_kernel<M, V, NW, RPL, D, GS, NB>;
    typedef PsumLayout<M> L;
    const size_t lds = (size_t)L::kBuffers * L::kBytes + 64;
    int st = set_max_lds(reinterpret_cast<const void*>(fn), lds);
    if (st != CODEGEMM_OK) return st;
    const dim3 grid((unsigned)g.NKS, (unsigned)g.NBLK, (unsigned)g.NG);
    hipLaunchKernelGGL(fn, grid, dim3(NW * kWave), lds, stream, CG_HEAD_ARGS(p), p);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}

template <int M, int V, bool GS>
int launch_gemm_batch_v(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    if constexpr (M <= 2) {
        // 14 gathering + 2 building wavefronts: blocks of 448 or 896 rows
        if (g.NW == 16 && g.RPL == 1 && g.NB == 2) return launch_gemm_batch_one<M, V, 16, 1, 2, GS, 2>(g, p, stream);
        if (g.NW == 16 && g.RPL == 2 && g.NB == 2) return launch_gemm_batch_one<M, V, 16, 2, 2, GS, 2>(g, p, stream);
    }
    if (g.NB != 0) return CODEGEMM_UNSUPPORTED;
    if (g.NW == 16 && g.RPL == 1) return launch_gemm_batch_one<M, V, 16, 1, 2, GS>(g, p, stream);
    if (g.NW == 8 && g.RPL == 1) return launch_gemm_batch_one<M, V, 8, 1, 2, GS>(g, p, stream);
    if (g.NW == 8 && g.RPL == 2) return launch_gemm_batch_one<M, V, 8, 2, 2, GS>(g, p, stream);
    if (g.NW == 8 && g.RPL == 4) return launch_gemm_batch_one<M, V, 8, 4, 2, GS>(g, p, stream);
    if (g.NW == 16 && g.RPL == 2) return launch_gemm_batch_one<M, V, 16, 2, 2, GS>(g, p, stream);
    return CODEGEMM_UNSUPPORTED;
}

template <int M, bool GS>
int launch_gemm_batch_m(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    if (g.v == 16) return launch_gemm_batch_v<M, 16, GS>(g, p, stream);
    if (g.v == 8) return launch_gemm_batch_v<M, 8, GS>(g, p, stream);
    if (g.v == 4) return launch_gemm_batch_v<M, 4, GS>(g, p, stream);
    return CODEGEMM_UNSUPPORTED;
}

int launch_gemm_batch_m1(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_batch_m2(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_batch_m3(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_batch_m4(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_batch_gs_m1(const Geometry& g, const GemmParams& p, hipStream_t stream);   // with group scales
int launch_gemm_batch_gs_m2(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_batch_gs_m3(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_batch_gs_m4(const Geometry& g, const GemmParams& p, hipStream_t stream);

}  // namespace cg
