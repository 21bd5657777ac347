// The hot path: fused Psumbook build + gather-by-code GEMV/GEMM (Section 3, Steps 1-3)
// with the row scale applied at the end, or group scales (Section 2.2, Step 1) applied as
// the partial sums are accumulated, for gfx950.  Included by one translation unit per
// number of codebooks and scale kind (gemm_m1.hip .. gemm_m4.hip, gemm_gs_m1.hip ..
// gemm_gs_m4.hip), which instantiate the kernels they need.
//
// Work decomposition.  A "unit" is 128 rows by 32 sub-vectors (32 * v weights along K);
// its packed codes are contiguous in HBM, and so are the units of consecutive K tiles
// of one 128-row granule.  One workgroup of NW (8, 14 or 16) wavefronts owns 16 * NW * RPL
// consecutive rows, i.e. RPL * NW/8 granules (3.5 of them with 14 wavefronts and RPL = 2:
// rows are indexed by 16-row pieces of a granule), and a contiguous range of K tiles (all
// of K when k_splits = 1), and streams through them:
//   * a half-wavefront (32 lanes) owns RPL words of 8 rows; its lane s works
//     on slot s of every K tile, so the 32 lanes always address 32 different slots = 32
//     different LDS banks, whatever the code values are, and the 8 * RPL accumulators
//     of a lane stay in registers for the whole range;
//   * the codes of the next D = 2 units are requested ahead (a register ring of 16-byte
//     loads): about what a compute unit can keep outstanding, so HBM streams continuously
//     and no wavefront stands blocked at the issue of a load while it should gather;
//   * while the lanes gather unit u from one Psumbook buffer in LDS, the matrix cores
//     build the Psumbook of unit u+1 (Eq. 2) into the other buffer: 32x32x8 fp16 MFMA
//     blocks whose centroid operands stay in registers for the whole kernel and whose
//     activation operand is 8 bytes per lane per unit.  One barrier per unit;
//   * at the end the 32 lanes of a half-wavefront are summed with a transposing DPP
//     reduction.  With k_splits = 1 that is the result: it is scaled and stored, and
//     no workgroup ever talks to another.  With k_splits > 1 each workgroup writes one
//     fp32 partial per row to the workspace and the last one to finish a row block
//     (atomic ticket) adds the partials in range order, scales and stores y.
// Batch rows are processed in groups of BG (1 or 2) per pass over the codes: the code
// words in registers are reused for the BG Psumbooks of a unit; groups are separate
// workgroups (grid.z).  Groups of 4 have a kernel of their own (gemm_batch_impl.h).
//
// LDS layout of one Psumbook buffer.  Rows of 256 bytes, one per centroid index,
// holding the 32 slots of two codebooks (codebook c: byte offset 128*(c%2)), grouped
// in "superplanes" of 256 rows (64 KB), one per pair of codebooks.  The byte address
//     (superplane << 16) | (code << 8) | (128*(c%2) + 4*slot)
// is assembled from a code byte by a single byte-permute instruction.
#pragma once

#include "cg_common.h"

// Ablation builds (diagnostic libraries libcodegemm_ablate_<mask>.so, never the production one)
// compile parts of the batch-1 gather kernel out to show what each costs on top of the code
// stream.  Their outputs are wrong on purpose.  Mask bits: 1 gather without its LDS reads,
// 2 no gather at all, 4 no Psumbook build after the first, 8 no exchange between workgroups.
#ifndef CODEGEMM_ABLATE
#define CODEGEMM_ABLATE 0
#endif

namespace cg {

constexpr int kMaxGroup = 4;     // layers one grouped launch can hold

// What differs between the layers of one launch: a plain call has one member, a grouped call
// (layers that share x and the format, e.g. the q, k and v projections) up to kMaxGroup, whose
// row blocks follow each other along grid.y.
struct Member {
    const uint8_t* packed;
    const _Float16* codebooks;
    const _Float16* scales;      // [N], one per output row; nullptr when group scales are used
    const uint8_t* gscales;      // packed group scales (see codegemm_pack_scales), or nullptr
    void* y;
    float* partials;             // [B][NKS][Npad]
    unsigned long long* pairs;   // [B][NKS - 1][Npad] words of the pairwise reduction, or nullptr: ticket and partials
    int N, NGR, Npad;
    int blk0;                    // first row block of this member in grid.y
};

struct GemmParams {
    const _Float16* x;
    uint32_t* counters;          // [groups][row blocks of all members][cstride], word 0 of each is the ticket counter
    int cstride;
    int B, K;
    int NKT, NKS, KPW;
    int y_fp32;
    int GPU, gshift;             // scale groups per unit; a lane's group in its unit = slot >> gshift
    unsigned long long* trace;   // [grid][24] timestamps (100 MHz) when built with CODEGEMM_TRACE, else unused
    int ngrp;                    // members in use (1 for a plain call)
    Member mem[kMaxGroup];
};

// The member a row block of the grid belongs to (uniform; constant indices only, so the table
// stays in the kernel-argument segment).
__device__ __forceinline__ Member member_of(const GemmParams& p, int grid_blk)
{
    Member m = p.mem[0];
    if (p.ngrp > 1) {
        if (grid_blk >= p.mem[1].blk0) m = p.mem[1];
        if (p.ngrp > 2 && grid_blk >= p.mem[2].blk0) m = p.mem[2];
        if (p.ngrp > 3 && grid_blk >= p.mem[3].blk0) m = p.mem[3];
        // lgkmcnt(0): the table loads have returned before the paths join, so that the path of a
        // plain call, whose early fields come preloaded, carries no wait on their account
        __builtin_amdgcn_s_waitcnt(0xc07f);
    }
    return m;
}

// What every workgroup needs before it can ask for its first codes, passed a second time as
// leading scalar kernel arguments.  The library is compiled with kernel-argument preloading
// (-mllvm -amdgpu-kernarg-preload-count): the leading scalar arguments arrive in scalar
// registers with the wavefront, so the first loads go out without a round trip to the
// kernel-argument segment (measured with a probe kernel: 260-300 clocks median, 630 for the
// slowest workgroup, against 8).  Structs are not preloaded, hence the copies (the fp16 pointers
// travel as void*, which keeps the kernel names readable in profiler output); firmware without
// the feature falls back to loading them, which the compiler arranges.
#define CG_HEAD_PARAMS const void* hx, const uint8_t* hpacked, const void* hcodebooks, const uint8_t* hgscales, \
                       int hK, int hNKT, int hKPW, int hB, int hNGR, int hmisc
#define CG_HEAD_ARGS(p) (p).x, (p).mem[0].packed, (p).mem[0].codebooks, (p).mem[0].gscales, (p).K, (p).NKT, (p).KPW, (p).B, \
                        (p).mem[0].NGR, ((p).ngrp | ((p).gshift << 8) | ((p).GPU << 16))

// The argument struct with the early fields taken from the leading scalars (member 0 starts at row block 0).
__device__ __forceinline__ GemmParams with_head(const GemmParams& pk, CG_HEAD_PARAMS)
{
    GemmParams p = pk;
    p.x = static_cast<const _Float16*>(hx); p.K = hK; p.NKT = hNKT; p.KPW = hKPW; p.B = hB;
    p.ngrp = hmisc & 0xff; p.gshift = (hmisc >> 8) & 0xff; p.GPU = (int)((unsigned)hmisc >> 16);
    p.mem[0].packed = hpacked; p.mem[0].codebooks = static_cast<const _Float16*>(hcodebooks); p.mem[0].gscales = hgscales;
    p.mem[0].NGR = hNGR; p.mem[0].blk0 = 0;
    return p;
}

#ifdef CODEGEMM_TRACE
#define CG_STAMP(k) do { if (p.trace && threadIdx.x == 0 && blockIdx.z == 0) p.trace[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 24 + (k)] = wall_clock64(); } while (0)
#else
#define CG_STAMP(k) do { } while (0)
#endif

template <int M>
struct PsumLayout {
    static constexpr int kSuperplanes = (M + 1) / 2;
    static constexpr int kBytes = kSuperplanes * 65536;                 // one buffer
    static constexpr int kBuffers = (2 * kBytes <= 131072) ? 2 : 1;     // double-buffer when it fits
    __host__ __device__ static constexpr int superplane(int c) { return c / 2; }
    __host__ __device__ static constexpr int sub_bytes(int c) { return 128 * (c % 2); }
};

typedef __attribute__((address_space(3))) float lds_float;

// One 32x32 block of the Psumbook on the matrix cores:
//   D[i][slot] = sum_k C[c][32*iblk + i][k] * x[slot][k]
// Lane l supplies row / column l%32 with k = 4*(l/32)..+3 (for v = 4 the upper half of
// the contraction is fed zeros) and receives D[8*blk + 4*(l/32) + e][l%32] in
// accumulator 4*blk + e; for fixed (blk, e) the 32 lanes of a half-wavefront write 32
// consecutive slots of one row.
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

// MFMA operand of one lane: 4 fp16 values per 32x32x8 pass.  v = 4 and v = 8 take one pass
// (for v = 4 the upper half of the contraction is fed zeros); v = 16 takes two passes, and
// the lane holds the 8 consecutive elements 8*(l/32)..+7 of its vector: elements ..+3 feed
// the first pass and +4..+7 the second, for both operands alike, so the two passes
// together contract over all 16 elements.
template <int V> struct Frag { typedef half4_t type; };
template <> struct Frag<16> { typedef half8_t type; };
template <int V> __host__ __device__ constexpr int frag_elems() { return V == 16 ? 8 : 4; }

// Stores a block's 16 accumulators per lane into the Psumbook buffer `buf` (codebook c, centroids 32*iblk..+31).
template <int M>
__device__ __forceinline__ void block_to_lds(float* buf, int c, int iblk, int lane, float16_t d)
{
    // The lane's first destination as an LDS byte address the optimiser cannot see through:
    // the 16 stores then differ only by small immediate offsets (and pair up into two-dword
    // writes) instead of each getting an address register of its own when the buffer's
    // constant offset does not fit an immediate.
    uint32_t dst = (uint32_t)reinterpret_cast<uintptr_t>((lds_float*)buf) +
                   (uint32_t)(PsumLayout<M>::superplane(c) * 65536 + PsumLayout<M>::sub_bytes(c) +
                              ((iblk * 32 + 4 * (lane >> 5)) * 64 + (lane & 31)) * 4);
    asm volatile("" : "+v"(dst));
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            *reinterpret_cast<lds_float*>(static_cast<uintptr_t>(dst + (uint32_t)(8 * blk + e) * 256u)) = d[4 * blk + e];
}

// One 32x32 block of a Psumbook: 32 centroids x 32 slots, contracted over the v elements.
template <int V>
__device__ __forceinline__ float16_t mfma_block(typename Frag<V>::type cfrag, typename Frag<V>::type xfrag)
{
    float16_t d = {0};
    if constexpr (V == 16) {
        d = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_shufflevector(cfrag, cfrag, 0, 1, 2, 3),
                                                 __builtin_shufflevector(xfrag, xfrag, 0, 1, 2, 3), d, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_shufflevector(cfrag, cfrag, 4, 5, 6, 7),
                                                 __builtin_shufflevector(xfrag, xfrag, 4, 5, 6, 7), d, 0, 0, 0);
    } else {
        d = __builtin_amdgcn_mfma_f32_32x32x8f16(cfrag, xfrag, d, 0, 0, 0);
    }
    return d;
}

template <int M, int V>
__device__ __forceinline__ void mfma_block_to_lds(float* buf, int c, int iblk, int lane,
                                                  typename Frag<V>::type cfrag, typename Frag<V>::type xfrag)
{
    block_to_lds<M>(buf, c, iblk, lane, mfma_block<V>(cfrag, xfrag));
}
// The fp16 Psumbook (plan field psum_dtype = 1): an entry is the pair of partial sums of one
// centroid index and slot for the two codebooks of a superplane, rounded to nearest-even
// fp16 and packed into one 32-bit word: codebook 2*sp in the low half, 2*sp + 1 in the
// high half.  A row is still 256 bytes per centroid index, now holding the 32 slots of both
// buffers (buffer parity at byte offset 128), so the byte address is
//     (superplane << 16) | (code << 8) | (128 * parity + 4 * slot + 2 * (c % 2)),
// again one byte-permute, and the bank of a lookup is again the slot.  The table of a unit is
// half the bytes: half the LDS writes per unit, and every format double-buffers in at most 128 KB.
template <int M>
struct PsumLayoutH {
    static constexpr int kSuperplanes = (M + 1) / 2;
    static constexpr int kBytes = kSuperplanes * 65536;                 // both buffers
};

typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;

// The 32x32 blocks (centroids 32*iblk..+31, all slots) of the two codebooks of superplane sp,
// packed and written for accumulator groups blk_lo..blk_hi-1 (4 groups of 8 centroid rows).
template <int M, int V>
__device__ __forceinline__ void mfma_pair_to_lds(float* planes, int sp, int iblk, int lane, int par, int blk_lo, int blk_hi,
                                                 typename Frag<V>::type c0, typename Frag<V>::type c1,
                                                 typename Frag<V>::type xfrag)
{
    float16_t d0 = {0}, d1 = {0};
    if constexpr (V == 16) {
        d0 = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_shufflevector(c0, c0, 0, 1, 2, 3),
                                                  __builtin_shufflevector(xfrag, xfrag, 0, 1, 2, 3), d0, 0, 0, 0);
        d0 = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_shufflevector(c0, c0, 4, 5, 6, 7),
                                                  __builtin_shufflevector(xfrag, xfrag, 4, 5, 6, 7), d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_shufflevector(c1, c1, 0, 1, 2, 3),
                                                  __builtin_shufflevector(xfrag, xfrag, 0, 1, 2, 3), d1, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_shufflevector(c1, c1, 4, 5, 6, 7),
                                                  __builtin_shufflevector(xfrag, xfrag, 4, 5, 6, 7), d1, 0, 0, 0);
    } else {
        d0 = __builtin_amdgcn_mfma_f32_32x32x8f16(c0, xfrag, d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_32x32x8f16(c1, xfrag, d1, 0, 0, 0);
    }
    uint32_t dst = (uint32_t)reinterpret_cast<uintptr_t>((lds_float*)planes) +
                   (uint32_t)(sp * 65536 + par * 128 + ((iblk * 32 + 4 * (lane >> 5)) * 64 + (lane & 31)) * 4);
    asm volatile("" : "+v"(dst));
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
        if (blk < blk_lo || blk >= blk_hi) continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const half2_t pr = {(_Float16)d0[4 * blk + e], (_Float16)d1[4 * blk + e]};
            *reinterpret_cast<lds_u32*>(static_cast<uintptr_t>(dst + (uint32_t)(8 * blk + e) * 256u)) = __builtin_bit_cast(uint32_t, pr);
        }
    }
}

// fp16 Psum lookup: same address assembly as psum_at; a 16-bit read (the bits land in the
// low half of the register, the high half is zero).
template <int k>
__device__ __forceinline__ uint32_t psum_h_at(uint32_t word, uint32_t off)
{
    const uint32_t addr = __builtin_amdgcn_perm(word, off, 0x0c020000u | ((4u + k) << 8));
    return *reinterpret_cast<const lds_u16*>(static_cast<uintptr_t>(addr));
}

// acc + psum (or acc + scale * psum) for an fp16 psum: one mixed-precision fused multiply-add
// that widens the fp16 operand exactly, so the vector-instruction count per lookup stays at
// two (address, accumulate) as with the fp32 table.
template <bool GS>
__device__ __forceinline__ float accumulate_h(float acc, uint32_t hbits, _Float16 scale)
{
    if constexpr (GS) {
        return __builtin_fmaf((float)scale, (float)__builtin_bit_cast(_Float16, (uint16_t)hbits), acc);
    } else {
        asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(hbits));
        return acc;
    }
}

// Psum lookup: the LDS byte address gets byte 0 from the low byte of `off`
// (sub-offset + 4*slot), byte 1 from code byte `k` of `word`, byte 2 from byte 2 of
// `off` (buffer and superplane), byte 3 zero; the read is a plain ds_read_b32 at that
// absolute address.
template <int k>
__device__ __forceinline__ float psum_at(uint32_t word, uint32_t off)
{
    const uint32_t addr = __builtin_amdgcn_perm(word, off, 0x0c020000u | ((4u + k) << 8));
    return *reinterpret_cast<const lds_float*>(static_cast<uintptr_t>(addr));
}

// The eight Psum lookups of one code word pair (8 rows, one codebook) and their additions as
// one instruction sequence that the compiler cannot stretch: address, read, address, read,
// ..., then each addition as soon as its read is back (LDS reads return in order, so once at
// most 7 - i accesses are outstanding, read i has arrived, whatever else was in flight
// before).  Used by the block shapes whose accumulators and code ring leave few registers:
// left to the scheduler, all reads of a unit are issued ahead of the first addition, their
// results stay live, and those shapes spill (measured: the 16-wavefront shapes with three or
// four codebooks, two batch rows, or 1024 rows).  The shapes that fit keep the compiler's
// schedule, which hides the LDS latency a little better (8192->28672, m = 2: 14.3 against 14.8 us).
#define CG_GATHER8_READS \
        "v_perm_b32 %8, %16, %18, %19\n\t"  "ds_read_b32 %8, %8\n\t"   \
        "v_perm_b32 %9, %16, %18, %20\n\t"  "ds_read_b32 %9, %9\n\t"   \
        "v_perm_b32 %10, %16, %18, %21\n\t" "ds_read_b32 %10, %10\n\t" \
        "v_perm_b32 %11, %16, %18, %22\n\t" "ds_read_b32 %11, %11\n\t" \
        "v_perm_b32 %12, %17, %18, %19\n\t" "ds_read_b32 %12, %12\n\t" \
        "v_perm_b32 %13, %17, %18, %20\n\t" "ds_read_b32 %13, %13\n\t" \
        "v_perm_b32 %14, %17, %18, %21\n\t" "ds_read_b32 %14, %14\n\t" \
        "v_perm_b32 %15, %17, %18, %22\n\t" "ds_read_b32 %15, %15\n\t"
#define CG_GATHER8_OUT(a) "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]), \
        "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3), "=&v"(t4), "=&v"(t5), "=&v"(t6), "=&v"(t7)
constexpr uint32_t kSel0 = 0x0c020400u, kSel1 = 0x0c020500u, kSel2 = 0x0c020600u, kSel3 = 0x0c020700u;   // byte k of the code word into address byte 1

__device__ __forceinline__ void gather8(float (&a)[8], uint32_t lo, uint32_t hi, uint32_t off)
{
    uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
    asm volatile(CG_GATHER8_READS
        "s_waitcnt lgkmcnt(7)\n\t" "v_add_f32 %0, %0, %8\n\t"
        "s_waitcnt lgkmcnt(6)\n\t" "v_add_f32 %1, %1, %9\n\t"
        "s_waitcnt lgkmcnt(5)\n\t" "v_add_f32 %2, %2, %10\n\t"
        "s_waitcnt lgkmcnt(4)\n\t" "v_add_f32 %3, %3, %11\n\t"
        "s_waitcnt lgkmcnt(3)\n\t" "v_add_f32 %4, %4, %12\n\t"
        "s_waitcnt lgkmcnt(2)\n\t" "v_add_f32 %5, %5, %13\n\t"
        "s_waitcnt lgkmcnt(1)\n\t" "v_add_f32 %6, %6, %14\n\t"
        "s_waitcnt lgkmcnt(0)\n\t" "v_add_f32 %7, %7, %15"
        : CG_GATHER8_OUT(a)
        : "v"(lo), "v"(hi), "v"(off), "s"(kSel0), "s"(kSel1), "s"(kSel2), "s"(kSel3)
        : "memory");
}

// The same with group scales: acc += scale[row] * psum as one mixed-precision fused
// multiply-add that widens the fp16 scale exactly (the scales of rows 2i and 2i + 1 are the
// low and high half of sc[i]).
__device__ __forceinline__ void gather8_scaled(float (&a)[8], uint32_t lo, uint32_t hi, uint32_t off, const uint32_t (&sc)[4])
{
    uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
    asm volatile(CG_GATHER8_READS
        "s_waitcnt lgkmcnt(7)\n\t" "v_fma_mix_f32 %0, %23, %8, %0 op_sel_hi:[1,0,0]\n\t"
        "s_waitcnt lgkmcnt(6)\n\t" "v_fma_mix_f32 %1, %23, %9, %1 op_sel:[1,0,0] op_sel_hi:[1,0,0]\n\t"
        "s_waitcnt lgkmcnt(5)\n\t" "v_fma_mix_f32 %2, %24, %10, %2 op_sel_hi:[1,0,0]\n\t"
        "s_waitcnt lgkmcnt(4)\n\t" "v_fma_mix_f32 %3, %24, %11, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t" "v_fma_mix_f32 %4, %25, %12, %4 op_sel_hi:[1,0,0]\n\t"
        "s_waitcnt lgkmcnt(2)\n\t" "v_fma_mix_f32 %5, %25, %13, %5 op_sel:[1,0,0] op_sel_hi:[1,0,0]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t" "v_fma_mix_f32 %6, %26, %14, %6 op_sel_hi:[1,0,0]\n\t"
        "s_waitcnt lgkmcnt(0)\n\t" "v_fma_mix_f32 %7, %26, %15, %7 op_sel:[1,0,0] op_sel_hi:[1,0,0]"
        : CG_GATHER8_OUT(a)
        : "v"(lo), "v"(hi), "v"(off), "s"(kSel0), "s"(kSel1), "s"(kSel2), "s"(kSel3),
          "v"(sc[0]), "v"(sc[1]), "v"(sc[2]), "v"(sc[3])
        : "memory");
}
#undef CG_GATHER8_READS
#undef CG_GATHER8_OUT

// Whether a block shape of the batch-1 kernel takes the fixed gather sequence above: the shapes
// that otherwise spill registers (128 per lane with 16 wavefronts, 256 with 8).
template <int M, int V, int NW, int RPL, int BG, bool GS>
__host__ __device__ constexpr bool fixed_gather()
{
    const int words = RPL * BG * M;                        // 8-accumulator groups times code words per unit
    if (NW == 8) return words >= 16;
    return words >= 8 || (V == 16 && M == 3 && RPL * BG == 2) || (GS && BG == 2 && RPL == 2);
}

// v + (v moved across lanes by a DPP control).  Lanes the control does not write add 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false);
    return v + __builtin_bit_cast(float, moved);
}

// One halving step of a transposing reduction: lanes are paired by the DPP control; the
// lane whose `upper` flag is set keeps the upper half of its n values, the other lane the
// lower half, and each adds the partner's copy of the half it keeps.
template <int CTRL, int N>
__device__ __forceinline__ void halve(float (&v)[N], bool upper)
{
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
        const float keep = upper ? v[i + N / 2] : v[i];
        const float send = upper ? v[i] : v[i + N / 2];
        const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), CTRL, 0xf, 0xf, false);
        v[i] = keep + __builtin_bit_cast(float, moved);
    }
}

// Sums NV (8 or 16) per-lane values over the 32 lanes of each half-wavefront.  On return
// lane l holds, in v[0], the total of value number l % NV.  Within a 16-lane row the lanes
// are paired by rotate-8, half-mirror, and two quad permutes (vector ALU only); each step
// halves the number of values a lane carries, so the whole reduction costs about 3*NV
// instructions instead of 5*NV.  The two rows of a half-wavefront are then added with one
// cross-lane shuffle.  The order of the additions is fixed.
template <int NV>
__device__ __forceinline__ float halfwave_transpose_sum(float (&v)[NV], int lane)
{
    static_assert(NV == 8 || NV == 16, "8 or 16 values");
    if constexpr (NV == 16) {
        halve<0x128, 16>(v, (lane & 8) != 0);              // row_ror:8
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = dpp_add<0x128, 0xf>(v[i]);
    }
    float (&v8)[8] = reinterpret_cast<float (&)[8]>(v);
    halve<0x141, 8>(v8, (lane & 4) != 0);                  // row_half_mirror: l <-> l ^ 7
    float (&v4)[4] = reinterpret_cast<float (&)[4]>(v);
    halve<0x4e, 4>(v4, (lane & 2) != 0);                   // quad_perm [2,3,0,1]: l <-> l ^ 2
    float (&v2)[2] = reinterpret_cast<float (&)[2]>(v);
    halve<0xb1, 2>(v2, (lane & 1) != 0);                   // quad_perm [1,0,3,2]: l <-> l ^ 1
    return v[0] + __shfl_xor(v[0], 16, kWave);
}

// End of a workgroup's work, shared by the gather kernels.  `stage` (LDS) holds the
// workgroup's BG x ROWS row totals over its K range.  With one K range they are scaled and
// stored.  Otherwise each workgroup stores its totals as fp32 partials, takes a ticket on
// the row block's counter, and the last one to arrive adds the partials of all K ranges in
// range order, scales and stores y.  Ends with the kernel: every path returns.
template <int NT, int BG, int ROWS>
__device__ __forceinline__ void finish_block(const GemmParams& p, const Member& mm, const float* stage, uint32_t* flag,
                                             int tid, int blk, int ks, int b0)
{
    CG_STAMP(16);
    __syncthreads();
    CG_STAMP(17);

    constexpr int PER_THREAD = (BG * ROWS + NT - 1) / NT;             // outputs per thread
    const int n_base = blk * ROWS;
    float mine[PER_THREAD];
    uint32_t scale_bits[PER_THREAD];
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        const int o = tid + i * NT;
        const int nn = n_base + o % ROWS;
        mine[i] = (o < BG * ROWS) ? stage[o] : 0.0f;
        // requested before any ticket round trip; with group scales the totals are already scaled
        scale_bits[i] = mm.scales ? reinterpret_cast<const uint16_t*>(mm.scales)[nn < mm.N ? nn : 0] : 0x3c00u;
    }
    // The scale is first touched where it is used (the pin keeps its conversion, and with it
    // the wait for the load, from being hoisted in front of the partial-sum stores).
    auto scale_of = [&](int i) -> float {
        uint32_t b = scale_bits[i];
        asm volatile("" : "+v"(b));
        return (float)__builtin_bit_cast(_Float16, (uint16_t)b);
    };
    auto store_y = [&](int row, int nn, float val) {
        if (p.y_fp32) static_cast<float*>(mm.y)[(size_t)row * mm.N + nn] = val;
        else static_cast<_Float16*>(mm.y)[(size_t)row * mm.N + nn] = (_Float16)val;
    };

#if CODEGEMM_ABLATE & 8
    const bool single = true;          // ablation build: no exchange between workgroups, every K range stores y
#else
    const bool single = p.NKS == 1;
#endif
    if (single) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int o = tid + i * NT;
            const int row = b0 + o / ROWS, nn = n_base + o % ROWS;
            if (o < BG * ROWS && row < p.B && nn < mm.N) store_y(row, nn, mine[i] * scale_of(i));
        }
        CG_STAMP(3);
        return;
    }

    if (mm.pairs) {
        // Pairwise reduction that carries the data in the atomics themselves.  K ranges 2i and 2i + 1
        // share a 64-bit word per output, zero between calls: each adds the bits of its fp32 partial
        // to its own half (+0.0 travels as -0.0, so that a half that has arrived is never zero) with
        // one device-scope add that returns the word as it was.  Whoever finds the other half there
        // holds both values: it clears the word, adds the two in range order and goes on to the next
        // level as range i; the other one is done.  One round trip per level, log2(NKS) levels, no
        // wait for a store to land, no counter, no barrier; the order of the additions is fixed.
        bool live[PER_THREAD];
        unsigned long long* word[PER_THREAD];
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int o = tid + i * NT;
            const int row = b0 + o / ROWS, nn = n_base + o % ROWS;
            live[i] = o < BG * ROWS && row < p.B && nn < mm.N;
            word[i] = mm.pairs + (size_t)(live[i] ? row : 0) * (p.NKS - 1) * mm.Npad + (live[i] ? nn : 0);
        }
        CG_STAMP(18);
        int k = ks;
        for (int span = p.NKS; span > 1; span >>= 1) {
            const int side = k & 1;
            unsigned long long old[PER_THREAD];
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) {
                uint32_t bits = __builtin_bit_cast(uint32_t, mine[i]);
                if (bits == 0u) bits = 0x80000000u;
                old[i] = 0;
                if (live[i])
                    old[i] = __hip_atomic_fetch_add(word[i] + (size_t)(k >> 1) * mm.Npad, (unsigned long long)bits << (32 * side),
                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) {
                const uint32_t other = (uint32_t)(old[i] >> (32 * (side ^ 1)));
                if (live[i] && other != 0u) {
                    __hip_atomic_store(word[i] + (size_t)(k >> 1) * mm.Npad, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const float ov = __builtin_bit_cast(float, other);
                    mine[i] = side ? ov + mine[i] : mine[i] + ov;
                } else {
                    live[i] = false;
                }
                word[i] += (size_t)(span >> 1) * mm.Npad;
            }
            if (span == p.NKS) CG_STAMP(19);
            k >>= 1;
        }
        CG_STAMP(20);
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int o = tid + i * NT;
            const int row = b0 + o / ROWS, nn = n_base + o % ROWS;
            if (live[i]) store_y(row, nn, (mine[i] + 0.0f) * scale_of(i));
        }
        if (live[0]) CG_STAMP(3);
        return;
    }

    // K ranges are combined through the workspace.  Every datum that crosses workgroups
    // is moved by device-scope atomic accesses (write-through stores, cache-bypassing
    // loads, one RMW on the counter), so no L2 write-back / invalidate is needed: each
    // thread waits for its own partial stores to be acknowledged, the barrier collects
    // that for the workgroup, and only then is the ticket taken.
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        const int o = tid + i * NT;
        const int row = b0 + o / ROWS, nn = n_base + o % ROWS;
        if (o < BG * ROWS && row < p.B && nn < mm.Npad)
            __hip_atomic_store(mm.partials + ((size_t)row * p.NKS + ks) * mm.Npad + nn, mine[i],
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    CG_STAMP(5);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    CG_STAMP(6);
    if (tid == 0) {
        uint32_t* ctr = p.counters + ((size_t)blockIdx.z * gridDim.y + mm.blk0 + blk) * p.cstride;
        const uint32_t old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = old == (uint32_t)(p.NKS - 1);
        if (last) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
        *flag = last ? 1u : 0u;
    }
    __syncthreads();
    CG_STAMP(7);
    if (*flag == 0u) return;
    // Last workgroup of this row block: add the partials of all K ranges in range order.
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        const int o = tid + i * NT;
        const int row = b0 + o / ROWS, nn = n_base + o % ROWS;
        if (o >= BG * ROWS || row >= p.B || nn >= mm.N) continue;
        const float* src = mm.partials + (size_t)row * p.NKS * mm.Npad + nn;
        if (p.NKS == 4) {
            // the order of the pairwise reduction, so that a launch gives the same bits whichever protocol its size selects
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[j] = __hip_atomic_load(src + (size_t)j * mm.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            store_y(row, nn, (((v[0] + v[1]) + (v[2] + v[3])) + 0.0f) * scale_of(i));
            continue;
        }
        float sum = 0.0f;
        int k2 = 0;
        for (; k2 + 32 <= p.NKS; k2 += 32) {            // 32 loads in flight, added in range order
            float v[32];
#pragma unroll
            for (int j = 0; j < 32; ++j)
                v[j] = __hip_atomic_load(src + (size_t)(k2 + j) * mm.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int j = 0; j < 32; ++j) sum += v[j];
        }
        for (; k2 + 16 <= p.NKS; k2 += 16) {
            float v[16];
#pragma unroll
            for (int j = 0; j < 16; ++j)
                v[j] = __hip_atomic_load(src + (size_t)(k2 + j) * mm.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int j = 0; j < 16; ++j) sum += v[j];
        }
        for (; k2 + 8 <= p.NKS; k2 += 8) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                v[j] = __hip_atomic_load(src + (size_t)(k2 + j) * mm.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int j = 0; j < 8; ++j) sum += v[j];
        }
        for (; k2 + 4 <= p.NKS; k2 += 4) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[j] = __hip_atomic_load(src + (size_t)(k2 + j) * mm.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int j = 0; j < 4; ++j) sum += v[j];
        }
        for (; k2 < p.NKS; ++k2)
            sum += __hip_atomic_load(src + (size_t)k2 * mm.Npad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        store_y(row, nn, sum * scale_of(i));
    }
    CG_STAMP(3);
}

// acc + scale * psum for group scales, acc + psum otherwise.
template <bool GS>
__device__ __forceinline__ float accumulate(float acc, float psum, _Float16 scale)
{
    if constexpr (GS) return __builtin_fmaf((float)scale, psum, acc);
    else return acc + psum;
}

template <int M, int V, int NW, int RPL, int BG, int D, bool GS, bool PH = false, int NB = 0>
__global__ void __launch_bounds__(NW * 64) gemm_kernel(CG_HEAD_PARAMS, const GemmParams pk)
{
    const GemmParams p = with_head(pk, hx, hpacked, hcodebooks, hgscales, hK, hNKT, hKPW, hB, hNGR, hmisc);
    constexpr int NTILES = 8 * M;                      // 32x32 MFMA blocks in one Psumbook
    constexpr int TPW = PH ? 1 : (NTILES + NW - 1) / NW;   // blocks per wavefront (fp32 Psumbook)
    // NB > 0: the last NB wavefronts build every Psumbook and do nothing else; the first NG
    // stream, gather and reduce and never touch the matrix cores.  A wavefront issues in program
    // order, so one that builds between two gathers delays its own next lookups and loads by the
    // length of its build; split up, the builders run a whole unit ahead of the gatherers.
    constexpr int NG = NW - NB;                        // wavefronts that own rows
    constexpr int PIECES = RPL * NG;                   // 16-row pieces (one row word of one wavefront) per workgroup
    typedef PsumLayout<M> L;
    typedef PsumLayoutH<M> LH;
    constexpr int NBUF = PH ? 2 : L::kBuffers;
    // fp16 Psumbook: block pairs (superplane, 32 centroids), each built by one wavefront, or by
    // two (each writing half of the rows) when there are more wavefronts than pairs
    constexpr int NPAIR = 8 * LH::kSuperplanes;
    constexpr int PPW = NPAIR >= NW ? NPAIR / NW : 1;
    constexpr int WPP = NPAIR >= NW ? 1 : NW / NPAIR;  // wavefronts per pair (1 or 2)
    static_assert(!PH || (NPAIR % NW == 0 || NW % NPAIR == 0), "pairs and wavefronts divide");
    static_assert(!PH || WPP <= 2, "at most two wavefronts per pair");
    static_assert(NW == 8 || NW == 14 || NW == 16, "8, 14 or 16 wavefronts");
    static_assert(!PH || NW != 14, "the fp16 Psumbook pairs up 8 or 16 wavefronts");
    static_assert((D & 1) == 0, "ring depth must be even (buffer parity is compile-time)");
    static_assert(NB == 0 || (!PH && BG == 1 && NBUF == 2 && NTILES % NB == 0),
                  "build-only wavefronts: one batch row, double-buffered fp32 Psumbook");

    extern __shared__ __align__(16) unsigned char smem[];
    float* planes = reinterpret_cast<float*>(smem);                     // NBUF buffers of L::kBytes
    uint32_t* flag = reinterpret_cast<uint32_t*>(smem + (PH ? LH::kBytes : NBUF * L::kBytes));

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and known to be: keeps buffer descriptors in scalar registers
    const int ks = blockIdx.x;
    const Member mm = member_of(p, blockIdx.y);        // the layer this workgroup works for
    const int blk = blockIdx.y - mm.blk0;              // its row block of PIECES x 16 rows
    const int b0 = blockIdx.z * BG;
    const int kt0 = ks * p.KPW;
    const int nq = min(p.KPW, p.NKT - kt0);            // units of this workgroup (>= 1 by construction)
    const int khalf = lane >> 5;
    const bool kvalid = 4 * khalf < V;
    typedef typename Frag<V>::type frag_t;
    constexpr int FE = frag_elems<V>();                // operand elements per lane
    const frag_t zero4 = {};

    CG_STAMP(0);
    // All streaming loads are bounds-checked buffer loads: a load past the end of this
    // workgroup's range returns zeros without touching memory.  That keeps every load
    // unconditional - the hardware returns loads in issue order and the compiler can count
    // outstanding loads exactly only along branch-free code - and it zero-fills the
    // activations of a ragged last K tile for free.
    constexpr uint32_t kRsrcFlags = 0x00020000u;       // raw 32-bit buffer, gfx9 family
    constexpr int kOutOfRange = 0x7ffffff0;
    //
    // Centroid operands of this wavefront's MFMA blocks: fixed for the whole kernel.
    frag_t cfrag[TPW];
    frag_t cpair[PH ? PPW : 1][2];                     // fp16 Psumbook: both codebooks of this wavefront's pairs
    if constexpr (NB > 0) {
#pragma unroll
        for (int i = 0; i < TPW; ++i) cfrag[i] = zero4;    // the builders keep their own (below)
    } else if constexpr (!PH) {
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            int tile = wave + i * NW;                      // c*8 + iblk
            if (tile >= NTILES) tile = NTILES - 1;
            cfrag[i] = *reinterpret_cast<const frag_t*>(mm.codebooks + (size_t)(tile * 32 + (lane & 31)) * V + (kvalid ? FE * khalf : 0));
        }
    } else {
#pragma unroll
        for (int i = 0; i < PPW; ++i) {
            const int pair = (WPP == 1) ? wave + i * NW : wave % NPAIR;        // sp*8 + iblk
            const int sp = pair / 8, iblk = pair % 8;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int c = min(2 * sp + h, M - 1);
                cpair[i][h] = *reinterpret_cast<const frag_t*>(mm.codebooks + (size_t)((c * 8 + iblk) * 32 + (lane & 31)) * V + (kvalid ? FE * khalf : 0));
                if (!kvalid || 2 * sp + h >= M) cpair[i][h] = zero4;           // an odd m leaves the last high half zero
            }
        }
    }
    // Activation operand: sub-vector (32*kt + l%32), elements 4*(l/32)..+3 (Step 1), read
    // through a descriptor that covers exactly this workgroup's K range of batch row bb.
    const int x_elems = min(nq * 32 * V, p.K - kt0 * 32 * V);
    __amdgpu_buffer_rsrc_t x_rsrc[BG];
#pragma unroll
    for (int bb = 0; bb < BG; ++bb) {
        const int row = min(b0 + bb, p.B - 1);
        x_rsrc[bb] = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(p.x + (size_t)row * p.K + (size_t)kt0 * 32 * V),
                                                       0, x_elems * 2, kRsrcFlags);
    }
    const int x_off0 = kvalid ? ((lane & 31) * V + FE * khalf) * 2 : kOutOfRange;
    auto load_x_raw = [&](int u, int bb) -> frag_t {
        if constexpr (V == 16) {
            const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc[bb], x_off0 + u * (32 * V * 2), 0, 0);
            return __builtin_bit_cast(frag_t, t);
        } else {
            const u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(x_rsrc[bb], x_off0 + u * (32 * V * 2), 0, 0);
            return __builtin_bit_cast(frag_t, t);
        }
    };
    // what the gathering wavefronts load: nothing when others build for them
    auto load_x = [&](int u, int bb) -> frag_t {
        if constexpr (NB > 0) return zero4;
        else return load_x_raw(u, bb);
    };
    // Codes of unit u for this lane: RPL words of 8*M bytes (8 rows x M codebooks at one slot).
    // Word q (q < RPL) of this wavefront is piece blk*PIECES + q*NW + wave of the matrix: rows
    // 16*piece .. 16*piece+15, i.e. row-lanes 2*(piece%8), +1 of granule piece/8.  With 8 or 16
    // wavefronts piece%8 = wave%8 for every q; with 14 it differs from word to word.
    constexpr int kUnitBytes = 128 * 32 * M;
    auto piece_of = [&](int q) -> int { return blk * PIECES + q * NG + wave; };
    auto granule_of = [&](int q) -> int { return piece_of(q) >> 3; };
    int entry[RPL];                                    // (row-lane, slot) index inside the unit
#pragma unroll
    for (int q = 0; q < RPL; ++q) entry[q] = (piece_of(q) & 7) * kWave + lane;
    __amdgpu_buffer_rsrc_t c_rsrc[RPL];
#pragma unroll
    for (int q = 0; q < RPL; ++q) {
        const int gr = granule_of(q);
        // a granule past the end of the matrix (ragged last block) gets an empty range: all codes read as 0
        const uint8_t* base = mm.packed + ((size_t)min(gr, mm.NGR - 1) * p.NKT + kt0) * kUnitBytes;
        c_rsrc[q] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, gr < mm.NGR ? nq * kUnitBytes : 0, kRsrcFlags);
    }
    auto load_codes = [&](uint32_t (&dst)[RPL][2 * M], int u) {
#pragma unroll
        for (int q = 0; q < RPL; ++q) {
#pragma unroll
            for (int part = 0; part < (M + 1) / 2; ++part) {
                if (2 * part + 1 == M) {
                    const u32x2_t t = __builtin_amdgcn_raw_buffer_load_b64(c_rsrc[q], u * kUnitBytes + part * 8192 + entry[q] * 8, 0, 2);
                    dst[q][4 * part + 0] = t.x;
                    dst[q][4 * part + 1] = t.y;
                } else {
                    const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(c_rsrc[q], u * kUnitBytes + part * 8192 + entry[q] * 16, 0, 2);
                    dst[q][4 * part + 0] = t.x;
                    dst[q][4 * part + 1] = t.y;
                    dst[q][4 * part + 2] = t.z;
                    dst[q][4 * part + 3] = t.w;
                }
            }
        }
    };
    // Group scales (Section 2.2, Step 1) of unit u for this lane: per row word, the 8 fp16
    // scales of its 8 rows for the group its slot belongs to, one 16-byte load.  They ride a
    // ring of their own, two units deep.
    constexpr int DS = 2;
    __amdgpu_buffer_rsrc_t s_rsrc[GS ? RPL : 1];
    int s_off[GS ? RPL : 1] = {};
    if constexpr (GS) {
#pragma unroll
        for (int q = 0; q < RPL; ++q) {
            const int gr = granule_of(q);
            const uint8_t* base = mm.gscales + ((size_t)min(gr, mm.NGR - 1) * p.NKT + kt0) * p.GPU * 256;
            s_rsrc[q] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, gr < mm.NGR ? nq * p.GPU * 256 : 0, kRsrcFlags);
        }
#pragma unroll
        for (int q = 0; q < RPL; ++q)
            s_off[q] = ((lane & 31) >> p.gshift) * 256 + ((piece_of(q) & 7) * 2 + khalf) * 16;
    }
    auto load_scales = [&](half8_t (&dst)[RPL], int u) {
#pragma unroll
        for (int q = 0; q < RPL; ++q)
            dst[q] = __builtin_bit_cast(half8_t, __builtin_amdgcn_raw_buffer_load_b128(s_rsrc[GS ? q : 0], u * p.GPU * 256 + s_off[GS ? q : 0], 0, 0));
    };
#if CODEGEMM_ABLATE & 4
    bool first_build = true;
#endif
    auto build = [&](float* buf, int par, frag_t xf) {
        if constexpr (NB > 0) return;                  // not this wavefront's job
#if CODEGEMM_ABLATE & 4
        // ablation build: only the first Psumbook is built; the activations are still consumed
        if (!first_build) { asm volatile("" :: "v"(xf)); return; }
        first_build = false;
#endif
        if constexpr (PH) {
#pragma unroll
            for (int i = 0; i < PPW; ++i) {
                const int pair = (WPP == 1) ? wave + i * NW : wave % NPAIR;
                const int half = (WPP == 1) ? 0 : wave / NPAIR;
                mfma_pair_to_lds<M, V>(planes, pair / 8, pair % 8, lane, par, WPP == 1 ? 0 : 2 * half, WPP == 1 ? 4 : 2 * half + 2,
                                       cpair[i][0], cpair[i][1], kvalid ? xf : zero4);
            }
        } else {
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int tile = wave + i * NW;
                if (NTILES % NW == 0 || tile < NTILES)
                    mfma_block_to_lds<M, V>(buf, tile / 8, tile % 8, lane, kvalid ? cfrag[i] : zero4, xf);
            }
        }
    };

    if constexpr (NB > 0) {
        if (wave >= NG) {
            // A builder: the blocks (wave - NG) + i * NB of every Psumbook, one unit ahead of the
            // gatherers, through the same barriers (one after the first table, one per unit).
            constexpr int TB = NTILES / NB;
            frag_t cb[TB];
#pragma unroll
            for (int i = 0; i < TB; ++i) {
                const int tile = (wave - NG) + i * NB;
                cb[i] = *reinterpret_cast<const frag_t*>(mm.codebooks + (size_t)(tile * 32 + (lane & 31)) * V + (kvalid ? FE * khalf : 0));
                if (!kvalid) cb[i] = zero4;
            }
            // software pipeline: the product of the next block is issued before the stores of the
            // current one, so the matrix core works while the LDS takes the stores
            auto build_all = [&](float* buf, frag_t xf) {
                float16_t cur = mfma_block<V>(cb[0], xf);
#pragma unroll
                for (int i = 0; i < TB; ++i) {
                    float16_t nxt = cur;
                    if (i + 1 < TB) nxt = mfma_block<V>(cb[i + 1], xf);
                    __builtin_amdgcn_sched_barrier(0);
                    const int tile = (wave - NG) + i * NB;
                    block_to_lds<M>(buf, tile / 8, tile % 8, lane, cur);
                    __builtin_amdgcn_sched_barrier(0);
                    cur = nxt;
                }
            };
            frag_t xs[2] = {load_x_raw(0, 0), load_x_raw(1, 0)};
            build_all(planes, xs[0]);
            xs[0] = load_x_raw(2, 0);
            __syncthreads();
#if CODEGEMM_ABLATE & 4
            constexpr bool kRebuild = false;   // ablation build: only the first Psumbook is built
#else
            constexpr bool kRebuild = true;
#endif
            // the gatherers' loop, barrier for barrier: while they gather unit u from buffer u % 2,
            // unit u + 1 is built into the other one
            for (int u0 = 0; u0 < nq; u0 += D) {
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const int u = u0 + d;
                    if (kRebuild && u + 1 < nq) build_all(planes + ((d + 1) & 1) * (L::kBytes / 4), xs[(d + 1) & 1]);
                    xs[(d + 1) & 1] = load_x_raw(u + 3, 0);
                    __syncthreads();
                }
            }
            finish_block<NW * kWave, BG, PIECES * 16>(p, mm, planes, flag, tid, blk, ks, b0);
            return;
        }
    }

    // Prologue: activations of the first D units, then the codes of the first unit only; the
    // rest of the code ring is requested after the first Psumbook has been written.  A
    // wavefront issues in program order and a compute unit takes about a microsecond to
    // accept a whole ring of code loads, so with the ring first the wavefronts that come
    // last would not even have asked for their operands by then (measured: the first
    // Psumbook 0.4 us earlier, calls 0.15-0.35 us shorter).
    frag_t xr[D][BG];
    uint32_t w[D][RPL][2 * M];
#pragma unroll
    for (int d = 0; d < D; ++d)
#pragma unroll
        for (int bb = 0; bb < BG; ++bb) xr[d][bb] = load_x(d, bb);
    __builtin_amdgcn_sched_barrier(0);
    // 8-wavefront workgroups serve the short calls, where the first Psumbook is on the critical
    // path: every wavefront's first operands go into the memory queues before anyone fills
    // them with codes (measured: -0.1 us there, nothing for the 16-wavefront streaming calls)
    if constexpr (NW == 8) __builtin_amdgcn_s_barrier();
    load_codes(w[0], 0);
    half8_t sc[GS ? DS : 1][RPL];
    if constexpr (GS) {
#pragma unroll
        for (int d = 0; d < DS; ++d) load_scales(sc[d], d);
    }
    __builtin_amdgcn_sched_barrier(0);

    float acc[BG][RPL][kRowsPerLane];
#pragma unroll
    for (int bb = 0; bb < BG; ++bb)
#pragma unroll
        for (int q = 0; q < RPL; ++q)
#pragma unroll
            for (int r = 0; r < kRowsPerLane; ++r) acc[bb][q][r] = 0.0f;

    // The Psumbook starts at the base of the kernel's LDS allocation (this kernel has no
    // static LDS, so that base is 0; it is added for form and must be a multiple of 64 KB).
    const uint32_t slot4 = (uint32_t)reinterpret_cast<uintptr_t>((lds_float*)planes) + (uint32_t)(lane & 31) * 4u;

    // Psumbook of (unit 0, batch row 0).
    CG_STAMP(2);
    build(planes, 0, xr[0][0]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int d = 1; d < D; ++d) load_codes(w[d], d);
    if (BG == 1) xr[0][0] = load_x(D, 0);
    __syncthreads();
    CG_STAMP(1);

    // Main loop over the sequence (unit u, batch row bb).  In every iteration the matrix
    // cores build the next Psumbook of the sequence while the lanes gather the current one.
    // Loads run unconditionally (past the end they return zeros without memory traffic); the
    // gather and the build are skipped for units past the end.
    for (int u0 = 0; u0 < nq; u0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int u = u0 + d;
#pragma unroll
            for (int bb = 0; bb < BG; ++bb) {
                const int par = (NBUF == 2) ? ((BG == 1) ? (d & 1) : (bb & 1)) : 0;   // buffer of the current Psumbook
                float* nxt = planes + ((NBUF == 2 && !PH) ? (par ^ 1) : 0) * (L::kBytes / 4);   // fp32 Psumbook: the other buffer
                const bool last_bb = (bb == BG - 1);
                const bool has_next = !last_bb || u + 1 < nq;
                // gather the current one (Step 3)
                if (u < nq) {
                    // Opaque to the optimiser: keeps the address arithmetic on the codes
                    // here instead of hoisting it out of the loops into registers.
#pragma unroll
                    for (int q = 0; q < RPL; ++q) {
#pragma unroll
                        for (int i = 0; i < 2 * M; ++i) asm volatile("" : "+v"(w[d][q][i]));
#pragma unroll
                        for (int c = 0; c < M; ++c) {
                            const uint32_t off = PH ? slot4 + (uint32_t)(2 * (c % 2) + 128 * par) + ((uint32_t)(c / 2) << 16)
                                                    : slot4 + (uint32_t)L::sub_bytes(c) +
                                                          ((uint32_t)(L::superplane(c) + par * L::kSuperplanes) << 16);
                            const uint32_t lo = w[d][q][2 * c], hi = w[d][q][2 * c + 1];
                            const half8_t sv = sc[GS ? d % DS : 0][q];
#if !CODEGEMM_ABLATE
                            if constexpr (!PH && fixed_gather<M, V, NW, RPL, BG, GS>()) {
                                if constexpr (GS) {
                                    const u32x4_t sw = __builtin_bit_cast(u32x4_t, sv);
                                    const uint32_t s4[4] = {sw.x, sw.y, sw.z, sw.w};
                                    gather8_scaled(acc[bb][q], lo, hi, off, s4);
                                } else {
                                    gather8(acc[bb][q], lo, hi, off);
                                }
                                continue;
                            }
#endif
#if CODEGEMM_ABLATE & 2
                            // ablation build: the code words are consumed, nothing is gathered
                            acc[bb][q][c & 7] += __builtin_bit_cast(float, (lo ^ hi) & 0x007fffffu);
                            (void)off; (void)sv;
                            continue;
#elif CODEGEMM_ABLATE & 1
                            // ablation build: address arithmetic and additions stay, the LDS reads go
#define CG_FAKE(k, wd) __builtin_bit_cast(float, __builtin_amdgcn_perm(wd, off, 0x0c020000u | ((4u + k) << 8)) & 0x007fffffu)
                            acc[bb][q][0] += CG_FAKE(0, lo); acc[bb][q][1] += CG_FAKE(1, lo);
                            acc[bb][q][2] += CG_FAKE(2, lo); acc[bb][q][3] += CG_FAKE(3, lo);
                            acc[bb][q][4] += CG_FAKE(0, hi); acc[bb][q][5] += CG_FAKE(1, hi);
                            acc[bb][q][6] += CG_FAKE(2, hi); acc[bb][q][7] += CG_FAKE(3, hi);
#undef CG_FAKE
                            (void)sv;
                            continue;
#endif
                            acc[bb][q][0] = PH ? accumulate_h<GS>(acc[bb][q][0], psum_h_at<0>(lo, off), sv[0]) : accumulate<GS>(acc[bb][q][0], psum_at<0>(lo, off), sv[0]);
                            acc[bb][q][1] = PH ? accumulate_h<GS>(acc[bb][q][1], psum_h_at<1>(lo, off), sv[1]) : accumulate<GS>(acc[bb][q][1], psum_at<1>(lo, off), sv[1]);
                            acc[bb][q][2] = PH ? accumulate_h<GS>(acc[bb][q][2], psum_h_at<2>(lo, off), sv[2]) : accumulate<GS>(acc[bb][q][2], psum_at<2>(lo, off), sv[2]);
                            acc[bb][q][3] = PH ? accumulate_h<GS>(acc[bb][q][3], psum_h_at<3>(lo, off), sv[3]) : accumulate<GS>(acc[bb][q][3], psum_at<3>(lo, off), sv[3]);
                            acc[bb][q][4] = PH ? accumulate_h<GS>(acc[bb][q][4], psum_h_at<0>(hi, off), sv[4]) : accumulate<GS>(acc[bb][q][4], psum_at<0>(hi, off), sv[4]);
                            acc[bb][q][5] = PH ? accumulate_h<GS>(acc[bb][q][5], psum_h_at<1>(hi, off), sv[5]) : accumulate<GS>(acc[bb][q][5], psum_at<1>(hi, off), sv[5]);
                            acc[bb][q][6] = PH ? accumulate_h<GS>(acc[bb][q][6], psum_h_at<2>(hi, off), sv[6]) : accumulate<GS>(acc[bb][q][6], psum_at<2>(hi, off), sv[6]);
                            acc[bb][q][7] = PH ? accumulate_h<GS>(acc[bb][q][7], psum_h_at<3>(hi, off), sv[7]) : accumulate<GS>(acc[bb][q][7], psum_at<3>(hi, off), sv[7]);
                        }
                    }
                }
                if (NBUF == 2) {
                    // build the next Psumbook of the sequence into the other buffer (after the
                    // gather in program order: the LDS reads that feed the accumulators go first)
                    if (has_next) {
                        if (last_bb) build(nxt, par ^ 1, xr[(d + 1) % D][0]);
                        else build(nxt, par ^ 1, xr[d][(bb + 1) % BG]);
                    }
                    if (BG == 1) xr[(d + 1) % D][0] = load_x(u + 1 + D, 0);   // its slot is free again
                }
                if (NBUF == 1) {
                    // single buffer: everyone must be done reading before it is rebuilt
                    __syncthreads();
                    if (has_next) {
                        if (last_bb) build(nxt, par ^ 1, xr[(d + 1) % D][0]);
                        else build(nxt, par ^ 1, xr[d][(bb + 1) % BG]);
                    }
                    if (BG == 1) xr[(d + 1) % D][0] = load_x(u + 1 + D, 0);
                }
                if (last_bb) load_codes(w[d], u + D);                       // refill the code ring
                if constexpr (GS) {
                    if (last_bb) load_scales(sc[d % DS], u + DS);
                }
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

    // Sum over the 32 slots (lanes) of each half-wavefront; the totals are parked in LDS
    // (the Psumbook is no longer needed), indexed by the row's position inside the
    // workgroup's block, so that the global stores and loads below are coalesced over all
    // threads.
    constexpr int ROWS = PIECES * 16;                                 // rows of this workgroup's block
    float* stage = planes;                                           // [BG][ROWS]
    {
        constexpr int NV = (RPL == 1) ? 8 : 16;                      // values reduced together
        const int idx = lane & (NV - 1);                             // value this lane ends up holding
#pragma unroll
        for (int q0 = 0; q0 < RPL; q0 += NV / 8) {
            const int q = q0 + idx / 8;
            const int local = (q * NG + wave) * 16 + khalf * kRowsPerLane + idx % 8;   // piece, half-wavefront, row
#pragma unroll
            for (int bb = 0; bb < BG; ++bb) {
                float v[NV];
#pragma unroll
                for (int i = 0; i < NV; ++i) v[i] = acc[bb][q0 + i / 8][i % 8];
                const float t = halfwave_transpose_sum<NV>(v, lane);
                if ((lane & 31) < NV) stage[bb * ROWS + local] = t;
            }
        }
    }
    finish_block<NW * kWave, BG, ROWS>(p, mm, stage, flag, tid, blk, ks, b0);
}

int set_max_lds(const void* fn, size_t bytes);

template <int M, int V, int NW, int RPL, int BG, int D, bool GS, bool PH = false, int NB = 0>
int launch_gemm_one(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    auto fn = gemm_kernel<M, V, NW, RPL, BG, D, GS, PH, NB>;
    typedef PsumLayout<M> L;
    const size_t lds = (PH ? (size_t)PsumLayoutH<M>::kBytes : (size_t)L::kBuffers * L::kBytes) + 64;
    int st = set_max_lds(reinterpret_cast<const void*>(fn), lds);
    if (st != CODEGEMM_OK) return st;
    const dim3 grid((unsigned)g.NKS, (unsigned)g.NBLK, (unsigned)g.NG);
    hipLaunchKernelGGL(fn, grid, dim3(NW * kWave), lds, stream, CG_HEAD_ARGS(p), p);
    return hipGetLastError() == hipSuccess ? CODEGEMM_OK : CODEGEMM_LAUNCH_FAILED;
}

// Instantiated (waves, row words per lane) pairs.  The code ring is two units deep everywhere.
// A compute unit keeps only about 32-40 KB of loads outstanding (measured: 16 wavefronts
// issue 32 KB of 16-byte loads in 400 clocks, 64 KB in 1300 and 128 KB in 3800 warm, 8800
// from HBM), and a wavefront that cannot issue its next load cannot build or gather either,
// so a deeper ring only parks the wavefronts in front of the memory pipeline: with 4 units
// the 70B calls took 0.6-2 us longer, with 6 units 50 % longer.
template <int M, int V, int BG, bool GS>
int launch_gemm_mvb(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    if constexpr (BG == 1 && M <= 2) {
        // 14 gathering + 2 building wavefronts: 448-row blocks
        if (g.NW == 16 && g.RPL == 2 && g.NB == 2) return launch_gemm_one<M, V, 16, 2, BG, 2, GS, false, 2>(g, p, stream);
    }
    if (g.NB != 0) return CODEGEMM_UNSUPPORTED;
    if (g.NW == 8 && g.RPL == 1) return launch_gemm_one<M, V, 8, 1, BG, 2, GS>(g, p, stream);
    if (g.NW == 16 && g.RPL == 1) return launch_gemm_one<M, V, 16, 1, BG, 2, GS>(g, p, stream);
    if constexpr (BG * M <= 4) {
        if (g.NW == 16 && g.RPL == 2) return launch_gemm_one<M, V, 16, 2, BG, 2, GS>(g, p, stream);
        // 448-row blocks: matrices whose height is 7 * 2^k (the Llama up/gate projections) then
        // divide into a number of workgroups that fills 256 compute units
        if (g.NW == 14 && g.RPL == 2) return launch_gemm_one<M, V, 14, 2, BG, 2, GS>(g, p, stream);
    }
    if constexpr (BG * M <= 8) {   // 8 wavefronts have twice the registers per lane
        if (g.NW == 8 && g.RPL == 2) return launch_gemm_one<M, V, 8, 2, BG, 2, GS>(g, p, stream);
    }
    if constexpr (BG == 1 && M <= 2 && !GS) {
        if (g.NW == 16 && g.RPL == 4) return launch_gemm_one<M, V, 16, 4, BG, 2, GS>(g, p, stream);
    }
    return CODEGEMM_UNSUPPORTED;
}

// fp16 Psumbook (batch rows one at a time): the same block shapes.
template <int M, int V, bool GS>
int launch_gemm_h_mv(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    if (g.NW == 8 && g.RPL == 1) return launch_gemm_one<M, V, 8, 1, 1, 2, GS, true>(g, p, stream);
    if (g.NW == 16 && g.RPL == 1) return launch_gemm_one<M, V, 16, 1, 1, 2, GS, true>(g, p, stream);
    if (g.NW == 8 && g.RPL == 2) return launch_gemm_one<M, V, 8, 2, 1, 2, GS, true>(g, p, stream);
    if constexpr (!GS) {   // with group scales the 16-wavefront, 2-row-word shape runs out of registers
        if (g.NW == 16 && g.RPL == 2) return launch_gemm_one<M, V, 16, 2, 1, 2, GS, true>(g, p, stream);
    }
    return CODEGEMM_UNSUPPORTED;
}

template <int M, bool GS>
int launch_gemm_h_m(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    if (g.BG != 1) return CODEGEMM_UNSUPPORTED;
    if (g.v == 16) return launch_gemm_h_mv<M, 16, GS>(g, p, stream);
    if (g.v == 8) return launch_gemm_h_mv<M, 8, GS>(g, p, stream);
    return launch_gemm_h_mv<M, 4, GS>(g, p, stream);
}

template <int M, bool GS>
int launch_gemm_m(const Geometry& g, const GemmParams& p, hipStream_t stream)
{
    if (g.v == 16) {
        switch (g.BG) {
            case 1: return launch_gemm_mvb<M, 16, 1, GS>(g, p, stream);
            case 2: return launch_gemm_mvb<M, 16, 2, GS>(g, p, stream);
        }
    } else if (g.v == 8) {
        switch (g.BG) {
            case 1: return launch_gemm_mvb<M, 8, 1, GS>(g, p, stream);
            case 2: return launch_gemm_mvb<M, 8, 2, GS>(g, p, stream);
        }
    } else {
        switch (g.BG) {
            case 1: return launch_gemm_mvb<M, 4, 1, GS>(g, p, stream);
            case 2: return launch_gemm_mvb<M, 4, 2, GS>(g, p, stream);
        }
    }
    return CODEGEMM_UNSUPPORTED;
}

int launch_gemm_m1(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_m2(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_m3(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_m4(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_gs_m1(const Geometry& g, const GemmParams& p, hipStream_t stream);   // with group scales
int launch_gemm_gs_m2(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_gs_m3(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_gs_m4(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_h_m1(const Geometry& g, const GemmParams& p, hipStream_t stream);      // fp16 Psumbook
int launch_gemm_h_m2(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_h_m3(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_h_m4(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_h_gs_m1(const Geometry& g, const GemmParams& p, hipStream_t stream);   // fp16 Psumbook, group scales
int launch_gemm_h_gs_m2(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_h_gs_m3(const Geometry& g, const GemmParams& p, hipStream_t stream);
int launch_gemm_h_gs_m4(const Geometry& g, const GemmParams& p, hipStream_t stream);

}  // namespace cg
