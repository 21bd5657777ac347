// Internal definitions shared by the translation units of libcodegemm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "codegemm.h"

namespace cg {

constexpr int kCentroids = 256;     // 2^b with b = 8
constexpr int kWave = 64;           // CDNA wavefront width
constexpr int kRowsPerLane = 8;     // output rows owned by one lane of the gather kernel
constexpr int kSlots = 32;          // sub-vectors per K tile = lanes of a half-wavefront
constexpr int kGranuleRows = 128;   // rows per packed unit: 16 half-wavefronts x 8 rows
// Ticket counters.  Every workspace starts with a counter area of fixed size, whatever the
// shape and plan of the calls that use it, so that calls of different shapes can share one
// workspace: a call leaves its counters at zero and never writes partial sums where another
// call keeps counters.  The counters of different row blocks lie kCounterStride words (256
// bytes) apart: device-scope atomics on words of one cache line are served one after the other
// (~0.2 us each), whoever issues them, and with the counters packed into one or two lines every
// ticket of a launch queued behind every other one (measured: 0.5-2 us per call).  Plans with
// more than 256 row blocks x batch groups AND several K ranges get a smaller stride.
constexpr int kCounterStride = 64;
constexpr int kCounterAreaWords = 16384;   // 64 KB
// Behind the counters: 64-bit words of the pairwise reduction between K ranges (2, 4 or 8 of them), which every call
// finds and leaves all zero like the counters.  Calls whose words do not fit use the ticket and the fp32 partials.
constexpr size_t kPairAreaBytes = 2u << 20;
constexpr int kMaxLds = 160 * 1024; // LDS per workgroup on gfx950
constexpr int kBatchPerLaunch = 32;         // batch rows one launch of a gather kernel takes; more rows = more launches
constexpr int kMaxBatch = 65535;            // grid limit of the comparator (one grid row per batch row)
constexpr int kMaxInFeatures = 1 << 22;     // K: a workgroup's code range (K/v/32 units of 4096 m bytes) and a row of
                                            // x stay below 2^31 bytes, which the 32-bit buffer offsets require
constexpr int kMaxOutFeatures = 1 << 24;    // N: row indices and padded row counts stay in 32-bit ints

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Derived sizes of one problem under one plan.
struct Geometry {
    int B, K, N, v, m, J;
    int NW;         // wavefronts per workgroup (8 or 16; 14 in the kernel for one or two batch rows)
    int NB;         // of the NW wavefronts, those that only build Psumbooks (0 or 2); the others own the rows
    int RPL;        // 8-row words per lane per unit (1, 2 or 4): the workgroup owns 16 * (NW - NB) * RPL rows
                    // (32 * NW * RPL in the batched kernel, BG = 4)
    int BG;         // batch rows per pass over the codes
    int NGR;        // ceil(N / 128) granules
    int NBLK;       // row blocks = workgroups along N: NGR over the granules per workgroup, rounded up
    int NKT;        // ceil(J / 32) K tiles
    int NKS;        // workgroups per row block (K ranges)
    int KPW;        // K tiles per workgroup: ceil(NKT / NKS)
    int NG;         // ceil(B / BG) batch groups
    int Npad;       // NGR * 128
    int g;          // normalisation group size along K, or -1
    int GPU;        // scale groups per 32-sub-vector unit: max(1, 32 * v / g); 0 when g = -1
    int gshift;     // a lane's group inside its unit = (sub-vector index in the unit) >> gshift
    bool y_fp32;
    bool psum_fp16;  // Psumbook stored as fp16 pairs (plan field psum_dtype)
};

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Offset of the packed byte that holds codes[c][n][j]  (see codegemm.h, packed layout).
__host__ __device__ inline size_t packed_offset(int c, int n, int j, int m, int NKT)
{
    const int granule = n / kGranuleRows;
    const int g = (n % kGranuleRows) / kRowsPerLane;       // row-lane: which half-wavefront
    const int r = n % kRowsPerLane;
    const int kt = j / kSlots;
    const int s = j % kSlots;
    const int part = c >> 1;
    const int part_bytes = (2 * part + 1 == m) ? 8 : 16;   // last part of an odd m holds one codebook
    size_t off = ((size_t)granule * NKT + kt) * (size_t)(kGranuleRows * kSlots * m);
    off += (size_t)part * 16 * 512 + (size_t)(g * kSlots + s) * part_bytes + (c & 1) * 8 + r;
    return off;
}

int make_geometry(const codegemm_desc* d, const codegemm_plan* plan, Geometry* g);   // status
size_t workspace_counter_bytes(const Geometry& g);   // the fixed area in front of the partial sums: counters, then pair words
size_t pair_words(const Geometry& g);                // 64-bit words the pairwise reduction of this problem needs; 0: not offered
int counter_stride(const Geometry& g);               // words between two row blocks' counters; 0: the plan does not fit

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

}  // namespace cg
