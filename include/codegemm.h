/*
 * codegemm.h - C ABI of the MI355X (gfx950) CodeGEMM library.
 *
 * Computes the linear layer  y = x W^T  for a weight matrix W (N x K) that is
 * stored codebook-quantized: every run of v consecutive weights along K is the
 * sum of m centroid vectors, one from each of m codebooks of 256 fp16 centroids,
 * selected by 8-bit codes, times an fp16 scale: one per output row (g = -1) or
 * one per run of g consecutive weights of a row
 * (CodeGEMM paper, Section 2.2: vector length v, number of codebooks m, bits
 * per code b = 8, normalisation group size g).
 *
 * The hot path never reconstructs W.  It builds a Psumbook (Section 3, Eq. 2)
 *     P[b][c][j][i] = sum_{k<v} C[c][i][k] * x[b][v*j + k]
 * in LDS, then gathers P by code and accumulates over j and c (Section 3,
 * Step 3), and multiplies by the row scale (g = -1) or scales every gathered
 * partial sum by the scale of its group as it is accumulated (g > 0).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HBM) unless marked "host".
 *     The descriptor and plan structs are host structs passed by pointer.
 *   - The caller owns every buffer.  The library allocates no device memory
 *     and never synchronises: work is enqueued on `stream` (a hipStream_t
 *     passed as void*; NULL = the default stream).  The only state it keeps
 *     between calls is per-process and mutex-guarded: a note of which kernels
 *     have had their LDS limit raised on which device (a one-time HIP
 *     attribute), and, once codegemm_gemm_static has been used on a device, the
 *     address of that device's copy of the library's static workspace.
 *   - Inputs are read-only.  Outputs are fully overwritten.  Buffers must not
 *     alias.  Every pointer must be 16-byte aligned.
 *   - Return value: CODEGEMM_OK (0) or a negative codegemm_status.  No entry
 *     point prints, throws or aborts.
 *
 * Canonical layouts (row-major, contiguous)
 *     x          [B][K]        fp16
 *     codes      [m][N][K/v]   uint8   (every value 0..255 is a valid centroid index)
 *     codebooks  [m][256][v]   fp16
 *     scales     [N]           fp16     (group_size = -1)
 *                [N][K/g]      fp16     (group_size = g > 0)
 *     y          [B][N]        fp16, or fp32 when CODEGEMM_FLAG_Y_FP32 is set
 *     psumbook   [B][m][K/v][256] fp32
 */
#ifndef CODEGEMM_H
#define CODEGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum codegemm_status {
    CODEGEMM_OK = 0,
    CODEGEMM_INVALID_ARG = -1,        /* NULL pointer, non-positive size, K % v != 0, misaligned pointer */
    CODEGEMM_UNSUPPORTED = -2,        /* v, m, b, g, batch or plan outside what the kernels implement   */
    CODEGEMM_WORKSPACE_TOO_SMALL = -3,
    CODEGEMM_LAUNCH_FAILED = -4       /* the HIP runtime rejected a launch or a memset                  */
} codegemm_status;

enum {
    CODEGEMM_FLAG_Y_FP32 = 1          /* y is float[B][N] instead of fp16 */
};

/* Problem descriptor (host struct). */
typedef struct codegemm_desc {
    int32_t batch;          /* B, 1..65535; more than 32 rows run as several   */
                            /* launches of up to 32 rows on the same stream    */
    int32_t in_features;    /* K, a positive multiple of vec_len, <= 2^22      */
    int32_t out_features;   /* N, 1..2^24                                      */
    int32_t vec_len;        /* v: 4, 8 or 16                                   */
    int32_t num_codebooks;  /* m: 1..4                                         */
    int32_t code_bits;      /* b: must be 8 (Section 6, Limitations)           */
    int32_t group_size;     /* g: -1 (one scale per output row), or v * 2^i    */
                            /* (i >= 0) dividing K: one scale per g weights     */
    int32_t flags;          /* CODEGEMM_FLAG_*                                 */
} codegemm_desc;

/*
 * Launch plan of codegemm_gemm (host struct).  The paper's tile is t_h rows by
 * t_w weights (Section 3); here one "unit" is 128 rows by 32 * v weights, and one
 * workgroup streams through a contiguous run of units of its rows (all of K when
 * k_splits = 1), rebuilding the Psumbook (m * 256 * 32 fp32 in LDS, double-
 * buffered for m <= 2) once per unit.
 */
typedef struct codegemm_plan {
    int32_t waves;          /* wavefronts per workgroup: 8, 14 or 16 (14: row_words = 2, batch_group  */
                            /* 1 or 2, fp32 Psumbook; its 448-row blocks divide heights of 7 * 2^k    */
                            /* rows into a number of workgroups that fills 256 compute units)         */
    int32_t row_words;      /* 8-row code words per lane per unit: 1, 2 or 4.  The workgroup owns     */
                            /* 16 * waves * row_words rows (32 * waves * row_words when batch_group   */
                            /* = 4).  Limits (registers): batch_group 1 or 2: row_words = 2 needs     */
                            /* batch_group * m <= 4 (<= 8 with waves = 8), row_words = 4 needs waves  */
                            /* = 16, batch_group = 1, m <= 2 and one scale per row; batch_group 4:    */
                            /* row_words = 4 needs waves = 8                                          */
    int32_t k_splits;       /* workgroups per row block, each taking a contiguous range of K tiles    */
                            /* (clamped to the number of K tiles).  1: every workgroup produces final */
                            /* outputs on its own.  > 1: partial sums are combined through the        */
                            /* workspace by the last workgroup to finish                               */
    int32_t batch_group;    /* batch rows handled per pass over the codes: 1, 2 or 4.  4 selects the  */
                            /* batched kernel (batch axis innermost in the Psumbook, 128-bit gathers) */
    int32_t psum_dtype;     /* number type the Psumbook is stored in (LDS): 0 = fp32 (default, exact     */
                            /* fp16 x fp16 products summed in fp32), 1 = fp16 (each partial sum rounded  */
                            /* to nearest-even fp16 after its fp32 accumulation; accumulation over K     */
                            /* stays fp32).  fp16 halves the LDS bytes written per unit and adds about   */
                            /* 3e-4 relative error to y; needs batch_group = 1, row_words <= 2, and with  */
                            /* group scales not (waves 16, row_words 2).                                 */
                            /* codegemm_default_plan never chooses it.                                    */
    int32_t build_waves;    /* 0: every wavefront builds its share of each Psumbook between two gathers.  */
                            /* 2 (waves = 16, row_words = 2, batch_group = 1, fp32 Psumbook, m <= 2): the */
                            /* last two wavefronts only build, one unit ahead; the other 14 stream,       */
                            /* gather and own the workgroup's 448 rows                                    */
    int32_t reserved[2];    /* must be zero */
} codegemm_plan;

enum {
    CODEGEMM_PSUM_FP32 = 0,
    CODEGEMM_PSUM_FP16 = 1
};

/* Fills *plan with the library's choice for this problem.  Host only, no GPU work. */
int codegemm_default_plan(const codegemm_desc *desc, codegemm_plan *plan);

/* Bytes of `workspace` codegemm_gemm needs under `plan` (NULL plan = default plan).
 * Returns 0 for an invalid descriptor or plan. */
size_t codegemm_workspace_bytes(const codegemm_desc *desc, const codegemm_plan *plan);

/* Bytes of the packed code buffer under `plan` (NULL = default).  0 if invalid. */
size_t codegemm_packed_codes_bytes(const codegemm_desc *desc, const codegemm_plan *plan);

/*
 * Prepares a workspace for codegemm_gemm: zero-fills it.  Must be enqueued once
 * after allocation, before the first codegemm_gemm that uses the workspace.
 * Every codegemm_gemm call leaves the workspace ready for the next call on the
 * same stream, so this is a one-time cost; the next call may have another
 * shape, format or plan (the workspace starts with a 64 KB area of ticket
 * counters and a 2 MB area of 64-bit words through which calls with two or four
 * K ranges combine their sums pairwise, both of which every call finds and
 * leaves all zero, followed by fp32 partial sums that need no initial value),
 * so one workspace of the largest codegemm_workspace_bytes() serves all layers
 * of a model.  A call that is aborted (device reset, killed process) can leave
 * the two areas non-zero: initialise again.  Two calls that use the same
 * workspace concurrently (different streams) race.
 */
int codegemm_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/*
 * Re-orders canonical codes [m][N][K/v] into the packed streaming layout the
 * gather kernel reads (offline, once per weight matrix), and back.
 *
 * Packed layout (independent of the plan).  Let J = K / v, NGR = ceil(N / 128),
 * NKT = ceil(J / 32).  The buffer is an array [NGR][NKT][part][16][32][bytes]:
 * one "unit" per 128-row granule rg and K tile kt (all units of a granule are
 * contiguous, in K order); inside a unit the index g = 0..15 selects 8 rows,
 * s = 0..31 a sub-vector of the tile, and the 8*m bytes of (g, s) are split
 * into parts of 16 bytes (two codebooks) plus, for odd m, a last part of 8
 * bytes (one codebook).  Within a part, byte 8*(c - c0) + r holds, for
 * codebook c and r = 0..7,
 *     codes[c][128*rg + 8*g + r][32*kt + s]
 * or 0 when that row or sub-vector lies outside the matrix.  A wavefront reads
 * 64 consecutive entries (two values of g, all 32 slots) with one 16-byte load
 * per lane, and the 32 lanes of each half-wavefront then address 32 different
 * slots of the Psumbook, which keeps the data-dependent LDS gathers free of
 * bank conflicts whatever the code values are.  Bytes are stored as such, so a
 * 32-bit word read from the buffer holds byte q in bits 8q..8q+7.
 *
 * Both calls are bit-exact: unpack(pack(codes)) == codes.
 */
int codegemm_pack_codes(const codegemm_desc *desc, const codegemm_plan *plan,
                        const uint8_t *codes, uint8_t *packed, void *stream);
int codegemm_unpack_codes(const codegemm_desc *desc, const codegemm_plan *plan,
                          const uint8_t *packed, uint8_t *codes, void *stream);

/*
 * The same two re-orderings on the host: `codes` and `packed` are HOST pointers,
 * the call is synchronous and touches no GPU (for packing a checkpoint where it
 * is loaded).  Byte for byte the result of the device calls.
 */
int codegemm_pack_codes_host(const codegemm_desc *desc, const uint8_t *codes, uint8_t *packed);
int codegemm_unpack_codes_host(const codegemm_desc *desc, const uint8_t *packed, uint8_t *codes);

/*
 * Scales of a layer with group_size = g > 0 (Section 2.2, Step 1), re-ordered
 * from the canonical [N][K/g] array into the layout the gather kernels read
 * next to the packed codes (offline, once per weight matrix).  With GPU =
 * max(1, 32 * v / g) groups per 32-sub-vector unit, the buffer is an array
 * [NGR][NKT][GPU][16][8] of fp16: entry (rg, kt, q, o, r) is the scale of row
 * 128*rg + 8*o + r for the group that holds sub-vector 32*kt + q*g/v (0 when
 * the row or the sub-vector lies outside the matrix), so the 8 rows a lane
 * owns are one 16-byte load.  codegemm_packed_scales_bytes returns 0 for an
 * invalid descriptor or for group_size = -1 (such layers pass scales [N] as is).
 */
size_t codegemm_packed_scales_bytes(const codegemm_desc *desc);
int codegemm_pack_scales(const codegemm_desc *desc, const void *scales, void *packed, void *stream);

/*
 * Section 3, Eq. 2, for the whole of K: psumbook[b][c][j][i] (fp32), from
 * x [B][K] fp16 and codebooks [m][256][v] fp16.  fp16 products are exact in
 * fp32 and are accumulated in fp32.  use_mfma != 0 computes the contraction on
 * the matrix cores (the (m*256) x (B*K/v) x v product), 0 on the vector ALU.
 */
int codegemm_psumbook_build(const codegemm_desc *desc, const void *x, const void *codebooks,
                            float *psumbook, int use_mfma, void *stream);

/*
 * The hot path (Section 3, Steps 1-3, then de-normalisation by the row scale):
 *     y[b][n] = scales[n] * sum_{c<m} sum_{j<K/v} P[b][c][j][ codes[c][n][j] ].
 * For group_size = g > 0,
 *     y[b][n] = sum_G scales[n][G] * sum_{c<m} sum_{j in G} P[b][c][j][ codes[c][n][j] ].
 * `packed_codes` is the output of codegemm_pack_codes.  `scales` is the
 * canonical [N] array when group_size = -1 and the output of
 * codegemm_pack_scales otherwise.
 * fp16 inputs, fp32 Psumbook (built on the matrix cores: fp16 products are exact
 * in fp32) and fp32 accumulation, y rounded to nearest-even fp16 (or stored as
 * fp32 under CODEGEMM_FLAG_Y_FP32).  Every sum is taken in a fixed order (also
 * across K ranges), so results are bit-reproducible.
 * `workspace` holds at least codegemm_workspace_bytes() bytes and has been
 * through codegemm_workspace_init once.  plan == NULL uses the default plan.
 */
int codegemm_gemm(const codegemm_desc *desc, const codegemm_plan *plan,
                  const void *x, const uint8_t *packed_codes, const void *codebooks,
                  const void *scales, void *y, void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * The hot path for up to 4 layers that read the same x in ONE kernel launch:
 * the q, k and v projections of a decoder block, or its gate and up projections
 * (the paper times a whole decoder block, Section 4.1 and its latency table; at
 * batch 1 a launch costs about as much as a small layer's data movement).  The
 * layers share in_features, the format (v, m, group_size), the batch and the
 * flags; each has its own out_features, packed codes, codebooks, scales and y.
 * Member i's result is bit-identical to codegemm_gemm on that layer alone with
 * the same plan.
 *   desc->out_features   the SUM of the members' out_features (checked);
 *   plan                 applies to every member; NULL = codegemm_default_plan(desc),
 *                        which suits since the launch fills the chip like one
 *                        layer of the summed height; batch <= 32;
 *   group[i]             device pointers as for codegemm_gemm, y [batch][out_features_i];
 *   workspace            codegemm_grouped_workspace_bytes() bytes, initialised once
 *                        with codegemm_workspace_init; any workspace may be shared
 *                        between grouped and plain calls on one stream.
 * Errors: CODEGEMM_INVALID_ARG (count outside 1..4, null or misaligned pointer,
 * out_features not summing to desc->out_features), CODEGEMM_UNSUPPORTED (batch > 32,
 * more than 65535 row blocks), CODEGEMM_WORKSPACE_TOO_SMALL.
 * codegemm_grouped_workspace_bytes returns 0 on any of the former two.
 */
typedef struct codegemm_group_member {
    int32_t out_features;
    int32_t reserved;             /* 0 */
    const uint8_t *packed_codes;  /* device, output of codegemm_pack_codes for this layer */
    const void *codebooks;        /* device, [m][256][v] fp16 */
    const void *scales;           /* device, [N] fp16 or the output of codegemm_pack_scales */
    void *y;                      /* device, [batch][out_features] */
} codegemm_group_member;

size_t codegemm_grouped_workspace_bytes(const codegemm_desc *desc, const codegemm_plan *plan,
                                        const int32_t *out_features, int32_t count);
int codegemm_gemm_grouped(const codegemm_desc *desc, const codegemm_plan *plan, const void *x,
                          const codegemm_group_member *group, int32_t count,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * codegemm_gemm for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same computation, same kernels and the same
 * bits in y as codegemm_gemm; the workspace is an array of
 * codegemm_static_workspace_limit() bytes (8 MiB) that lives inside the loaded
 * library, one per GPU, until the process ends.  The call allocates nothing.
 * Returns CODEGEMM_WORKSPACE_TOO_SMALL when codegemm_workspace_bytes(desc, plan)
 * exceeds that limit (about batch * k_splits * N > 1.5 million).  The first call on
 * a device looks the array up and clears its counter and pair-word areas on `stream`; make
 * that call outside graph capture.  All calls on one GPU share the array: two
 * that overlap in time (different streams, or graphs replayed concurrently)
 * race; calls on one stream, of any shapes and plans, do not.
 */
size_t codegemm_static_workspace_limit(void);
int codegemm_gemm_static(const codegemm_desc *desc, const codegemm_plan *plan,
                         const void *x, const uint8_t *packed_codes, const void *codebooks,
                         const void *scales, void *y, void *stream);

/*
 * Dequantization-based comparator (Section 2.3: the whole codebook sits in LDS,
 * each code fetches its centroid vector, which is multiplied with the matching
 * activations; O(N*B*K) multiply-adds).  Same result as codegemm_gemm up to
 * fp32 summation order.  `codes` is the canonical [m][N][K/v] array and `scales`
 * the canonical [N] or [N][K/g] array.  Needs no workspace.
 */
int codegemm_dequant_gemm(const codegemm_desc *desc, const void *x, const uint8_t *codes,
                          const void *codebooks, const void *scales, void *y, void *stream);

/* Static, NUL-terminated description of a status code.  Host only. */
const char *codegemm_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CODEGEMM_H */
