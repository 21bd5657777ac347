// Host-side logic: argument validation, launch plan, buffer sizes, status strings.
#include "cg_common.h"

namespace cg {

static int validate_desc(const codegemm_desc* d)
{
    if (!d) return CODEGEMM_INVALID_ARG;
    if (d->batch < 1 || d->in_features < 1 || d->out_features < 1) return CODEGEMM_INVALID_ARG;
    if (d->vec_len != 4 && d->vec_len != 8 && d->vec_len != 16) return CODEGEMM_UNSUPPORTED;
    if (d->num_codebooks < 1 || d->num_codebooks > 4) return CODEGEMM_UNSUPPORTED;
    if (d->code_bits != 8) return CODEGEMM_UNSUPPORTED;
    // Every byte offset the kernels form (a workgroup's code range, a row of x) stays below 2^31.
    if (d->batch > kMaxBatch || d->in_features > kMaxInFeatures || d->out_features > kMaxOutFeatures)
        return CODEGEMM_UNSUPPORTED;
    if (d->in_features % d->vec_len) return CODEGEMM_INVALID_ARG;
    if (d->group_size != -1) {
        // one scale per g = v * 2^i weights, groups tiling K exactly
        const int g = d->group_size;
        if (g < d->vec_len || g % d->vec_len) return CODEGEMM_UNSUPPORTED;
        const int ratio = g / d->vec_len;
        if (ratio & (ratio - 1)) return CODEGEMM_UNSUPPORTED;
        if (d->in_features % g) return CODEGEMM_INVALID_ARG;
    }
    if (d->flags & ~CODEGEMM_FLAG_Y_FP32) return CODEGEMM_INVALID_ARG;
    return CODEGEMM_OK;
}

static int validate_plan(const codegemm_desc* d, const codegemm_plan* p)
{
    if (p->waves != 8 && p->waves != 14 && p->waves != 16) return CODEGEMM_UNSUPPORTED;
    if (p->waves == 14) {
        // 448-row blocks: gather kernel for one or two batch rows only, fp32 Psumbook, registers as for 16 wavefronts
        if (p->row_words != 2 || p->batch_group > 2 || p->psum_dtype != CODEGEMM_PSUM_FP32) return CODEGEMM_UNSUPPORTED;
    }
    if (p->row_words != 1 && p->row_words != 2 && p->row_words != 4) return CODEGEMM_UNSUPPORTED;
    if (p->row_words == 4 && p->waves != 16 && p->batch_group != 4) return CODEGEMM_UNSUPPORTED;
    if (p->k_splits < 1) return CODEGEMM_UNSUPPORTED;
    if (p->batch_group != 1 && p->batch_group != 2 && p->batch_group != 4) return CODEGEMM_UNSUPPORTED;
    for (int i = 0; i < 2; ++i)
        if (p->reserved[i]) return CODEGEMM_INVALID_ARG;
    if (p->build_waves != 0 && p->build_waves != 2) return CODEGEMM_UNSUPPORTED;
    if (p->build_waves == 2) {
        // 14 gathering + 2 building wavefronts: a double-buffered fp32 Psumbook (one or two codebooks); one batch
        // row per pass with two row words, or the batched kernel with one or two
        if (p->waves != 16 || p->psum_dtype != CODEGEMM_PSUM_FP32 || d->num_codebooks > 2) return CODEGEMM_UNSUPPORTED;
        if (p->batch_group == 1 ? p->row_words != 2 : (p->batch_group != 4 || p->row_words > 2)) return CODEGEMM_UNSUPPORTED;
    }
    if (p->psum_dtype != CODEGEMM_PSUM_FP32 && p->psum_dtype != CODEGEMM_PSUM_FP16) return CODEGEMM_UNSUPPORTED;
    if (p->psum_dtype == CODEGEMM_PSUM_FP16) {
        if (p->batch_group != 1 || p->row_words > 2) return CODEGEMM_UNSUPPORTED;
        if (d->group_size > 0 && p->waves == 16 && p->row_words == 2) return CODEGEMM_UNSUPPORTED;   // registers
        return CODEGEMM_OK;
    }
    const int m = d->num_codebooks;
    if (p->batch_group == 4) {
        // the batched kernel: 32 accumulators per row word
        if (p->row_words == 4 && p->waves != 8) return CODEGEMM_UNSUPPORTED;
        return CODEGEMM_OK;
    }
    if (p->row_words >= 2 && p->batch_group * m > (p->waves == 8 ? 8 : 4)) return CODEGEMM_UNSUPPORTED;   // accumulators + code ring must fit in registers
    if (p->row_words == 4 && (p->batch_group != 1 || m > 2 || d->group_size > 0)) return CODEGEMM_UNSUPPORTED;
    return CODEGEMM_OK;
}

// Library's own choice.  One workgroup per compute unit is resident (its Psumbook
// buffers take 128 KB of LDS).  A workgroup must stream about 32 KB of codes per K tile
// to keep up with its share of HBM, so blocks are 512 rows tall when the batch and the
// number of codebooks leave registers for it; the K ranges are then cut to give close
// to, but not more than, 256 workgroups.
static void choose_plan(const codegemm_desc* d, codegemm_plan* p)
{
    *p = codegemm_plan{};
    const int m = d->num_codebooks;
    const int J = d->in_features / d->vec_len;
    const int ngr = ceil_div(d->out_features, kGranuleRows);
    const int nkt = ceil_div(J, kSlots);
    const double code_positions = (double)d->out_features * J;
    // Two batch rows: the batch-1 kernel with the code words reused for a second Psumbook, except on
    // large matrices, where the batched kernel wins even with two of its four batch lanes idle
    // (8192->28672: 32.7 -> 25.6 us; 8192^2: 11.4 against 12.0)
    const int batch = d->batch < kBatchPerLaunch ? d->batch : kBatchPerLaunch;
    p->batch_group = batch == 1 ? 1 : ((batch == 2 && code_positions < 16e6) ? 2 : 4);
    if (p->batch_group == 4) {
        // LDS- and ALU-bound.  Every workgroup rebuilds the Psumbook of its tiles, and LDS
        // writes are slow, so blocks are 1024 rows tall when there are at least two batch
        // groups to fill the chip with, 512 otherwise; K ranges are cut so that all batch
        // groups together give close to, but not more than, 256 workgroups.
        const int groups = ceil_div(batch, 4);
        auto fill = [&](int waves, int row_words, int* k_splits) {      // workgroups of a block shape
            const int nblk = ceil_div(ngr * kGranuleRows, waves * row_words * 32) * groups;
            int nks = 256 / nblk;
            if (nks > nkt) nks = nkt;
            if (nks < 1) nks = 1;
            *k_splits = ceil_div(nkt, ceil_div(nkt, nks));
            return nblk * *k_splits;
        };
        p->waves = 16;
        p->row_words = groups >= 2 ? 2 : 1;
        if (groups == 1) {
            // one batch group: 1024-row blocks only if every workgroup still gets 4 units of K
            // from at most 16 K ranges
            // (8192->28672 at batch 4: 32.4 -> 27.5 us; with 1 unit each they lose: 13.0 -> 16.6)
            const int nblk2 = ceil_div(ngr, 8);
            int nks2 = 256 / nblk2;
            if (nks2 > nkt) nks2 = nkt;
            if (nks2 < 1) nks2 = 1;
            if (ceil_div(nkt, nks2) >= 4 && nks2 <= 16) p->row_words = 2;   // (28 ranges: 30.1 -> 32.7 us)
        }
        // The 1024-row shape with 16 wavefronts has 128 registers per lane: with group scales, or
        // three and more codebooks, its 64 accumulators and the scale ring no longer fit and it
        // spills (8192->28672, m2v8g128, batch 8: 93 us against 56 us with 512-row blocks).
        if (p->row_words == 2 && (d->group_size > 0 || m >= 3)) p->row_words = 1;
        // Small matrices: a shorter block when the taller one leaves most of the chip idle
        // (2048^2 at batch 8: 32 workgroups of 1024 rows 19.5 us, 128 of 256 rows 7.8 us).
        int ks = 1;
        int wgs = fill(p->waves, p->row_words, &ks);
        if (wgs < 192 && p->row_words == 2) {
            int ks1 = 1;
            const int w1 = fill(16, 1, &ks1);
            if (w1 > wgs) { p->row_words = 1; wgs = w1; ks = ks1; }
        }
        if (wgs < 192 || ks > 32) {
            // also when the chip is only filled by cutting K into more than 32 ranges: the last
            // workgroup of a row block then adds that many partial sums per output
            // (8192->2048, v4 m1, batch 4: 64 ranges 13.2 us)
            int ks8 = 1;
            const int w8 = fill(8, 1, &ks8);
            if (w8 > wgs || (w8 >= 192 && ks8 < ks)) { p->waves = 8; p->row_words = 1; wgs = w8; ks = ks8; }
        }
        p->k_splits = ks;
        // Heights that 448 (896) rows divide, one or two codebooks: 14 of the 16 wavefronts own the rows
        // and 2 build every tile's Psumbook one tile ahead; the blocks then also fill 256 compute units
        // where 512 (1024) rows give 224 (4096->14336 v8 m2, batch 4 / 8 / 16 / 32: -5 / -9 / -12 / -11 %;
        // 8192->28672 m2v8g128 batch 4 / 8: -9 / -10 %).  With a ragged last block it loses (8192 rows: +10 %).
        if (p->waves == 16 && m <= 2) {
            const int rows = 14 * p->row_words * 32;
            const int nblk14 = ceil_div(d->out_features, rows);
            if ((long long)nblk14 * rows * 50 <= (long long)ngr * kGranuleRows * 51) {        // at most 2 % of padding
                int ks14 = 1;
                const int wgs14 = fill(14, p->row_words, &ks14);
                if (wgs14 >= wgs && wgs14 >= 192) {
                    p->k_splits = ks14;
                    p->build_waves = 2;
                }
            }
        }
        return;
    }
    // 512-row blocks for large matrices with up to three codebooks, 256-row blocks (more, shorter
    // K ranges; twice the registers per lane) otherwise -- from plan sweeps on the Llama-3 shapes
    p->waves = (code_positions >= 16e6 && p->batch_group * m <= 4) ? 16 : 8;
    p->row_words = (p->batch_group * m <= (p->waves == 8 ? 8 : 4)) ? 2 : 1;
    // K ranges: as many as give close to, but not more than, 256 workgroups (one per compute
    // unit).  When K is too short for that with 2 row words, blocks of half the height double
    // the workgroups (plan sweeps: 1024-output shapes -0.3 us).
    auto ranges = [&](int row_words, int* workgroups) {
        const int nblk = ceil_div(ngr * kGranuleRows, row_words * p->waves * 16);
        int nks = 256 / nblk;
        if (nks > nkt) nks = nkt;
        if (nks < 1) nks = 1;
        nks = ceil_div(nkt, ceil_div(nkt, nks));          // no empty K range
        *workgroups = nblk * nks;
        return nks;
    };
    int wgs = 0;
    p->k_splits = ranges(p->row_words, &wgs);
    // 448-row blocks (14 wavefronts) when they fill more of the 256 compute units: heights of
    // 7 * 2^k rows (the Llama up/gate projections) divide into 224 workgroups of 512 rows but
    // into 256 of 448.  Measured at 8192->28672: -2 % to -5 % for one and three codebooks and with
    // group scales; with two or four codebooks and one scale per row a tie or a loss (+0.1 us),
    // because the 8m MFMA blocks of a Psumbook then divide evenly over 16 wavefronts and not over 14.
    // With one or two codebooks the 448 rows go to 14 of 16 wavefronts and the other two build
    // every Psumbook, one unit ahead (build_waves = 2), when a workgroup has at least four units
    // to stream: 8192->28672 v8 m1 10.0 -> 9.8 us, v4 m1 15.3 -> 14.0, v4 m1 g128 19.3 -> 17.0,
    // m2v8g128 15.6 -> 15.2 against the 14-wavefront shape (two codebooks, one scale per row: 14.5 both).
    if (p->waves == 16 && p->row_words == 2 && ((m & 1) || d->group_size > 0)) {
        p->waves = 14;
        int wgs14 = 0;
        const int nks14 = ranges(2, &wgs14);
        if (wgs14 > wgs && wgs >= 192) {
            p->k_splits = nks14;
            if (m <= 2 && ceil_div(nkt, nks14) >= 4) {
                p->waves = 16;
                p->build_waves = 2;
            }
            return;
        }
        p->waves = 16;
    }
    if (p->row_words == 2 && wgs <= 128) {
        int wgs1 = 0;
        const int nks1 = ranges(1, &wgs1);
        if (wgs1 > wgs) {
            p->row_words = 1;
            p->k_splits = nks1;
        }
    }
}

int make_geometry(const codegemm_desc* d, const codegemm_plan* plan, Geometry* g)
{
    int st = validate_desc(d);
    if (st) return st;
    codegemm_plan local;
    if (!plan) {
        choose_plan(d, &local);
        plan = &local;
    }
    st = validate_plan(d, plan);
    if (st) return st;
    g->B = d->batch < kBatchPerLaunch ? d->batch : kBatchPerLaunch;   // larger batches run as several launches
    g->K = d->in_features;
    g->N = d->out_features;
    g->v = d->vec_len;
    g->m = d->num_codebooks;
    g->J = g->K / g->v;
    g->NW = plan->waves;
    g->NB = plan->build_waves;
    g->RPL = plan->row_words;
    g->BG = plan->batch_group;
    g->psum_fp16 = plan->psum_dtype == CODEGEMM_PSUM_FP16;
    g->NGR = ceil_div(g->N, kGranuleRows);
    // rows per workgroup: 16 per wavefront and row word (32 in the batched kernel)
    g->NBLK = ceil_div(g->NGR * kGranuleRows, g->RPL * (g->NW - g->NB) * (g->BG == 4 ? 32 : 16));
    g->NKT = ceil_div(g->J, kSlots);
    int nks = plan->k_splits < g->NKT ? plan->k_splits : g->NKT;
    g->KPW = ceil_div(g->NKT, nks);
    g->NKS = ceil_div(g->NKT, g->KPW);          // no empty K range
    g->NG = ceil_div(g->B, g->BG);
    g->Npad = g->NGR * kGranuleRows;
    if (counter_stride(*g) == 0) return CODEGEMM_UNSUPPORTED;   // > 16384 row blocks x batch groups with several K ranges
    g->y_fp32 = (d->flags & CODEGEMM_FLAG_Y_FP32) != 0;
    g->g = d->group_size;
    g->GPU = 0;
    g->gshift = 0;
    if (g->g > 0) {
        const int ratio = g->g / g->v;                 // sub-vectors per group, a power of two
        g->GPU = ratio >= kSlots ? 1 : kSlots / ratio;
        while ((1 << g->gshift) < ratio && g->gshift < 5) ++g->gshift;
    }
    return CODEGEMM_OK;
}

size_t workspace_counter_bytes(const Geometry&)
{
    return (size_t)kCounterAreaWords * sizeof(uint32_t) + kPairAreaBytes;
}

size_t pair_words(const Geometry& g)
{
    // Measured per level: one add that returns, on every output of the launch at once, takes 0.8-0.9 us, the ticket
    // protocol 1.9 us whatever the number of ranges: two ranges gain 0.95 us, four 0.2 us, eight lose 0.35 us.
    // The batched kernel, with four times the outputs per workgroup, takes it for two ranges (8192->28672, batch 8:
    // 54.1 -> 53.1 us).
    if (g.NKS != 2 && (g.NKS != 4 || g.BG == 4)) return 0;
    return (size_t)g.B * (g.NKS - 1) * g.Npad;
}

int counter_stride(const Geometry& g)
{
    if (g.NKS == 1) return kCounterStride;             // no counter is touched
    const long long blocks = (long long)g.NG * g.NBLK;
    int stride = kCounterStride;
    while (stride > 1 && blocks * stride > kCounterAreaWords) stride /= 2;
    return blocks * stride <= kCounterAreaWords ? stride : 0;
}

}  // namespace cg

using namespace cg;

extern "C" int codegemm_default_plan(const codegemm_desc* desc, codegemm_plan* plan)
{
    if (!plan) return CODEGEMM_INVALID_ARG;
    int st = validate_desc(desc);
    if (st) return st;
    choose_plan(desc, plan);
    return validate_plan(desc, plan);
}

extern "C" size_t codegemm_workspace_bytes(const codegemm_desc* desc, const codegemm_plan* plan)
{
    Geometry g;
    if (make_geometry(desc, plan, &g)) return 0;
    size_t bytes = workspace_counter_bytes(g) + (size_t)g.B * g.NKS * g.Npad * sizeof(float);
    if (desc->batch > kBatchPerLaunch && desc->batch % kBatchPerLaunch) {
        // the last launch of a large batch has fewer rows and, under the default plan, other K ranges
        codegemm_desc tail = *desc;
        tail.batch = desc->batch % kBatchPerLaunch;
        if (make_geometry(&tail, plan, &g)) return 0;
        const size_t b2 = workspace_counter_bytes(g) + (size_t)g.B * g.NKS * g.Npad * sizeof(float);
        if (b2 > bytes) bytes = b2;
    }
    return bytes;
}

extern "C" size_t codegemm_packed_codes_bytes(const codegemm_desc* desc, const codegemm_plan* plan)
{
    Geometry g;
    if (make_geometry(desc, plan, &g)) return 0;
    return (size_t)g.NGR * g.NKT * kGranuleRows * kSlots * g.m;
}

extern "C" size_t codegemm_packed_scales_bytes(const codegemm_desc* desc)
{
    Geometry g;
    if (make_geometry(desc, nullptr, &g) || g.g <= 0) return 0;
    return (size_t)g.NGR * g.NKT * g.GPU * 256;
}

extern "C" const char* codegemm_status_string(int status)
{
    switch (status) {
        case CODEGEMM_OK: return "ok";
        case CODEGEMM_INVALID_ARG: return "invalid argument";
        case CODEGEMM_UNSUPPORTED: return "unsupported format, batch or plan";
        case CODEGEMM_WORKSPACE_TOO_SMALL: return "workspace too small";
        case CODEGEMM_LAUNCH_FAILED: return "HIP launch failed";
        default: return "unknown status";
    }
}
