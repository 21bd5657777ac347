// Host-side logic: argument validation, launch plan, buffer sizes, status strings.
#include "cg_common.h"

namespace cg {

static int validate_desc(const codegemm_desc* d)
{
    if (!d) return CODEGEMM_INVALID_ARG;
    if (d->batch < 1 || d->in_features < 1 || d->out_features < 1) return CODEGEMM_INVALID_ARG;
    if (d->vec_len != 4 && d->vec_len != 8) return CODEGEMM_UNSUPPORTED;
    if (d->num_codebooks < 1 || d->num_codebooks > 4) return CODEGEMM_UNSUPPORTED;
    if (d->code_bits != 8 || d->group_size != -1) return CODEGEMM_UNSUPPORTED;
    if (d->batch > 32) return CODEGEMM_UNSUPPORTED;
    if (d->in_features % d->vec_len) return CODEGEMM_INVALID_ARG;
    if (d->flags & ~CODEGEMM_FLAG_Y_FP32) return CODEGEMM_INVALID_ARG;
    return CODEGEMM_OK;
}

static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

static int validate_plan(const codegemm_desc* d, const codegemm_plan* p)
{
    if (p->slots != 32 && p->slots != 64) return CODEGEMM_UNSUPPORTED;
    if (!pow2(p->row_waves) || !pow2(p->k_waves)) return CODEGEMM_UNSUPPORTED;
    if (p->row_waves * p->k_waves > 16) return CODEGEMM_UNSUPPORTED;
    if (p->slots % p->k_waves) return CODEGEMM_UNSUPPORTED;
    const int nstep = p->slots / p->k_waves;
    if (nstep != 4 && nstep != 8 && nstep != 16) return CODEGEMM_UNSUPPORTED;
    if (p->build != 0 && p->build != 1) return CODEGEMM_UNSUPPORTED;
    for (int i = 0; i < 4; ++i)
        if (p->reserved[i]) return CODEGEMM_INVALID_ARG;
    const size_t planes = (size_t)d->num_codebooks * kCentroids * p->slots * sizeof(float);
    const size_t staging = (size_t)d->num_codebooks * kCentroids * d->vec_len * 2 + (size_t)p->slots * d->vec_len * 2;
    if (planes + staging + 64 > (size_t)kMaxLds) return CODEGEMM_UNSUPPORTED;
    return CODEGEMM_OK;
}

// Library's own choice of tile shape.  A tile is 512*row_waves rows by `slots`
// sub-vectors.  The Psumbook is rebuilt once per tile, so tall tiles amortise the
// build; but the grid must still cover the 256 compute units, so the tile height
// is reduced until there are at least that many tiles.
static void choose_plan(const codegemm_desc* d, codegemm_plan* p)
{
    *p = codegemm_plan{};
    const int m = d->num_codebooks;
    const int J = d->in_features / d->vec_len;
    p->slots = (m <= 2) ? 64 : 32;
    const int nrb = ceil_div(d->out_features, kBlockRows);
    const int nkt = ceil_div(J, p->slots);
    int rw = 4;
    while (rw > 1 && (long)ceil_div(nrb, rw) * nkt < 224) rw >>= 1;
    p->row_waves = rw;
    int jw = 16 / rw;
    if (p->slots / jw < 4) jw = p->slots / 4;
    p->k_waves = jw;
    p->build = 0;
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
    g->B = d->batch;
    g->K = d->in_features;
    g->N = d->out_features;
    g->v = d->vec_len;
    g->m = d->num_codebooks;
    g->J = g->K / g->v;
    g->S = plan->slots;
    g->RW = plan->row_waves;
    g->JW = plan->k_waves;
    g->NSTEP = g->S / g->JW;
    g->NRB = ceil_div(g->N, kBlockRows);
    g->NKT = ceil_div(g->J, g->S);
    g->NRT = ceil_div(g->NRB, g->RW);
    g->Npad = g->NRB * kBlockRows;
    g->build = plan->build;
    g->y_fp32 = (d->flags & CODEGEMM_FLAG_Y_FP32) != 0;
    return CODEGEMM_OK;
}

size_t workspace_counter_bytes(const Geometry& g)
{
    return ((size_t)g.NRT * sizeof(uint32_t) + 255) & ~(size_t)255;
}

size_t lds_bytes_gemm(const Geometry& g)
{
    return (size_t)g.m * kCentroids * g.S * sizeof(float)      // Psumbook planes
           + (size_t)g.m * kCentroids * g.v * 2                // codebook staging (fp16)
           + (size_t)g.S * g.v * 2                             // x slice staging (fp16)
           + 64;                                               // flags
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
    return workspace_counter_bytes(g) + (size_t)g.B * g.NKT * g.Npad * sizeof(float);
}

extern "C" size_t codegemm_packed_codes_bytes(const codegemm_desc* desc, const codegemm_plan* plan)
{
    Geometry g;
    if (make_geometry(desc, plan, &g)) return 0;
    return (size_t)g.NRB * g.NKT * g.S * step_bytes(g.m);
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
