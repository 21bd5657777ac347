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

static int validate_plan(const codegemm_desc* d, const codegemm_plan* p)
{
    const int m = d->num_codebooks;
    if (p->slots != 32 && p->slots != 64) return CODEGEMM_UNSUPPORTED;
    if (p->waves != 8 && p->waves != 16) return CODEGEMM_UNSUPPORTED;
    if (p->slots == 64 && m > 2) return CODEGEMM_UNSUPPORTED;                 // Psumbook would exceed LDS
    if ((p->slots / p->waves) * m > 8) return CODEGEMM_UNSUPPORTED;           // code ring must fit in registers
    if (p->k_splits < 1) return CODEGEMM_UNSUPPORTED;
    if (p->batch_group != 1 && p->batch_group != 2 && p->batch_group != 4) return CODEGEMM_UNSUPPORTED;
    for (int i = 0; i < 4; ++i)
        if (p->reserved[i]) return CODEGEMM_INVALID_ARG;
    return CODEGEMM_OK;
}

// Library's own choice.  One workgroup per compute unit is resident (its two Psumbook
// buffers take 128 KB of LDS), so the K ranges are cut to give close to, but not more
// than, 256 workgroups, each streaming a contiguous run of units.
static void choose_plan(const codegemm_desc* d, codegemm_plan* p)
{
    *p = codegemm_plan{};
    const int m = d->num_codebooks;
    const int J = d->in_features / d->vec_len;
    p->slots = (m == 1) ? 64 : 32;
    p->waves = 16;
    const int nrb = ceil_div(d->out_features, kBlockRows);
    const int nkt = ceil_div(J, p->slots);
    int nks = 256 / nrb;
    if (nks < 1) nks = 1;
    if (nks > nkt) nks = nkt;
    const int kpw = ceil_div(nkt, nks);
    p->k_splits = ceil_div(nkt, kpw);             // no empty K range
    p->batch_group = d->batch == 1 ? 1 : (d->batch == 2 ? 2 : 4);
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
    g->NW = plan->waves;
    g->BG = plan->batch_group;
    g->NRB = ceil_div(g->N, kBlockRows);
    g->NKT = ceil_div(g->J, g->S);
    int nks = plan->k_splits < g->NKT ? plan->k_splits : g->NKT;
    g->KPW = ceil_div(g->NKT, nks);
    g->NKS = ceil_div(g->NKT, g->KPW);          // no empty K range
    g->NG = ceil_div(g->B, g->BG);
    g->Npad = g->NRB * kBlockRows;
    g->y_fp32 = (d->flags & CODEGEMM_FLAG_Y_FP32) != 0;
    return CODEGEMM_OK;
}

size_t workspace_counter_bytes(const Geometry& g)
{
    return ((size_t)g.NG * g.NRB * sizeof(uint32_t) + 255) & ~(size_t)255;
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
    return workspace_counter_bytes(g) + (size_t)g.B * g.NKS * g.Npad * sizeof(float);
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
