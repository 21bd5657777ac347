// C entry point of the hot path: validation, plan -> kernel instance, launch.
#include <mutex>
#include <utility>
#include <vector>

#include "gemm_batch_impl.h"

namespace cg {

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
    // The gather kernels form absolute LDS addresses with the Psumbook at offset 0 of the
    // workgroup's allocation: a kernel that also had static LDS would have its dynamic part moved.
    hipFuncAttributes attr;
    if (hipFuncGetAttributes(&attr, fn) != hipSuccess) return CODEGEMM_LAUNCH_FAILED;
    if (attr.sharedSizeBytes != 0) return CODEGEMM_UNSUPPORTED;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess)
        return CODEGEMM_LAUNCH_FAILED;
    done.emplace_back(fn, dev);
    return CODEGEMM_OK;
}

}  // namespace cg

using namespace cg;

// Workspace of codegemm_gemm_static: one array per GPU, held by the loaded library until
// the process ends.  In host code the array's name only stands for the symbol; its device
// address is looked up once per device and used from then on.
constexpr size_t kStaticWorkspaceBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device; on first use there, the ticket
// counters at its start are cleared on `stream` (a fill kernel), ahead of the caller's launch.
int static_workspace(void** out, hipStream_t stream)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CODEGEMM_LAUNCH_FAILED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CODEGEMM_LAUNCH_FAILED;
        const int st = codegemm_workspace_init(ptr, (size_t)kCounterAreaWords * sizeof(uint32_t) + kPairAreaBytes, stream);
        if (st) return st;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CODEGEMM_OK;
}
}  // namespace

#ifdef CODEGEMM_TRACE
#include "codegemm_trace.h"
static uint64_t* g_trace = nullptr;
extern "C" void codegemm_set_trace(uint64_t* stamps) { g_trace = stamps; }
#endif

// Kernel instance for a geometry -> launch.  g.NBLK is the number of row blocks of all members of p.
static int dispatch(const Geometry& g, const GemmParams& p, hipStream_t s)
{
    if (g.BG == 4) {
        switch (g.m) {
            case 1: return g.g > 0 ? launch_gemm_batch_gs_m1(g, p, s) : launch_gemm_batch_m1(g, p, s);
            case 2: return g.g > 0 ? launch_gemm_batch_gs_m2(g, p, s) : launch_gemm_batch_m2(g, p, s);
            case 3: return g.g > 0 ? launch_gemm_batch_gs_m3(g, p, s) : launch_gemm_batch_m3(g, p, s);
            case 4: return g.g > 0 ? launch_gemm_batch_gs_m4(g, p, s) : launch_gemm_batch_m4(g, p, s);
        }
        return CODEGEMM_UNSUPPORTED;
    }
    if (g.psum_fp16) {
        switch (g.m) {
            case 1: return g.g > 0 ? launch_gemm_h_gs_m1(g, p, s) : launch_gemm_h_m1(g, p, s);
            case 2: return g.g > 0 ? launch_gemm_h_gs_m2(g, p, s) : launch_gemm_h_m2(g, p, s);
            case 3: return g.g > 0 ? launch_gemm_h_gs_m3(g, p, s) : launch_gemm_h_m3(g, p, s);
            case 4: return g.g > 0 ? launch_gemm_h_gs_m4(g, p, s) : launch_gemm_h_m4(g, p, s);
        }
        return CODEGEMM_UNSUPPORTED;
    }
    if (g.g > 0) {
        switch (g.m) {
            case 1: return launch_gemm_gs_m1(g, p, s);
            case 2: return launch_gemm_gs_m2(g, p, s);
            case 3: return launch_gemm_gs_m3(g, p, s);
            case 4: return launch_gemm_gs_m4(g, p, s);
        }
        return CODEGEMM_UNSUPPORTED;
    }
    switch (g.m) {
        case 1: return launch_gemm_m1(g, p, s);
        case 2: return launch_gemm_m2(g, p, s);
        case 3: return launch_gemm_m3(g, p, s);
        case 4: return launch_gemm_m4(g, p, s);
    }
    return CODEGEMM_UNSUPPORTED;
}

// The fields of the kernel arguments that all members of a launch share.
static void fill_common(GemmParams* p, const Geometry& g, const void* x, void* workspace)
{
    p->x = static_cast<const _Float16*>(x);
    p->GPU = g.GPU;
    p->gshift = g.gshift;
    p->counters = static_cast<uint32_t*>(workspace);
    p->cstride = counter_stride(g);
    p->B = g.B; p->K = g.K;
    p->NKT = g.NKT; p->NKS = g.NKS; p->KPW = g.KPW;
    p->y_fp32 = g.y_fp32 ? 1 : 0;
    p->trace = nullptr;
#ifdef CODEGEMM_TRACE
    p->trace = reinterpret_cast<unsigned long long*>(g_trace);
#endif
    p->ngrp = 1;
    for (int i = 0; i < kMaxGroup; ++i) p->mem[i] = Member{};
}

static void fill_member(Member* mm, const Geometry& g, const uint8_t* packed_codes, const void* codebooks,
                        const void* scales, void* y, float* partials, unsigned long long* pairs, int blk0)
{
    mm->pairs = pairs;
    mm->packed = packed_codes;
    mm->codebooks = static_cast<const _Float16*>(codebooks);
    mm->scales = g.g > 0 ? nullptr : static_cast<const _Float16*>(scales);
    mm->gscales = g.g > 0 ? static_cast<const uint8_t*>(scales) : nullptr;
    mm->y = y;
    mm->partials = partials;
    mm->N = g.N; mm->NGR = g.NGR; mm->Npad = g.Npad;
    mm->blk0 = blk0;
}

// One launch: at most kBatchPerLaunch batch rows.
static int gemm_launch(const codegemm_desc* desc, const codegemm_plan* plan, const void* x,
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
    const size_t need = cbytes + (size_t)g.B * g.NKS * g.Npad * sizeof(float);
    if (workspace_bytes < need) return CODEGEMM_WORKSPACE_TOO_SMALL;

    GemmParams p;
    fill_common(&p, g, x, workspace);
    // the pairwise reduction where its words fit into their area, else ticket and partials
    unsigned long long* pairs = reinterpret_cast<unsigned long long*>(static_cast<unsigned char*>(workspace) + (size_t)kCounterAreaWords * sizeof(uint32_t));
    const size_t pw = pair_words(g);
    if (pw == 0 || pw * 8 > kPairAreaBytes) pairs = nullptr;
    fill_member(&p.mem[0], g, packed_codes, codebooks, scales, y,
                reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + cbytes), pairs, 0);
    return dispatch(g, p, static_cast<hipStream_t>(stream));
}

extern "C" int codegemm_gemm(const codegemm_desc* desc, const codegemm_plan* plan, const void* x,
                             const uint8_t* packed_codes, const void* codebooks, const void* scales,
                             void* y, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!desc || desc->batch <= kBatchPerLaunch)
        return gemm_launch(desc, plan, x, packed_codes, codebooks, scales, y, workspace, workspace_bytes, stream);
    // A larger batch runs as consecutive launches of up to kBatchPerLaunch rows on the same
    // stream, sharing the workspace (launches on one stream do not overlap).  Row offsets of
    // x and y are multiples of 64 bytes, so the alignment of the pointers carries over.
    Geometry g;
    int st = make_geometry(desc, plan, &g);
    if (st) return st;
    if (!x || !y) return CODEGEMM_INVALID_ARG;
    const size_t ysize = g.y_fp32 ? sizeof(float) : sizeof(_Float16);
    for (int b0 = 0; b0 < desc->batch; b0 += kBatchPerLaunch) {
        codegemm_desc part = *desc;
        part.batch = desc->batch - b0 < kBatchPerLaunch ? desc->batch - b0 : kBatchPerLaunch;
        st = gemm_launch(&part, plan, static_cast<const unsigned char*>(x) + (size_t)b0 * g.K * sizeof(_Float16),
                         packed_codes, codebooks, scales, static_cast<unsigned char*>(y) + (size_t)b0 * g.N * ysize,
                         workspace, workspace_bytes, stream);
        if (st) return st;
    }
    return CODEGEMM_OK;
}

extern "C" size_t codegemm_static_workspace_limit(void) { return kStaticWorkspaceBytes; }

extern "C" int codegemm_gemm_static(const codegemm_desc* desc, const codegemm_plan* plan, const void* x,
                                    const uint8_t* packed_codes, const void* codebooks, const void* scales,
                                    void* y, void* stream)
{
    const size_t need = codegemm_workspace_bytes(desc, plan);
    if (need == 0) {
        Geometry g;
        const int st = make_geometry(desc, plan, &g);
        return st ? st : CODEGEMM_INVALID_ARG;
    }
    if (need > kStaticWorkspaceBytes) return CODEGEMM_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    const int st = static_workspace(&ws, static_cast<hipStream_t>(stream));
    if (st) return st;
    return codegemm_gemm(desc, plan, x, packed_codes, codebooks, scales, y, ws, kStaticWorkspaceBytes, stream);
}

// ---- several layers that share x in one launch ----------------------------------------------

// Geometry of the members of a group under one plan, and the geometry of the whole launch (row
// blocks summed).  The plan has to suit every member, and a launch takes at most kBatchPerLaunch rows.
static int group_geometry(const codegemm_desc* desc, const codegemm_plan* plan, const int32_t* out_features,
                          int count, Geometry* members, Geometry* whole)
{
    if (!desc || !out_features) return CODEGEMM_INVALID_ARG;
    if (count < 1 || count > kMaxGroup) return CODEGEMM_INVALID_ARG;
    if (desc->batch > kBatchPerLaunch) return CODEGEMM_UNSUPPORTED;
    codegemm_plan of_sum;
    if (!plan) {   // the default plan of one layer of the summed height, for every member
        const int st = codegemm_default_plan(desc, &of_sum);
        if (st) return st;
        plan = &of_sum;
    }
    long long total = 0;
    for (int i = 0; i < count; ++i) {
        codegemm_desc d = *desc;
        d.out_features = out_features[i];
        const int st = make_geometry(&d, plan, &members[i]);
        if (st) return st;
        total += out_features[i];
    }
    if (total != desc->out_features) return CODEGEMM_INVALID_ARG;
    *whole = members[0];
    whole->N = (int)total;
    whole->NBLK = 0; whole->NGR = 0; whole->Npad = 0;
    for (int i = 0; i < count; ++i) {
        whole->NBLK += members[i].NBLK;
        whole->NGR += members[i].NGR;
        whole->Npad += members[i].Npad;
    }
    if (whole->NBLK > 65535 || counter_stride(*whole) == 0) return CODEGEMM_UNSUPPORTED;
    return CODEGEMM_OK;
}

extern "C" size_t codegemm_grouped_workspace_bytes(const codegemm_desc* desc, const codegemm_plan* plan,
                                                   const int32_t* out_features, int32_t count)
{
    Geometry members[kMaxGroup], whole;
    if (group_geometry(desc, plan, out_features, count, members, &whole)) return 0;
    return workspace_counter_bytes(whole) + (size_t)whole.B * whole.NKS * whole.Npad * sizeof(float);
}

extern "C" int codegemm_gemm_grouped(const codegemm_desc* desc, const codegemm_plan* plan, const void* x,
                                     const codegemm_group_member* group, int32_t count,
                                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!group || count < 1 || count > kMaxGroup) return CODEGEMM_INVALID_ARG;
    int32_t out_features[kMaxGroup];
    for (int i = 0; i < count; ++i) out_features[i] = group[i].out_features;
    Geometry members[kMaxGroup], whole;
    int st = group_geometry(desc, plan, out_features, count, members, &whole);
    if (st) return st;
    if (!x || !workspace || misaligned(x) || misaligned(workspace)) return CODEGEMM_INVALID_ARG;
    for (int i = 0; i < count; ++i) {
        const codegemm_group_member& gm = group[i];
        if (!gm.packed_codes || !gm.codebooks || !gm.scales || !gm.y) return CODEGEMM_INVALID_ARG;
        if (misaligned(gm.packed_codes) || misaligned(gm.codebooks) || misaligned(gm.scales) || misaligned(gm.y))
            return CODEGEMM_INVALID_ARG;
    }
    const size_t cbytes = workspace_counter_bytes(whole);
    const size_t need = cbytes + (size_t)whole.B * whole.NKS * whole.Npad * sizeof(float);
    if (workspace_bytes < need) return CODEGEMM_WORKSPACE_TOO_SMALL;

    GemmParams p;
    fill_common(&p, whole, x, workspace);
    p.ngrp = count;
    float* partials = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + cbytes);
    unsigned long long* pairs = reinterpret_cast<unsigned long long*>(static_cast<unsigned char*>(workspace) + (size_t)kCounterAreaWords * sizeof(uint32_t));
    const size_t pw = pair_words(whole);               // whole.Npad is the sum over the members
    if (pw == 0 || pw * 8 > kPairAreaBytes) pairs = nullptr;
    int blk0 = 0;
    for (int i = 0; i < count; ++i) {
        fill_member(&p.mem[i], members[i], group[i].packed_codes, group[i].codebooks, group[i].scales,
                    group[i].y, partials, pairs, blk0);
        if (pairs) pairs += pair_words(members[i]);
        partials += (size_t)whole.B * whole.NKS * members[i].Npad;
        blk0 += members[i].NBLK;
    }
    return dispatch(whole, p, static_cast<hipStream_t>(stream));
}
