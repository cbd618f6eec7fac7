// Choice of the plan's centre order by measurement (Sec. 3.3.2 ends with the remark that, for configurations the
// analysis does not cover, the order in which the triplets are processed can be selected by auto-tuning before the
// massive executions).  The public triplet arrays are always in (k, o, i) order; what can differ is which centres
// share a tile of the plan: index order or a Z-order curve (PCPP_PLAN_SPATIAL).  pcpp_tune_plan_order builds both
// plans for the caller's cloud and layer shape, times the forward pass (and the input gradient when asked for) on
// each, and reports the faster one.  Features and weights are zeros: none of the kernels' timing depends on values.
#include "pcpp_internal.h"

namespace pcpp {

namespace {

constexpr int TUNE_REPS = 3;

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

struct TuneLayout {
    size_t tri_o, tri_i, tri_k, seg, plan, plan_bytes, build_ws, build_ws_bytes, src, w, dst, mvmr_ws, mvmr_ws_bytes, bytes;
};

TuneLayout tune_layout(int64_t n_in, int64_t n_out, int t, int64_t n_t, int c_in, int c_out, int dtype, int ops)
{
    const int K = t * t * t;
    const size_t s = dtype == PCPP_BF16 ? 2 : 4;
    TuneLayout l{};
    size_t at = 0;
    auto take = [&](size_t b) { const size_t o = at; at += align256(b); return o; };
    const size_t cap = (size_t)(n_t > 0 ? n_t : 1);
    l.tri_o = take(cap * 4); l.tri_i = take(cap * 4); l.tri_k = take(cap * 4);
    l.seg = take((size_t)(K + 1) * 8);
    const size_t pa = pcpp_plan_bytes(n_in, n_out, t, n_t, ops), pb = pcpp_plan_bytes(n_in, n_out, t, n_t, ops | PCPP_PLAN_SPATIAL);
    l.plan_bytes = pa > pb ? pa : pb;
    l.plan = take(l.plan_bytes);
    l.build_ws_bytes = pcpp_build_triplets_workspace_bytes_for(n_in, n_out, t, n_t);
    l.build_ws = take(l.build_ws_bytes);
    const size_t rows_a = (size_t)n_in * c_in, rows_b = (size_t)n_out * c_out;
    l.src = take((rows_a > rows_b ? rows_a : rows_b) * s);
    l.w = take((size_t)K * c_in * c_out * s);
    l.dst = take((rows_a > rows_b ? rows_a : rows_b) * 4);
    const size_t wa = pcpp_mvmr_workspace_bytes(0, n_in, n_out, n_t, c_in, c_out, K, dtype);
    const size_t wb = pcpp_mvmr_workspace_bytes(1, n_in, n_out, n_t, c_in, c_out, K, dtype);
    l.mvmr_ws_bytes = wa > wb ? wa : wb;
    l.mvmr_ws = take(l.mvmr_ws_bytes);
    l.bytes = at;
    return l;
}

__global__ void tune_zero(uint32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

int fail(int code, const char *msg)
{
    set_error("%s", msg);
    return code;
}

struct Events {
    hipEvent_t a = nullptr, b = nullptr;
    ~Events()
    {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

}  // namespace

}  // namespace pcpp

using namespace pcpp;

extern "C" {

PCPP_API size_t pcpp_tune_workspace_bytes(int64_t n_in, int64_t n_out, int t, int64_t n_triplets, int c_in, int c_out,
                                          int in_dtype, int ops)
{
    if (n_in < 0 || n_out < 0 || t < 1 || t > PCPP_MAX_T || n_triplets < 0 || c_in < 1 || c_out < 1) return 0;
    return tune_layout(n_in, n_out, t, n_triplets, c_in, c_out, in_dtype, ops).bytes;
}

PCPP_API int pcpp_tune_plan_order(const float *in_xyz, int64_t n_in, const float *out_xyz, int64_t n_out, float radius,
                                  int t, int build_flags, int64_t n_triplets, int c_in, int c_out, int in_dtype, int ops,
                                  void *workspace, size_t workspace_bytes, int *best_plan_flags, float *ms_index_order,
                                  float *ms_spatial_order, void *stream_)
{
    if (!best_plan_flags) return fail(PCPP_ERR_INVALID_ARG, "pcpp_tune_plan_order: best_plan_flags is NULL");
    if ((ops & ~(PCPP_PLAN_FWD | PCPP_PLAN_BWD_INPUT)) || !(ops & PCPP_PLAN_FWD))
        return fail(PCPP_ERR_INVALID_ARG, "pcpp_tune_plan_order: ops must be PCPP_PLAN_FWD, optionally with PCPP_PLAN_BWD_INPUT");
    if (build_flags & ~PCPP_BUILD_VOXEL)
        return fail(PCPP_ERR_INVALID_ARG, "pcpp_tune_plan_order: build_flags may hold PCPP_BUILD_VOXEL only");
    if (in_dtype != PCPP_F32 && in_dtype != PCPP_BF16)
        return fail(PCPP_ERR_INVALID_ARG, "pcpp_tune_plan_order: unknown dtype");
    if (n_in < 0 || n_out < 0 || t < 1 || t > PCPP_MAX_T || n_triplets < 0 || c_in < 1 || c_out < 1)
        return fail(PCPP_ERR_INVALID_ARG, "pcpp_tune_plan_order: bad sizes");
    const TuneLayout l = tune_layout(n_in, n_out, t, n_triplets, c_in, c_out, in_dtype, ops);
    if (!workspace || workspace_bytes < l.bytes || (reinterpret_cast<uintptr_t>(workspace) & 255))
        return fail(PCPP_ERR_WORKSPACE, "pcpp_tune_plan_order: workspace missing, misaligned or smaller than pcpp_tune_workspace_bytes");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int K = t * t * t;
    char *ws = static_cast<char *>(workspace);
    int32_t *tri_o = reinterpret_cast<int32_t *>(ws + l.tri_o), *tri_i = reinterpret_cast<int32_t *>(ws + l.tri_i),
            *tri_k = reinterpret_cast<int32_t *>(ws + l.tri_k);
    int64_t *seg = reinterpret_cast<int64_t *>(ws + l.seg);
    // zeros for the features, the weights and nothing else (the destination is overwritten)
    const size_t zero_words = (l.dst - l.src) / 4;
    tune_zero<<<1024, 256, 0, stream>>>(reinterpret_cast<uint32_t *>(ws + l.src), zero_words);
    PCPP_HIP_CHECK(hipGetLastError());
    Events ev;
    PCPP_HIP_CHECK(hipEventCreate(&ev.a));
    PCPP_HIP_CHECK(hipEventCreate(&ev.b));
    float ms[2] = {0.f, 0.f};
    for (int v = 0; v < 2; ++v) {
        const int flags = ops | (v ? PCPP_PLAN_SPATIAL : 0);
        int64_t n_t = 0;
        int rc = pcpp_build_triplets(in_xyz, n_in, out_xyz, n_out, radius, t, tri_o, tri_i, tri_k, n_triplets, seg, &n_t,
                                     ws + l.plan, l.plan_bytes, flags | build_flags, ws + l.build_ws, l.build_ws_bytes, stream);
        if (rc != PCPP_OK) return rc;
        if (n_t != n_triplets)
            return fail(PCPP_ERR_INVALID_ARG, "pcpp_tune_plan_order: n_triplets is not the number of triplets of this cloud");
        const size_t plan_bytes = pcpp_plan_bytes(n_in, n_out, t, n_t, flags);
        auto pass = [&]() -> int {
            int r = pcpp_mvmr_fwd(ws + l.src, ws + l.w, ws + l.dst, in_dtype, PCPP_F32, n_in, n_out, c_in, c_out, K, tri_o, tri_i,
                                  tri_k, seg, n_t, ws + l.plan, plan_bytes, flags, ws + l.mvmr_ws, l.mvmr_ws_bytes, stream);
            if (r == PCPP_OK && (ops & PCPP_PLAN_BWD_INPUT))
                r = pcpp_mvmr_bwd_input(ws + l.src, ws + l.w, ws + l.dst, in_dtype, PCPP_F32, n_in, n_out, c_in, c_out, K, tri_o,
                                        tri_i, tri_k, seg, n_t, ws + l.plan, plan_bytes, flags, ws + l.mvmr_ws,
                                        l.mvmr_ws_bytes, stream);
            return r;
        };
        if ((rc = pass()) != PCPP_OK) return rc;                 // warm-up
        PCPP_HIP_CHECK(hipEventRecord(ev.a, stream));
        for (int r = 0; r < TUNE_REPS; ++r)
            if ((rc = pass()) != PCPP_OK) return rc;
        PCPP_HIP_CHECK(hipEventRecord(ev.b, stream));
        PCPP_HIP_CHECK(hipEventSynchronize(ev.b));
        PCPP_HIP_CHECK(hipEventElapsedTime(&ms[v], ev.a, ev.b));
        ms[v] /= TUNE_REPS;
    }
    if (ms_index_order) *ms_index_order = ms[0];
    if (ms_spatial_order) *ms_spatial_order = ms[1];
    *best_plan_flags = ops | (ms[1] < ms[0] ? PCPP_PLAN_SPATIAL : 0);
    return PCPP_OK;
}

}  // extern "C"
