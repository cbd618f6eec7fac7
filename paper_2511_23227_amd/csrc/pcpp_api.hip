// C ABI entry points of the three MVMR compute calls: argument checks and dispatch.
// (pcpp_build_triplets lives in build_triplets.hip.)
#include <stdarg.h>
#include <stdio.h>

#include "pcpp_internal.h"

namespace pcpp {

static thread_local char g_error[512] = "no error";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

namespace {

size_t elem_size(int dtype) { return dtype == PCPP_F32 ? 4 : 2; }

int check_common(const char *fn, const void *a, const void *b, const void *c, int in_dtype, int out_dtype,
                 int64_t n_in, int64_t n_out, int c_in, int c_out, int K, const int32_t *tri_o,
                 const int32_t *tri_i, const int32_t *tri_k, const int64_t *seg_offsets, int64_t n_triplets,
                 const void *plan)
{
    if (n_in < 0 || n_out < 0 || n_triplets < 0 || K < 1) {
        set_error("%s: negative size or K < 1", fn);
        return PCPP_ERR_INVALID_ARG;
    }
    if ((n_in > 0 && n_out > 0 && (!a || !c)) || !b) {
        set_error("%s: null tensor pointer", fn);
        return PCPP_ERR_INVALID_ARG;
    }
    if (n_triplets > 0 && (!tri_o || !tri_i || !tri_k || !seg_offsets)) {
        set_error("%s: null triplet arrays", fn);
        return PCPP_ERR_INVALID_ARG;
    }
    if (!plan) {
        set_error("%s: plan is NULL (build it with pcpp_build_triplets)", fn);
        return PCPP_ERR_INVALID_ARG;
    }
    if ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c)) & 15) {
        set_error("%s: tensors must be 16-byte aligned", fn);
        return PCPP_ERR_INVALID_ARG;
    }
    if (reinterpret_cast<uintptr_t>(plan) & 255) {
        set_error("%s: plan must be 256-byte aligned", fn);
        return PCPP_ERR_INVALID_ARG;
    }
    if (K > MAX_K || c_in < 1 || c_out < 1 || c_in > 1024 || c_out > 1024) {
        set_error("%s: K must be <= %d and channel counts in 1..1024", fn, MAX_K);
        return PCPP_ERR_UNSUPPORTED;
    }
    if ((in_dtype != PCPP_F32 && in_dtype != PCPP_BF16) || (out_dtype != PCPP_F32 && out_dtype != PCPP_BF16) ||
        (in_dtype == PCPP_F32 && out_dtype == PCPP_BF16)) {
        set_error("%s: unsupported dtype combination in=%d out=%d", fn, in_dtype, out_dtype);
        return PCPP_ERR_UNSUPPORTED;
    }
    if (n_in >= INT32_MAX || n_out >= INT32_MAX || n_triplets >= INT32_MAX) {
        set_error("%s: sizes must be below 2^31", fn);
        return PCPP_ERR_UNSUPPORTED;
    }
    return PCPP_OK;
}

// t from K = t^3 (the plan layout is keyed on it)
int cube_root(int K)
{
    for (int t = 1; t <= PCPP_MAX_T; ++t)
        if (t * t * t == K) return t;
    return -1;
}

PlanSideView side_view(const void *plan, const SideLayout &s)
{
    const char *pb = static_cast<const char *>(plan);
    PlanSideView v;
    v.tile_ptr = reinterpret_cast<const uint32_t *>(pb + s.tile_ptr_off);
    v.run_start = reinterpret_cast<const uint32_t *>(pb + s.run_start_off);
    v.gather = reinterpret_cast<const int32_t *>(pb + s.gather_off);
    v.n_tiles = s.n_tiles;
    return v;
}

}  // namespace
}  // namespace pcpp

using namespace pcpp;

extern "C" {

const char *pcpp_last_error(void) { return g_error; }

int pcpp_version(void) { return 100; }

size_t pcpp_mvmr_workspace_bytes(int op, int64_t n_in, int64_t n_out, int64_t n_triplets, int c_in, int c_out, int K,
                                 int in_dtype)
{
    if (n_in < 0 || n_out < 0 || n_triplets < 0 || c_in < 1 || c_out < 1 || K < 1) return 0;
    switch (op) {
    case 0:                                                                     // W in fragment order
    case 1: return align_up((size_t)K * c_out * c_in * (in_dtype == PCPP_F32 ? 6 : 2));   // W / W^T in fragment order (fp32: up to three bf16 terms)
    case 2: {                                                                   // partial dW per range of centres
        const size_t g = mvmr_weight_workspace_bytes(n_out, c_in, c_out, K);
        const size_t m = mvmr_weight_mfma_workspace_bytes(n_triplets, c_in, c_out, K, in_dtype);
        return g > m ? g : m;
    }
    default: return 0;
    }
}

int pcpp_mvmr_fwd(const void *x, const void *w, void *out, int in_dtype, int out_dtype, int64_t n_in,
                  int64_t n_out, int c_in, int c_out, int K, const int32_t *tri_o, const int32_t *tri_i,
                  const int32_t *tri_k, const int64_t *seg_offsets, int64_t n_triplets, const void *plan,
                  void *workspace, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = check_common("pcpp_mvmr_fwd", x, w, out, in_dtype, out_dtype, n_in, n_out, c_in, c_out, K, tri_o, tri_i,
                          tri_k, seg_offsets, n_triplets, plan);
    if (rc != PCPP_OK) return rc;
    const int t = cube_root(K);
    if (t < 0) { set_error("pcpp_mvmr_fwd: K must be a cube"); return PCPP_ERR_INVALID_ARG; }
    if (n_out == 0) return PCPP_OK;
    // the forward side of the plan is laid out first whenever it is present, whatever else was requested
    const PlanLayout pl = plan_layout(n_in, n_out, K, n_triplets, PCPP_PLAN_FWD);
    MvmrArgs a{};
    a.feat = x; a.w = w; a.dst = out; a.dense = nullptr;
    a.in_dtype = in_dtype; a.out_dtype = out_dtype;
    a.n_src = n_in; a.n_centres = n_out; a.c_src = c_in; a.c_dst = c_out; a.K = K;
    a.gather = tri_i; a.side = side_view(plan, pl.fwd); a.n_triplets = n_triplets;
    if (mvmr_rows_sel_supported(a)) {
        const size_t need = pcpp_mvmr_workspace_bytes(0, n_in, n_out, n_triplets, c_in, c_out, K, in_dtype);
        if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
            set_error("pcpp_mvmr_fwd: workspace missing, misaligned or smaller than %zu bytes", need);
            return PCPP_ERR_WORKSPACE;
        }
        if ((rc = mvmr_rows_sel_pack_w(w, workspace, K, c_in, c_out, c_in, 1, in_dtype, stream)) != PCPP_OK) return rc;
        a.w = workspace;
        return mvmr_rows_sel(a, stream);
    }
    return mvmr_rows_generic(a, stream);
}

int pcpp_mvmr_bwd_input(const void *dy, const void *w, void *dx, int in_dtype, int out_dtype, int64_t n_in,
                        int64_t n_out, int c_in, int c_out, int K, const int32_t *tri_o, const int32_t *tri_i,
                        const int32_t *tri_k, const int64_t *seg_offsets, int64_t n_triplets, const void *plan,
                        void *workspace, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = check_common("pcpp_mvmr_bwd_input", dy, w, dx, in_dtype, out_dtype, n_in, n_out, c_in, c_out, K, tri_o,
                          tri_i, tri_k, seg_offsets, n_triplets, plan);
    if (rc != PCPP_OK) return rc;
    const int t = cube_root(K);
    if (t < 0) { set_error("pcpp_mvmr_bwd_input: K must be a cube"); return PCPP_ERR_INVALID_ARG; }
    const size_t need = pcpp_mvmr_workspace_bytes(1, n_in, n_out, n_triplets, c_in, c_out, K, in_dtype);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
        set_error("pcpp_mvmr_bwd_input: workspace missing, misaligned or smaller than %zu bytes", need);
        return PCPP_ERR_WORKSPACE;
    }
    if (n_in == 0) return PCPP_OK;
    const PlanLayout pl = plan_layout(n_in, n_out, K, n_triplets, PCPP_PLAN_FWD | PCPP_PLAN_BWD_INPUT);
    MvmrArgs a{};
    a.feat = dy; a.w = workspace; a.dst = dx; a.dense = nullptr;
    a.in_dtype = in_dtype; a.out_dtype = out_dtype;
    a.n_src = n_out; a.n_centres = n_in; a.c_src = c_out; a.c_dst = c_in; a.K = K;
    a.side = side_view(plan, pl.bwd); a.gather = a.side.gather; a.n_triplets = n_triplets;
    // W[k] is [c_out][c_in]; the rows kernel wants (dst = c_in, src = c_out) = W[k]^T
    if (mvmr_rows_sel_supported(a)) {
        if ((rc = mvmr_rows_sel_pack_w(w, workspace, K, c_out, c_in, 1, c_in, in_dtype, stream)) != PCPP_OK) return rc;
        return mvmr_rows_sel(a, stream);
    }
    if ((rc = transpose_w(w, workspace, K, c_out, c_in, in_dtype, stream)) != PCPP_OK) return rc;
    return mvmr_rows_generic(a, stream);
}

int pcpp_mvmr_bwd_weight(const void *x, const void *dy, float *dw, int in_dtype, int64_t n_in, int64_t n_out,
                         int c_in, int c_out, int K, const int32_t *tri_o, const int32_t *tri_i,
                         const int32_t *tri_k, const int64_t *seg_offsets, int64_t n_triplets, const void *plan,
                         void *workspace, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = check_common("pcpp_mvmr_bwd_weight", x, dw, dy, in_dtype, PCPP_F32, n_in, n_out, c_in, c_out, K, tri_o,
                          tri_i, tri_k, seg_offsets, n_triplets, plan);
    if (rc != PCPP_OK) return rc;
    const int t = cube_root(K);
    if (t < 0) { set_error("pcpp_mvmr_bwd_weight: K must be a cube"); return PCPP_ERR_INVALID_ARG; }
    const size_t need = pcpp_mvmr_workspace_bytes(2, n_in, n_out, n_triplets, c_in, c_out, K, in_dtype);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
        set_error("pcpp_mvmr_bwd_weight: workspace missing, misaligned or smaller than %zu bytes", need);
        return PCPP_ERR_WORKSPACE;
    }
    const PlanLayout pl = plan_layout(n_in, n_out, K, n_triplets, PCPP_PLAN_FWD);
    MvmrArgs a{};
    a.feat = x; a.w = nullptr; a.dst = nullptr; a.dense = dy;
    a.in_dtype = in_dtype; a.out_dtype = PCPP_F32;
    a.n_src = n_in; a.n_centres = n_out; a.c_src = c_in; a.c_dst = c_out; a.K = K;
    a.gather = tri_i; a.side = side_view(plan, pl.fwd); a.n_triplets = n_triplets;
    bool handled = false;
    if (n_triplets == 0) return fill_u32(reinterpret_cast<uint32_t *>(dw), 0u, (int64_t)K * c_out * c_in, stream);
    rc = mvmr_weight_mfma(a, dw, tri_o, seg_offsets, workspace, workspace_bytes, stream, &handled);
    if (rc != PCPP_OK || handled) return rc;
    return mvmr_weight_generic(a, dw, workspace, workspace_bytes, stream);
}

}  // extern "C"
