// C ABI entry points of the three MVMR compute calls: argument checks and dispatch.
// (pcpp_build_triplets lives in build_triplets.hip.)
#include <stdarg.h>
#include <stdio.h>

#include <mutex>
#include <vector>

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

// Kernels that need more dynamic LDS than the default limit have the limit raised once per device; the table only
// remembers what has already been asked for, so that the attribute call is not repeated on every launch.
int raise_lds_limit(const void *kernel, size_t bytes)
{
    struct Entry { const void *kernel; int device; size_t bytes; };
    static std::mutex mu;
    static std::vector<Entry> done;
    int dev = 0;
    PCPP_HIP_CHECK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    for (Entry &e : done)
        if (e.kernel == kernel && e.device == dev) {
            if (e.bytes >= bytes) return PCPP_OK;
            PCPP_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
            e.bytes = bytes;
            return PCPP_OK;
        }
    PCPP_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    done.push_back(Entry{kernel, dev, bytes});
    return PCPP_OK;
}

namespace {

int check_common(const char *fn, const void *a, const void *b, const void *c, int in_dtype, int out_dtype,
                 int64_t n_in, int64_t n_out, int c_in, int c_out, int K, const int32_t *tri_o,
                 const int32_t *tri_i, const int32_t *tri_k, const int64_t *seg_offsets, int64_t n_triplets,
                 const void *plan, size_t plan_bytes, int plan_flags, int need_flags)
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
    if ((plan_flags & ~PLAN_FLAG_MASK) || (plan_flags & need_flags) != need_flags) {
        set_error("%s: plan_flags 0x%x lack the part this call reads (0x%x) or hold unknown bits", fn, plan_flags,
                  need_flags);
        return PCPP_ERR_INVALID_ARG;
    }
    int t = 1;
    while (t * t * t < K) ++t;
    if (t * t * t != K) {
        set_error("%s: K must be a cube", fn);
        return PCPP_ERR_INVALID_ARG;
    }
    const size_t need = plan_layout(n_in, n_out, K, n_triplets, plan_flags).bytes;
    if (plan_bytes < need) {
        set_error("%s: plan buffer has %zu bytes, these sizes and flags need %zu", fn, plan_bytes, need);
        return PCPP_ERR_WORKSPACE;
    }
    return PCPP_OK;
}

PlanSideView side_view(const void *plan, const SideLayout &s, bool spatial)
{
    const char *pb = static_cast<const char *>(plan);
    PlanSideView v;
    v.tile_ptr = reinterpret_cast<const uint32_t *>(pb + s.tile_ptr_off);
    v.run_start = reinterpret_cast<const uint32_t *>(pb + s.run_start_off);
    v.gather = s.gather_index >= 0 ? reinterpret_cast<const int32_t *>(pb + s.gather_off) : nullptr;
    v.perm = spatial ? reinterpret_cast<const int32_t *>(pb + s.perm_off) : nullptr;
    v.n_tiles = s.n_tiles;
    return v;
}

// Device memory that the entry point which allocates nothing uses in place of a caller's workspace (packed
// weights).  One copy per device, held until the process ends; calls that overlap on one device would race on it.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)24 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mu;
void *scratch_ptr[MAX_DEVICES];      // the array's address on each device, once asked for

int static_scratch(void **out)
{
    int dev = 0;
    PCPP_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) {
        set_error("pcpp_mvmr_fwd_static: device index %d out of range", dev);
        return PCPP_ERR_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        PCPP_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return PCPP_OK;
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
                  size_t plan_bytes, int plan_flags, void *workspace, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = check_common("pcpp_mvmr_fwd", x, w, out, in_dtype, out_dtype, n_in, n_out, c_in, c_out, K, tri_o, tri_i,
                          tri_k, seg_offsets, n_triplets, plan, plan_bytes, plan_flags, PCPP_PLAN_FWD);
    if (rc != PCPP_OK) return rc;
    if (n_out == 0) return PCPP_OK;
    const bool spatial = (plan_flags & PCPP_PLAN_SPATIAL) != 0;
    const PlanLayout pl = plan_layout(n_in, n_out, K, n_triplets, plan_flags);
    MvmrArgs a{};
    a.feat = x; a.w = w; a.dst = out; a.dense = nullptr;
    a.in_dtype = in_dtype; a.out_dtype = out_dtype;
    a.n_src = n_in; a.n_centres = n_out; a.c_src = c_in; a.c_dst = c_out; a.K = K;
    a.side = side_view(plan, pl.fwd, spatial); a.gather = a.side.gather ? a.side.gather : tri_i;
    a.n_triplets = n_triplets;
    const bool pc = mvmr_rows_pc_usable(a);
    if (pc || mvmr_rows_sel_supported(a)) {
        const size_t need = pcpp_mvmr_workspace_bytes(0, n_in, n_out, n_triplets, c_in, c_out, K, in_dtype);
        if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
            set_error("pcpp_mvmr_fwd: workspace missing, misaligned or smaller than %zu bytes", need);
            return PCPP_ERR_WORKSPACE;
        }
        if (pc) {
            if ((rc = mvmr_rows_pc_pack_w(w, workspace, K, c_in, c_out, c_in, 1, stream)) != PCPP_OK) return rc;
            a.w = workspace;
            return mvmr_rows_pc(a, stream);
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
                        size_t plan_bytes, int plan_flags, void *workspace, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = check_common("pcpp_mvmr_bwd_input", dy, w, dx, in_dtype, out_dtype, n_in, n_out, c_in, c_out, K, tri_o,
                          tri_i, tri_k, seg_offsets, n_triplets, plan, plan_bytes, plan_flags,
                          PCPP_PLAN_FWD | PCPP_PLAN_BWD_INPUT);
    if (rc != PCPP_OK) return rc;
    const size_t need = pcpp_mvmr_workspace_bytes(1, n_in, n_out, n_triplets, c_in, c_out, K, in_dtype);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
        set_error("pcpp_mvmr_bwd_input: workspace missing, misaligned or smaller than %zu bytes", need);
        return PCPP_ERR_WORKSPACE;
    }
    if (n_in == 0) return PCPP_OK;
    const PlanLayout pl = plan_layout(n_in, n_out, K, n_triplets, plan_flags);
    MvmrArgs a{};
    a.feat = dy; a.w = workspace; a.dst = dx; a.dense = nullptr;
    a.in_dtype = in_dtype; a.out_dtype = out_dtype;
    a.n_src = n_out; a.n_centres = n_in; a.c_src = c_out; a.c_dst = c_in; a.K = K;
    a.side = side_view(plan, pl.bwd, (plan_flags & PCPP_PLAN_SPATIAL) != 0); a.gather = a.side.gather;
    a.n_triplets = n_triplets;
    // W[k] is [c_out][c_in]; the rows kernel wants (dst = c_in, src = c_out) = W[k]^T
    if (mvmr_rows_pc_usable(a)) {
        if ((rc = mvmr_rows_pc_pack_w(w, workspace, K, c_out, c_in, 1, c_in, stream)) != PCPP_OK) return rc;
        return mvmr_rows_pc(a, stream);
    }
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
                         size_t plan_bytes, int plan_flags, void *workspace, size_t workspace_bytes, void *stream_)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = check_common("pcpp_mvmr_bwd_weight", x, dw, dy, in_dtype, PCPP_F32, n_in, n_out, c_in, c_out, K, tri_o,
                          tri_i, tri_k, seg_offsets, n_triplets, plan, plan_bytes, plan_flags, PCPP_PLAN_FWD);
    if (rc != PCPP_OK) return rc;
    const size_t need = pcpp_mvmr_workspace_bytes(2, n_in, n_out, n_triplets, c_in, c_out, K, in_dtype);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255)) {
        set_error("pcpp_mvmr_bwd_weight: workspace missing, misaligned or smaller than %zu bytes", need);
        return PCPP_ERR_WORKSPACE;
    }
    const PlanLayout pl = plan_layout(n_in, n_out, K, n_triplets, plan_flags);
    MvmrArgs a{};
    a.feat = x; a.w = nullptr; a.dst = nullptr; a.dense = dy;
    a.in_dtype = in_dtype; a.out_dtype = PCPP_F32;
    a.n_src = n_in; a.n_centres = n_out; a.c_src = c_in; a.c_dst = c_out; a.K = K;
    a.side = side_view(plan, pl.fwd, (plan_flags & PCPP_PLAN_SPATIAL) != 0); a.gather = a.side.gather ? a.side.gather : tri_i;
    a.n_triplets = n_triplets;
    bool handled = false;
    if (n_triplets == 0) return fill_u32(reinterpret_cast<uint32_t *>(dw), 0u, (int64_t)K * c_out * c_in, stream);
    MvmrArgs am = a;
    am.gather = tri_i;                               // the matrix-core kernels walk the public (k, o, i) list
    rc = mvmr_weight_mfma(am, dw, tri_o, seg_offsets, workspace, workspace_bytes, stream, &handled);
    if (rc != PCPP_OK || handled) return rc;
    return mvmr_weight_generic(a, dw, workspace, workspace_bytes, stream);
}

size_t pcpp_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int pcpp_mvmr_fwd_static(const void *x, const void *w, void *out, int in_dtype, int out_dtype, int64_t n_in,
                         int64_t n_out, int c_in, int c_out, int K, const int32_t *tri_o, const int32_t *tri_i,
                         const int32_t *tri_k, const int64_t *seg_offsets, int64_t n_triplets, const void *plan,
                         size_t plan_bytes, int plan_flags, void *stream_)
{
    const size_t need = pcpp_mvmr_workspace_bytes(0, n_in, n_out, n_triplets, c_in, c_out, K, in_dtype);
    if (need > STATIC_SCRATCH_BYTES) {
        set_error("pcpp_mvmr_fwd_static: the packed weights need %zu bytes, the library's own scratch holds %zu", need,
                  STATIC_SCRATCH_BYTES);
        return PCPP_ERR_UNSUPPORTED;
    }
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != PCPP_OK) return rc;
    return pcpp_mvmr_fwd(x, w, out, in_dtype, out_dtype, n_in, n_out, c_in, c_out, K, tri_o, tri_i, tri_k, seg_offsets,
                         n_triplets, plan, plan_bytes, plan_flags, ws, STATIC_SCRATCH_BYTES, stream_);
}

}  // extern "C"
