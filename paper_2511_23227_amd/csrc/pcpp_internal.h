// Internal declarations shared by the translation units of libpcpp.so (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pcpp.h"

namespace pcpp {

// Centres are processed in tiles of TILE consecutive indices; the per-(cell, centre) neighbour
// counts and the per-(cell, tile) offsets of a plan use this granularity.
constexpr int TILE = 64;
constexpr int MAX_K = PCPP_MAX_T * PCPP_MAX_T * PCPP_MAX_T;

void set_error(const char *fmt, ...);

#define PCPP_HIP_CHECK(expr)                                                              \
    do {                                                                                  \
        hipError_t e_ = (expr);                                                           \
        if (e_ != hipSuccess) {                                                           \
            ::pcpp::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_),      \
                              __FILE__, __LINE__);                                        \
            return PCPP_ERR_HIP;                                                          \
        }                                                                                 \
    } while (0)

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// One side of a plan: triplets grouped around `n_centres` centres (outputs for the forward /
// weight-gradient side, inputs for the input-gradient side).
//   tile_ptr  uint32 [K * n_tiles + 1]  start of the (cell k, tile) run in the side's triplet
//                                       order, k-major; last entry = |T|
//   run_start uint32 [n_tiles][K][TILE] start of the (cell k, centre tile*TILE + a) run; it ends where
//                                       the next centre's run starts (for a = TILE-1: at the end of
//                                       the (k, tile) run)
//   gather    int32  [|T|]              (input-gradient side only) output index of each triplet in
//                                       (k, i, o) order; the forward side gathers through tri_i
struct SideLayout {
    int64_t n_centres = 0;
    int64_t n_tiles = 0;
    size_t tile_ptr_off = 0;
    size_t run_start_off = 0;
    size_t gather_off = 0;
    size_t end = 0;
};

struct PlanLayout {
    SideLayout fwd;   // valid if flags & PCPP_PLAN_FWD
    SideLayout bwd;   // valid if flags & PCPP_PLAN_BWD_INPUT
    size_t bytes = 0;
};

PlanLayout plan_layout(int64_t n_in, int64_t n_out, int K, int64_t n_triplets, int flags);

struct PlanSideView {
    const uint32_t *tile_ptr;
    const uint32_t *run_start;
    const int32_t *gather;
    int64_t n_tiles;
};

// ---- device-wide exclusive scan of uint32 (scan.hip) ------------------------------------------
// out[i] = sum_{j<i} in[j] for i in [0, n]; out has n+1 entries (out may alias in when it has
// room for n+1).  scratch: scan_scratch_bytes(n) bytes that are all zero when the scan starts (it
// leaves them non-zero: zero them again before the next scan, or give every scan its own).
// total64 (device, optional) receives the 64-bit total.
size_t scan_scratch_bytes(int64_t n);
int scan_exclusive_u32(const uint32_t *in, uint32_t *out, int64_t n, void *scratch,
                       unsigned long long *total64, hipStream_t stream);
int fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t stream);
int fill_u64(unsigned long long *p, unsigned long long v, int64_t n, hipStream_t stream);

// ---- MVMR kernels (mvmr_generic.hip, mvmr_rows.hip, mvmr_weight.hip) -------------------------
struct MvmrArgs {
    const void *feat;        // gathered tensor: x (fwd, bwd_weight) or dy (bwd_input), [n_src, c_src]
    const void *w;           // fwd: W [K][c_dst][c_src];  bwd_input: W^T [K][c_dst][c_src] (already transposed)
    void *dst;               // [n_centres, c_dst]
    const void *dense;       // bwd_weight only: dy [n_centres, c_dense]
    int in_dtype, out_dtype;
    int64_t n_src, n_centres;
    int c_src, c_dst;
    int K;
    const int32_t *gather;   // source row of each triplet in the side's order
    PlanSideView side;
    int64_t n_triplets;
};

int mvmr_rows_generic(const MvmrArgs &a, hipStream_t stream);              // fwd and bwd_input
// rows kernels with both the run sums and the W product on the matrix cores (mvmr_rows.hip)
bool mvmr_rows_sel_supported(const MvmrArgs &a);
int mvmr_rows_sel_pack_w(const void *w, void *packed, int K, int c_src, int c_dst, int stride_d, int stride_s,
                         int dtype, hipStream_t stream);
int mvmr_rows_sel(const MvmrArgs &a, hipStream_t stream);   // a.w = weights packed by mvmr_rows_sel_pack_w
int transpose_w(const void *w, void *wt, int K, int c_out, int c_in, int dtype, hipStream_t stream);
int mvmr_weight_generic(const MvmrArgs &a, float *dw, void *workspace, size_t workspace_bytes,
                        hipStream_t stream);
size_t mvmr_weight_workspace_bytes(int64_t n_centres, int c_in, int c_out, int K);
int mvmr_weight_mfma(const MvmrArgs &a, float *dw, const int32_t *tri_o, const int64_t *seg_offsets, void *workspace,
                     size_t workspace_bytes, hipStream_t stream, bool *handled);
size_t mvmr_weight_mfma_workspace_bytes(int64_t n_triplets, int c_in, int c_out, int K, int in_dtype);

}  // namespace pcpp
