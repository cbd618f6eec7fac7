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
// weight-gradient side, inputs for the input-gradient side).  A centre's position in the side's order is its
// slot; slots are the centre indices themselves, or, in a plan built with PCPP_PLAN_SPATIAL, positions along a
// space-filling curve (perm[slot] = centre index).
//   perm      int32  [n_centres]           (spatial plans only) centre index of each slot
//   tile_ptr  uint32 [K * n_tiles + 1]     start of the (cell k, tile) run in the side's triplet
//                                          order, k-major; last entry = |T|
//   run_start uint32 [n_tiles][K][TILE]    start of the (cell k, slot tile*TILE + a) run; it ends where
//                                          the next slot's run starts (for a = TILE-1: at the end of
//                                          the (k, tile) run)
//   gather    int32  [|T|]                 source row of each triplet in (k, slot, source) order, bit 31 set on
//                                          the last triplet of a (k, slot) run.  The input-gradient side always has
//                                          one; the forward side has one in spatial plans and otherwise gathers
//                                          through tri_i.  These arrays follow everything else, one after the
//                                          other, each align_up(|T| * 4) bytes: `gather_index` counts them.
struct SideLayout {
    int64_t n_centres = 0;
    int64_t n_tiles = 0;
    size_t perm_off = 0;
    size_t tile_ptr_off = 0;
    size_t run_start_off = 0;
    int gather_index = -1;       // position among the |T|-sized arrays, -1: none
    size_t gather_off = 0;       // = tail_off + gather_index * align_up(n_triplets * 4)
};

struct PlanLayout {
    SideLayout fwd;   // valid if flags & PCPP_PLAN_FWD
    SideLayout bwd;   // valid if flags & PCPP_PLAN_BWD_INPUT
    size_t tail_off = 0;    // start of the |T|-sized arrays
    int n_tail = 0;         // how many there are
    size_t bytes = 0;
};

constexpr int PLAN_FLAG_MASK = PCPP_PLAN_FWD | PCPP_PLAN_BWD_INPUT | PCPP_PLAN_SPATIAL;
constexpr uint32_t GATHER_LAST = 0x80000000u;     // flag on the last triplet of a run in a plan's gather array
constexpr uint32_t GATHER_INDEX = 0x7fffffffu;

PlanLayout plan_layout(int64_t n_in, int64_t n_out, int K, int64_t n_triplets, int flags);

struct PlanSideView {
    const uint32_t *tile_ptr;
    const uint32_t *run_start;
    const int32_t *gather;     // NULL when the side gathers through tri_i
    const int32_t *perm;       // NULL when slots are centre indices
    int64_t n_tiles;
};

// Raise a kernel's dynamic LDS limit to `bytes` (once per kernel and device; later calls with no more are free).
int raise_lds_limit(const void *kernel, size_t bytes);

// ---- spatial order of a point set (spatial_order.hip) ----------------------------------------
// perm[slot] = index of the point at that position along a Morton curve of cells of pitch `pitch`.
// scratch: spatial_order_scratch_bytes(n) bytes, 256-byte aligned; scan_status: SPATIAL_ORDER_SCANS consecutive
// regions of scan_scratch_bytes(spatial_order_scan_items(n)) bytes, all zero when the call starts.
constexpr int SPATIAL_ORDER_SCANS = 3;
size_t spatial_order_scratch_bytes(int64_t n);
int64_t spatial_order_scan_items(int64_t n);
int spatial_order(const float *xyz, int64_t n, double pitch, int32_t *perm, void *scratch, void *scan_status,
                  size_t scan_stride, uint32_t *err, hipStream_t stream);

// ---- device-wide exclusive scan of uint32 (scan.hip) ------------------------------------------
// out[i] = sum_{j<i} in[j] for i in [0, n]; out has n+1 entries (out may alias in when it has
// room for n+1).  scratch: scan_scratch_bytes(n) bytes that are all zero when the scan starts (it
// leaves them non-zero: zero them again before the next scan, or give every scan its own).
// total64 (device, optional) receives the 64-bit total.
size_t scan_scratch_bytes(int64_t n);
// err (device, optional): set to 1 if a wait inside the scan ran out (the results are then undefined);
// when it is already set the last block stores ~0 as the total.
int scan_exclusive_u32(const uint32_t *in, uint32_t *out, int64_t n, void *scratch,
                       unsigned long long *total64, uint32_t *err, hipStream_t stream);
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
// wide layers with producer and consumer waves (mvmr_rows_pc.hip); needs a plan side with its own gather array
bool mvmr_rows_pc_usable(const MvmrArgs &a);
int mvmr_rows_pc_pack_w(const void *w, void *packed, int K, int c_src, int c_dst, int stride_d, int stride_s,
                        hipStream_t stream);
int mvmr_rows_pc(const MvmrArgs &a, hipStream_t stream);   // a.w = weights packed by mvmr_rows_pc_pack_w
int transpose_w(const void *w, void *wt, int K, int c_out, int c_in, int dtype, hipStream_t stream);
int mvmr_weight_generic(const MvmrArgs &a, float *dw, void *workspace, size_t workspace_bytes,
                        hipStream_t stream);
size_t mvmr_weight_workspace_bytes(int64_t n_centres, int c_in, int c_out, int K);
int mvmr_weight_mfma(const MvmrArgs &a, float *dw, const int32_t *tri_o, const int64_t *seg_offsets, void *workspace,
                     size_t workspace_bytes, hipStream_t stream, bool *handled);
size_t mvmr_weight_mfma_workspace_bytes(int64_t n_triplets, int c_in, int c_out, int K, int in_dtype);

}  // namespace pcpp
