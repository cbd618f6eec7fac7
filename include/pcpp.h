/*
 * pcpp -- convolution on native points (PointCNN++) as MVMR, MI355X (gfx950) only.
 *
 * C ABI of libpcpp.so.  Plain pointers and sizes; every pointer is a DEVICE pointer unless the
 * comment says HOST.  The caller owns every buffer (inputs, outputs, plan, workspace).  The calls
 * below allocate no device or host memory and keep no data between calls; the only thing the
 * library remembers is, per kernel and device, that it has raised that kernel's dynamic LDS limit
 * (an idempotent attribute of the loaded code).  pcpp_build_triplets creates one event and destroys
 * it before it returns.
 *
 * Notation (paper -> here): output index i -> o, input index j -> i, kernel cell k;
 * t = kernel resolution per axis, K = t^3; T = the triplet set {(o, i, k)}.
 *
 * Conventions shared by all calls
 *   - return value: PCPP_OK or a negative PCPP_ERR_* code; pcpp_last_error() gives a message for
 *     the calling thread.  Nothing is printed, nothing throws.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls are asynchronous on it, except
 *     pcpp_build_triplets, which waits once for the triplet count.
 *   - outputs are overwritten, never accumulated into; rows without a triplet are zero.
 *   - indices are int32 (n_in, n_out, |T| < 2^31), segment offsets int64, coordinates fp32.
 *   - feature tensors are row-major, 16-byte aligned; dtype codes below.
 *   - feature tensors (x, dy, w) must hold finite values.  The matrix-core kernels form the sum of the
 *     source rows of a (cell, output) run as a product with a 0/1 selection matrix or stage it beside other
 *     rows, so an Inf or NaN in one source row can reach destination rows that have no triplet with it
 *     (within the same group of up to 128 consecutive centres).  Coordinates must be finite too.
 */
#ifndef PCPP_H_
#define PCPP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define PCPP_API __attribute__((visibility("default")))
#else
#define PCPP_API
#endif

#define PCPP_OK                 0
#define PCPP_ERR_INVALID_ARG   -1  /* null pointer, negative size, t < 1, bad radius, misaligned    */
#define PCPP_ERR_CAPACITY      -2  /* triplet buffers too small; *n_triplets holds the needed count */
#define PCPP_ERR_WORKSPACE     -3  /* workspace or plan buffer smaller than the matching *_bytes()  */
#define PCPP_ERR_UNSUPPORTED   -4  /* dtype / shape outside what the library handles                */
#define PCPP_ERR_HIP           -5  /* a HIP runtime call failed, or a device-side wait ran out      */

#define PCPP_F32   0   /* IEEE binary32                    */
#define PCPP_BF16  1   /* bfloat16, round-to-nearest-even  */

/* plan_flags: which parts of a plan pcpp_build_triplets writes, and how.  The same value must be passed
 * to every compute call that reads the plan. */
#define PCPP_PLAN_FWD        1   /* what pcpp_mvmr_fwd and pcpp_mvmr_bwd_weight read */
#define PCPP_PLAN_BWD_INPUT  2   /* what pcpp_mvmr_bwd_input reads (only together with PCPP_PLAN_FWD) */
#define PCPP_PLAN_SPATIAL    4   /* the plan groups the centres along a space-filling curve computed by the
                                    library instead of in index order: the centres a kernel block owns are then
                                    neighbours in space whatever the caller's point order, which wide layers need
                                    (they share source rows and weight slices through the caches).  The public
                                    triplet arrays, every result and every tolerance are unchanged; the build
                                    takes about a third longer. */
/* testing aids, accepted in plan_flags by pcpp_build_triplets only; results are identical with or without */
#define PCPP_BUILD_TEST_SHORT_LISTS  0x100  /* keep at most 40 neighbours of a centre on chip: longer lists take
                                               the path that ranks by scanning the candidates again          */
#define PCPP_BUILD_TEST_WIDE_KEYS    0x200  /* treat cell and index as too wide to share one 32-bit word, as for
                                               clouds of 2^24 points or more                                  */

#define PCPP_BUILD_VOXEL             0x400  /* accepted in plan_flags by pcpp_build_triplets[_batched]: build the triplets
                                               of the degraded operator of Sec. 3.2 ("Voxel Convolution as a Special
                                               Case"; "Ours (degraded)" in Sec. 4.2), i.e. sparse voxel convolution:
                                               `radius` is then the pitch v of a global voxelisation, t must be odd,
                                               voxel of a coordinate = floor((double)p / (double)v); input i is a
                                               neighbour of output o iff their voxels differ by at most h = (t-1)/2
                                               along every axis, and k = ((dx+h)*t + dy+h)*t + dz+h with (dx, dy, dz) the
                                               voxel offset input minus output.  Everything else (order of T, plan,
                                               compute calls) is unchanged. */

#define PCPP_MAX_T  6            /* K = t^3 <= 216 */

/* Message for the last error returned on the calling thread (never NULL). HOST. */
PCPP_API const char *pcpp_last_error(void);

/* Library version, major*100 + minor. */
PCPP_API int pcpp_version(void);

/* ---------------------------------------------------------------------------------------------
 * Triplet construction: Sec. 3.2 "Definition" with the fixed radius search of Sec. 4.1, followed
 * by the reordering of Sec. 3.3.2 (sort by kernel cell; here by (k, o, i)).
 *
 * (o, i, k) is in T iff |in_xyz[i] - out_xyz[o]|^2 <= r^2, the test being evaluated in binary64
 * on the binary32 coordinates as (dx*dx + dy*dy) + dz*dz <= (double)r*(double)r without fused
 * multiply-add.  k is the cell of d = in - out in the t x t x t grid tiling [-r, r]^3 around the
 * output point: c_a = clamp(floor((d_a + r) * (t / (2r))), 0, t-1), k = (c_x*t + c_y)*t + c_z.
 *
 * Outputs
 *   tri_o, tri_i, tri_k  [capacity] int32: T in ascending (k, o, i) order.  All three NULL =>
 *                        count only (capacity, seg_offsets and plan are ignored).
 *   seg_offsets          [K+1] int64: start of each cell's run; seg_offsets[K] = |T|.
 *   n_triplets           HOST int64: |T|, also set when PCPP_ERR_CAPACITY is returned.  If it points into
 *                        pinned host memory (hipHostMalloc) the device writes the count straight into it
 *                        and the second pass is queued without waiting for the host; with pageable memory
 *                        the call copies the count synchronously first (same results, the GPU idles for one
 *                        round trip).
 *   plan                 optional opaque buffer of pcpp_plan_bytes(...) bytes that the three
 *                        compute calls need: per-(cell, centre) neighbour runs and tile offsets
 *                        for the forward / weight-gradient pass (PCPP_PLAN_FWD) and the same
 *                        triplets regrouped by (k, i, o) for the input gradient
 *                        (PCPP_PLAN_BWD_INPUT).  plan_flags selects the parts; NULL => none.
 *   workspace            scratch of pcpp_build_triplets_workspace_bytes(...) bytes, 256-byte
 *                        aligned; contents are undefined afterwards.  With at least
 *                        pcpp_build_triplets_workspace_bytes_for(..., capacity) bytes the neighbours
 *                        found while counting are kept and the second pass does not search again
 *                        (same results, about a third less time); a plan in spatial order, which groups
 *                        the same neighbourhoods a second time, then regroups those lists instead of
 *                        searching twice.
 * in_xyz [n_in,3] and out_xyz [n_out,3] may alias (outputs at the inputs).
 * Errors: INVALID_ARG (null xyz with n > 0, radius not finite or <= 0, t outside 1..PCPP_MAX_T,
 * some but not all tri_* NULL, unknown flag bits), CAPACITY, WORKSPACE, UNSUPPORTED (|T| >= 2^31), HIP.
 * Non-finite coordinates are not supported (undefined triplets, no fault).
 * ------------------------------------------------------------------------------------------- */
PCPP_API size_t pcpp_build_triplets_workspace_bytes(int64_t n_in, int64_t n_out, int t);
PCPP_API size_t pcpp_build_triplets_workspace_bytes_for(int64_t n_in, int64_t n_out, int t, int64_t capacity);
PCPP_API size_t pcpp_plan_bytes(int64_t n_in, int64_t n_out, int t, int64_t n_triplets, int plan_flags);

PCPP_API int pcpp_build_triplets(const float *in_xyz, int64_t n_in,
                                 const float *out_xyz, int64_t n_out,
                                 float radius, int t,
                                 int32_t *tri_o, int32_t *tri_i, int32_t *tri_k, int64_t capacity,
                                 int64_t *seg_offsets,
                                 int64_t *n_triplets,
                                 void *plan, size_t plan_bytes, int plan_flags,
                                 void *workspace, size_t workspace_bytes,
                                 void *stream);

/* ---------------------------------------------------------------------------------------------
 * Triplet construction over a batch of clouds held as concatenated arrays plus offsets (the jagged batch
 * representation of Sec. 4.1, implementation details): cloud b owns inputs [in_batch_offsets[b],
 * in_batch_offsets[b+1]) and outputs [out_batch_offsets[b], out_batch_offsets[b+1]); a triplet pairs points of the same
 * cloud only, whatever their coordinates.  Both offset arrays are DEVICE int32 [n_batches + 1], ascending, first
 * entry 0, last entry n_in / n_out; both NULL (with n_batches = 1) is pcpp_build_triplets.  Triplet indices refer to
 * the concatenated arrays, so the compute calls take the whole batch as one cloud.  1 <= n_batches <= 65536.
 * Everything else as pcpp_build_triplets.
 * ------------------------------------------------------------------------------------------- */
PCPP_API int pcpp_build_triplets_batched(const float *in_xyz, int64_t n_in,
                                         const float *out_xyz, int64_t n_out,
                                         const int32_t *in_batch_offsets, const int32_t *out_batch_offsets,
                                         int n_batches,
                                         float radius, int t,
                                         int32_t *tri_o, int32_t *tri_i, int32_t *tri_k, int64_t capacity,
                                         int64_t *seg_offsets,
                                         int64_t *n_triplets,
                                         void *plan, size_t plan_bytes, int plan_flags,
                                         void *workspace, size_t workspace_bytes,
                                         void *stream);

/* ---------------------------------------------------------------------------------------------
 * Voxel-grid down-sampling that keeps original coordinates (Sec. 4.1, implementation details): the output points
 * of a strided layer.  For every occupied voxel of pitch `pitch` (voxel of a coordinate = floor((double)p /
 * (double)pitch)) the point with the lowest index is kept.
 *   kept    [n] int32 (room for all points): indices of the kept points, ascending
 *   n_kept  HOST int64: their number (pinned host memory is written by the device, as in pcpp_build_triplets)
 *   workspace: pcpp_voxel_subsample_workspace_bytes(n) bytes, 256-byte aligned
 * The call waits for its result.  A strided layer is then pcpp_build_triplets with out_xyz = the kept points'
 * coordinates; the up-sampling layer of a decoder is the same call with the roles of the two point sets swapped
 * (more outputs than inputs is an ordinary case).
 * Errors: INVALID_ARG, WORKSPACE, UNSUPPORTED (n >= 2^31), HIP.  Coordinates beyond 2^20 voxels from the origin fall
 * into the outermost voxel.
 * ------------------------------------------------------------------------------------------- */
PCPP_API size_t pcpp_voxel_subsample_workspace_bytes(int64_t n);
PCPP_API int pcpp_voxel_subsample(const float *xyz, int64_t n, float pitch, int32_t *kept, int64_t *n_kept,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * MVMR forward, Eq. (1) of Sec. 3.1.1:  out[o, :] = sum_{(o,i,k) in T} W[k] x[i, :].
 *   x   [n_in , c_in ]  in_dtype        w  [K, c_out, c_in] in_dtype (the paper's layout, Sec. 3.3.2)
 *   out [n_out, c_out]  out_dtype (PCPP_F32, or PCPP_BF16 when in_dtype is PCPP_BF16)
 * Products are accumulated in fp32.  tri_* / seg_offsets / plan must be exactly what one
 * pcpp_build_triplets call produced for these n_in, n_out, K with these plan_flags (which must include
 * PCPP_PLAN_FWD); anything else is undefined behaviour.  plan_bytes is the size of the plan buffer.
 * workspace: pcpp_mvmr_workspace_bytes(...) bytes, 256-byte aligned.
 * Errors: INVALID_ARG (also: plan_flags lack the part this call reads), WORKSPACE (also: plan_bytes smaller
 * than pcpp_plan_bytes for these sizes and flags), UNSUPPORTED (c_in or c_out < 1 or > 1024, dtype combination).
 * ------------------------------------------------------------------------------------------- */
PCPP_API size_t pcpp_mvmr_workspace_bytes(int op /*0 fwd, 1 bwd_input, 2 bwd_weight*/, int64_t n_in, int64_t n_out,
                                          int64_t n_triplets, int c_in, int c_out, int K, int in_dtype);

PCPP_API int pcpp_mvmr_fwd(const void *x, const void *w, void *out, int in_dtype, int out_dtype,
                           int64_t n_in, int64_t n_out, int c_in, int c_out, int K,
                           const int32_t *tri_o, const int32_t *tri_i, const int32_t *tri_k,
                           const int64_t *seg_offsets, int64_t n_triplets,
                           const void *plan, size_t plan_bytes, int plan_flags,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * MVMR backward w.r.t. the input features, first gradient equation of Sec. 3.3.3:
 *   dx[i, :] = sum_{(o,i,k) in T} W[k]^T dy[o, :].
 *   dy [n_out, c_out] in_dtype,  w [K, c_out, c_in] in_dtype,  dx [n_in, c_in] out_dtype.
 * Needs a plan built with PCPP_PLAN_BWD_INPUT.  Otherwise as pcpp_mvmr_fwd.
 * ------------------------------------------------------------------------------------------- */
PCPP_API int pcpp_mvmr_bwd_input(const void *dy, const void *w, void *dx, int in_dtype, int out_dtype,
                                 int64_t n_in, int64_t n_out, int c_in, int c_out, int K,
                                 const int32_t *tri_o, const int32_t *tri_i, const int32_t *tri_k,
                                 const int64_t *seg_offsets, int64_t n_triplets,
                                 const void *plan, size_t plan_bytes, int plan_flags,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Backward w.r.t. the weights (VVOR), Eq. (5) of Sec. 3.3.3:
 *   dw[k] = sum_{(o,i,k) in T} dy[o, :] (outer) x[i, :],   dw [K, c_out, c_in] always fp32.
 * Cells with no triplet get exact zeros.  Needs a plan built with PCPP_PLAN_FWD.
 * ------------------------------------------------------------------------------------------- */
PCPP_API int pcpp_mvmr_bwd_weight(const void *x, const void *dy, float *dw, int in_dtype,
                                  int64_t n_in, int64_t n_out, int c_in, int c_out, int K,
                                  const int32_t *tri_o, const int32_t *tri_i, const int32_t *tri_k,
                                  const int64_t *seg_offsets, int64_t n_triplets,
                                  const void *plan, size_t plan_bytes, int plan_flags,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * pcpp_mvmr_fwd for callers that cannot provide scratch memory or let the library allocate it: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same arguments
 * and same results as pcpp_mvmr_fwd without the workspace: the packed weights go to a device array of
 * pcpp_static_scratch_bytes() bytes (24 MiB) that is part of the loaded library, one copy per GPU, held until
 * the process ends.  The call allocates nothing and creates nothing.
 * Limits: K * c_out * c_in * (2 bytes for bf16, 6 for fp32) must fit that array, otherwise UNSUPPORTED is
 * returned and nothing is launched.  Every call on a GPU uses that GPU's one array, so two calls that overlap
 * in time on one GPU (different streams or threads) race; calls on one stream are ordered and safe.
 * ------------------------------------------------------------------------------------------- */
PCPP_API size_t pcpp_static_scratch_bytes(void);
PCPP_API int pcpp_mvmr_fwd_static(const void *x, const void *w, void *out, int in_dtype, int out_dtype,
                                  int64_t n_in, int64_t n_out, int c_in, int c_out, int K,
                                  const int32_t *tri_o, const int32_t *tri_i, const int32_t *tri_k,
                                  const int64_t *seg_offsets, int64_t n_triplets,
                                  const void *plan, size_t plan_bytes, int plan_flags, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Choice of the processing order by measurement.  Sec. 3.3.2 ends with the remark that for configurations outside
 * its analysis the order in which the triplets are processed can be selected by auto-tuning before the massive
 * executions.  Here the public arrays are always in (k, o, i) order; what can differ is which centres share a tile
 * of the plan: index order, or positions along a Z-order curve (PCPP_PLAN_SPATIAL).  The call builds both plans for
 * this cloud, times pcpp_mvmr_fwd (and pcpp_mvmr_bwd_input when ops holds PCPP_PLAN_BWD_INPUT) on zero-filled
 * features of this layer shape, three passes each after a warm-up, and reports
 *   best_plan_flags  HOST int: ops, with PCPP_PLAN_SPATIAL added when that order was faster
 *   ms_index_order, ms_spatial_order  HOST float, optional: the time of one pass in either order
 * n_triplets must be |T| of this cloud (from a counting call of pcpp_build_triplets); build_flags is 0 or
 * PCPP_BUILD_VOXEL; ops is PCPP_PLAN_FWD or PCPP_PLAN_FWD | PCPP_PLAN_BWD_INPUT.  workspace:
 * pcpp_tune_workspace_bytes(...) bytes (device, 256-byte aligned; room for the triplets, the larger plan, the build's
 * workspace and the layer's tensors).  The call waits for its result and creates two events for the timing; it is
 * meant to run once per layer configuration, not per step.
 * Errors: INVALID_ARG, WORKSPACE, and whatever the calls it makes return.
 * ------------------------------------------------------------------------------------------- */
PCPP_API size_t pcpp_tune_workspace_bytes(int64_t n_in, int64_t n_out, int t, int64_t n_triplets, int c_in, int c_out,
                                          int in_dtype, int ops);
PCPP_API int pcpp_tune_plan_order(const float *in_xyz, int64_t n_in, const float *out_xyz, int64_t n_out, float radius,
                                  int t, int build_flags, int64_t n_triplets, int c_in, int c_out, int in_dtype, int ops,
                                  void *workspace, size_t workspace_bytes, int *best_plan_flags, float *ms_index_order,
                                  float *ms_spatial_order, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PCPP_H_ */
