// Shape-generic MVMR kernels (any channel counts, fp32 or bf16 storage, fp32 accumulation).
// They are the fallback for shapes without a matrix-core kernel.
//
// All three operations start from the same step: for a cell k and a tile of TILE consecutive
// centres, the source rows of every (k, centre) run are summed on chip,
//     S_k[c] = sum_{(c, s, k) in T} feat[s]
// which is legal because Eq. (1) is linear: out[o] = sum_k W[k] (sum_{i in cell k of o} x[i]).
// Then
//   rows kernel   (Eq. (1) forward; Sec. 3.3.3 input gradient with W^T):  dst[c] += W[k] S_k[c]
//   weight kernel (Eq. (5)):                                            dW[k] += dense[c] (x) S_k[c]
// Every destination row is owned by one block and written once: no atomics, fixed summation order.
#include "pcpp_internal.h"

namespace pcpp {

namespace {

constexpr int THREADS = 256;
constexpr int CH = 64;             // channel chunk handled per block / per staging step
constexpr int XS_STRIDE = CH + 1;  // padded row stride of the on-chip tiles

__device__ inline float bf16_to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

__device__ inline uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T> __device__ inline float load_f(const T *p, size_t idx);
template <> __device__ inline float load_f<float>(const float *p, size_t idx) { return p[idx]; }
template <> __device__ inline float load_f<uint16_t>(const uint16_t *p, size_t idx) { return bf16_to_f32(p[idx]); }

// Start and length of each centre's run inside the (k, tile) run [run_begin, run_end), from the plan.
// Called by the whole block; the results are visible after the next __syncthreads().
__device__ inline void stage_runs(const PlanSideView &side, int K, int64_t tile, int k, uint32_t run_end,
                                  uint32_t *row_start, uint32_t *row_cnt)
{
    if (threadIdx.x < TILE) {
        const int lane = threadIdx.x;
        const uint32_t *rs = side.run_start + ((size_t)tile * K + k) * TILE;
        const uint32_t st = rs[lane];
        const uint32_t en = lane < TILE - 1 ? rs[lane + 1] : run_end;
        row_cnt[lane] = en - st;
        row_start[lane] = st;
    }
}

// S[r][c] for r < TILE, c in [c0, c0 + CH): thread (r = tid / 4, q = tid % 4) sums 16 channels.
template <typename T>
__device__ inline void presum_chunk(const T *__restrict__ feat, int c_src, int c0, const int32_t *__restrict__ gather,
                                    const uint32_t *row_start, const uint32_t *row_cnt, float *S)
{
    const int r = threadIdx.x >> 2, q = threadIdx.x & 3;
    float s[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) s[e] = 0.f;
    const uint32_t n = row_cnt[r], st = row_start[r];
    for (uint32_t j = 0; j < n; ++j) {
        const size_t row = (size_t)((uint32_t)gather[st + j] & GATHER_INDEX) * c_src;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int c = c0 + q * 16 + e;
            if (c < c_src) s[e] += load_f<T>(feat, row + c);
        }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) S[r * XS_STRIDE + q * 16 + e] = s[e];
}

// grid = (n_tiles, ceil(c_dst / CH)); each block owns TILE centres x CH destination channels
template <typename TIn, typename TOut>
__global__ __launch_bounds__(THREADS) void rows_kernel(const TIn *__restrict__ feat, const TIn *__restrict__ w,
                                                       TOut *__restrict__ dst, int64_t n_centres, int c_src, int c_dst,
                                                       int K, const int32_t *__restrict__ gather, PlanSideView side)
{
    __shared__ float S[TILE * XS_STRIDE];
    __shared__ uint32_t row_start[TILE], row_cnt[TILE];
    const int64_t tile = blockIdx.x;
    const int d0 = blockIdx.y * CH;
    const int rg = threadIdx.x >> 4, cg = threadIdx.x & 15;   // rows rg*4..+3, channels d0 + cg + 16 j
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k = 0; k < K; ++k) {
        const uint32_t a = side.tile_ptr[(size_t)k * side.n_tiles + tile];
        const uint32_t b = side.tile_ptr[(size_t)k * side.n_tiles + tile + 1];
        if (a == b) continue;                                  // block-uniform
        __syncthreads();
        stage_runs(side, K, tile, k, b, row_start, row_cnt);
        for (int c0 = 0; c0 < c_src; c0 += CH) {
            __syncthreads();
            presum_chunk<TIn>(feat, c_src, c0, gather, row_start, row_cnt, S);
            __syncthreads();
            const int cmax = c_src - c0 < CH ? c_src - c0 : CH;
            for (int c = 0; c < cmax; ++c) {
                float xv[4], wv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) xv[i] = S[(rg * 4 + i) * XS_STRIDE + c];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int co = d0 + cg + 16 * j;
                    wv[j] = co < c_dst ? load_f<TIn>(w, ((size_t)k * c_dst + co) * c_src + c0 + c) : 0.f;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] += xv[i] * wv[j];
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t slot = tile * TILE + rg * 4 + i;
        if (slot >= n_centres) continue;
        const int64_t row = side.perm ? (int64_t)side.perm[slot] : slot;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int co = d0 + cg + 16 * j;
            if (co >= c_dst) continue;
            if constexpr (sizeof(TOut) == 4) dst[(size_t)row * c_dst + co] = acc[i][j];
            else dst[(size_t)row * c_dst + co] = f32_to_bf16(acc[i][j]);
        }
    }
}

// grid = (K, n_ranges, chunks_out * chunks_in); each block owns one CH x CH block of dW[k] over a
// range of tiles and writes its partial sum to part[range][k][c_out][c_in]
template <typename T>
__global__ __launch_bounds__(THREADS) void weight_kernel(const T *__restrict__ feat, const T *__restrict__ dense,
                                                         float *__restrict__ part, int64_t n_centres, int c_in,
                                                         int c_out, int K, const int32_t *__restrict__ gather,
                                                         PlanSideView side, int tiles_per_range, int chunks_in)
{
    __shared__ float S[TILE * XS_STRIDE];      // summed source rows  [r][ci]
    __shared__ float D[TILE * XS_STRIDE];      // dense rows (dy)     [r][co]
    __shared__ uint32_t row_start[TILE], row_cnt[TILE];
    const int k = blockIdx.x;
    const int range = blockIdx.y;
    const int co0 = (blockIdx.z / chunks_in) * CH, ci0 = (blockIdx.z % chunks_in) * CH;
    const int og = threadIdx.x >> 4, ig = threadIdx.x & 15;   // co = co0 + og + 16 i, ci = ci0 + ig + 16 j
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    const int64_t t_begin = (int64_t)range * tiles_per_range;
    int64_t t_end = t_begin + tiles_per_range;
    if (t_end > side.n_tiles) t_end = side.n_tiles;
    for (int64_t tile = t_begin; tile < t_end; ++tile) {
        const uint32_t a = side.tile_ptr[(size_t)k * side.n_tiles + tile];
        const uint32_t b = side.tile_ptr[(size_t)k * side.n_tiles + tile + 1];
        if (a == b) continue;                                  // block-uniform
        __syncthreads();
        stage_runs(side, K, tile, k, b, row_start, row_cnt);
        __syncthreads();
        presum_chunk<T>(feat, c_in, ci0, gather, row_start, row_cnt, S);
        {
            const int r = threadIdx.x >> 2, q = threadIdx.x & 3;
            const int64_t slot = tile * TILE + r;
            const int64_t row = (slot < n_centres && side.perm) ? (int64_t)side.perm[slot] : slot;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int c = co0 + q * 16 + e;
                D[r * XS_STRIDE + q * 16 + e] =
                    (slot < n_centres && c < c_out) ? load_f<T>(dense, (size_t)row * c_out + c) : 0.f;
            }
        }
        __syncthreads();
        for (int r = 0; r < TILE; ++r) {
            float dv[4], sv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) dv[i] = D[r * XS_STRIDE + og + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) sv[j] = S[r * XS_STRIDE + ig + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += dv[i] * sv[j];
        }
    }
    float *dstp = part + ((size_t)range * K + k) * c_out * c_in;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int co = co0 + og + 16 * i;
        if (co >= c_out) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ci = ci0 + ig + 16 * j;
            if (ci < c_in) dstp[(size_t)co * c_in + ci] = acc[i][j];
        }
    }
}

// dw[e] = sum over ranges of part[range][e], in range order
__global__ void reduce_partials(const float *__restrict__ part, float *__restrict__ dw, size_t n, int n_ranges)
{
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    float s = 0.f;
    for (int r = 0; r < n_ranges; ++r) s += part[(size_t)r * n + e];
    dw[e] = s;
}

template <typename T>
__global__ void transpose_kernel(const T *__restrict__ w, T *__restrict__ wt, int c_out, int c_in)
{
    __shared__ T tile[32][33];
    const size_t base = (size_t)blockIdx.z * c_out * c_in;
    int ci = blockIdx.x * 32 + threadIdx.x;
    for (int dy = threadIdx.y; dy < 32; dy += blockDim.y) {
        int co = blockIdx.y * 32 + dy;
        if (co < c_out && ci < c_in) tile[dy][threadIdx.x] = w[base + (size_t)co * c_in + ci];
    }
    __syncthreads();
    int co = blockIdx.y * 32 + threadIdx.x;
    for (int dy = threadIdx.y; dy < 32; dy += blockDim.y) {
        int ci2 = blockIdx.x * 32 + dy;
        if (co < c_out && ci2 < c_in) wt[base + (size_t)ci2 * c_out + co] = tile[threadIdx.x][dy];
    }
}

int weight_ranges(int64_t n_tiles, int c_in, int c_out, int K)
{
    if (n_tiles <= 0) return 1;
    int64_t r = 2048 / K;
    if (r < 1) r = 1;
    if (r > n_tiles) r = n_tiles;
    const size_t per = (size_t)K * c_out * c_in * sizeof(float);
    const size_t cap = (size_t)256 << 20;
    while (r > 1 && (size_t)r * per > cap) --r;
    return (int)r;
}

}  // namespace

size_t mvmr_weight_workspace_bytes(int64_t n_centres, int c_in, int c_out, int K)
{
    const int64_t n_tiles = ceil_div(n_centres, TILE);
    return align_up((size_t)weight_ranges(n_tiles, c_in, c_out, K) * K * c_out * c_in * sizeof(float));
}

int mvmr_rows_generic(const MvmrArgs &a, hipStream_t stream)
{
    if (a.side.n_tiles <= 0) return PCPP_OK;
    dim3 grid((unsigned)a.side.n_tiles, (unsigned)ceil_div(a.c_dst, CH));
    if (a.in_dtype == PCPP_F32) {
        rows_kernel<float, float><<<grid, THREADS, 0, stream>>>(
            static_cast<const float *>(a.feat), static_cast<const float *>(a.w), static_cast<float *>(a.dst),
            a.n_centres, a.c_src, a.c_dst, a.K, a.gather, a.side);
    } else if (a.out_dtype == PCPP_F32) {
        rows_kernel<uint16_t, float><<<grid, THREADS, 0, stream>>>(
            static_cast<const uint16_t *>(a.feat), static_cast<const uint16_t *>(a.w), static_cast<float *>(a.dst),
            a.n_centres, a.c_src, a.c_dst, a.K, a.gather, a.side);
    } else {
        rows_kernel<uint16_t, uint16_t><<<grid, THREADS, 0, stream>>>(
            static_cast<const uint16_t *>(a.feat), static_cast<const uint16_t *>(a.w),
            static_cast<uint16_t *>(a.dst), a.n_centres, a.c_src, a.c_dst, a.K, a.gather, a.side);
    }
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

int mvmr_weight_generic(const MvmrArgs &a, float *dw, void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    const int c_in = a.c_src, c_out = a.c_dst;
    const size_t n = (size_t)a.K * c_out * c_in;
    if (a.side.n_tiles <= 0) return fill_u32(reinterpret_cast<uint32_t *>(dw), 0u, (int64_t)n, stream);
    const int n_ranges = weight_ranges(a.side.n_tiles, c_in, c_out, a.K);
    if (workspace_bytes < (size_t)n_ranges * n * sizeof(float)) {
        set_error("pcpp_mvmr_bwd_weight: workspace has %zu bytes, needs %zu", workspace_bytes,
                  (size_t)n_ranges * n * sizeof(float));
        return PCPP_ERR_WORKSPACE;
    }
    const int tiles_per_range = (int)ceil_div(a.side.n_tiles, n_ranges);
    const int chunks_in = (int)ceil_div(c_in, CH), chunks_out = (int)ceil_div(c_out, CH);
    dim3 grid((unsigned)a.K, (unsigned)n_ranges, (unsigned)(chunks_in * chunks_out));
    float *part = static_cast<float *>(workspace);
    if (a.in_dtype == PCPP_F32)
        weight_kernel<float><<<grid, THREADS, 0, stream>>>(static_cast<const float *>(a.feat),
                                                           static_cast<const float *>(a.dense), part, a.n_centres,
                                                           c_in, c_out, a.K, a.gather, a.side, tiles_per_range,
                                                           chunks_in);
    else
        weight_kernel<uint16_t><<<grid, THREADS, 0, stream>>>(static_cast<const uint16_t *>(a.feat),
                                                              static_cast<const uint16_t *>(a.dense), part,
                                                              a.n_centres, c_in, c_out, a.K, a.gather, a.side,
                                                              tiles_per_range, chunks_in);
    PCPP_HIP_CHECK(hipGetLastError());
    reduce_partials<<<(unsigned)ceil_div((int64_t)n, 256), 256, 0, stream>>>(part, dw, n, n_ranges);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

int transpose_w(const void *w, void *wt, int K, int c_out, int c_in, int dtype, hipStream_t stream)
{
    dim3 grid((unsigned)ceil_div(c_in, 32), (unsigned)ceil_div(c_out, 32), (unsigned)K), block(32, 8);
    if (dtype == PCPP_F32)
        transpose_kernel<float><<<grid, block, 0, stream>>>(static_cast<const float *>(w), static_cast<float *>(wt),
                                                            c_out, c_in);
    else
        transpose_kernel<uint16_t><<<grid, block, 0, stream>>>(static_cast<const uint16_t *>(w),
                                                               static_cast<uint16_t *>(wt), c_out, c_in);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

}  // namespace pcpp
