// Matrix-core (MFMA) MVMR kernels for gfx950.
//
// Rows kernel (Eq. (1) forward; Sec. 3.3.3 input gradient with W^T): a block of four waves owns 32
// consecutive centres and every destination channel; wave w takes the kernel cells k = w, w+4, ...
// For each of its cells a wave
//   1. sums the source rows of each (k, centre) run in fp32 registers -- the lanes are laid out so that
//      the summed tile already is the MFMA A operand: lane (m = lane % 32, h = lane / 32) holds
//      channels [h*C/2, (h+1)*C/2) of centre m -- no LDS and no barrier on this path;
//   2. multiplies the 32 x C_SRC tile by W[k]^T on the matrix cores into fp32 accumulators that stay
//      in registers for the whole cell loop.
// Run bounds and gather indices of the next cell are fetched while the rows of the current one are in
// flight.  The reduction index of the MFMA is permuted (step s of half h <-> channel h*C/2 + s, or the
// s-th group of 8 for bf16) identically for both operands, so every lane reads contiguous memory.
// The four waves' accumulators are added in wave order through LDS and each destination row is
// written once: no atomics, fixed summation order.
//
// Weight kernel (Eq. (5), VVOR): dW[k] = sum over the cell's run of dy[o] (x) x[i].  The triplet list
// is cut into equal chunks, one per wave; the reduction index of the MFMA is the triplet, both
// operands are rows read straight from memory (lane <-> channel), partial sums per chunk go to the
// workspace and are added in a fixed order by a second kernel.
#include <stdlib.h>

#include "pcpp_internal.h"

namespace pcpp {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int WAVES = 4;
constexpr int ROWS = 32;   // centres per wave

// Per-lane predicated 16-byte load through a buffer descriptor: a lane whose offset is OOB_OFFSET is out
// of the descriptor's range, reads zeros and causes no memory traffic, so runs of different lengths
// need no branches around their loads.
constexpr uint32_t OOB_OFFSET = 0xffffff00u;
constexpr size_t MAX_BUFFER_BYTES = 0xfffff000u;

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

__device__ inline v4u buffer_load16(__amdgpu_buffer_rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
}

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

// MFMA register layouts used below (wave64):
//   v_mfma_f32_32x32x2_f32 :  A: lane (m = l%32, h = l/32) gives A[m][h];  B: lane (n, h) gives B[h][n]
//   v_mfma_f32_32x32x16_bf16: A: lane (m, h) gives A[m][8h .. 8h+7];       B: lane (n, h) gives B[8h .. 8h+7][n]
//   D (both): lane l, register j -> row 8*(j/4) + 4*(l/32) + j%4, column l%32.

// Re-lays W for the rows kernel so that each MFMA B fragment is one contiguous 1 KiB wave load:
//   packed[((k*NB + b)*NV + v)*64 + lane] (16 bytes) = W(k, dst = b*32 + lane%32, src = (lane/32)*HALF + v*E .. +E)
// with E = 16 / element size.  W(k, d, s) is read at w[k*c_dst*c_src + d*stride_d + s*stride_s], which
// covers both W[k][c_out][c_in] as stored (forward) and its transpose (input gradient).
template <typename T>
__global__ void pack_w_kernel(const T *__restrict__ w, T *__restrict__ packed, int K, int c_src, int c_dst,
                              int stride_d, int stride_s)
{
    constexpr int E = 16 / sizeof(T);
    const int half = c_src / 2, nv = half / E, nb = c_dst / 32;
    const int64_t total = (int64_t)K * nb * nv * 64;
    const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (piece >= total) return;
    const int lane = (int)(piece & 63);
    int64_t r = piece >> 6;
    const int v = (int)(r % nv); r /= nv;
    const int b = (int)(r % nb);
    const int k = (int)(r / nb);
    const int d = b * 32 + (lane & 31);
    const int s0 = (lane >> 5) * half + v * E;
    const T *src = w + (size_t)k * c_dst * c_src + (size_t)d * stride_d;
    T *dst = packed + piece * E;
#pragma unroll
    for (int e = 0; e < E; ++e) dst[e] = src[(size_t)(s0 + e) * stride_s];
}

// KW = kernel cells per wave (compile time): the cell loop is fully unrolled so that the run bounds and
// the first J gather indices of every cell are fetched up front, leaving one memory round trip per cell.
template <bool BF16, int C_SRC, int C_DST, int J, int KW, bool PIPE, int NW, typename TOut>
__global__ __launch_bounds__(NW * 64) void rows_kernel(const void *__restrict__ feat_, const void *__restrict__ w_,
                                                          TOut *__restrict__ dst, int64_t n_centres, int K,
                                                          const int32_t *__restrict__ gather, uint32_t last_triplet,
                                                          uint32_t feat_bytes, PlanSideView side, int dbg)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr uint32_t ROWB = C_SRC * ES;    // bytes per source row
    constexpr int HALF = C_SRC / 2;          // channels per lane
    constexpr int NV = HALF * ES / 16;       // 16-byte loads per source row per lane
    constexpr int NB = C_DST / 32;           // 32-wide destination blocks
    extern __shared__ float red[];           // [NW - 1][NB * 16][64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int64_t blk = blockIdx.x;          // 32-centre block
    const int64_t row0 = blk * ROWS;
    const int64_t tile = blk >> 1;
    const int sub = (int)(blk & 1) * ROWS;   // offset of the block inside its 64-centre tile
    const bool last_in_tile = (sub + m) == TILE - 1;
    const __amdgpu_buffer_rsrc_t frs = make_rsrc(feat_, feat_bytes);
    const uint32_t lane_off = (uint32_t)h * HALF * ES;
    // W is pre-packed in fragment order: [k][b][v][lane][16 bytes] (see pack_w_kernel)
    const v4u *wfrag = static_cast<const v4u *>(w_) + lane;
    const uint32_t *runs = side.run_start + (size_t)tile * K * TILE + sub + m;
    const uint32_t *tends = side.tile_ptr + tile + 1;

    // run bounds of centre m for this wave's cells, then the first J gather indices of each run
    uint32_t st[KW], cn[KW];
#pragma unroll
    for (int t = 0; t < KW; ++t) {
        const int k = wave + NW * t;
        const int kc = k < K ? k : K - 1;
        const uint32_t *pe = last_in_tile ? tends + (size_t)kc * side.n_tiles : runs + (size_t)kc * TILE + 1;
        st[t] = (dbg & 8) ? 0u : runs[(size_t)kc * TILE];
        cn[t] = (dbg & 8) ? 0u : *pe;
    }
#pragma unroll
    for (int t = 0; t < KW; ++t) cn[t] = (wave + NW * t) < K ? cn[t] - st[t] : 0u;
    int32_t idx[KW][J];
#pragma unroll
    for (int t = 0; t < KW; ++t)
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const uint32_t p = st[t] + j;
            idx[t][j] = (dbg & 8) ? 0 : gather[p < last_triplet ? p : last_triplet];
        }
    // keep the index loads here, ahead of the cell loop (they would otherwise be sunk next to their uses)
#pragma unroll
    for (int t = 0; t < KW; ++t)
#pragma unroll
        for (int j = 0; j < J; ++j) asm volatile("" : "+v"(idx[t][j]));

    v16f acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[b][j] = 0.f;

    // Two cells in flight: the loads of cell t+1 (W fragments and the first J rows of every run) are
    // issued before the rows of cell t are consumed.  Lanes past the end of their run read through an
    // out-of-range buffer offset (zeros, no traffic), so the issue step has no branches.
    v4u bw[PIPE ? 2 : 1][NB][NV];
    v4u rv[PIPE ? 2 : 1][J][NV];
    auto issue = [&](int t, int buf) {
        const int k = wave + NW * t;
        const int kc = k < K ? k : K - 1;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < NV; ++v)
                bw[buf][b][v] = (dbg & 16) ? v4u{1u, 2u, 3u, 4u} : wfrag[(((size_t)((dbg & 2) ? 0 : kc) * NB + b) * NV + v) * 64];
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const uint32_t off = ((uint32_t)j < cn[t] && !(dbg & 1)) ? (uint32_t)idx[t][j] * ROWB + lane_off : OOB_OFFSET;
#pragma unroll
            for (int v = 0; v < NV; ++v) rv[buf][j][v] = buffer_load16(frs, off + v * 16);
        }
    };
    if constexpr (PIPE) issue(0, 0);
#pragma unroll
    for (int t = 0; t < KW; ++t) {
        const int buf = PIPE ? (t & 1) : 0;
        if constexpr (PIPE) {
            if (t + 1 < KW) issue(t + 1, buf ^ 1);
        } else {
            issue(t, 0);
        }
        const uint32_t cn_c = cn[t], st_c = st[t];
        float xs[HALF];
#pragma unroll
        for (int c = 0; c < HALF; ++c) xs[c] = 0.f;
        auto add_row = [&](const v4u (&r)[NV]) {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if constexpr (BF16) {
                        xs[v * 8 + 2 * e] += __uint_as_float(r[v][e] << 16);
                        xs[v * 8 + 2 * e + 1] += __uint_as_float(r[v][e] & 0xffff0000u);
                    } else {
                        xs[v * 4 + e] += __uint_as_float(r[v][e]);
                    }
                }
        };
#pragma unroll
        for (int j = 0; j < J; ++j) add_row(rv[buf][j]);
        // runs longer than J
        for (uint32_t j0 = J; j0 < cn_c; j0 += J) {
            int32_t ix[J];
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint32_t p = st_c + j0 + j;
                ix[j] = gather[p < last_triplet ? p : last_triplet];
            }
            v4u rr[J][NV];
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint32_t off = j0 + j < cn_c ? (uint32_t)ix[j] * ROWB + lane_off : OOB_OFFSET;
#pragma unroll
                for (int v = 0; v < NV; ++v) rr[j][v] = buffer_load16(frs, off + v * 16);
            }
#pragma unroll
            for (int j = 0; j < J; ++j) add_row(rr[j]);
        }
        if (dbg & 4) { acc[0][0] += xs[0] + __uint_as_float(bw[buf][0][0][0]); continue; }
        if constexpr (BF16) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                v4u a;
#pragma unroll
                for (int e = 0; e < 4; ++e) a[e] = pack_bf16x2(xs[v * 8 + 2 * e], xs[v * 8 + 2 * e + 1]);
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a),
                                                                     __builtin_bit_cast(v8bf, bw[buf][b][v]), acc[b], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[v * 4 + e], __uint_as_float(bw[buf][b][v][e]),
                                                                      acc[b], 0, 0, 0);
        }
    }

    // add the four waves' accumulators in wave order, wave 0 writes the rows
    if (wave > 0) {
        float *mine = red + (size_t)(wave - 1) * NB * 16 * 64;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int j = 0; j < 16; ++j) mine[(b * 16 + j) * 64 + lane] = acc[b][j];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            float v = acc[b][j];
#pragma unroll
            for (int wv = 0; wv < NW - 1; ++wv) v += red[((size_t)wv * NB * 16 + b * 16 + j) * 64 + lane];
            const int64_t row = row0 + 8 * (j / 4) + 4 * h + (j % 4);
            if (row < n_centres) {
                if constexpr (sizeof(TOut) == 4) dst[(size_t)row * C_DST + b * 32 + m] = v;
                else dst[(size_t)row * C_DST + b * 32 + m] = (uint16_t)(pack_bf16x2(v, 0.f) & 0xffffu);
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Rows kernel for wide layers (bf16, C_SRC a multiple of 64, large K): here W[k] is too large to be
// re-read per 32 centres, so a block of eight waves owns 256 consecutive centres (32 per wave) and
// shares every W[k] through LDS.  The work is a sequence of steps (cell k, 64-channel chunk c of the
// source row); per step the block copies the 64 x C_DST slice of W[k] (fragment order, 16 B per lane)
// into one of two LDS buffers while each wave gathers and sums the matching 128-byte slice of its
// centres' source rows, then every wave multiplies its 32 x 64 tile with the shared slice.  One
// barrier per step; cells without a triplet in the block's 256 centres are skipped by the whole block.
//   packed W layout: piece ((((k*NCH + c)*NB + b)*4 + v)*64 + lane) =
//                    W(k, dst = b*32 + lane%32, src = c*64 + (lane/32)*32 + v*8 .. +8)
// ---------------------------------------------------------------------------------------------
constexpr int BIG_WAVES = 8;

template <int C_SRC, int C_DST, int J, typename TOut>
__global__ __launch_bounds__(BIG_WAVES * 64) void rows_big_kernel(const void *__restrict__ feat_,
                                                                  const void *__restrict__ w_, TOut *__restrict__ dst,
                                                                  int64_t n_centres, int K,
                                                                  const int32_t *__restrict__ gather,
                                                                  uint32_t last_triplet, uint32_t feat_bytes,
                                                                  PlanSideView side)
{
    constexpr uint32_t ROWB = C_SRC * 2;
    constexpr int NCH = C_SRC / 64;                  // source chunks
    constexpr int NB = C_DST / 32;                   // destination blocks
    constexpr int PIECES = NB * 4 * 64;              // 16-byte pieces of one W slice
    constexpr int PPT = PIECES / (BIG_WAVES * 64);   // pieces copied per thread
    extern __shared__ __attribute__((aligned(16))) char lds[];   // 2 * PIECES * 16 bytes
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int64_t blk = (int64_t)blockIdx.x * BIG_WAVES + wave;   // 32-centre block of this wave
    const int64_t row0 = blk * ROWS;
    const bool valid = row0 < n_centres;                          // wave-uniform
    int64_t tile = blk >> 1;
    if (tile >= side.n_tiles) tile = side.n_tiles - 1;
    const int sub = (int)(blk & 1) * ROWS;
    const bool last_in_tile = (sub + m) == TILE - 1;
    const __amdgpu_buffer_rsrc_t frs = make_rsrc(feat_, feat_bytes);
    const v4u *wsrc = static_cast<const v4u *>(w_) + threadIdx.x;
    const uint32_t *runs = side.run_start + (size_t)tile * K * TILE + sub + m;
    const uint32_t *tends = side.tile_ptr + tile + 1;
    const int64_t t0 = (int64_t)blockIdx.x * (BIG_WAVES / 2);
    const int64_t t1 = t0 + BIG_WAVES / 2 < side.n_tiles ? t0 + BIG_WAVES / 2 : side.n_tiles;

    v16f acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[b][j] = 0.f;

    int step = 0;
    for (int k = 0; k < K; ++k) {
        // any triplet of cell k among the block's centres?  (block-uniform)
        if (side.tile_ptr[(size_t)k * side.n_tiles + t0] == side.tile_ptr[(size_t)k * side.n_tiles + t1]) continue;
        uint32_t st_c = runs[(size_t)k * TILE];
        uint32_t cn_c = (last_in_tile ? tends[(size_t)k * side.n_tiles] : runs[(size_t)k * TILE + 1]) - st_c;
        if (!valid) cn_c = 0;
        int32_t idx[J];
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const uint32_t p = st_c + j;
            idx[j] = gather[p < last_triplet ? p : last_triplet];
        }
        const bool any = __ballot(cn_c != 0) != 0;
#pragma unroll 1
        for (int c = 0; c < NCH; ++c, ++step) {
            char *buf = lds + (size_t)(step & 1) * PIECES * 16;
            // this thread's share of the W slice
            v4u wr[PPT];
            const v4u *ws = wsrc + ((size_t)k * NCH + c) * PIECES;
#pragma unroll
            for (int q = 0; q < PPT; ++q) wr[q] = ws[q * BIG_WAVES * 64];
            // the matching slice of this centre's source rows
            const uint32_t slice_off = (uint32_t)(c * 64 + h * 32) * 2;
            v4u rv[J][4];
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const uint32_t off = (uint32_t)j < cn_c ? (uint32_t)idx[j] * ROWB + slice_off : OOB_OFFSET;
#pragma unroll
                for (int v = 0; v < 4; ++v) rv[j][v] = buffer_load16(frs, off + v * 16);
            }
#pragma unroll
            for (int q = 0; q < PPT; ++q)
                *reinterpret_cast<v4u *>(buf + (size_t)(threadIdx.x + q * BIG_WAVES * 64) * 16) = wr[q];
            float xs[32];
#pragma unroll
            for (int e = 0; e < 32; ++e) xs[e] = 0.f;
            auto add_row = [&](const v4u (&r)[4]) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        xs[v * 8 + 2 * e] += __uint_as_float(r[v][e] << 16);
                        xs[v * 8 + 2 * e + 1] += __uint_as_float(r[v][e] & 0xffff0000u);
                    }
            };
#pragma unroll
            for (int j = 0; j < J; ++j) add_row(rv[j]);
            for (uint32_t j0 = J; j0 < cn_c; j0 += J) {           // runs longer than J
                int32_t ix[J];
#pragma unroll
                for (int j = 0; j < J; ++j) {
                    const uint32_t p = st_c + j0 + j;
                    ix[j] = gather[p < last_triplet ? p : last_triplet];
                }
                v4u rr[J][4];
#pragma unroll
                for (int j = 0; j < J; ++j) {
                    const uint32_t off = j0 + j < cn_c ? (uint32_t)ix[j] * ROWB + slice_off : OOB_OFFSET;
#pragma unroll
                    for (int v = 0; v < 4; ++v) rr[j][v] = buffer_load16(frs, off + v * 16);
                }
#pragma unroll
                for (int j = 0; j < J; ++j) add_row(rr[j]);
            }
            v4u a[4];
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int e = 0; e < 4; ++e) a[v][e] = pack_bf16x2(xs[v * 8 + 2 * e], xs[v * 8 + 2 * e + 1]);
            __syncthreads();                                      // the slice is complete in LDS
            if (any) {
                const v4u *bl = reinterpret_cast<const v4u *>(buf) + lane;
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a[v]),
                                                                         __builtin_bit_cast(v8bf, bl[(b * 4 + v) * 64]),
                                                                         acc[b], 0, 0, 0);
            }
        }
    }
    if (!valid) return;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t row = row0 + 8 * (j / 4) + 4 * h + (j % 4);
            if (row < n_centres) {
                if constexpr (sizeof(TOut) == 4) dst[(size_t)row * C_DST + b * 32 + m] = acc[b][j];
                else dst[(size_t)row * C_DST + b * 32 + m] = (uint16_t)(pack_bf16x2(acc[b][j], 0.f) & 0xffffu);
            }
        }
}

// W slices for rows_big_kernel (layout in its header comment)
__global__ void pack_w_big_kernel(const uint16_t *__restrict__ w, uint16_t *__restrict__ packed, int K, int c_src,
                                  int c_dst, int stride_d, int stride_s)
{
    const int nch = c_src / 64, nb = c_dst / 32;
    const int64_t total = (int64_t)K * nch * nb * 4 * 64;
    const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (piece >= total) return;
    const int lane = (int)(piece & 63);
    int64_t r = piece >> 6;
    const int v = (int)(r & 3); r >>= 2;
    const int b = (int)(r % nb); r /= nb;
    const int c = (int)(r % nch);
    const int k = (int)(r / nch);
    const int d = b * 32 + (lane & 31);
    const int s0 = c * 64 + (lane >> 5) * 32 + v * 8;
    const uint16_t *src = w + (size_t)k * c_dst * c_src + (size_t)d * stride_d;
    uint16_t *dstp = packed + piece * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) dstp[e] = src[(size_t)(s0 + e) * stride_s];
}

// ---------------------------------------------------------------------------------------------
// Weight gradient (VVOR), Eq. (5).  Wave c owns triplets [c*chunk, (c+1)*chunk) of the (k, o, i)
// ordered list.  A chunk usually lies inside one cell's run; where a run starts inside the chunk the
// accumulator is flushed and restarted.  Slots of the partial buffer:
//   slot c               sum for the cell of the chunk's first triplet
//   slot n_chunks + k    sum for cell k over the part of its run that starts inside a chunk
// fp32: one MFMA step consumes 2 triplets: lane (c, h) supplies channel c of dy[o] and of x[i] of
// triplet 2 s + h.  bf16: one step consumes 16 triplets; a lane reads one dword (2 channels) per
// triplet and the even / odd channels form separate 32-wide blocks of the operand.
// ---------------------------------------------------------------------------------------------
// Wide layers: a wave owns a SUB_OUT x SUB_IN block of dW[k]; the n_sub waves that share a chunk are
// consecutive, so their re-reads of the same rows are served by the L1 / L2 caches.
template <bool BF16, int C_IN, int C_OUT, int SUB_IN, int SUB_OUT>
__global__ __launch_bounds__(WAVES * 64) void weight_kernel(const void *__restrict__ x_, const void *__restrict__ dy_,
                                                            float *__restrict__ part,
                                                            const int32_t *__restrict__ tri_o,
                                                            const int32_t *__restrict__ tri_i,
                                                            const int64_t *__restrict__ seg, int K, int64_t n_triplets,
                                                            int chunk, int64_t n_chunks)
{
    constexpr int NBI = SUB_IN / 32, NBO = SUB_OUT / 32;
    constexpr int N_SUB_IN = C_IN / SUB_IN, N_SUB = N_SUB_IN * (C_OUT / SUB_OUT);
    constexpr int STEP = BF16 ? 16 : 2;      // triplets per MFMA step
    constexpr int NS = 32 / STEP;            // steps per batch of 32 triplets
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int64_t gw = (int64_t)blockIdx.x * WAVES + wave;
    const int64_t chunk_id = gw / N_SUB;
    const int sub = (int)(gw % N_SUB);
    const int ci0 = (sub % N_SUB_IN) * SUB_IN, co0 = (sub / N_SUB_IN) * SUB_OUT;
    if (chunk_id >= n_chunks) return;
    int64_t p = chunk_id * chunk;
    int64_t p_end = p + chunk;
    if (p_end > n_triplets) p_end = n_triplets;

    // cell of the first triplet: the k with seg[k] <= p < seg[k+1]
    int k = 0;
    for (int kb = 0; kb < K; kb += 64) {
        const int kk = kb + lane;
        const bool hit = kk < K && seg[kk] <= p && p < seg[kk + 1];
        const unsigned long long msk = __ballot(hit);
        if (msk) { k = kb + __ffsll((long long)msk) - 1; break; }
    }

    v16f acc[NBO][NBI];
    bool first = true;
    while (p < p_end) {
        int64_t q = seg[k + 1];
        if (q > p_end) q = p_end;
        if (q <= p) { ++k; continue; }       // empty run
#pragma unroll
        for (int bo = 0; bo < NBO; ++bo)
#pragma unroll
            for (int bi = 0; bi < NBI; ++bi)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[bo][bi][j] = 0.f;

        for (int64_t b0 = p; b0 < q; b0 += 32) {
            const int n = (int)(q - b0 < 32 ? q - b0 : 32);
            // lanes 0..31 hold o of triplet b0 + lane, lanes 32..63 hold i of triplet b0 + lane - 32
            int32_t oi = 0;
            if (c < n) oi = h == 0 ? tri_o[b0 + c] : tri_i[b0 + c];
            if constexpr (!BF16) {
                float a[NBO][NS], b[NBI][NS];
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const int t = 2 * s + h;
                    const int32_t o = __shfl(oi, t, 64), i = __shfl(oi, 32 + t, 64);
                    const float *dyr = static_cast<const float *>(dy_) + (size_t)o * C_OUT + co0 + c;
                    const float *xr = static_cast<const float *>(x_) + (size_t)i * C_IN + ci0 + c;
#pragma unroll
                    for (int bo = 0; bo < NBO; ++bo) a[bo][s] = t < n ? dyr[bo * 32] : 0.f;
#pragma unroll
                    for (int bi = 0; bi < NBI; ++bi) b[bi][s] = t < n ? xr[bi * 32] : 0.f;
                }
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int bo = 0; bo < NBO; ++bo)
#pragma unroll
                        for (int bi = 0; bi < NBI; ++bi)
                            acc[bo][bi] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[bo][s], b[bi][s], acc[bo][bi], 0, 0, 0);
            } else {
                // block index of the operand = 2 * q + parity: channel 2 * (c + 32 q) + parity
                constexpr int QO = SUB_OUT / 64, QI = SUB_IN / 64;
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    uint32_t dyw[QO][8], xw[QI][8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int t = 16 * s + 8 * h + e;
                        const int32_t o = __shfl(oi, t, 64), i = __shfl(oi, 32 + t, 64);
                        const uint32_t *dyr = static_cast<const uint32_t *>(dy_) + (size_t)o * (C_OUT / 2) + co0 / 2 + c;
                        const uint32_t *xr = static_cast<const uint32_t *>(x_) + (size_t)i * (C_IN / 2) + ci0 / 2 + c;
#pragma unroll
                        for (int qo = 0; qo < QO; ++qo) dyw[qo][e] = t < n ? dyr[qo * 32] : 0u;
#pragma unroll
                        for (int qi = 0; qi < QI; ++qi) xw[qi][e] = t < n ? xr[qi * 32] : 0u;
                    }
                    v4u av[NBO], bv[NBI];
#pragma unroll
                    for (int qo = 0; qo < QO; ++qo)
#pragma unroll
                        for (int e2 = 0; e2 < 4; ++e2) {
                            av[2 * qo][e2] = (dyw[qo][2 * e2] & 0xffffu) | (dyw[qo][2 * e2 + 1] << 16);
                            av[2 * qo + 1][e2] = (dyw[qo][2 * e2] >> 16) | (dyw[qo][2 * e2 + 1] & 0xffff0000u);
                        }
#pragma unroll
                    for (int qi = 0; qi < QI; ++qi)
#pragma unroll
                        for (int e2 = 0; e2 < 4; ++e2) {
                            bv[2 * qi][e2] = (xw[qi][2 * e2] & 0xffffu) | (xw[qi][2 * e2 + 1] << 16);
                            bv[2 * qi + 1][e2] = (xw[qi][2 * e2] >> 16) | (xw[qi][2 * e2 + 1] & 0xffff0000u);
                        }
#pragma unroll
                    for (int bo = 0; bo < NBO; ++bo)
#pragma unroll
                        for (int bi = 0; bi < NBI; ++bi)
                            acc[bo][bi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, av[bo]),
                                                                                  __builtin_bit_cast(v8bf, bv[bi]),
                                                                                  acc[bo][bi], 0, 0, 0);
                }
            }
        }
        // flush
        float *dstp = part + (size_t)(first ? chunk_id : n_chunks + k) * C_OUT * C_IN;
#pragma unroll
        for (int bo = 0; bo < NBO; ++bo)
#pragma unroll
            for (int bi = 0; bi < NBI; ++bi)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int r = 8 * (j / 4) + 4 * h + (j % 4);
                    int co, ci;
                    if constexpr (BF16) {
                        co = co0 + 2 * (r + 32 * (bo >> 1)) + (bo & 1);
                        ci = ci0 + 2 * (c + 32 * (bi >> 1)) + (bi & 1);
                    } else {
                        co = co0 + bo * 32 + r;
                        ci = ci0 + bi * 32 + c;
                    }
                    dstp[(size_t)co * C_IN + ci] = acc[bo][bi][j];
                }
        first = false;
        p = q;
        ++k;
    }
}

// dw[k][e] = (partial of the run's head, if it starts inside a chunk) + partials of the chunks whose first
// triplet lies in run k.  16 threads share one element: thread g adds chunks c0+g, c0+g+16, ... in
// ascending order and the 16 sums are then added in order of g, so the result is reproducible.
// grid = (ceil(c_out*c_in / 16), K), block = 256
__global__ __launch_bounds__(256) void weight_reduce(const float *__restrict__ part, float *__restrict__ dw,
                                                     const int64_t *__restrict__ seg, int n_elem, int chunk,
                                                     int64_t n_chunks)
{
    __shared__ float sums[16][17];
    const int el = threadIdx.x & 15, g = threadIdx.x >> 4;
    const int e = blockIdx.x * 16 + el;
    const int k = blockIdx.y;
    const int64_t s = seg[k], t = seg[k + 1];
    float v = 0.f;
    if (t > s && e < n_elem) {
        const int64_t c0 = (s + chunk - 1) / chunk, c1 = (t + chunk - 1) / chunk;
        for (int64_t c = c0 + g; c < c1; c += 16) v += part[(size_t)c * n_elem + e];
    }
    sums[g][el] = v;
    __syncthreads();
    if (g == 0 && e < n_elem) {
        float r = (t > s && s % chunk != 0) ? part[(size_t)(n_chunks + k) * n_elem + e] : 0.f;
#pragma unroll
        for (int gg = 0; gg < 16; ++gg) r += sums[gg][el];
        dw[(size_t)k * n_elem + e] = r;
    }
}

// triplets per chunk: at least 512, grown so that there are at most about 8192 chunks (2048 for wide
// layers, whose partial sums are large)
int weight_chunk(int64_t n_triplets, int c_in, int c_out)
{
    const int64_t max_chunks = (int64_t)c_in * c_out >= 128 * 128 ? 2048 : 8192;
    int chunk = 512;
    while ((n_triplets + chunk - 1) / chunk > max_chunks) chunk *= 2;
    return chunk;
}

template <bool BF16, int C_IN, int C_OUT, int SUB_IN = C_IN, int SUB_OUT = C_OUT>
int launch_weight(const MvmrArgs &a, float *dw, const int32_t *tri_o, const int64_t *seg, void *workspace,
                  size_t workspace_bytes, hipStream_t stream)
{
    const int n_elem = C_IN * C_OUT;
    const int chunk = weight_chunk(a.n_triplets, C_IN, C_OUT);
    const int64_t n_chunks = ceil_div(a.n_triplets, chunk);
    constexpr int N_SUB = (C_IN / SUB_IN) * (C_OUT / SUB_OUT);
    const size_t need = (size_t)(n_chunks + a.K) * n_elem * sizeof(float);
    if (workspace_bytes < need) {
        set_error("pcpp_mvmr_bwd_weight: workspace has %zu bytes, needs %zu", workspace_bytes, need);
        return PCPP_ERR_WORKSPACE;
    }
    float *part = static_cast<float *>(workspace);
    if (n_chunks > 0) {
        weight_kernel<BF16, C_IN, C_OUT, SUB_IN, SUB_OUT><<<(unsigned)ceil_div(n_chunks * N_SUB, WAVES), WAVES * 64, 0, stream>>>(
            a.feat, a.dense, part, tri_o, a.gather, seg, a.K, a.n_triplets, chunk, n_chunks);
        PCPP_HIP_CHECK(hipGetLastError());
    }
    dim3 grid((unsigned)ceil_div(n_elem, 16), (unsigned)a.K);
    weight_reduce<<<grid, 256, 0, stream>>>(part, dw, seg, n_elem, chunk, n_chunks);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

bool weight_shape_supported(int in_dtype, int c_in, int c_out)
{
    if (in_dtype == PCPP_F32) return (c_in == 32 && c_out == 32) || (c_in == 64 && c_out == 64);
    return (c_in == 64 && c_out == 64) || (c_in == 64 && c_out == 128) || (c_in == 128 && c_out == 128) ||
           (c_in == 256 && c_out == 256);
}

int rows_env(const char *name, int dflt)
{
    const char *e = getenv(name);
    return e ? atoi(e) : dflt;
}

template <bool BF16, int C_SRC, int C_DST, int J, int KW, bool PIPE, int NW>
int launch_rows_cfg(const MvmrArgs &a, hipStream_t stream)
{
    const int64_t blocks = ceil_div(a.n_centres, ROWS);
    const size_t lds = (size_t)(NW - 1) * (C_DST / 32) * 16 * 64 * sizeof(float);
    const uint32_t last = (uint32_t)(a.n_triplets - 1);
    const uint32_t feat_bytes = (uint32_t)((size_t)a.n_src * C_SRC * (BF16 ? 2 : 4));
    if (a.out_dtype == PCPP_F32) {
        rows_kernel<BF16, C_SRC, C_DST, J, KW, PIPE, NW, float><<<(unsigned)blocks, NW * 64, lds, stream>>>(
            a.feat, a.w, static_cast<float *>(a.dst), a.n_centres, a.K, a.gather, last, feat_bytes, a.side, rows_env("PCPP_ROWS_DBG", 0));
    } else {
        rows_kernel<BF16, C_SRC, C_DST, J, KW, PIPE, NW, uint16_t><<<(unsigned)blocks, NW * 64, lds, stream>>>(
            a.feat, a.w, static_cast<uint16_t *>(a.dst), a.n_centres, a.K, a.gather, last, feat_bytes, a.side, rows_env("PCPP_ROWS_DBG", 0));
    }
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

// K <= 28: either 4 waves x 7 cells or 8 waves x 4 cells per 32-centre block
template <bool BF16, int C_SRC, int C_DST, int J>
int launch_rows_k28(const MvmrArgs &a, hipStream_t stream)
{
    static const int nw = rows_env("PCPP_ROWS_NW", 4), pipe = rows_env("PCPP_ROWS_PIPE", 0);
    if (nw == 8) return pipe ? launch_rows_cfg<BF16, C_SRC, C_DST, J, 4, true, 8>(a, stream)
                             : launch_rows_cfg<BF16, C_SRC, C_DST, J, 4, false, 8>(a, stream);
    return pipe ? launch_rows_cfg<BF16, C_SRC, C_DST, J, 7, true, 4>(a, stream)
                : launch_rows_cfg<BF16, C_SRC, C_DST, J, 7, false, 4>(a, stream);
}

// cells per wave: 7 covers K <= 28 (t <= 3); larger kernels fall back to the generic path
template <bool BF16, int C_SRC, int C_DST, int J>
int launch_rows(const MvmrArgs &a, hipStream_t stream, bool *handled)
{
    if ((size_t)a.n_src * C_SRC * (BF16 ? 2 : 4) > MAX_BUFFER_BYTES) { *handled = false; return PCPP_OK; }
    if (a.K <= 4 * 2) return launch_rows_cfg<BF16, C_SRC, C_DST, J, 2, false, 4>(a, stream);
    if (a.K <= 4 * 7) return launch_rows_k28<BF16, C_SRC, C_DST, J>(a, stream);
    *handled = false;
    return PCPP_OK;
}

}  // namespace

// wide bf16 layers with any K: rows_big_kernel
bool rows_big_shape(const MvmrArgs &a)
{
    return a.in_dtype == PCPP_BF16 && ((a.c_src == 256 && a.c_dst == 256) || (a.c_src == 128 && a.c_dst == 128));
}

template <int C_SRC, int C_DST>
int launch_rows_big(const MvmrArgs &a, hipStream_t stream)
{
    constexpr int J = 2;
    const int64_t blocks = ceil_div(ceil_div(a.n_centres, ROWS), BIG_WAVES);
    const size_t lds = (size_t)2 * (C_DST / 32) * 4 * 64 * 16;
    const uint32_t last = (uint32_t)(a.n_triplets - 1);
    const uint32_t feat_bytes = (uint32_t)((size_t)a.n_src * C_SRC * 2);
    if (a.out_dtype == PCPP_F32) {
        auto kern = rows_big_kernel<C_SRC, C_DST, J, float>;
        PCPP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        kern<<<(unsigned)blocks, BIG_WAVES * 64, lds, stream>>>(a.feat, a.w, static_cast<float *>(a.dst), a.n_centres,
                                                                a.K, a.gather, last, feat_bytes, a.side);
    } else {
        auto kern = rows_big_kernel<C_SRC, C_DST, J, uint16_t>;
        PCPP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        kern<<<(unsigned)blocks, BIG_WAVES * 64, lds, stream>>>(a.feat, a.w, static_cast<uint16_t *>(a.dst),
                                                                a.n_centres, a.K, a.gather, last, feat_bytes, a.side);
    }
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

bool mvmr_rows_mfma_supported(const MvmrArgs &a)
{
    if (a.n_triplets <= 0) return false;
    if (rows_big_shape(a)) return (size_t)a.n_src * a.c_src * 2 <= MAX_BUFFER_BYTES;
    if (a.K > 28) return false;
    const size_t es = a.in_dtype == PCPP_BF16 ? 2 : 4;
    if ((size_t)a.n_src * a.c_src * es > MAX_BUFFER_BYTES) return false;
    if (a.in_dtype == PCPP_F32 && a.out_dtype == PCPP_F32)
        return (a.c_src == 32 && a.c_dst == 32) || (a.c_src == 16 && a.c_dst == 32) || (a.c_src == 64 && a.c_dst == 64);
    if (a.in_dtype == PCPP_BF16)
        return (a.c_src == 64 && a.c_dst == 64) || (a.c_src == 64 && a.c_dst == 128) ||
               (a.c_src == 128 && a.c_dst == 64) || (a.c_src == 32 && a.c_dst == 32);
    return false;
}

// Packs W(k, d, s) = w[k*c_dst*c_src + d*stride_d + s*stride_s] into `packed` (K*c_dst*c_src elements).
int mvmr_pack_w(const void *w, void *packed, int K, int c_src, int c_dst, int stride_d, int stride_s, int dtype,
                hipStream_t stream)
{
    const int e = dtype == PCPP_BF16 ? 8 : 4;
    const int64_t total = (int64_t)K * (c_dst / 32) * (c_src / 2 / e) * 64;
    const unsigned blocks = (unsigned)ceil_div(total, 256);
    if (dtype == PCPP_BF16 && ((c_src == 256 && c_dst == 256) || (c_src == 128 && c_dst == 128))) {
        pack_w_big_kernel<<<blocks, 256, 0, stream>>>(static_cast<const uint16_t *>(w), static_cast<uint16_t *>(packed),
                                                      K, c_src, c_dst, stride_d, stride_s);
        PCPP_HIP_CHECK(hipGetLastError());
        return PCPP_OK;
    }
    if (dtype == PCPP_BF16)
        pack_w_kernel<uint16_t><<<blocks, 256, 0, stream>>>(static_cast<const uint16_t *>(w),
                                                            static_cast<uint16_t *>(packed), K, c_src, c_dst,
                                                            stride_d, stride_s);
    else
        pack_w_kernel<float><<<blocks, 256, 0, stream>>>(static_cast<const float *>(w), static_cast<float *>(packed),
                                                         K, c_src, c_dst, stride_d, stride_s);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

// a.w must be the packed weights
int mvmr_rows_mfma(const MvmrArgs &a, hipStream_t stream, bool *handled)
{
    *handled = true;
    if (!mvmr_rows_mfma_supported(a)) { *handled = false; return PCPP_OK; }
    if (rows_big_shape(a)) {
        if (a.c_src == 256) return launch_rows_big<256, 256>(a, stream);
        return launch_rows_big<128, 128>(a, stream);
    }
    if (a.in_dtype == PCPP_F32 && a.out_dtype == PCPP_F32) {
        if (a.c_src == 32 && a.c_dst == 32) return launch_rows<false, 32, 32, 2>(a, stream, handled);
        if (a.c_src == 16 && a.c_dst == 32) return launch_rows<false, 16, 32, 2>(a, stream, handled);
        if (a.c_src == 64 && a.c_dst == 64) return launch_rows<false, 64, 64, 2>(a, stream, handled);
    } else if (a.in_dtype == PCPP_BF16) {
        if (a.c_src == 64 && a.c_dst == 64) return launch_rows<true, 64, 64, 2>(a, stream, handled);
        if (a.c_src == 64 && a.c_dst == 128) return launch_rows<true, 64, 128, 2>(a, stream, handled);
        if (a.c_src == 128 && a.c_dst == 64) return launch_rows<true, 128, 64, 1>(a, stream, handled);
        if (a.c_src == 32 && a.c_dst == 32) return launch_rows<true, 32, 32, 2>(a, stream, handled);
    }
    *handled = false;
    return PCPP_OK;
}

// c_src = c_in (x), c_dst = c_out (dy, passed as `dense`); gather = tri_i
int mvmr_weight_mfma(const MvmrArgs &a, float *dw, const int32_t *tri_o, const int64_t *seg, void *workspace,
                     size_t workspace_bytes, hipStream_t stream, bool *handled)
{
    *handled = true;
    if (a.in_dtype == PCPP_F32) {
        if (a.c_src == 32 && a.c_dst == 32) return launch_weight<false, 32, 32>(a, dw, tri_o, seg, workspace, workspace_bytes, stream);
        if (a.c_src == 64 && a.c_dst == 64) return launch_weight<false, 64, 64>(a, dw, tri_o, seg, workspace, workspace_bytes, stream);
    } else {
        if (a.c_src == 64 && a.c_dst == 64) return launch_weight<true, 64, 64>(a, dw, tri_o, seg, workspace, workspace_bytes, stream);
        if (a.c_src == 64 && a.c_dst == 128) return launch_weight<true, 64, 128>(a, dw, tri_o, seg, workspace, workspace_bytes, stream);
        if (a.c_src == 128 && a.c_dst == 128) return launch_weight<true, 128, 128, 64, 128>(a, dw, tri_o, seg, workspace, workspace_bytes, stream);
        if (a.c_src == 256 && a.c_dst == 256) return launch_weight<true, 256, 256, 64, 128>(a, dw, tri_o, seg, workspace, workspace_bytes, stream);
    }
    *handled = false;
    return PCPP_OK;
}

size_t mvmr_weight_mfma_workspace_bytes(int64_t n_triplets, int c_in, int c_out, int K, int in_dtype)
{
    if (!weight_shape_supported(in_dtype, c_in, c_out)) return 0;
    const int chunk = weight_chunk(n_triplets, c_in, c_out);
    return align_up((size_t)(ceil_div(n_triplets, chunk) + K) * c_in * c_out * sizeof(float));
}

}  // namespace pcpp
