// MVMR rows kernel (Eq. (1) forward; Sec. 3.3.3 input gradient with W^T) on the matrix cores.
//
// Eq. (1) is linear, so out[o] = sum_k W[k] S_k[o] with S_k[o] = sum of x[i] over the (k, o) run.  Both
// factors of that expression are matrix products and both run on the MFMA units:
//
//   stage 1 (sum of each run)   S_k^T [channel][centre] = X_g^T [channel][triplet] . Sel^T [triplet][centre]
//       X_g = the source rows of the (cell, 32-centre block) run, one row per triplet, read densely
//       (a half-wave reads one 128-byte row, lane <-> channel); Sel[centre][triplet] = 1 when the triplet
//       belongs to the centre's run, built in registers from the run bounds.  Products with 1.0 are exact,
//       so this is the fp32 sum of the rows; run lengths never cause divergence and every loaded byte
//       is used.  fp32 inputs are split exactly into three bf16 terms (8 + 8 + 8 significant bits).
//   stage 2 (Eq. (1))           acc [centre][c_dst] += S_k [centre][channel] . W[k]^T
//       The stage-1 accumulator layout (lane <-> centre, register <-> channel) is the A-operand layout of
//       the second MFMA up to a permutation of the reduction index, which is folded into the order in
//       which W is packed.  bf16: the fp32 sums are rounded to bf16 once (v_cvt_pk_bf16_f32).
//
// A block of NW waves owns 32 consecutive centres and all destination channels; wave w takes cells
// w, w + NW, ...; the partial accumulators are added in wave order through LDS and every destination
// row is written once: no atomics, fixed summation order.
//
// MFMA layouts (wave64), v_mfma_f32_32x32x16_bf16: A: lane (M = l%32, h = l/32) holds A[M][8h .. 8h+7];
// B: lane (N = l%32, h) holds B[8h .. 8h+7][N]; D: lane l, register j -> M = 8*(j/4) + 4*(l/32) + j%4, N = l%32.
// v_mfma_f32_32x32x2_f32: A: lane (M, h) holds A[M][h]; B: lane (N, h) holds B[h][N]; D as above.
#include <stdlib.h>

#include "pcpp_internal.h"

namespace pcpp {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int ROWS = 32;                         // centres per block
constexpr uint32_t OOB_OFFSET = 0xffffff00u;     // buffer offset past any descriptor: reads zero, no traffic
constexpr size_t MAX_BUFFER_BYTES = 0xfffff000u;

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

__device__ inline uint32_t cvt_pk_bf16(float lo, float hi)
{
    const v2f v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, v2bf));   // round to nearest even
}

// Source channel of element e of packed piece pc for lane-half h (see the header comment and rows_kernel).
//   fp32: piece pc = g*4 + v      : 4 floats, channel 32 g + 8 v + 4 h + e
//   bf16: piece pc = (g*2+par)*2+s: 8 bf16, dword column d = 32 g + 8 (2 s + e/4) + 4 h + e%4, channel 2 d + par
template <bool BF16>
__host__ __device__ inline int packed_channel(int pc, int h, int e)
{
    if constexpr (BF16) {
        const int s = pc & 1, par = (pc >> 1) & 1, g = pc >> 2;
        const int d = 32 * g + 8 * (2 * s + (e >> 2)) + 4 * h + (e & 3);
        return 2 * d + par;
    } else {
        const int v = pc & 3, g = pc >> 2;
        return 32 * g + 8 * v + 4 * h + e;
    }
}

// packed[(((k*NB + b)*NPC + pc)*64 + lane)*16 bytes] = W(k, dst = b*32 + lane%32, src = packed_channel(pc, lane/32, e))
// with W(k, d, s) read at w[k*c_dst*c_src + d*stride_d + s*stride_s] (covers W as stored and its transpose).
template <typename T>
__global__ void pack_w_sel_kernel(const T *__restrict__ w, T *__restrict__ packed, int K, int c_src, int c_dst,
                                  int stride_d, int stride_s)
{
    constexpr bool BF16 = sizeof(T) == 2;
    constexpr int E = 16 / sizeof(T);
    const int nb = c_dst / 32, npc = c_src / E / 2;   // pieces per (k, b): every lane-half covers c_src / 2 channels
    const int64_t total = (int64_t)K * nb * npc * 64;
    const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (piece >= total) return;
    const int lane = (int)(piece & 63);
    int64_t r = piece >> 6;
    const int pc = (int)(r % npc); r /= npc;
    const int b = (int)(r % nb);
    const int k = (int)(r / nb);
    const int d = b * 32 + (lane & 31);
    const T *src = w + (size_t)k * c_dst * c_src + (size_t)d * stride_d;
    T *dst = packed + piece * E;
#pragma unroll
    for (int e = 0; e < E; ++e) dst[e] = src[(size_t)packed_channel<BF16>(pc, lane >> 5, e) * stride_s];
}

template <bool BF16, int C_SRC, int C_DST, int NW, typename TOut>
__global__ __launch_bounds__(NW * 64) void rows_kernel(const void *__restrict__ feat_, const void *__restrict__ w_,
                                                       TOut *__restrict__ dst, int64_t n_centres, int K,
                                                       const int32_t *__restrict__ gather, uint32_t last_triplet,
                                                       uint32_t feat_bytes, PlanSideView side)
{
    constexpr int DW = BF16 ? C_SRC / 2 : C_SRC;     // dwords per source row
    constexpr int NG = DW / 32;                      // lane c reads dword columns c + 32 g
    constexpr int NP = BF16 ? 2 : 1;                 // even / odd channel of a dword (bf16)
    constexpr int NS1 = NG * NP;                     // stage-1 accumulator blocks of 32 channels
    constexpr int NB = C_DST / 32;                   // destination blocks
    constexpr int NPC = BF16 ? NS1 * 2 : NG * 4;     // packed W pieces per (cell, destination block)
    constexpr uint32_t ROWB = DW * 4;
    constexpr int RED_FLOATS = (NW - 1) * NB * 16 * 64;
    extern __shared__ __attribute__((aligned(16))) float smem[];   // [RED_FLOATS] reduction + [256] selection table (v4u)
    float *red = smem;
    v4u *sel_tab = reinterpret_cast<v4u *>(smem + RED_FLOATS);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;          // c: channel column in stage 1, centre in stage 2
    const int64_t blk = blockIdx.x;
    const int64_t row0 = blk * ROWS;
    const int64_t tile = blk >> 1;
    const int sub = (int)(blk & 1) * ROWS;           // offset of the block inside its 64-centre tile
    const bool last_in_tile = (sub + c) == TILE - 1;
    const __amdgpu_buffer_rsrc_t frs = make_rsrc(feat_, feat_bytes);
    const v4u *wfrag = static_cast<const v4u *>(w_) + lane;
    const uint32_t *runs = side.run_start + (size_t)tile * K * TILE + sub + c;
    const uint32_t *tends = side.tile_ptr + tile + 1;

    // selection table: entry b (8 bits) -> eight bf16 values, element e = 1.0 if bit e of b is set
    for (int b = threadIdx.x; b < 256; b += NW * 64) {
        v4u v;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            v[q] = (((b >> (2 * q)) & 1) ? 0x3f80u : 0u) | (((b >> (2 * q + 1)) & 1) ? 0x3f800000u : 0u);
        sel_tab[b] = v;
    }

    // Run bounds of centre c in cell k (clamped to a valid cell; cells >= K are masked by the caller).
    auto load_runs = [&](int k, uint32_t &st, uint32_t &en) {
        const int kc = k < K ? k : K - 1;
        const uint32_t *pe = last_in_tile ? tends + (size_t)kc * side.n_tiles : runs + (size_t)kc * TILE + 1;
        st = runs[(size_t)kc * TILE];
        en = *pe;
    };
    // Software pipeline over this wave's cells k = wave, wave + NW, ...: run bounds are fetched two cells
    // ahead and the gather indices of the block's first 64 triplets one cell ahead of the rows.
    uint32_t st_c, en_c, st_n, en_n;
    load_runs(wave, st_c, en_c);
    load_runs(wave + NW, st_n, en_n);
    uint32_t bs_c = __builtin_amdgcn_readlane(st_c, 0);
    int32_t iv_c;
    {
        const uint32_t p = bs_c + lane;
        iv_c = gather[p < last_triplet ? p : last_triplet];
    }
    __syncthreads();                                 // selection table complete

    v16f acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[b][j] = 0.f;

    for (int k = wave; k < K; k += NW) {
        // prefetch: bounds of cell k + 2 NW, gather indices of cell k + NW
        uint32_t st_nn, en_nn;
        load_runs(k + 2 * NW, st_nn, en_nn);
        const uint32_t bs_n = __builtin_amdgcn_readlane(st_n, 0);
        int32_t iv_n;
        {
            const uint32_t p = bs_n + lane;
            iv_n = gather[p < last_triplet ? p : last_triplet];
        }
        const uint32_t cn_c = en_c - st_c;
        const uint32_t n = __builtin_amdgcn_readlane(en_c, 31) - bs_c;   // triplets of the block in cell k
        if (n != 0) {                                                    // wave-uniform
            // ---- stage 1: sums of the runs, groups of 64 triplets = 4 steps of 16 ------------------
            v16f d1[NS1];
#pragma unroll
            for (int s = 0; s < NS1; ++s)
#pragma unroll
                for (int j = 0; j < 16; ++j) d1[s][j] = 0.f;
            const int rel = (int)(st_c - bs_c);      // this centre's run, relative to the block's run
            int32_t ivc = iv_c;
            // W[k] fragments for stage 2, requested now so that they arrive during stage 1
            const v4u *wk = wfrag + (size_t)k * NB * NPC * 64;
            v4u bw[NB][NPC];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int pc = 0; pc < NPC; ++pc) bw[b][pc] = wk[(b * NPC + pc) * 64];
            for (uint32_t g0 = 0; g0 < n; g0 += 64) {
                if (g0 != 0) {                       // source rows of the next 64 triplets
                    const uint32_t p = bs_c + g0 + lane;
                    ivc = gather[p < last_triplet ? p : last_triplet];
                }
                // byte offset of triplet g0 + lane's source row, out of range past the end of the run
                const uint32_t offv = g0 + lane < n ? (uint32_t)ivc * ROWB : OOB_OFFSET;
                // bits of this centre's run inside the group: triplets [lo, hi) of the 64
                int lo = rel - (int)g0, hi = lo + (int)cn_c;
                lo = lo < 0 ? 0 : (lo > 64 ? 64 : lo);
                hi = hi < 0 ? 0 : (hi > 64 ? 64 : hi);
                const unsigned long long run_bits =
                    (hi >= 64 ? ~0ull : ((1ull << hi) - 1ull)) & ~(lo >= 64 ? ~0ull : ((1ull << lo) - 1ull));
                const uint32_t steps = n - g0 >= 64 ? 4u : (n - g0 + 15u) / 16u;   // wave-uniform
                // all loads of the group first: lane (c, h) reads dword column c (+32 g) of triplets 16 p + 8 h + e
                uint32_t xv[4][8][NG];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    if ((uint32_t)p < steps) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const uint32_t off = (uint32_t)__shfl((int)offv, 16 * p + 8 * h + e, 64) + (uint32_t)c * 4;
#pragma unroll
                            for (int g = 0; g < NG; ++g)
                                xv[p][e][g] = __builtin_amdgcn_raw_buffer_load_b32(frs, (int)(off + g * 128), 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    if ((uint32_t)p < steps) {
                        // selection operand: lane (centre c, h), element e = 1.0 when triplet 16 p + 8 h + e is in the run
                        const v8bf selv =
                            __builtin_bit_cast(v8bf, sel_tab[(uint32_t)(run_bits >> (16 * p + 8 * h)) & 0xffu]);
#pragma unroll
                        for (int g = 0; g < NG; ++g) {
                            if constexpr (BF16) {
                                v4u ev, od;
#pragma unroll
                                for (int q = 0; q < 4; ++q) {
                                    ev[q] = __builtin_amdgcn_perm(xv[p][2 * q + 1][g], xv[p][2 * q][g], 0x05040100u);
                                    od[q] = __builtin_amdgcn_perm(xv[p][2 * q + 1][g], xv[p][2 * q][g], 0x07060302u);
                                }
                                d1[2 * g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, ev), selv, d1[2 * g], 0, 0, 0);
                                d1[2 * g + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, od), selv, d1[2 * g + 1], 0, 0, 0);
                            } else {
                                // x = x1 + x2 + x3 exactly, each term a bf16 (8 significant bits)
                                v4u p1, p2, p3;
                                uint32_t a1[8], a2[8], a3[8];
#pragma unroll
                                for (int e = 0; e < 8; ++e) {
                                    const float x = __uint_as_float(xv[p][e][g]);
                                    a1[e] = xv[p][e][g] & 0xffff0000u;
                                    const float r1 = x - __uint_as_float(a1[e]);
                                    a2[e] = __float_as_uint(r1) & 0xffff0000u;
                                    a3[e] = __float_as_uint(r1 - __uint_as_float(a2[e]));
                                }
#pragma unroll
                                for (int q = 0; q < 4; ++q) {
                                    p1[q] = __builtin_amdgcn_perm(a1[2 * q + 1], a1[2 * q], 0x07060302u);
                                    p2[q] = __builtin_amdgcn_perm(a2[2 * q + 1], a2[2 * q], 0x07060302u);
                                    p3[q] = __builtin_amdgcn_perm(a3[2 * q + 1], a3[2 * q], 0x07060302u);
                                }
                                d1[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, p1), selv, d1[g], 0, 0, 0);
                                d1[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, p2), selv, d1[g], 0, 0, 0);
                                d1[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, p3), selv, d1[g], 0, 0, 0);
                            }
                        }
                    }
                }
            }

            // ---- stage 2: acc += S_k . W[k]^T; d1[s][j] of lane (centre, h) is channel column 8 (j/4) + 4 h + j%4 ----
            if constexpr (BF16) {
#pragma unroll
                for (int s = 0; s < NS1; ++s)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        v4u a;
#pragma unroll
                        for (int q = 0; q < 4; ++q) a[q] = cvt_pk_bf16(d1[s][8 * s2 + 2 * q], d1[s][8 * s2 + 2 * q + 1]);
#pragma unroll
                        for (int b = 0; b < NB; ++b)
                            acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, bw[b][s * 2 + s2]), acc[b], 0, 0, 0);
                    }
            } else {
#pragma unroll
                for (int g = 0; g < NG; ++g)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
#pragma unroll
                            for (int b = 0; b < NB; ++b)
                                acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(d1[g][4 * v + e],
                                                                              __uint_as_float(bw[b][g * 4 + v][e]), acc[b], 0, 0, 0);
            }
        }
        // rotate the pipeline
        st_c = st_n; en_c = en_n; bs_c = bs_n; iv_c = iv_n;
        st_n = st_nn; en_n = en_nn;
    }

    // add the waves' accumulators in wave order, wave 0 writes the rows
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
                if constexpr (sizeof(TOut) == 4) dst[(size_t)row * C_DST + b * 32 + c] = v;
                else dst[(size_t)row * C_DST + b * 32 + c] = (uint16_t)(cvt_pk_bf16(v, 0.f) & 0xffffu);
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Wide layers (bf16, C_SRC a multiple of 64 with at least 3 chunks, any K): W[k] is too large to be
// re-read per 32 centres, so a block of eight waves owns 256 consecutive centres (32 per wave) and
// shares W through LDS.  The work is a sequence of steps (active cell k, 64-channel chunk c of the
// source row).  Per step every wave runs stage 1 on the matching 128-byte slice of its triplets'
// source rows and stage 2 against the 64 x C_DST slice of W[k] held in one of two LDS buffers.
// Everything a step needs was requested one step earlier: the W slice (global -> registers -> LDS),
// the first 32 triplets' row slices, and -- spread over a cell's chunks -- the run bounds and gather
// indices of the next active cell.  One barrier per step; cells without a triplet among the block's
// 256 centres are skipped by the whole block.
//   packed W: piece (((k*NCH + c)*NB + b)*4 + v)*64 + lane = W(k, b*32 + lane%32, packed_channel(c*4 + v, lane/32, e))
// ---------------------------------------------------------------------------------------------
constexpr int WIDE_WAVES = 8;

__global__ void pack_w_wide_kernel(const uint16_t *__restrict__ w, uint16_t *__restrict__ packed, int K, int c_src,
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
    const uint16_t *src = w + (size_t)k * c_dst * c_src + (size_t)d * stride_d;
    uint16_t *dstp = packed + piece * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) dstp[e] = src[(size_t)packed_channel<true>(c * 4 + v, lane >> 5, e) * stride_s];
}

template <int C_SRC, int C_DST, typename TOut>
__global__ __launch_bounds__(WIDE_WAVES * 64) void rows_wide_kernel(const void *__restrict__ feat_,
                                                                    const void *__restrict__ w_, TOut *__restrict__ dst,
                                                                    int64_t n_centres, int K,
                                                                    const int32_t *__restrict__ gather,
                                                                    uint32_t last_triplet, uint32_t feat_bytes,
                                                                    PlanSideView side)
{
    constexpr uint32_t ROWB = C_SRC * 2;
    constexpr int NCH = C_SRC / 64;                  // source chunks of 32 dwords
    constexpr int NB = C_DST / 32;                   // destination blocks
    constexpr int PIECES = NB * 4 * 64;              // 16-byte pieces of one W slice
    constexpr int PPT = PIECES / (WIDE_WAVES * 64);  // pieces copied per thread
    static_assert(NCH >= 3 && PPT >= 1, "shape not supported by the wide kernel");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    v4u *wbuf = reinterpret_cast<v4u *>(lds);                    // [2][PIECES]
    v4u *sel_tab = wbuf + 2 * PIECES;                            // [256]
    int *act = reinterpret_cast<int *>(sel_tab + 256);           // [256] active cells, [256] = their number
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int64_t blk = (int64_t)blockIdx.x * WIDE_WAVES + wave;  // 32-centre block of this wave
    const int64_t row0 = blk * ROWS;
    const bool valid = row0 < n_centres;                          // wave-uniform
    int64_t tile = blk >> 1;
    if (tile >= side.n_tiles) tile = side.n_tiles - 1;
    const int sub = (int)(blk & 1) * ROWS;
    const bool last_in_tile = (sub + c) == TILE - 1;
    const __amdgpu_buffer_rsrc_t frs = make_rsrc(feat_, feat_bytes);
    const v4u *wsrc = static_cast<const v4u *>(w_) + threadIdx.x;
    const uint32_t *runs = side.run_start + (size_t)tile * K * TILE + sub + c;
    const uint32_t *tends = side.tile_ptr + tile + 1;
    const int64_t t0 = (int64_t)blockIdx.x * (WIDE_WAVES / 2);
    const int64_t t1 = t0 + WIDE_WAVES / 2 < side.n_tiles ? t0 + WIDE_WAVES / 2 : side.n_tiles;

    for (int b = threadIdx.x; b < 256; b += WIDE_WAVES * 64) {
        v4u v;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            v[q] = (((b >> (2 * q)) & 1) ? 0x3f80u : 0u) | (((b >> (2 * q + 1)) & 1) ? 0x3f800000u : 0u);
        sel_tab[b] = v;
    }
    if (wave == 0) {                                              // cells with a triplet among the 256 centres
        int cnt = 0;
        for (int kb = 0; kb < K; kb += 64) {
            const int k = kb + lane;
            const bool a = k < K && side.tile_ptr[(size_t)k * side.n_tiles + t0] != side.tile_ptr[(size_t)k * side.n_tiles + t1];
            const unsigned long long m = __ballot(a);
            if (a) act[cnt + __popcll(m & ((1ull << lane) - 1ull))] = k;
            cnt += __popcll(m);
        }
        if (lane == 0) act[256] = cnt;
    }
    __syncthreads();
    const int n_act = act[256];
    const int total_steps = n_act * NCH;

    auto load_runs = [&](int k, uint32_t &st, uint32_t &en) {
        const uint32_t *pe = last_in_tile ? tends + (size_t)k * side.n_tiles : runs + (size_t)k * TILE + 1;
        st = runs[(size_t)k * TILE];
        en = *pe;
    };
    auto row_offsets = [&](int32_t iv, uint32_t n) -> uint32_t {   // byte offset of triplet `lane`'s source row
        return (uint32_t)lane < n ? (uint32_t)iv * ROWB : OOB_OFFSET;
    };

    v16f acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[b][j] = 0.f;

    if (total_steps > 0) {
        // first active cell, unpipelined
        uint32_t st_c, en_c;
        load_runs(act[0], st_c, en_c);
        uint32_t bs_c = __builtin_amdgcn_readlane(st_c, 0);
        uint32_t n_c = valid ? __builtin_amdgcn_readlane(en_c, 31) - bs_c : 0u;
        uint32_t cn_c = valid ? en_c - st_c : 0u;
        uint32_t offv_c;
        {
            const uint32_t p = bs_c + lane;
            offv_c = row_offsets(gather[p < last_triplet ? p : last_triplet], n_c);
        }
        uint32_t st_n = 0, en_n = 0, bs_n = 0, n_n = 0;
        int32_t iv_n = 0;
        // W slice of step 0 and the first 32 triplets' row slices of step 0
        v4u wr[PPT];
#pragma unroll
        for (int q = 0; q < PPT; ++q) wr[q] = wsrc[(size_t)act[0] * NCH * PIECES + q * WIDE_WAVES * 64];
        uint32_t xa[2][8];
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                xa[p][e] = __builtin_amdgcn_raw_buffer_load_b32(
                    frs, (int)((uint32_t)__shfl((int)offv_c, 16 * p + 8 * h + e, 64) + (uint32_t)c * 4), 0, 0);

        for (int s = 0; s < total_steps; ++s) {
            const int j = s / NCH, ch = s % NCH;
            const int k = act[j];
            v4u *buf = wbuf + (size_t)(s & 1) * PIECES;
            // (1) this step's W slice into LDS, next step's slice requested
#pragma unroll
            for (int q = 0; q < PPT; ++q) buf[threadIdx.x + q * WIDE_WAVES * 64] = wr[q];
            if (s + 1 < total_steps) {
                const size_t nxt = ((size_t)act[(s + 1) / NCH] * NCH + (s + 1) % NCH) * PIECES;
#pragma unroll
                for (int q = 0; q < PPT; ++q) wr[q] = wsrc[nxt + q * WIDE_WAVES * 64];
            }
            // (2) next active cell: run bounds at chunk 0, gather indices at chunk 1, used from the last chunk on
            const bool more = j + 1 < n_act;
            if (ch == 0 && more) load_runs(act[j + 1], st_n, en_n);
            if (ch == 1 && more) {
                bs_n = __builtin_amdgcn_readlane(st_n, 0);
                n_n = valid ? __builtin_amdgcn_readlane(en_n, 31) - bs_n : 0u;
                const uint32_t p = bs_n + lane;
                iv_n = gather[p < last_triplet ? p : last_triplet];
            }
            uint32_t offv_n = OOB_OFFSET;
            if (ch == NCH - 1 && more) offv_n = row_offsets(iv_n, n_n);
            // (3) triplets 32..63 of this step (not prefetched) and the first 32 of the next step
            const uint32_t slice = (uint32_t)ch * 128 + (uint32_t)c * 4;
            uint32_t xe[2][8];
            if (n_c > 32) {
#pragma unroll
                for (int p = 0; p < 2; ++p)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        xe[p][e] = __builtin_amdgcn_raw_buffer_load_b32(
                            frs, (int)((uint32_t)__shfl((int)offv_c, 32 + 16 * p + 8 * h + e, 64) + slice), 0, 0);
            }
            uint32_t xb[2][8];
            {
                const uint32_t offv = ch == NCH - 1 ? offv_n : offv_c;
                const uint32_t nslice = (uint32_t)((ch + 1) % NCH) * 128 + (uint32_t)c * 4;
#pragma unroll
                for (int p = 0; p < 2; ++p)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        xb[p][e] = __builtin_amdgcn_raw_buffer_load_b32(
                            frs, (int)((uint32_t)__shfl((int)offv, 16 * p + 8 * h + e, 64) + nslice), 0, 0);
            }
            // (4) stage 1: sums of the runs for this 64-channel slice
            v16f d1[2];
#pragma unroll
            for (int par = 0; par < 2; ++par)
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) d1[par][jj] = 0.f;
            if (n_c != 0) {
                const int rel = (int)(st_c - bs_c);
                auto run_window = [&](uint32_t g0) -> unsigned long long {
                    int lo = rel - (int)g0, hi = lo + (int)cn_c;
                    lo = lo < 0 ? 0 : (lo > 64 ? 64 : lo);
                    hi = hi < 0 ? 0 : (hi > 64 ? 64 : hi);
                    return (hi >= 64 ? ~0ull : ((1ull << hi) - 1ull)) & ~(lo >= 64 ? ~0ull : ((1ull << lo) - 1ull));
                };
                auto sel_step = [&](const uint32_t (&x)[8], unsigned long long bits, int p) {
                    const v8bf selv = __builtin_bit_cast(v8bf, sel_tab[(uint32_t)(bits >> (16 * p + 8 * h)) & 0xffu]);
                    v4u ev, od;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        ev[q] = __builtin_amdgcn_perm(x[2 * q + 1], x[2 * q], 0x05040100u);
                        od[q] = __builtin_amdgcn_perm(x[2 * q + 1], x[2 * q], 0x07060302u);
                    }
                    d1[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, ev), selv, d1[0], 0, 0, 0);
                    d1[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, od), selv, d1[1], 0, 0, 0);
                };
                const unsigned long long bits0 = run_window(0);
                sel_step(xa[0], bits0, 0);
                if (n_c > 16) sel_step(xa[1], bits0, 1);
                if (n_c > 32) sel_step(xe[0], bits0, 2);
                if (n_c > 48) sel_step(xe[1], bits0, 3);
                for (uint32_t g0 = 64; g0 < n_c; g0 += 64) {     // rare: more than 64 triplets of the block in one cell
                    const uint32_t p = bs_c + g0 + lane;
                    const uint32_t offv = g0 + lane < n_c ? (uint32_t)gather[p < last_triplet ? p : last_triplet] * ROWB
                                                          : OOB_OFFSET;
                    const unsigned long long bits = run_window(g0);
#pragma unroll
                    for (int p4 = 0; p4 < 4; ++p4) {
                        if (g0 + 16 * p4 < n_c) {
                            uint32_t x[8];
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                x[e] = __builtin_amdgcn_raw_buffer_load_b32(
                                    frs, (int)((uint32_t)__shfl((int)offv, 16 * p4 + 8 * h + e, 64) + slice), 0, 0);
                            sel_step(x, bits, p4);
                        }
                    }
                }
            }
            v4u a[4];
#pragma unroll
            for (int par = 0; par < 2; ++par)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        a[par * 2 + s2][q] = cvt_pk_bf16(d1[par][8 * s2 + 2 * q], d1[par][8 * s2 + 2 * q + 1]);
            __syncthreads();                                      // the W slice is complete in LDS
            // (5) stage 2 against the shared slice
            if (n_c != 0) {
                const v4u *bl = buf + lane;
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a[v]),
                                                                         __builtin_bit_cast(v8bf, bl[(b * 4 + v) * 64]),
                                                                         acc[b], 0, 0, 0);
            }
            // (6) rotate
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int e = 0; e < 8; ++e) xa[p][e] = xb[p][e];
            if (ch == NCH - 1 && more) {
                st_c = st_n; en_c = en_n; bs_c = bs_n; n_c = n_n;
                cn_c = valid ? en_c - st_c : 0u;
                offv_c = offv_n;
            }
            (void)k;
        }
    }
    if (!valid) return;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t row = row0 + 8 * (j / 4) + 4 * h + (j % 4);
            if (row < n_centres) {
                if constexpr (sizeof(TOut) == 4) dst[(size_t)row * C_DST + b * 32 + c] = acc[b][j];
                else dst[(size_t)row * C_DST + b * 32 + c] = (uint16_t)(cvt_pk_bf16(acc[b][j], 0.f) & 0xffffu);
            }
        }
}

template <int C_SRC, int C_DST>
int launch_wide(const MvmrArgs &a, hipStream_t stream)
{
    const int64_t blocks = ceil_div(ceil_div(a.n_centres, ROWS), WIDE_WAVES);
    const size_t lds = (size_t)2 * (C_DST / 32) * 4 * 64 * 16 + 256 * 16 + 257 * sizeof(int);
    const uint32_t last = (uint32_t)(a.n_triplets - 1);
    const uint32_t feat_bytes = (uint32_t)((size_t)a.n_src * C_SRC * 2);
    if (a.out_dtype == PCPP_F32) {
        auto kern = rows_wide_kernel<C_SRC, C_DST, float>;
        PCPP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        kern<<<(unsigned)blocks, WIDE_WAVES * 64, lds, stream>>>(a.feat, a.w, static_cast<float *>(a.dst), a.n_centres,
                                                                 a.K, a.gather, last, feat_bytes, a.side);
    } else {
        auto kern = rows_wide_kernel<C_SRC, C_DST, uint16_t>;
        PCPP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        kern<<<(unsigned)blocks, WIDE_WAVES * 64, lds, stream>>>(a.feat, a.w, static_cast<uint16_t *>(a.dst),
                                                                 a.n_centres, a.K, a.gather, last, feat_bytes, a.side);
    }
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

bool wide_shape(const MvmrArgs &a) { return a.in_dtype == PCPP_BF16 && a.c_src == 256 && a.c_dst == 256; }

template <bool BF16, int C_SRC, int C_DST, int NW>
int launch(const MvmrArgs &a, hipStream_t stream)
{
    const int64_t blocks = ceil_div(a.n_centres, ROWS);
    const size_t lds = (size_t)(NW - 1) * (C_DST / 32) * 16 * 64 * sizeof(float) + 256 * 16;
    const uint32_t last = (uint32_t)(a.n_triplets - 1);
    const uint32_t feat_bytes = (uint32_t)((size_t)a.n_src * C_SRC * (BF16 ? 2 : 4));
    if (a.out_dtype == PCPP_F32) {
        rows_kernel<BF16, C_SRC, C_DST, NW, float><<<(unsigned)blocks, NW * 64, lds, stream>>>(
            a.feat, a.w, static_cast<float *>(a.dst), a.n_centres, a.K, a.gather, last, feat_bytes, a.side);
    } else {
        rows_kernel<BF16, C_SRC, C_DST, NW, uint16_t><<<(unsigned)blocks, NW * 64, lds, stream>>>(
            a.feat, a.w, static_cast<uint16_t *>(a.dst), a.n_centres, a.K, a.gather, last, feat_bytes, a.side);
    }
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

template <bool BF16, int C_SRC, int C_DST>
int launch_k(const MvmrArgs &a, hipStream_t stream)
{
    static const int nw = [] { const char *e = getenv("PCPP_ROWS_NW"); return e ? atoi(e) : 2; }();
    if (nw == 8) return launch<BF16, C_SRC, C_DST, 8>(a, stream);
    if (nw == 2) return launch<BF16, C_SRC, C_DST, 2>(a, stream);
    if (nw == 1) return launch<BF16, C_SRC, C_DST, 1>(a, stream);
    return launch<BF16, C_SRC, C_DST, 4>(a, stream);
}

}  // namespace

bool mvmr_rows_sel_supported(const MvmrArgs &a)
{
    if (a.n_triplets <= 0) return false;
    const size_t es = a.in_dtype == PCPP_BF16 ? 2 : 4;
    if ((size_t)a.n_src * a.c_src * es > MAX_BUFFER_BYTES) return false;
    if (wide_shape(a)) return true;
    if (a.K > 64) return false;                      // narrow layers with many cells: generic path
    if (a.in_dtype == PCPP_F32 && a.out_dtype == PCPP_F32)
        return (a.c_src == 32 && a.c_dst == 32) || (a.c_src == 64 && a.c_dst == 64);
    if (a.in_dtype == PCPP_BF16)
        return (a.c_src == 64 && a.c_dst == 64) || (a.c_src == 64 && a.c_dst == 128) || (a.c_src == 128 && a.c_dst == 64);
    return false;
}

int mvmr_rows_sel_pack_w(const void *w, void *packed, int K, int c_src, int c_dst, int stride_d, int stride_s,
                         int dtype, hipStream_t stream)
{
    const int e = dtype == PCPP_BF16 ? 8 : 4;
    const int64_t total = (int64_t)K * (c_dst / 32) * (c_src / e / 2) * 64;
    const unsigned blocks = (unsigned)ceil_div(total, 256);
    if (dtype == PCPP_BF16 && c_src == 256 && c_dst == 256) {
        pack_w_wide_kernel<<<blocks, 256, 0, stream>>>(static_cast<const uint16_t *>(w), static_cast<uint16_t *>(packed),
                                                       K, c_src, c_dst, stride_d, stride_s);
        PCPP_HIP_CHECK(hipGetLastError());
        return PCPP_OK;
    }
    if (dtype == PCPP_BF16)
        pack_w_sel_kernel<uint16_t><<<blocks, 256, 0, stream>>>(static_cast<const uint16_t *>(w),
                                                                static_cast<uint16_t *>(packed), K, c_src, c_dst,
                                                                stride_d, stride_s);
    else
        pack_w_sel_kernel<float><<<blocks, 256, 0, stream>>>(static_cast<const float *>(w),
                                                             static_cast<float *>(packed), K, c_src, c_dst, stride_d,
                                                             stride_s);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

// a.w must be the weights packed by mvmr_rows_sel_pack_w
int mvmr_rows_sel(const MvmrArgs &a, hipStream_t stream)
{
    if (wide_shape(a)) return launch_wide<256, 256>(a, stream);
    if (a.in_dtype == PCPP_F32) {
        if (a.c_src == 32 && a.c_dst == 32) return launch_k<false, 32, 32>(a, stream);
        if (a.c_src == 64 && a.c_dst == 64) return launch_k<false, 64, 64>(a, stream);
    } else {
        if (a.c_src == 64 && a.c_dst == 64) return launch_k<true, 64, 64>(a, stream);
        if (a.c_src == 64 && a.c_dst == 128) return launch_k<true, 64, 128>(a, stream);
        if (a.c_src == 128 && a.c_dst == 64) return launch_k<true, 128, 64>(a, stream);
    }
    set_error("mvmr_rows_sel: unsupported shape");
    return PCPP_ERR_UNSUPPORTED;
}

}  // namespace pcpp
