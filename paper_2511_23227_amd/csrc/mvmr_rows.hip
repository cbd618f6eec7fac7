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
#include "mvmr_rows_common.h"

namespace pcpp {

namespace {

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

// fp32 layers whose stage 2 runs on the bf16 matrix cores: W is stored as three bf16 terms, W = w1 + w2 + w3
// exactly (8 + 8 + 8 significant bits).  Piece (k*NB + b)*(3*KS) + kap*3 + t, lane (dst = b*32 + lane%32,
// h = lane/32), element e = term t of W(k, dst, channel 8 (2 kap + e/4) + 4 h + e%4).
constexpr bool split_f32_shape(bool bf16, int c_src, int c_dst) { return !bf16 && c_src == 32 && c_dst == 32; }

__global__ void pack_w_split_kernel(const float *__restrict__ w, uint16_t *__restrict__ packed, int K, int c_src,
                                    int c_dst, int stride_d, int stride_s)
{
    const int nb = c_dst / 32, ks = c_src / 16;      // reduction steps of 16 channels
    const int64_t total = (int64_t)K * nb * ks * 3 * 64;
    const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (piece >= total) return;
    const int lane = (int)(piece & 63);
    int64_t r = piece >> 6;
    const int t = (int)(r % 3); r /= 3;
    const int kap = (int)(r % ks); r /= ks;
    const int b = (int)(r % nb);
    const int k = (int)(r / nb);
    const int d = b * 32 + (lane & 31), h = lane >> 5;
    const float *src = w + (size_t)k * c_dst * c_src + (size_t)d * stride_d;
    uint16_t *dstp = packed + piece * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float x = src[(size_t)(8 * (2 * kap + (e >> 2)) + 4 * h + (e & 3)) * stride_s];
        const uint32_t a1 = __float_as_uint(x) & 0xffff0000u;
        const float r1 = x - __uint_as_float(a1);
        const uint32_t a2 = __float_as_uint(r1) & 0xffff0000u;
        const uint32_t a3 = __float_as_uint(r1 - __uint_as_float(a2));
        dstp[e] = (uint16_t)((t == 0 ? a1 : (t == 1 ? a2 : a3)) >> 16);
    }
}

// Waves per SIMD the register allocation must leave room for: these layers are bound by memory latency and sit
// just above a register-count step without this (measured per shape; 128 -> 64 is better left alone).
constexpr int rows_min_waves(bool bf16, int c_src, int c_dst)
{
    return (!bf16 && c_src == 32 && c_dst == 32) ? 4 : ((bf16 && c_src == 64 && c_dst == 64) ? 3 : ((bf16 && c_src == 64 && c_dst == 128) ? 2 : 1));
}

// NWIN = windows of 64 triplets per (cell, block) whose gather indices are requested one cell ahead: 1, or 3 for clouds
// with many neighbours per cell, where the rows of the second and third window would otherwise wait for an index
// load on top of their own round trip.  (A variant of its own because the layers with few neighbours per cell sit at
// a register-count step and lose a wave per SIMD, or spill, to the four registers that the indices take.)
template <bool BF16, int C_SRC, int C_DST, int NW, int NWIN, typename TOut>
__global__ __launch_bounds__(NW * 64, rows_min_waves(BF16, C_SRC, C_DST)) void rows_kernel(const void *__restrict__ feat_, const void *__restrict__ w_,
                                                       TOut *__restrict__ dst, int64_t n_centres, int K,
                                                       const int32_t *__restrict__ gather, uint32_t last_triplet,
                                                       uint32_t feat_bytes, PlanSideView side)
{
    constexpr int DW = BF16 ? C_SRC / 2 : C_SRC;     // dwords per source row
    constexpr int NG = DW / 32;                      // lane c reads dword columns c + 32 g
    constexpr int NP = BF16 ? 2 : 1;                 // even / odd channel of a dword (bf16)
    constexpr int NS1 = NG * NP;                     // stage-1 accumulator blocks of 32 channels
    constexpr int NB = C_DST / 32;                   // destination blocks
    constexpr bool SPLIT = split_f32_shape(BF16, C_SRC, C_DST);   // fp32 stage 2 as products of bf16 terms
    constexpr int NPC = BF16 ? NS1 * 2 : (SPLIT ? 3 * (C_SRC / 16) : NG * 4);   // packed W pieces per (cell, destination block)
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
    // gather indices of the block's first, second and third 64 triplets in the cell (the later ones only when the
    // cell has that many: a load that is not needed still costs the layers with few neighbours per cell)
    int32_t iv_c, iw_c = 0, ix_c = 0;
    auto load_indices = [&](uint32_t bs, uint32_t n_cell, int32_t &iv, int32_t &iw, int32_t &ix) {
        const uint32_t p = bs + lane;
        iv = gather[p < last_triplet ? p : last_triplet];
        if (NWIN > 1 && n_cell > 64u) iw = gather[p + 64u < last_triplet ? p + 64u : last_triplet];      // wave-uniform
        if (NWIN > 1 && n_cell > 128u) ix = gather[p + 128u < last_triplet ? p + 128u : last_triplet];
    };
    load_indices(bs_c, (uint32_t)__builtin_amdgcn_readlane(en_c, 31) - bs_c, iv_c, iw_c, ix_c);
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
        int32_t iv_n, iw_n = 0, ix_n = 0;
        load_indices(bs_n, (uint32_t)__builtin_amdgcn_readlane(en_n, 31) - bs_n, iv_n, iw_n, ix_n);
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
            constexpr int NPC_EARLY = SPLIT ? NPC / 2 : NPC;   // the split form fetches its second half after stage 1
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int pc = 0; pc < NPC_EARLY; ++pc) bw[b][pc] = wk[(b * NPC + pc) * 64];
            for (uint32_t g0 = 0; g0 < n; g0 += 64) {
                if (NWIN > 1 && g0 == 64) {          // the second and third 64 triplets: asked for one cell ahead, so that
                    ivc = iw_c;                      // their rows do not wait for an index load on top of their own
                } else if (NWIN > 1 && g0 == 128) {
                    ivc = ix_c;
                } else if (g0 != 0) {                // source rows of the next 64 triplets
                    const uint32_t p = bs_c + g0 + lane;
                    ivc = gather[p < last_triplet ? p : last_triplet];
                }
                // byte offset of triplet g0 + lane's source row, out of range past the end of the run
                const uint32_t offv = g0 + lane < n ? ((uint32_t)ivc & GATHER_INDEX) * ROWB : OOB_OFFSET;
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
            } else if constexpr (SPLIT) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int pc = NPC_EARLY; pc < NPC; ++pc) bw[b][pc] = wk[(b * NPC + pc) * 64];
                // S = s1 + s2 + s3 and W = w1 + w2 + w3 exactly, each term a bf16; the six products of weight
                // 2^-16 or more relative to s1 w1 are accumulated in fp32, smallest first.  Registers 8 kap ..
                // 8 kap + 7 of lane (centre, h) are the channels 8 (2 kap + e/4) + 4 h + e%4 of reduction step kap.
                static_assert(NG == 1, "split stage 2 is written for 32 source channels");
#pragma unroll
                for (int kap = 0; kap < 2; ++kap) {
                    uint32_t t1[8], t2[8], t3[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float x = d1[0][8 * kap + j];
                        t1[j] = __float_as_uint(x) & 0xffff0000u;
                        const float r1 = x - __uint_as_float(t1[j]);
                        t2[j] = __float_as_uint(r1) & 0xffff0000u;
                        t3[j] = __float_as_uint(r1 - __uint_as_float(t2[j]));
                    }
                    v4u a1, a2, a3;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        a1[q] = __builtin_amdgcn_perm(t1[2 * q + 1], t1[2 * q], 0x07060302u);
                        a2[q] = __builtin_amdgcn_perm(t2[2 * q + 1], t2[2 * q], 0x07060302u);
                        a3[q] = __builtin_amdgcn_perm(t3[2 * q + 1], t3[2 * q], 0x07060302u);
                    }
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const v8bf w1 = __builtin_bit_cast(v8bf, bw[b][kap * 3 + 0]);
                        const v8bf w2 = __builtin_bit_cast(v8bf, bw[b][kap * 3 + 1]);
                        const v8bf w3 = __builtin_bit_cast(v8bf, bw[b][kap * 3 + 2]);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a3), w1, acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a1), w3, acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a2), w2, acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a2), w1, acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a1), w2, acc[b], 0, 0, 0);
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a1), w1, acc[b], 0, 0, 0);
                    }
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
        st_c = st_n; en_c = en_n; bs_c = bs_n; iv_c = iv_n; iw_c = iw_n; ix_c = ix_n;
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
            const int64_t slot = row0 + 8 * (j / 4) + 4 * h + (j % 4);
            if (slot < n_centres) {
                const int64_t row = side.perm ? (int64_t)side.perm[slot] : slot;
                if constexpr (sizeof(TOut) == 4) dst[(size_t)row * C_DST + b * 32 + c] = v;
                else dst[(size_t)row * C_DST + b * 32 + c] = (uint16_t)(cvt_pk_bf16(v, 0.f) & 0xffffu);
            }
        }
}

template <bool BF16, int C_SRC, int C_DST, int NW, int NWIN>
int launch(const MvmrArgs &a, hipStream_t stream)
{
    const int64_t blocks = ceil_div(a.n_centres, ROWS);
    const size_t lds = (size_t)(NW - 1) * (C_DST / 32) * 16 * 64 * sizeof(float) + 256 * 16;
    const uint32_t last = (uint32_t)(a.n_triplets - 1);
    const uint32_t feat_bytes = (uint32_t)((size_t)a.n_src * C_SRC * (BF16 ? 2 : 4));
    if (a.out_dtype == PCPP_F32) {
        rows_kernel<BF16, C_SRC, C_DST, NW, NWIN, float><<<(unsigned)blocks, NW * 64, lds, stream>>>(
            a.feat, a.w, static_cast<float *>(a.dst), a.n_centres, a.K, a.gather, last, feat_bytes, a.side);
    } else {
        rows_kernel<BF16, C_SRC, C_DST, NW, NWIN, uint16_t><<<(unsigned)blocks, NW * 64, lds, stream>>>(
            a.feat, a.w, static_cast<uint16_t *>(a.dst), a.n_centres, a.K, a.gather, last, feat_bytes, a.side);
    }
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

// two waves per block of 32 centres measured best on the benchmark scenes (one wave: too little in flight
// per block; four: more partial accumulators to add than work to share)
template <bool BF16, int C_SRC, int C_DST>
int launch_k(const MvmrArgs &a, hipStream_t stream)
{
    // (64 -> 128 and 128 -> 64: one wave per block measured 10 % and 3 % faster on the strided scene, forward and
    // input gradient -- twice the blocks, and no partial sums to add)
    constexpr int NW = (BF16 && ((C_SRC == 64 && C_DST == 128) || (C_SRC == 128 && C_DST == 64))) ? 1 : 2;
    // more than 48 triplets per (cell, block of 32 centres) on average: index windows ahead
    if (a.n_triplets * ROWS > 48 * a.n_centres * (int64_t)a.K) return launch<BF16, C_SRC, C_DST, NW, 3>(a, stream);
    return launch<BF16, C_SRC, C_DST, NW, 1>(a, stream);
}

}  // namespace

bool mvmr_rows_sel_supported(const MvmrArgs &a)
{
    if (a.n_triplets <= 0) return false;
    const size_t es = a.in_dtype == PCPP_BF16 ? 2 : 4;
    if ((size_t)a.n_src * a.c_src * es > MAX_BUFFER_BYTES) return false;
    if (mvmr_rows_wide_shape(a)) return true;
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
    if (dtype == PCPP_BF16 && c_src == 256 && c_dst == 256)
        return mvmr_rows_wide_pack_w(w, packed, K, c_src, c_dst, stride_d, stride_s, stream);
    if (split_f32_shape(dtype == PCPP_BF16, c_src, c_dst)) {
        const int64_t pieces = (int64_t)K * (c_dst / 32) * (c_src / 16) * 3 * 64;
        pack_w_split_kernel<<<(unsigned)ceil_div(pieces, 256), 256, 0, stream>>>(
            static_cast<const float *>(w), static_cast<uint16_t *>(packed), K, c_src, c_dst, stride_d, stride_s);
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
    if (mvmr_rows_wide_shape(a)) return mvmr_rows_wide(a, stream);
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
