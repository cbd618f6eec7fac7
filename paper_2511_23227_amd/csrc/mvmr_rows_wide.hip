// MVMR rows kernel for wide layers (Eq. (1) forward; Sec. 3.3.3 input gradient with W^T): the run sums and the
// product with W[k] both on the matrix cores, W shared by 256 centres through LDS.
//
// Compiled with MFMA results selected into ordinary vector registers by default: the 256 accumulator
// registers of stage 2 then move to the accumulation half of the register file while the short-lived
// stage-1 results stay beside their consumers.
#include "mvmr_rows_common.h"

namespace pcpp {

namespace {

// ---------------------------------------------------------------------------------------------
// Wide layers (bf16, 256 -> 256 channels, any K): W[k] is too large to be re-read per 32 centres, so a
// block of four waves -- one per SIMD, 512 registers per lane, the accumulators in the upper half --
// owns 256 consecutive centres (one 64-centre tile = two 32-centre sub-blocks per wave) and shares W
// through LDS.  The work is a sequence of steps (active cell k, 64-channel chunk of the source row).
// Per step every wave runs stage 1 on the matching 128-byte slice of its triplets' source rows and
// stage 2 against the 64 x C_DST slice of W[k] held in one of two LDS buffers; a W fragment read from
// LDS feeds four MFMAs.  Everything a step needs was requested one step earlier: the W slice (global ->
// registers -> LDS), the row slices of the first 64 triplets of either sub-block (a ring of two
// 32-triplet slots per sub-block, each refilled as soon as it has been consumed) and -- spread over a
// cell's chunks -- the run bounds and gather indices of the next active cell.  One barrier per step;
// cells without a triplet among the block's 256 centres are skipped by the whole block.
//
// Both stages use v_mfma_f32_16x16x32_bf16 (A: lane (M = l%16, g = l/16) holds A[M][8g .. 8g+7]; B: lane
// (N = l%16, g) holds B[8g .. 8g+7][N]; D: lane l, register j -> M = 4g + j, N = l%16), which lets a
// lane read 8 bytes (four channels) of a row: 16 lanes cover the 128-byte slice of one triplet and one
// load instruction covers four triplets.
//   stage 1, pass of 32 triplets: lane (m, g), load i reads channels 4m .. 4m+3 of triplet 8g + i; MFMA q
//       (q = 0..3) takes channel 4m + q as A[m][8g + i] against Sel^T[8g + i][centre]; its D register j of
//       lane (centre, g) is the run sum of channel 16g + 4j + q.
//   stage 2: A[centre][8g + e] = run sum of channel 16g + 8 kap + e (kap = 0, 1), two MFMAs per 64-channel
//       chunk and 16 destination channels.
//   packed W: piece ((((k*NCH + ch)*NDB + db)*2 + kap)*64 + lane), element e
//             = W(k, dst 16 db + lane%16, src 64 ch + 16 (lane/16) + 8 kap + e)
// Blocks are renumbered so that the blocks resident on one XCD (block index modulo 8) cover a contiguous
// range of centres: neighbouring centres share source rows, which then meet in that XCD's L2.
// ---------------------------------------------------------------------------------------------
constexpr int WIDE_WAVES = 4;
constexpr int WIDE_ROWS = WIDE_WAVES * TILE;     // centres per block
constexpr int NUM_XCD = 8;

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

__global__ void pack_w_wide_kernel(const uint16_t *__restrict__ w, uint16_t *__restrict__ packed, int K, int c_src,
                                   int c_dst, int stride_d, int stride_s)
{
    const int nch = c_src / 64, ndb = c_dst / 16;
    const int64_t total = (int64_t)K * nch * ndb * 2 * 64;
    const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (piece >= total) return;
    const int lane = (int)(piece & 63);
    int64_t r = piece >> 6;
    const int kap = (int)(r & 1); r >>= 1;
    const int db = (int)(r % ndb); r /= ndb;
    const int ch = (int)(r % nch);
    const int k = (int)(r / nch);
    const int d = db * 16 + (lane & 15);
    const int s0 = ch * 64 + 16 * (lane >> 4) + 8 * kap;
    const uint16_t *src = w + (size_t)k * c_dst * c_src + (size_t)d * stride_d;
    uint16_t *dstp = packed + piece * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) dstp[e] = src[(size_t)(s0 + e) * stride_s];
}

// acc[sb][half][db] += A(sub-block sb, half) . W fragment, for the sub-blocks that have triplets in the cell
template <bool HAS0, bool HAS1, int NDB>
__device__ inline void wide_stage2(v4f (&acc)[2][2][NDB], const v4u (&a)[2][2][2], const v4u *bl)
{
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int kap = 0; kap < 2; ++kap) {
            const v8bf bw = __builtin_bit_cast(v8bf, bl[(db * 2 + kap) * 64]);
            if constexpr (HAS0) {
                acc[0][0][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a[0][0][kap]), bw, acc[0][0][db], 0, 0, 0);
                acc[0][1][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a[0][1][kap]), bw, acc[0][1][db], 0, 0, 0);
            }
            if constexpr (HAS1) {
                acc[1][0][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a[1][0][kap]), bw, acc[1][0][db], 0, 0, 0);
                acc[1][1][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a[1][1][kap]), bw, acc[1][1][db], 0, 0, 0);
            }
        }
}

template <int C_SRC, int C_DST, typename TOut>
__global__ __launch_bounds__(WIDE_WAVES * 64) void rows_wide_kernel(const void *__restrict__ feat_,
                                                                    const void *__restrict__ w_, TOut *__restrict__ dst,
                                                                    int64_t n_centres, int K,
                                                                    const int32_t *__restrict__ gather,
                                                                    uint32_t last_triplet, uint32_t feat_bytes,
                                                                    PlanSideView side, int64_t n_blocks)
{
    constexpr uint32_t ROWB = C_SRC * 2;
    constexpr int NCH = C_SRC / 64;                  // 64-channel chunks of a source row
    constexpr int NDB = C_DST / 16;                  // destination blocks of 16 channels
    constexpr int PIECES = NDB * 2 * 64;             // 16-byte pieces of one W slice
    constexpr int PPT = PIECES / (WIDE_WAVES * 64);  // pieces copied per thread
    static_assert(NCH >= 3 && PPT >= 1, "shape not supported by the wide kernel");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    v4u *wbuf = reinterpret_cast<v4u *>(lds);                    // [2][PIECES]
    v4u *sel_tab = wbuf + 2 * PIECES;                            // [256]
    int *act = reinterpret_cast<int *>(sel_tab + 256);           // [256] active cells, [256] = their number
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int64_t per_xcd = gridDim.x / NUM_XCD;
    const int64_t vb = (int64_t)(blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
    if (vb >= n_blocks) return;                                   // whole block, before any barrier
    const int64_t t0 = vb * WIDE_WAVES;
    const int64_t t1 = t0 + WIDE_WAVES < side.n_tiles ? t0 + WIDE_WAVES : side.n_tiles;
    const bool wvalid = t0 + wave < side.n_tiles;                 // wave-uniform: the wave's tile exists
    const int64_t tile = wvalid ? t0 + wave : side.n_tiles - 1;
    const int64_t row0 = (t0 + wave) * TILE;
    const __amdgpu_buffer_rsrc_t frs = make_rsrc(feat_, feat_bytes);
    const v4u *wsrc = static_cast<const v4u *>(w_) + threadIdx.x;
    const uint32_t *runs = side.run_start + (size_t)tile * K * TILE + lane;
    const uint32_t *tends = side.tile_ptr + tile + 1;

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

    v4f acc[2][2][NDB];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int db = 0; db < NDB; ++db) acc[sb][hf][db] = v4f{0.f, 0.f, 0.f, 0.f};

    if (total_steps > 0) {
        // A cell as seen by this wave: per sub-block the start bs and length cnt of its triplet list, and for
        // the two centres this lane serves as selection column (n and 16 + n of the sub-block) the run
        // [rel, rel + len) inside that list.
        struct Cell {
            uint32_t bs[2], cnt[2];
            int rel[2][2];
            uint32_t len[2][2];
        };
        // st: start of the run of centre `lane` of the tile; tend: end of the tile's triplets in the cell
        auto describe = [&](uint32_t st, uint32_t tend, Cell &c) {
            const uint32_t te = __builtin_amdgcn_readfirstlane(tend);
            const uint32_t nx = (uint32_t)__shfl((int)st, (lane + 1) & 63, 64);
            const uint32_t en = lane == 63 ? te : nx;
            c.bs[0] = __builtin_amdgcn_readlane(st, 0);
            c.bs[1] = __builtin_amdgcn_readlane(st, 32);
            c.cnt[0] = wvalid ? c.bs[1] - c.bs[0] : 0u;
            c.cnt[1] = wvalid ? te - c.bs[1] : 0u;
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const int src = 32 * sb + 16 * hf + n;
                    const uint32_t s = (uint32_t)__shfl((int)st, src, 64), e = (uint32_t)__shfl((int)en, src, 64);
                    c.rel[sb][hf] = (int)(s - c.bs[sb]);
                    c.len[sb][hf] = e - s;
                }
        };
        // byte offset of the source row of triplet first + lane, out of range past the end of the list
        auto row_offsets = [&](uint32_t first, uint32_t left) -> uint32_t {
            const uint32_t p = first + lane;
            const int32_t iv = gather[p < last_triplet ? p : last_triplet];
            return (uint32_t)lane < left ? ((uint32_t)iv & GATHER_INDEX) * ROWB : OOB_OFFSET;
        };
        // triplets [lo, lo + len) of a run as a bit mask over the 64 triplets starting at g0
        auto run_window = [&](int rel, uint32_t len, uint32_t g0) -> unsigned long long {
            int lo = rel - (int)g0, hi = lo + (int)len;
            lo = lo < 0 ? 0 : (lo > 64 ? 64 : lo);
            hi = hi < 0 ? 0 : (hi > 64 ? 64 : hi);
            return (hi >= 64 ? ~0ull : ((1ull << hi) - 1ull)) & ~(lo >= 64 ? ~0ull : ((1ull << lo) - 1ull));
        };
        // pass p (32 triplets) of a group of 64: lane (m, g), load i <- channels 4m .. 4m+3 of triplet 32p + 8g + i
        auto refill = [&](v2u (&x)[8], uint32_t offv, int p, uint32_t slice) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                x[i] = __builtin_amdgcn_raw_buffer_load_b64(
                    frs, (int)((uint32_t)__shfl((int)offv, 32 * p + 8 * g + i, 64) + slice), 0, 0);
        };

        Cell cur;
        describe(runs[(size_t)act[0] * TILE], tends[(size_t)act[0] * side.n_tiles], cur);
        uint32_t off0[2], off1[2];                   // row offsets of triplets lane and 64 + lane of either list
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            off0[sb] = row_offsets(cur.bs[sb], cur.cnt[sb]);
            off1[sb] = cur.cnt[sb] > 64 ? row_offsets(cur.bs[sb] + 64, cur.cnt[sb] - 64) : OOB_OFFSET;
        }
        v2u xq[2][2][8];                             // [sub-block][slot][load]
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
#pragma unroll
                for (int i = 0; i < 8; ++i) xq[sb][p][i] = v2u{0u, 0u};
                if (cur.cnt[sb] > 32u * p) refill(xq[sb][p], off0[sb], p, (uint32_t)n * 8);
            }
        v4u wr[PPT];
#pragma unroll
        for (int q = 0; q < PPT; ++q) wr[q] = wsrc[(size_t)act[0] * NCH * PIECES + q * WIDE_WAVES * 64];
        uint32_t st_n = 0, tend_n = 0;               // next active cell: bounds as loaded, list starts and lengths
        uint32_t nbs[2] = {0u, 0u}, ncnt[2] = {0u, 0u};
        uint32_t noff0[2] = {OOB_OFFSET, OOB_OFFSET}, noff1[2] = {OOB_OFFSET, OOB_OFFSET};

        for (int s = 0; s < total_steps; ++s) {
            const int j = s / NCH, ch = s % NCH;
            const bool more = j + 1 < n_act, last_chunk = ch == NCH - 1;
            v4u *buf = wbuf + (size_t)(s & 1) * PIECES;
            // (1) this step's W slice into LDS, next step's slice requested
#pragma unroll
            for (int q = 0; q < PPT; ++q) buf[threadIdx.x + q * WIDE_WAVES * 64] = wr[q];
            if (s + 1 < total_steps) {
                const size_t nxt_slice = ((size_t)act[(s + 1) / NCH] * NCH + (s + 1) % NCH) * PIECES;
#pragma unroll
                for (int q = 0; q < PPT; ++q) wr[q] = wsrc[nxt_slice + q * WIDE_WAVES * 64];
            }
            // (2) next active cell: run bounds at chunk 0, lists and gather indices at chunk 1, used from the last chunk on
            if (ch == 0 && more) {
                const int kn = act[j + 1];
                st_n = runs[(size_t)kn * TILE];
                tend_n = tends[(size_t)kn * side.n_tiles];
            }
            if (ch == 1 && more) {
                const uint32_t te = __builtin_amdgcn_readfirstlane(tend_n);
                nbs[0] = __builtin_amdgcn_readlane(st_n, 0);
                nbs[1] = __builtin_amdgcn_readlane(st_n, 32);
                ncnt[0] = wvalid ? nbs[1] - nbs[0] : 0u;
                ncnt[1] = wvalid ? te - nbs[1] : 0u;
#pragma unroll
                for (int sb = 0; sb < 2; ++sb) {
                    noff0[sb] = row_offsets(nbs[sb], ncnt[sb]);
                    noff1[sb] = ncnt[sb] > 64 ? row_offsets(nbs[sb] + 64, ncnt[sb] - 64) : OOB_OFFSET;
                }
            }
            const bool to_next = last_chunk && more;
            const uint32_t slice = (uint32_t)ch * 128 + (uint32_t)n * 8;
            const uint32_t nslice = (uint32_t)((ch + 1) % NCH) * 128 + (uint32_t)n * 8;
            // (3) stage 1 per sub-block: sums of the runs for this 64-channel slice; every consumed slot is
            //     refilled with the next group of this step (lists longer than 64) or with the next step's rows
            v4u a[2][2][2];
#pragma unroll
            for (int sb = 0; sb < 2; ++sb) {
                const uint32_t cnt = cur.cnt[sb];
                const uint32_t f_off = last_chunk ? (more ? noff0[sb] : OOB_OFFSET) : off0[sb];
                const uint32_t f_cnt = last_chunk ? (more ? ncnt[sb] : 0u) : cnt;
                v4f d1[4][2];
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) d1[q][hf] = v4f{0.f, 0.f, 0.f, 0.f};
                for (uint32_t g0 = 0;; g0 += 64) {
                    const uint32_t rem = cnt - g0;                 // triplets from g0 on (cnt >= g0)
                    const bool again = rem > 64;                   // wave-uniform
                    uint32_t r_off = f_off, r_cnt = f_cnt, r_slice = nslice;
                    if (again) {
                        r_off = g0 == 0 ? off1[sb] : row_offsets(cur.bs[sb] + g0 + 64, rem - 64);
                        r_cnt = rem - 64;
                        r_slice = slice;
                    }
                    const unsigned long long m0 = run_window(cur.rel[sb][0], cur.len[sb][0], g0);
                    const unsigned long long m1 = run_window(cur.rel[sb][1], cur.len[sb][1], g0);
#pragma unroll
                    for (int p = 0; p < 2; ++p) {
                        if (rem > 32u * p) {
                            const v8bf sel0 = __builtin_bit_cast(v8bf, sel_tab[(uint32_t)(m0 >> (32 * p + 8 * g)) & 0xffu]);
                            const v8bf sel1 = __builtin_bit_cast(v8bf, sel_tab[(uint32_t)(m1 >> (32 * p + 8 * g)) & 0xffu]);
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                v4u av;
#pragma unroll
                                for (int wd = 0; wd < 4; ++wd)
                                    av[wd] = __builtin_amdgcn_perm(xq[sb][p][2 * wd + 1][q >> 1], xq[sb][p][2 * wd][q >> 1],
                                                                   (q & 1) ? 0x07060302u : 0x05040100u);
                                d1[q][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, av), sel0, d1[q][0], 0, 0, 0);
                                d1[q][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, av), sel1, d1[q][1], 0, 0, 0);
                            }
                        }
                        if (r_cnt > 32u * p) refill(xq[sb][p], r_off, p, r_slice);
                    }
                    if (!again) break;
                }
                // A operands of stage 2: element e = 2 wd, 2 wd + 1 of slice kap is channel 16g + 8 kap + e
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                    for (int kap = 0; kap < 2; ++kap)
#pragma unroll
                        for (int wd = 0; wd < 4; ++wd)
                            a[sb][hf][kap][wd] = cvt_pk_bf16(d1[2 * (wd & 1)][hf][2 * kap + (wd >> 1)],
                                                             d1[2 * (wd & 1) + 1][hf][2 * kap + (wd >> 1)]);
            }
            __syncthreads();                                      // the W slice is complete in LDS
            // (4) stage 2 against the shared slice
            {
                const v4u *bl = buf + lane;
                const bool has0 = cur.cnt[0] != 0, has1 = cur.cnt[1] != 0;
                if (has0 && has1) wide_stage2<true, true, NDB>(acc, a, bl);
                else if (has0) wide_stage2<true, false, NDB>(acc, a, bl);
                else if (has1) wide_stage2<false, true, NDB>(acc, a, bl);
            }
            // (5) rotate to the next cell
            if (to_next) {
                describe(st_n, tend_n, cur);
#pragma unroll
                for (int sb = 0; sb < 2; ++sb) { off0[sb] = noff0[sb]; off1[sb] = noff1[sb]; }
            }
        }
    }
    if (!wvalid) return;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t slot = row0 + 32 * sb + 16 * hf + 4 * g + j;
                    if (slot < n_centres) {
                        const int64_t row = side.perm ? (int64_t)side.perm[slot] : slot;
                        const float v = acc[sb][hf][db][j];
                        if constexpr (sizeof(TOut) == 4) dst[(size_t)row * C_DST + db * 16 + n] = v;
                        else dst[(size_t)row * C_DST + db * 16 + n] = (uint16_t)(cvt_pk_bf16(v, 0.f) & 0xffffu);
                    }
                }
}

template <int C_SRC, int C_DST>
int launch_wide(const MvmrArgs &a, hipStream_t stream)
{
    const int64_t n_blocks = ceil_div(a.n_centres, WIDE_ROWS);
    const int64_t grid = ceil_div(n_blocks, NUM_XCD) * NUM_XCD;
    const size_t lds = (size_t)2 * (C_DST / 16) * 2 * 64 * 16 + 256 * 16 + 257 * sizeof(int);
    const uint32_t last = (uint32_t)(a.n_triplets - 1);
    const uint32_t feat_bytes = (uint32_t)((size_t)a.n_src * C_SRC * 2);
    if (a.out_dtype == PCPP_F32) {
        auto kern = rows_wide_kernel<C_SRC, C_DST, float>;
        if (int rc = raise_lds_limit(reinterpret_cast<const void *>(kern), lds)) return rc;
        kern<<<(unsigned)grid, WIDE_WAVES * 64, lds, stream>>>(a.feat, a.w, static_cast<float *>(a.dst), a.n_centres,
                                                               a.K, a.gather, last, feat_bytes, a.side, n_blocks);
    } else {
        auto kern = rows_wide_kernel<C_SRC, C_DST, uint16_t>;
        if (int rc = raise_lds_limit(reinterpret_cast<const void *>(kern), lds)) return rc;
        kern<<<(unsigned)grid, WIDE_WAVES * 64, lds, stream>>>(a.feat, a.w, static_cast<uint16_t *>(a.dst),
                                                               a.n_centres, a.K, a.gather, last, feat_bytes, a.side,
                                                               n_blocks);
    }
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

}  // namespace

bool mvmr_rows_wide_shape(const MvmrArgs &a) { return a.in_dtype == PCPP_BF16 && a.c_src == 256 && a.c_dst == 256; }

int mvmr_rows_wide_pack_w(const void *w, void *packed, int K, int c_src, int c_dst, int stride_d, int stride_s,
                          hipStream_t stream)
{
    const int64_t total = (int64_t)K * c_dst * c_src / 8;          // 16-byte pieces
    pack_w_wide_kernel<<<(unsigned)ceil_div(total, 256), 256, 0, stream>>>(
        static_cast<const uint16_t *>(w), static_cast<uint16_t *>(packed), K, c_src, c_dst, stride_d, stride_s);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

int mvmr_rows_wide(const MvmrArgs &a, hipStream_t stream) { return launch_wide<256, 256>(a, stream); }

}  // namespace pcpp
