// MVMR rows kernel for wide layers with separate producer and consumer waves (Eq. (1) forward; Sec. 3.3.3 input
// gradient with W^T).
//
// Eq. (1) is linear, so out[o] = sum_k W[k] S_k[o] with S_k[o] = the sum of x[i] over the (k, o) run.  A block owns
// 128 consecutive slots of the plan's centre order (two tiles) and walks the kernel cells that hold a triplet for
// any of them.  Per cell,
//   producer waves (four, one per SIMD; each serves 32 centres) gather the source rows of their centres' runs --
//       one 512-byte row per load instruction, lane <-> four channels -- add them up in fp32 on the vector ALUs,
//       round each run's sum to bf16 once and store it as row `centre` of an LDS tile S[128][C_src];
//   consumer waves (four, one per SIMD; each owns 64 destination channels of all 128 centres, 128 accumulator
//       registers) multiply the tile by their slice of W[k] on the matrix cores, acc += S . W[k]^T, in groups of 16
//       centres; groups in which no centre has a triplet in the cell are skipped (inside a group that is not, the
//       producers store rows of zeros for the centres without one).
// The two run one cell apart on two LDS tiles, one barrier per cell: while the matrix cores work on cell j the
// rows of cell j + 1 are in flight.  A consumer's W slice (64 x C_src of the 16.4 MB at K = 125) comes straight from
// memory / L2 into registers in fragment order, three 32-channel chunks ahead of its use (a ring of four); nothing
// but S goes through LDS.  A wave issues at most one instruction every four cycles, so the consumers' inner unit
// (one group of 16 centres x 32 source channels: four MFMAs, 64 cycles of the matrix pipe) holds little else: a
// test of the group's bit, the four MFMAs and one LDS read at a fixed offset that fetches the group's A piece of
// the next chunk; all waiting is one explicit instruction per chunk.  Every destination row is accumulated in registers across all cells and written once by its owner: no
// atomics, fixed summation order.
//
// v_mfma_f32_16x16x32_bf16 (A: lane (M = l%16, g = l/16) holds A[M][8g .. 8g+7]; B: lane (N = l%16, g) holds
// B[8g .. 8g+7][N]; D: lane l, register j -> M = 4g + j, N = l%16):
//   A = S[16 centres][32 channels], read from LDS as one 16-byte piece per lane (row pitch C_src * 2 + 16 bytes, which
//       spreads the sixteen rows of a piece over the banks);
//   B = W[k][16 destination channels][32 source channels], 16 bytes per lane from the packed copy
//       packed piece (((k * NQ + q) * NC32 + c) * 4 + cg) * 64 + lane, element e
//             = W(k, dst 64 q + 16 cg + lane%16, src 32 c + 8 (lane/16) + e)
// The gather array of the plan side must carry GATHER_LAST on the last triplet of every (cell, centre) run.
#include "mvmr_rows_common.h"

namespace pcpp {

namespace {

constexpr int PC_ROWS = 128;                      // centres per block
constexpr int PC_PROD = 4, PC_CONS = 4;           // producer and consumer waves
constexpr int PC_THREADS = (PC_PROD + PC_CONS) * 64;
constexpr int PC_GROUPS = PC_ROWS / 16;
constexpr int PC_SLOTS = 32;                      // rows a producer wave keeps in flight
constexpr int NUM_XCD = 8;

typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

__global__ void pack_w_pc_kernel(const uint16_t *__restrict__ w, uint16_t *__restrict__ packed, int K, int c_src,
                                 int c_dst, int stride_d, int stride_s)
{
    const int nch = c_src / 64, nq = c_dst / 64;
    const int64_t total = (int64_t)K * nq * nch * 2 * 4 * 64;
    const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (piece >= total) return;
    const int lane = (int)(piece & 63);
    int64_t r = piece >> 6;
    const int cg = (int)(r & 3); r >>= 2;
    const int ks = (int)(r & 1); r >>= 1;
    const int ch = (int)(r % nch); r /= nch;
    const int q = (int)(r % nq);
    const int k = (int)(r / nq);
    const int d = 64 * q + 16 * cg + (lane & 15);
    const int s0 = 64 * ch + 32 * ks + 8 * (lane >> 4);
    const uint16_t *src = w + (size_t)k * c_dst * c_src + (size_t)d * stride_d;
    uint16_t *dstp = packed + piece * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) dstp[e] = src[(size_t)(s0 + e) * stride_s];
}

// all LDS traffic of the waves done, then the block's barrier; the compiler keeps memory operations on their side
// of it.  (Deliberately no wait for outstanding global loads: the prefetches of both roles stay in flight.)
__device__ inline void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// c += a . b on the matrix cores, 16 x 16 x 32 bf16, with the accumulator pinned to the accumulation registers and
// updated in place: the 128 accumulator registers of a consumer wave then never compete with the operands for
// ordinary vector registers, whatever the control flow around the call looks like.
__device__ inline void mfma_16x16x32_acc(v4f &c, const v4u &a, const v4u &b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

template <int NCH, typename TOut>
__global__ __launch_bounds__(PC_THREADS) void rows_pc_kernel(const void *__restrict__ feat_, const void *__restrict__ w_,
                                                             TOut *__restrict__ dst, int64_t n_centres, int K,
                                                             const int32_t *__restrict__ gather, uint32_t last_triplet,
                                                             uint32_t feat_bytes, PlanSideView side, int64_t n_blocks)
{
    constexpr int C_SRC = 64 * NCH, C_DST = 64 * PC_CONS;
    constexpr uint32_t ROWB = C_SRC * 2;              // bytes of a source row
    constexpr uint32_t SROW = ROWB + 16;              // pitch of the LDS tile
    constexpr uint32_t SBUF = PC_ROWS * SROW;
    static_assert(C_SRC == 256, "a producer lane holds four channels: rows of 256 channels");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char *S = lds;                                                 // [2][PC_ROWS][SROW]
    uint32_t *hasrun = reinterpret_cast<uint32_t *>(lds + 2 * SBUF);   // [2][4]: bit c of word p = centre 32 p + c has a run
    int *act = reinterpret_cast<int *>(hasrun + 8);                // active cells, act[MAX_K] = their number
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t per_xcd = gridDim.x / NUM_XCD;
    const int64_t vb = (int64_t)(blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
    if (vb >= n_blocks) return;                                    // whole block, before any barrier
    const int64_t t0 = vb * (PC_ROWS / TILE);
    const int64_t t1 = t0 + PC_ROWS / TILE < side.n_tiles ? t0 + PC_ROWS / TILE : side.n_tiles;

    if (wave == 0) {                                               // cells with a triplet among the 128 centres
        int cnt = 0;
        for (int kb = 0; kb < K; kb += 64) {
            const int k = kb + lane;
            const bool a = k < K && side.tile_ptr[(size_t)k * side.n_tiles + t0] != side.tile_ptr[(size_t)k * side.n_tiles + t1];
            const unsigned long long m = __ballot(a);
            if (a) act[cnt + __popcll(m & ((1ull << lane) - 1ull))] = k;
            cnt += __popcll(m);
        }
        if (lane == 0) act[MAX_K] = cnt;
    }
    __syncthreads();
    const int n_act = act[MAX_K];

    if (wave < PC_PROD) {
        // ------------------------------------------------------------------------------------------------
        // producer: centres 32 p .. 32 p + 31 of the block
        // ------------------------------------------------------------------------------------------------
        const int p = wave;
        const int64_t tile = t0 + (p >> 1);
        const bool pvalid = tile < side.n_tiles;                   // wave-uniform
        const int64_t tl = pvalid ? tile : side.n_tiles - 1;
        const int cl = (p & 1) * 32 + (lane & 31);                 // this lane's centre inside the tile (lanes 32.. repeat)
        const uint32_t *runs = side.run_start + (size_t)tl * K * TILE + cl;
        const uint32_t *tends = side.tile_ptr + tl + 1;
        const bool last_in_tile = cl == TILE - 1;
        const __amdgpu_buffer_rsrc_t frs = make_rsrc(feat_, feat_bytes);
        char *Smine = S + (size_t)(32 * p) * SROW + lane * 8;

        // bounds of the runs of cell act[j] (clamped; steps past the end are masked by their callers)
        auto load_bounds = [&](int j, uint32_t &st, uint32_t &en) {
            const int k = act[j < n_act ? j : (n_act > 0 ? n_act - 1 : 0)];
            st = runs[(size_t)k * TILE];
            en = last_in_tile ? tends[(size_t)k * side.n_tiles] : runs[(size_t)k * TILE + 1];
        };
        // gather words of triplets first + lane (clamped to the list)
        auto load_gather = [&](uint32_t first) -> uint32_t {
            const uint32_t t = first + (uint32_t)lane;
            return (uint32_t)gather[t < last_triplet ? t : last_triplet];
        };
        v2u xq[PC_SLOTS];
        // rows of triplets [base, base + 32) of a 64-triplet window whose gather words are gv; n = triplets left from
        // base.  Rows past the end of the list are not requested (whole groups of eight) or read as zeros.
        auto issue_rows = [&](uint32_t gv, int half, uint32_t n) {
            const uint32_t offv = ((uint32_t)(lane & 31) < n && (lane >> 5) == half) ? (gv & GATHER_INDEX) * ROWB : OOB_OFFSET;
#pragma unroll
            for (int j = 0; j < PC_SLOTS; ++j) {
                if ((j & 7) == 0 && (uint32_t)j >= n) break;                                       // wave-uniform
                const uint32_t off = (uint32_t)__builtin_amdgcn_readlane((int)offv, 32 * half + j);   // uniform
                xq[j] = __builtin_amdgcn_raw_buffer_load_b64(frs, (int)(off + (uint32_t)lane * 8u), 0, 0);
            }
        };
        // (1, 0) and (0, 1) as pairs of bf16, kept in scalar registers: as immediate operands of the dot instruction
        // their halves would be at the assembler's discretion
        uint32_t sel_lo = 0x00003f80u, sel_hi = 0x3f800000u;
        asm volatile("" : "+s"(sel_lo), "+s"(sel_hi));
        const v2bf one_lo = __builtin_bit_cast(v2bf, sel_lo), one_hi = __builtin_bit_cast(v2bf, sel_hi);

        if (n_act > 0) {
            uint32_t st_c, en_c, st_n, en_n, st_nn, en_nn;
            load_bounds(0, st_c, en_c);
            load_bounds(1, st_n, en_n);
            load_bounds(2, st_nn, en_nn);
            uint32_t s0_c = __builtin_amdgcn_readfirstlane(st_c);
            uint32_t n_c = pvalid ? (uint32_t)__builtin_amdgcn_readlane((int)en_c, 31) - s0_c : 0u;
            uint32_t gv_c = load_gather(s0_c);
            uint32_t s0_n = __builtin_amdgcn_readfirstlane(st_n);
            uint32_t gv_n = load_gather(s0_n);
            issue_rows(gv_c, 0, n_c);

            for (int s = 0; s < n_act; ++s) {
                // bounds three cells ahead, gather words two cells ahead
                uint32_t st_3, en_3;
                load_bounds(s + 3, st_3, en_3);
                const uint32_t s0_nn = __builtin_amdgcn_readfirstlane(st_nn);
                const uint32_t gv_nn = load_gather(s0_nn);

                // ---- sums of this cell's runs -> S[s & 1] ------------------------------------------------
                char *Sb = Smine + (size_t)(s & 1) * SBUF;
                uint32_t hm = __builtin_amdgcn_readfirstlane(pvalid ? (uint32_t)(__ballot(en_c != st_c) & 0xffffffffull) : 0u);
                if (lane == 0) hasrun[(s & 1) * 4 + p] = hm;
                {   // rows of zeros for the centres without a run inside a group of 16 that has one
                    uint32_t z = ~hm & (((hm & 0xffffu) ? 0xffffu : 0u) | ((hm >> 16) ? 0xffff0000u : 0u));
                    while (z) {                            // wave-uniform
                        const int c = __builtin_ctz(z);
                        z &= z - 1u;
                        *reinterpret_cast<v2u *>(Sb + (size_t)c * SROW) = v2u{0u, 0u};
                    }
                }
                float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
                uint32_t fresh = 1u;                       // no row has gone into the sums since the last run ended
                uint32_t gv_w = gv_c;                      // gather words of the current 64-triplet window
                for (uint32_t base = 0; base < n_c; base += PC_SLOTS) {
                    const int half = (int)((base >> 5) & 1u);
                    if (base != 0) {                       // later passes are not prefetched
                        if (half == 0) gv_w = load_gather(s0_c + base);
                        issue_rows(gv_w, half, n_c - base);
                    }
                    const uint32_t left = n_c - base < PC_SLOTS ? n_c - base : PC_SLOTS;
                    const unsigned long long fl = __ballot((gv_w & GATHER_LAST) != 0u && (lane >> 5) == half &&
                                                           (uint32_t)(lane & 31) < left);
                    // (all wave-uniform; said explicitly so that the tests below are scalar branches)
                    const uint32_t flags = __builtin_amdgcn_readfirstlane((uint32_t)(fl >> (32 * half)));   // bit j: a run ends at row j
                    const uint32_t single = __builtin_amdgcn_readfirstlane(flags & ((flags << 1) | fresh));  // ... and it began there too
                    fresh = __builtin_amdgcn_readfirstlane((flags >> (left - 1u)) & 1u);
#pragma unroll
                    for (int j = 0; j < PC_SLOTS; ++j) {
                        if ((j & 7) == 0 && (uint32_t)j >= left) break;            // wave-uniform
                        const v2u v = xq[j];
                        uint32_t v_lo = v[0], v_hi = v[1];
                        asm volatile("" : "+v"(v_lo), "+v"(v_hi));   // two separate operands for the dot instructions below
                        if ((single >> j) & 1u) {                                  // wave-uniform: a run of one row is its own sum
                            const int c = __builtin_ctz(hm);
                            hm &= hm - 1u;
                            *reinterpret_cast<v2u *>(Sb + (size_t)c * SROW) = v2u{v_lo, v_hi};
                        } else {
                            // fp32 sums: lane <-> channels 4 lane .. 4 lane + 3; one dot product with (1, 0) or (0, 1) per channel
#ifndef PC_NO_DOT
                            a0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, v_lo), one_lo, a0, false);
                            a1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, v_lo), one_hi, a1, false);
                            a2 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, v_hi), one_lo, a2, false);
                            a3 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, v_hi), one_hi, a3, false);
#else
                            a0 += __uint_as_float(v_lo << 16);
                            a1 += __uint_as_float(v_lo & 0xffff0000u);
                            a2 += __uint_as_float(v_hi << 16);
                            a3 += __uint_as_float(v_hi & 0xffff0000u);
#endif
                            if ((flags >> j) & 1u) {                               // wave-uniform: the run ends here
                                const int c = __builtin_ctz(hm);
                                hm &= hm - 1u;
                                *reinterpret_cast<v2u *>(Sb + (size_t)c * SROW) = v2u{cvt_pk_bf16(a0, a1), cvt_pk_bf16(a2, a3)};
                                a0 = a1 = a2 = a3 = 0.f;
                            }
                        }
                    }
                }
                // ---- rows of the next cell ------------------------------------------------------------
                const uint32_t n_n = (pvalid && s + 1 < n_act) ? (uint32_t)__builtin_amdgcn_readlane((int)en_n, 31) - s0_n : 0u;
                issue_rows(gv_n, 0, n_n);
                lds_barrier();
                st_c = st_n; en_c = en_n; s0_c = s0_n; n_c = n_n; gv_c = gv_n;
                st_n = st_nn; en_n = en_nn; s0_n = s0_nn; gv_n = gv_nn;
                st_nn = st_3; en_nn = en_3;
            }
        }
        lds_barrier();                                     // the consumers' last cell
        return;
    }

    // ----------------------------------------------------------------------------------------------------
    // consumer: destination channels 64 q .. 64 q + 63 of all 128 centres
    // ----------------------------------------------------------------------------------------------------
    const int q = wave - PC_PROD;
    const int m = lane & 15, g4 = lane >> 4;
    constexpr int NC32 = 2 * NCH;                          // 32-channel chunks of a source row
    constexpr size_t W_CELL = (size_t)PC_CONS * NC32 * 4 * 64;
    static_assert(NC32 % 4 == 0, "the ring of four chunks must close over a cell");
    // s_waitcnt immediate: [3:0] and [15:14] vector-memory count, [6:4] export count, [11:8] LDS / scalar count.
    // All LDS reads done, and all vector-memory loads but the twelve newest.
    constexpr int WAIT_CHUNK = 0x007C;
    const v4u *wq = static_cast<const v4u *>(w_) + (size_t)q * NC32 * 4 * 64 + lane;     // + k * W_CELL
    v4f acc[PC_GROUPS][4];
#pragma unroll
    for (int g = 0; g < PC_GROUPS; ++g)
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) acc[g][cg] = v4f{0.f, 0.f, 0.f, 0.f};
    v4u wb[4][4];                                          // ring of four 32-channel chunks of the slice: [chunk & 3][cg]
    if (n_act > 0) {
#pragma unroll
        for (int c = 0; c < 3; ++c)
#pragma unroll
            for (int cg = 0; cg < 4; ++cg) wb[c][cg] = wq[(size_t)act[0] * W_CELL + (c * 4 + cg) * 64];
    }
    lds_barrier();                                         // iteration 0: the producers fill the first tile
    const uint32_t a_lane = (uint32_t)m * SROW + (uint32_t)g4 * 16u;
    for (int s = 0; s < n_act; ++s) {
        const char *Sb = S + (size_t)(s & 1) * SBUF + a_lane;
        const uint32_t h0 = hasrun[(s & 1) * 4 + 0], h1 = hasrun[(s & 1) * 4 + 1], h2 = hasrun[(s & 1) * 4 + 2],
                       h3 = hasrun[(s & 1) * 4 + 3];
        // groups of 16 centres with a run in this cell
        uint32_t ag = 0;
        ag |= (h0 & 0xffffu) ? 1u : 0u;  ag |= (h0 >> 16) ? 2u : 0u;
        ag |= (h1 & 0xffffu) ? 4u : 0u;  ag |= (h1 >> 16) ? 8u : 0u;
        ag |= (h2 & 0xffffu) ? 16u : 0u; ag |= (h2 >> 16) ? 32u : 0u;
        ag |= (h3 & 0xffffu) ? 64u : 0u; ag |= (h3 >> 16) ? 128u : 0u;
        ag = __builtin_amdgcn_readfirstlane(ag);
        const v4u *w_this = wq + (size_t)act[s] * W_CELL;
        const v4u *w_next = wq + (size_t)act[s + 1 < n_act ? s + 1 : s] * W_CELL;
        // The work of a cell is a sequence of units (chunk ch, active group g), ch-major, four MFMAs each.  Every
        // group keeps one A piece in registers; a unit requests the group's piece of the next chunk right after its
        // MFMAs, so that it has a whole chunk's time to arrive.
        v4u piece[PC_GROUPS];
#pragma unroll
        for (int g = 0; g < PC_GROUPS; ++g)
            if ((ag >> g) & 1u) piece[g] = *reinterpret_cast<const v4u *>(Sb + (size_t)g * 16 * SROW);
#pragma unroll
        for (int ch = 0; ch < NC32; ++ch) {
            // W three chunks ahead (the next cell's first chunks after the last ones of this cell); then one wait for
            // everything this chunk reads: its own W pieces (all loads but the twelve newest) and the A pieces
            {
                const v4u *src = ch + 3 < NC32 ? w_this + (size_t)(ch + 3) * 4 * 64 : w_next + (size_t)(ch + 3 - NC32) * 4 * 64;
#pragma unroll
                for (int cg = 0; cg < 4; ++cg) wb[(ch + 3) & 3][cg] = src[cg * 64];
            }
            __builtin_amdgcn_s_waitcnt(WAIT_CHUNK);
#pragma unroll
            for (int g = 0; g < PC_GROUPS; ++g) {
                if (!((ag >> g) & 1u)) continue;           // wave-uniform
#pragma unroll
                for (int cg = 0; cg < 4; ++cg) mfma_16x16x32_acc(acc[g][cg], piece[g], wb[ch & 3][cg]);
                if (ch + 1 < NC32) piece[g] = *reinterpret_cast<const v4u *>(Sb + (size_t)g * 16 * SROW + (ch + 1) * 64);
            }
        }
        lds_barrier();
    }
    // the matrix cores' last results must have landed before ordinary instructions read the accumulators (the
    // compiler cannot see inside the MFMA statements, so the wait states are spelled out)
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    // every row once, by its owner
    const int64_t slot0 = vb * PC_ROWS;
#pragma unroll
    for (int g = 0; g < PC_GROUPS; ++g)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t slot = slot0 + 16 * g + 4 * g4 + j;
            if (slot < n_centres) {
                const int64_t row = side.perm ? (int64_t)side.perm[slot] : slot;
#pragma unroll
                for (int cg = 0; cg < 4; ++cg) {
                    const float v = acc[g][cg][j];
                    const size_t at = (size_t)row * C_DST + 64 * q + 16 * cg + m;
                    if constexpr (sizeof(TOut) == 4) dst[at] = v;
                    else dst[at] = (uint16_t)(cvt_pk_bf16(v, 0.f) & 0xffffu);
                }
            }
        }
}

}  // namespace

bool mvmr_rows_pc_usable(const MvmrArgs &a)
{
    return a.n_triplets > 0 && a.in_dtype == PCPP_BF16 && a.c_src == 256 && a.c_dst == 256 && a.side.gather != nullptr &&
           (size_t)a.n_src * a.c_src * 2 <= MAX_BUFFER_BYTES;
}

int mvmr_rows_pc_pack_w(const void *w, void *packed, int K, int c_src, int c_dst, int stride_d, int stride_s,
                        hipStream_t stream)
{
    const int64_t total = (int64_t)K * c_dst * c_src / 8;          // 16-byte pieces
    pack_w_pc_kernel<<<(unsigned)ceil_div(total, 256), 256, 0, stream>>>(
        static_cast<const uint16_t *>(w), static_cast<uint16_t *>(packed), K, c_src, c_dst, stride_d, stride_s);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

int mvmr_rows_pc(const MvmrArgs &a, hipStream_t stream)
{
    constexpr int NCH = 4;
    const int64_t n_blocks = ceil_div(a.n_centres, PC_ROWS);
    const int64_t grid = ceil_div(n_blocks, NUM_XCD) * NUM_XCD;
    const size_t lds = (size_t)2 * PC_ROWS * (64 * NCH * 2 + 16) + 8 * sizeof(uint32_t) + (MAX_K + 1) * sizeof(int);
    const uint32_t last = (uint32_t)(a.n_triplets - 1);
    const uint32_t feat_bytes = (uint32_t)((size_t)a.n_src * a.c_src * 2);
    if (a.out_dtype == PCPP_F32) {
        auto kern = rows_pc_kernel<NCH, float>;
        if (int rc = raise_lds_limit(reinterpret_cast<const void *>(kern), lds)) return rc;
        kern<<<(unsigned)grid, PC_THREADS, lds, stream>>>(a.feat, a.w, static_cast<float *>(a.dst), a.n_centres, a.K,
                                                          a.gather, last, feat_bytes, a.side, n_blocks);
    } else {
        auto kern = rows_pc_kernel<NCH, uint16_t>;
        if (int rc = raise_lds_limit(reinterpret_cast<const void *>(kern), lds)) return rc;
        kern<<<(unsigned)grid, PC_THREADS, lds, stream>>>(a.feat, a.w, static_cast<uint16_t *>(a.dst), a.n_centres,
                                                          a.K, a.gather, last, feat_bytes, a.side, n_blocks);
    }
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

}  // namespace pcpp
