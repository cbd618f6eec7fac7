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
#include <type_traits>

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

// One A piece from LDS.  The read is outside the compiler's bookkeeping of outstanding memory operations, and so
// are the waits for it (lds_wait): a consumer keeps exactly one read per active group in flight, in the order in
// which the pieces are used, so "all but the newest two have arrived" is enough whenever three or more groups are
// active -- a count the compiler cannot know and would replace by a wait for everything.
template <int OFFSET>
__device__ inline void lds_read_piece(v4u &dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFFSET));
}
template <int N>
__device__ inline void lds_wait()
{
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
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
    uint32_t *rank_tab = hasrun + 8;                               // [PC_PROD][32]: a producer's centres with a run, in order
    int *act = reinterpret_cast<int *>(rank_tab + PC_PROD * 32);   // active cells, act[MAX_K] = their number
    constexpr uint32_t DUMMY_OFF = 2 * SBUF + (8 + PC_PROD * 32) * 4 + (MAX_K + 1) * 4 + 12;   // [PC_PROD][ROWB]: where rows
    static_assert(DUMMY_OFF % 16 == 0, "alignment of the scratch rows");                       // past a list's end are stored
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
                // Straight-line code per row (a taken branch costs a wave more than the dozen instructions it would
                // skip): every row is added to the four fp32 sums of its lane (lane <-> channels 4 lane .. 4 lane + 3;
                // v_dot2c_f32_bf16 would halve the instructions but runs at a quarter of the rate), the sums so far are
                // rounded to bf16 and stored to the
                // S row of the run's centre -- the store of the run's last row is the one that stays -- and the sums are
                // cleared behind a run's last row.
                const uint32_t hm = __builtin_amdgcn_readfirstlane(pvalid ? (uint32_t)(__ballot(en_c != st_c) & 0xffffffffull) : 0u);
                if (lane == 0) hasrun[(s & 1) * 4 + p] = hm;
                {   // rows of zeros for the centres without a run inside a group of 16 that has one: lane (c, half)
                    // clears half a row
                    const uint32_t z = ~hm & (((hm & 0xffffu) ? 0xffffu : 0u) | ((hm >> 16) ? 0xffff0000u : 0u));
                    if ((z >> (lane & 31)) & 1u) {
                        char *zp = S + (size_t)(s & 1) * SBUF + (size_t)(32 * p + (lane & 31)) * SROW + (lane >> 5) * 256;
#pragma unroll
                        for (int e = 0; e < 16; ++e) *reinterpret_cast<v4u *>(zp + 16 * e) = v4u{0u, 0u, 0u, 0u};
                    }
                }
                // the centres with a run, by rank: the run that ends r-th belongs to centre tab[r]
                uint32_t *tab = rank_tab + p * 32;
                if (lane < 32 && ((hm >> lane) & 1u)) tab[__popc(hm & ((1u << lane) - 1u))] = (uint32_t)lane;
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
                float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
                uint32_t ends_before = 0u;                 // runs that ended in earlier passes
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
                    const uint32_t flags = __builtin_amdgcn_readfirstlane((uint32_t)(fl >> (32 * half)));   // bit j: a run ends at row j
                    // lane j: where row j's sums go (byte offset of its centre's S row in the block's LDS; rows past the
                    // end of the list, which are zeros, go to a scratch row)
                    const uint32_t rk = ends_before + (uint32_t)__popc(flags & ((1u << (lane & 31)) - 1u));
                    const uint32_t ctr = tab[rk < 32u ? rk : 31u] & 31u;
                    const uint32_t dsto = (uint32_t)(lane & 31) < left ? (uint32_t)(s & 1) * SBUF + (32u * p + ctr) * SROW
                                                                       : DUMMY_OFF + (uint32_t)p * ROWB;
                    ends_before += (uint32_t)__popc(flags);
#pragma unroll
                    for (int j = 0; j < PC_SLOTS; ++j) {
                        if ((j & 7) == 0 && (uint32_t)j >= left) break;            // wave-uniform
                        const v2u v = xq[j];
                        a0 += __uint_as_float(v[0] << 16);
                        a1 += __uint_as_float(v[0] & 0xffff0000u);
                        a2 += __uint_as_float(v[1] << 16);
                        a3 += __uint_as_float(v[1] & 0xffff0000u);
                        const uint32_t off = (uint32_t)__builtin_amdgcn_readlane((int)dsto, j);
                        *reinterpret_cast<v2u *>(lds + off + lane * 8) = v2u{cvt_pk_bf16(a0, a1), cvt_pk_bf16(a2, a3)};
                        // all-ones while the run goes on, zero behind its last row (wave-uniform, a scalar)
                        const uint32_t keep = ((flags >> j) & 1u) - 1u;
                        a0 = __uint_as_float(__float_as_uint(a0) & keep);
                        a1 = __uint_as_float(__float_as_uint(a1) & keep);
                        a2 = __uint_as_float(__float_as_uint(a2) & keep);
                        a3 = __uint_as_float(__float_as_uint(a3) & keep);
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
    // All vector-memory loads but the twelve newest done.
    constexpr int WAIT_W = 0x0F7C;
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
        // MFMAs, so the piece a unit needs is always the oldest read in flight and n_ag - 1 newer ones follow it.
        const int n_ag = __builtin_popcount(ag);
        const uint32_t sb_addr = (uint32_t)(uintptr_t)(Sb - lds);       // the dynamic LDS block starts at address 0 (no static LDS)
        v4u piece[PC_GROUPS];
        constexpr int GROW = 16 * (int)SROW;
#define PCPP_PC_FIRST(g) if ((ag >> g) & 1u) lds_read_piece<g * GROW>(piece[g], sb_addr);
        PCPP_PC_FIRST(0) PCPP_PC_FIRST(1) PCPP_PC_FIRST(2) PCPP_PC_FIRST(3)
        PCPP_PC_FIRST(4) PCPP_PC_FIRST(5) PCPP_PC_FIRST(6) PCPP_PC_FIRST(7)
#undef PCPP_PC_FIRST
        auto chunk = [&](auto ch_tag) {
            constexpr int ch = decltype(ch_tag)::value;
            // W three chunks ahead (the next cell's first chunks after the last ones of this cell), then wait for this
            // chunk's W pieces: all loads but the twelve newest
            {
                constexpr int pre = (ch + 3) % NC32;       // chunk to request: of this cell, or of the next one
                const v4u *src = (ch + 3 < NC32 ? w_this : w_next) + (size_t)pre * 4 * 64;
#pragma unroll
                for (int cg = 0; cg < 4; ++cg) wb[(ch + 3) & 3][cg] = src[cg * 64];
            }
            __builtin_amdgcn_s_waitcnt(WAIT_W);
            if (n_ag < 3) lds_wait<0>();                   // wave-uniform
            auto unit = [&](auto g_tag) {
                constexpr int g = decltype(g_tag)::value;
                uint32_t on = (ag >> g) & 1u;
                asm volatile("" : "+s"(on));               // a scalar, tested by a scalar branch
                if (!on) return;
                lds_wait<2>();
#pragma unroll
                for (int cg = 0; cg < 4; ++cg) mfma_16x16x32_acc(acc[g][cg], piece[g], wb[ch & 3][cg]);
                if constexpr (ch + 1 < NC32) lds_read_piece<g * GROW + (ch + 1) * 64>(piece[g], sb_addr);
            };
            unit(std::integral_constant<int, 0>{}); unit(std::integral_constant<int, 1>{});
            unit(std::integral_constant<int, 2>{}); unit(std::integral_constant<int, 3>{});
            unit(std::integral_constant<int, 4>{}); unit(std::integral_constant<int, 5>{});
            unit(std::integral_constant<int, 6>{}); unit(std::integral_constant<int, 7>{});
        };
        static_assert(NC32 == 8 && PC_GROUPS == 8, "the chunk and unit sequences are written out for eight of each");
        chunk(std::integral_constant<int, 0>{}); chunk(std::integral_constant<int, 1>{});
        chunk(std::integral_constant<int, 2>{}); chunk(std::integral_constant<int, 3>{});
        chunk(std::integral_constant<int, 4>{}); chunk(std::integral_constant<int, 5>{});
        chunk(std::integral_constant<int, 6>{}); chunk(std::integral_constant<int, 7>{});
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
    const size_t lds = (size_t)2 * PC_ROWS * (64 * NCH * 2 + 16) + (8 + PC_PROD * 32) * sizeof(uint32_t) + (MAX_K + 1) * sizeof(int) + 12 + PC_PROD * 64 * NCH * 2;
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
