// MVMR rows kernel for wide layers with separate producer and consumer waves (Eq. (1) forward; Sec. 3.3.3 input
// gradient with W^T).
//
// Eq. (1) is linear, so out[o] = sum_k W[k] S_k[o] with S_k[o] = the sum of x[i] over the (k, o) run.  A block owns
// 128 consecutive slots of the plan's centre order (two tiles) and walks the kernel cells that hold a triplet for
// any of them.  Per cell,
//   producer waves (four, one per SIMD) gather the source rows of the block's runs -- the cell's triplets of the
//       block are one contiguous piece of the list, cut into four shares at run boundaries; one 512-byte row per
//       load instruction, lane <-> four channels -- add them up in fp32 on the vector ALUs, round each run's sum to
//       bf16 once and store it as row `centre` of an LDS tile S[128][C_src]; centres without a run get rows of zeros;
//   consumer waves (four, one per SIMD; each owns 64 destination channels of all 128 centres, 128 accumulator
//       registers) multiply the tile by their slice of W[k] on the matrix cores, acc += S . W[k]^T, chunk of 32
//       source channels by chunk; per chunk, one test per quarter of the block (32 centres) skips the quarters
//       that hold no triplet in the cell (3.0 of 4 do on this workload; within a quarter the rows of centres
//       without a run are zeros and are multiplied all the same).  A test per group of 16 centres was slower: it
//       costs the in-order wave about as much as the 64 cycles of the matrix pipe that it saves.
// The two run one cell apart on two LDS tiles, one barrier per cell: while the matrix cores work on cell j the
// rows of cell j + 1 are in flight.  A consumer's W slice (64 x C_src of the 16.4 MB at K = 125) comes straight from
// memory / L2 into registers in fragment order, three 32-channel chunks ahead of its use (a ring of four); nothing
// but S goes through LDS.  Every destination row is accumulated in registers across all cells and written once by
// its owner: no atomics, fixed summation order.
//
// What bounds it: the matrix pipe needs 256 x 16 = 4096 cycles for a cell in which every quarter holds a triplet;
// the consumer's loads of W and of S add about 1500 (each is an instruction of the same in-order wave), and in a
// cell with few rows the 32 loads of its W slice, three chunks ahead, are what it waits for.  A producer spends about 70 cycles per row when
// alone on its SIMD (10 vector instructions for the sums, two conversions, and a 512-byte LDS store that costs
// 24) and about 105 beside a wave that issues MFMAs back to back, since both issue through the SIMD's vector
// port; with the per-cell bookkeeping a producer's cell takes about as long as a consumer's.
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
constexpr int PC_STEP = 4;                        // rows are requested and added in groups of this many
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
    uint32_t *rank_tab = reinterpret_cast<uint32_t *>(lds + 2 * SBUF);   // [PC_PROD][PC_ROWS]: per producer, the block's centres with a run, in order
    int *act = reinterpret_cast<int *>(rank_tab + PC_PROD * PC_ROWS);   // active cells, act[MAX_K] = their number
    uint32_t *qmask = reinterpret_cast<uint32_t *>(act + MAX_K + 1);    // [2]: per LDS tile, bit q = centres 32 q .. 32 q + 31 hold a run
    constexpr uint32_t DUMMY_OFF = 2 * SBUF + PC_PROD * PC_ROWS * 4 + (MAX_K + 1) * 4 + 12;   // [PC_PROD][ROWB]: where rows
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
        // producer.  The triplets of a cell that belong to the block's 128 centres are one contiguous piece of the
        // list (consecutive tiles of one cell follow each other); the four producers cut it into quarters at run
        // boundaries -- producer p takes the runs that start in the p-th quarter -- so that each adds up about the
        // same number of rows whatever the distribution of the neighbours over the centres.  (The barrier at the end
        // of a cell waits for the slowest of the four.)  Rows of zeros for centres without a run: producer p clears
        // those among centres 32 p .. 32 p + 31.
        // ------------------------------------------------------------------------------------------------
        const int p = wave;
        const bool b_valid = t0 + 1 < side.n_tiles;                // the block's second tile exists (uniform)
        const int64_t tile_b = b_valid ? t0 + 1 : t0;
        const uint32_t *runs_a = side.run_start + (size_t)t0 * K * TILE + lane;
        const uint32_t *runs_b = side.run_start + (size_t)tile_b * K * TILE + lane;
        const uint32_t *tends_a = side.tile_ptr + t0 + 1, *tends_b = side.tile_ptr + tile_b + 1;
        const bool last_in_tile = lane == TILE - 1;
        const __amdgpu_buffer_rsrc_t frs = make_rsrc(feat_, feat_bytes);
        const unsigned long long below = (1ull << lane) - 1ull;

        struct Bounds { uint32_t st_a, en_a, st_b, en_b; };        // lane <-> centre `lane` of tile a and of tile b
        // bounds of the runs of cell act[j] (clamped; steps past the end are masked by their callers)
        auto load_bounds = [&](int j) -> Bounds {
            const int k = act[j < n_act ? j : (n_act > 0 ? n_act - 1 : 0)];
            Bounds b;
            b.st_a = runs_a[(size_t)k * TILE];
            b.en_a = last_in_tile ? tends_a[(size_t)k * side.n_tiles] : runs_a[(size_t)k * TILE + 1];
            b.st_b = runs_b[(size_t)k * TILE];
            b.en_b = last_in_tile ? tends_b[(size_t)k * side.n_tiles] : runs_b[(size_t)k * TILE + 1];
            return b;
        };
        struct Share { uint32_t first, n, rank; };                 // this producer's triplets and the rank of its first run
        auto share_of = [&](const Bounds &b) -> Share {
            const unsigned long long m_a = __ballot(b.en_a != b.st_a);
            const unsigned long long m_b = b_valid ? __ballot(b.en_b != b.st_b) : 0ull;
            const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)b.st_a, 0);
            const uint32_t b1 = (uint32_t)__builtin_amdgcn_readlane((int)(b_valid ? b.en_b : b.en_a), 63);
            const uint32_t nb = b1 - b0;
            // the first run that starts at or behind x: its first triplet and its rank among the block's runs
            auto first_run = [&](uint32_t x, uint32_t &start, uint32_t &rank) {
                const unsigned long long c_a = __ballot(b.en_a != b.st_a && b.st_a >= x);
                const unsigned long long c_b = b_valid ? __ballot(b.en_b != b.st_b && b.st_b >= x) : 0ull;
                if (c_a) {
                    const int i = __builtin_ctzll(c_a);
                    start = (uint32_t)__builtin_amdgcn_readlane((int)b.st_a, i);
                    rank = (uint32_t)__popcll(m_a & ((1ull << i) - 1ull));
                } else if (c_b) {
                    const int i = __builtin_ctzll(c_b);
                    start = (uint32_t)__builtin_amdgcn_readlane((int)b.st_b, i);
                    rank = (uint32_t)__popcll(m_a) + (uint32_t)__popcll(m_b & ((1ull << i) - 1ull));
                } else {
                    start = b1;
                    rank = 0u;
                }
            };
            Share sh;
            uint32_t stop, stop_rank;
            first_run(b0 + ((nb * (uint32_t)p) >> 2), sh.first, sh.rank);
            if (p + 1 < PC_PROD) first_run(b0 + ((nb * (uint32_t)(p + 1)) >> 2), stop, stop_rank);
            else stop = b1;
            sh.first = __builtin_amdgcn_readfirstlane(sh.first);
            sh.rank = __builtin_amdgcn_readfirstlane(sh.rank);
            sh.n = __builtin_amdgcn_readfirstlane(stop) - sh.first;
            return sh;
        };
        // gather words of triplets first + lane (clamped to the list)
        auto load_gather = [&](uint32_t first) -> uint32_t {
            const uint32_t t = first + (uint32_t)lane;
            return (uint32_t)gather[t < last_triplet ? t : last_triplet];
        };
        v2u xq[PC_SLOTS];
        // rows of triplets [base, base + 32) of a 64-triplet window whose gather words are gv; n = triplets left from
        // base.  Whole groups of PC_STEP are requested; the rows behind the share's end inside the last group repeat a
        // row of the share (their sums go to a scratch row).  A row's offset travels in a scalar register, so a
        // request is two instructions: lane j's offset to the scalar file, then the load of 8 bytes per lane.
        auto issue_rows = [&](uint32_t gv, int half, uint32_t n) {
            const uint32_t src = (uint32_t)(lane & 31) < n ? gv : (uint32_t)__builtin_amdgcn_readlane((int)gv, 32 * half);
            const uint32_t offv = (src & GATHER_INDEX) * ROWB;
#pragma unroll
            for (int j0 = 0; j0 < PC_SLOTS; j0 += PC_STEP) {
                if ((uint32_t)j0 >= n) break;                                                     // wave-uniform
                uint32_t off[PC_STEP];
#pragma unroll
                for (int j = 0; j < PC_STEP; ++j) off[j] = (uint32_t)__builtin_amdgcn_readlane((int)offv, 32 * half + j0 + j);
#pragma unroll
                for (int j = 0; j < PC_STEP; ++j)
                    xq[j0 + j] = __builtin_amdgcn_raw_buffer_load_b64(frs, (int)((uint32_t)lane * 8u), (int)off[j], 0);
            }
        };

        if (n_act > 0) {
            Bounds bd_c = load_bounds(0), bd_n = load_bounds(1), bd_nn = load_bounds(2);
            Share sh_c = share_of(bd_c);
            uint32_t gv_c = load_gather(sh_c.first), gx_c = load_gather(sh_c.first + 64u);   // first and second window
            Share sh_n = share_of(bd_n);
            if (n_act < 2) sh_n.n = 0u;
            uint32_t gv_n = load_gather(sh_n.first), gx_n = load_gather(sh_n.first + 64u);
            issue_rows(gv_c, 0, sh_c.n);

            uint32_t dirty0 = ~0u, dirty1 = ~0u;           // per LDS tile: rows of this producer's centres that are not zeros
            for (int s = 0; s < n_act; ++s) {
                // ---- sums of this cell's runs -> S[s & 1] ------------------------------------------------
                // Straight-line code per row (a taken branch costs a wave more than the dozen instructions it would
                // skip): every row is added to the four fp32 sums of its lane (lane <-> channels 4 lane .. 4 lane + 3;
                // v_dot2c_f32_bf16 would halve the instructions but runs at a quarter of the rate), the sums so far are
                // rounded to bf16 and stored to the S row of the run's centre -- the store of the run's last row is the
                // one that stays -- and the row behind a run's last one starts new sums (one fused multiply-add per
                // channel does both; a non-finite sum therefore spoils the later runs of this producer in the cell,
                // all of them rows of this block's centres).
                const unsigned long long m_a = __ballot(bd_c.en_a != bd_c.st_a);
                const unsigned long long m_b = b_valid ? __ballot(bd_c.en_b != bd_c.st_b) : 0ull;
                {   // rows of zeros for the centres 32 p .. 32 p + 31 without a run in this cell, unless the row is still
                    // zero from the tile's last use two cells ago: lane (c, half) clears half a row
                    const uint32_t has = (uint32_t)((p < 2 ? m_a : m_b) >> (32 * (p & 1)));
                    const uint32_t z = ~has & ((s & 1) ? dirty1 : dirty0);
                    if (s & 1) dirty1 = has; else dirty0 = has;
                    if ((z >> (lane & 31)) & 1u) {
                        char *zp = S + (size_t)(s & 1) * SBUF + (size_t)(32 * p + (lane & 31)) * SROW + (lane >> 5) * 256;
#pragma unroll
                        for (int e = 0; e < 16; ++e) *reinterpret_cast<v4u *>(zp + 16 * e) = v4u{0u, 0u, 0u, 0u};
                    }
                }
                if (p == 0 && lane == 0)
                    qmask[s & 1] = ((uint32_t)m_a != 0u) | (((uint32_t)(m_a >> 32) != 0u) << 1) |
                                   (((uint32_t)m_b != 0u) << 2) | (((uint32_t)(m_b >> 32) != 0u) << 3);
                // the block's centres with a run, by rank: the run that ends r-th belongs to centre tab[r]
                uint32_t *tab = rank_tab + p * PC_ROWS;
                if ((m_a >> lane) & 1ull) tab[__popcll(m_a & below)] = (uint32_t)lane;
                if ((m_b >> lane) & 1ull) tab[__popcll(m_a) + __popcll(m_b & below)] = (uint32_t)(TILE + lane);
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
                const uint32_t n_c = sh_c.n;
                float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f, keep = 0.f;
                uint32_t ends_before = sh_c.rank;          // runs that ended before the rows of this pass
                // Rows travel in passes of 32 through the 32 row registers.  The first pass of a cell was requested
                // during the previous cell; every later pass is requested group by group during the pass before it, each
                // group into the registers that the current pass has just added up, so that shares of more than 32
                // rows (a third of the cells, and the ones that set the pace) do not wait out a memory round trip.  A
                // pass that refills always requests all eight groups, and the passes of a share are written out one
                // behind the other without a loop: the number of row loads younger than the one a group needs is
                // then a constant that the compiler can see (28 while refilling, fewer in a share's last pass), and
                // it waits for exactly that.  The gather words of the first 128 triplets of a share are prefetched;
                // beyond that (rare) the passes are requested one at a time.
                // pass over `left` (<= 32) rows whose gather words are half `half` of gv_w; when REFILL, the n_next rows of
                // the pass behind it (gather words: the other half, of g_next) are requested on the way
                auto pass = [&](int half, uint32_t left, uint32_t gv_w, uint32_t g_next, uint32_t n_next, auto refill_c) {
                    constexpr bool REFILL = decltype(refill_c)::value;
                    const int nhalf = half ^ 1;
                    uint32_t off_next = 0u;                // lane 32 nhalf + j: row j of the next pass
                    if (REFILL) {
                        const uint32_t src_next = (uint32_t)(lane & 31) < n_next ? g_next
                                                                                 : (uint32_t)__builtin_amdgcn_readlane((int)g_next, 32 * nhalf);
                        off_next = (src_next & GATHER_INDEX) * ROWB;
                    }
                    const unsigned long long fl = __ballot((gv_w & GATHER_LAST) != 0u && (lane >> 5) == half &&
                                                           (uint32_t)(lane & 31) < left);
                    const uint32_t flags = __builtin_amdgcn_readfirstlane((uint32_t)(fl >> (32 * half)));   // bit j: a run ends at row j
                    // lane j: where row j's sums go (byte offset of its centre's S row in the block's LDS; rows past the
                    // end of the share go to a scratch row)
                    const uint32_t rk = ends_before + (uint32_t)__popc(flags & ((1u << (lane & 31)) - 1u));
                    const uint32_t ctr = tab[rk < (uint32_t)PC_ROWS ? rk : (uint32_t)PC_ROWS - 1u] & (uint32_t)(PC_ROWS - 1);
                    const uint32_t dsto = (uint32_t)(lane & 31) < left ? (uint32_t)(s & 1) * SBUF + ctr * SROW
                                                                       : DUMMY_OFF + (uint32_t)p * ROWB;
                    ends_before += (uint32_t)__popc(flags);
#pragma unroll
                    for (int j0 = 0; j0 < PC_SLOTS; j0 += PC_STEP) {
                        if (!REFILL && (uint32_t)j0 >= left) break;                // wave-uniform
                        uint32_t at[PC_STEP];                                      // where the lane's 8 bytes of row j go
#pragma unroll
                        for (int j = 0; j < PC_STEP; ++j) at[j] = (uint32_t)__builtin_amdgcn_readlane((int)dsto, j0 + j) + (uint32_t)lane * 8u;
#pragma unroll
                        for (int j = 0; j < PC_STEP; ++j) asm volatile("" : "+v"(at[j]));   // all here, off the sums' critical path
#pragma unroll
                        for (int j = 0; j < PC_STEP; ++j) {
                            const v2u v = xq[j0 + j];
                            // sums = sums * keep + row: keep is 1 inside a run and 0 for the row behind a run's last one
                            a0 = __builtin_fmaf(a0, keep, __uint_as_float(v[0] << 16));
                            a1 = __builtin_fmaf(a1, keep, __uint_as_float(v[0] & 0xffff0000u));
                            a2 = __builtin_fmaf(a2, keep, __uint_as_float(v[1] << 16));
                            a3 = __builtin_fmaf(a3, keep, __uint_as_float(v[1] & 0xffff0000u));
                            *reinterpret_cast<v2u *>(lds + at[j]) = v2u{cvt_pk_bf16(a0, a1), cvt_pk_bf16(a2, a3)};
                            keep = __uint_as_float((((flags >> (j0 + j)) & 1u) ^ 1u) * 0x3f800000u);   // wave-uniform, a scalar
                        }
                        if (REFILL) {
                            uint32_t off[PC_STEP];
#pragma unroll
                            for (int j = 0; j < PC_STEP; ++j) off[j] = (uint32_t)__builtin_amdgcn_readlane((int)off_next, 32 * nhalf + j0 + j);
#pragma unroll
                            for (int j = 0; j < PC_STEP; ++j)
                                xq[j0 + j] = __builtin_amdgcn_raw_buffer_load_b64(frs, (int)((uint32_t)lane * 8u), (int)off[j], 0);
                        }
                    }
                };
                constexpr uint32_t PREFETCHED = 4u * PC_SLOTS;      // triplets whose gather words gv_c and gx_c hold
                const uint32_t n_main = n_c < PREFETCHED ? n_c : PREFETCHED;
                const std::true_type yes{};
                const std::false_type no{};
                if (n_main > PC_SLOTS) {
                    pass(0, PC_SLOTS, gv_c, gv_c, n_main - PC_SLOTS, yes);
                    if (n_main > 2u * PC_SLOTS) {
                        pass(1, PC_SLOTS, gv_c, gx_c, n_main - 2u * PC_SLOTS, yes);
                        if (n_main > 3u * PC_SLOTS) {
                            pass(0, PC_SLOTS, gx_c, gx_c, n_main - 3u * PC_SLOTS, yes);
                            pass(1, n_main - 3u * PC_SLOTS, gx_c, gx_c, 0u, no);
                        } else {
                            pass(0, n_main - 2u * PC_SLOTS, gx_c, gx_c, 0u, no);
                        }
                    } else {
                        pass(1, n_main - PC_SLOTS, gv_c, gx_c, 0u, no);
                    }
                } else if (n_main > 0u) {
                    pass(0, n_main, gv_c, gv_c, 0u, no);
                }
                for (uint32_t base = PREFETCHED; base < n_c; base += PC_SLOTS) {      // rare: one pass at a time
                    const uint32_t gv_t = load_gather(sh_c.first + base);
                    const uint32_t left = n_c - base < PC_SLOTS ? n_c - base : PC_SLOTS;
                    issue_rows(gv_t, 0, left);
                    pass(0, left, gv_t, gv_t, 0u, no);
                }
                // ---- bounds three cells ahead, share and gather words two cells ahead, rows of the next cell --------
                // (Behind the sums on purpose: the waits for rows that the compiler places between them are sized for
                // the path on which the rows were requested a moment ago, and a load requested in front of the sums
                // would be waited for there at its full latency, every cell.)
                const Bounds bd_3 = load_bounds(s + 3);
                Share sh_nn = share_of(bd_nn);
                if (s + 2 >= n_act) sh_nn.n = 0u;
                const uint32_t gv_nn = load_gather(sh_nn.first), gx_nn = load_gather(sh_nn.first + 64u);
                issue_rows(gv_n, 0, sh_n.n);
                lds_barrier();
                bd_c = bd_n; sh_c = sh_n; gv_c = gv_n; gx_c = gx_n;
                bd_n = bd_nn; sh_n = sh_nn; gv_n = gv_nn; gx_n = gx_nn;
                bd_nn = bd_3;
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
    constexpr int GROW = 16 * (int)SROW;
    for (int s = 0; s < n_act; ++s) {
        const char *Sb = S + (size_t)(s & 1) * SBUF + a_lane;
        const v4u *w_this = wq + (size_t)act[s] * W_CELL;
        const v4u *w_next = wq + (size_t)act[s + 1 < n_act ? s + 1 : s] * W_CELL;
        // The work of a cell is up to 64 units (chunk ch, group g of 16 centres), ch-major, four MFMAs each.  Every
        // group keeps one A piece in registers and requests its piece of the next chunk right after its MFMAs.  One
        // test per chunk and quarter of the block (32 centres) skips the quarters without a triplet in the cell: those
        // are the cells with few rows, where the producers are quick and the consumers set the pace.  (A second,
        // branch-free copy of the loop for the cells in which all four quarters hold a triplet made the register
        // allocator spill the accumulators.)
        const uint32_t qm = __builtin_amdgcn_readfirstlane(qmask[s & 1]);
        auto cell = [&](auto dense_c) {
            constexpr bool DENSE = decltype(dense_c)::value;
            v4u piece[PC_GROUPS];
#pragma unroll
            for (int g = 0; g < PC_GROUPS; ++g)
                if (DENSE || ((qm >> (g >> 1)) & 1u)) piece[g] = *reinterpret_cast<const v4u *>(Sb + g * GROW);
#pragma unroll
            for (int ch = 0; ch < NC32; ++ch) {
                // W three chunks ahead (the next cell's first chunks after the last ones of this cell)
                {
                    const int pre = (ch + 3) % NC32;
                    const v4u *src = (ch + 3 < NC32 ? w_this : w_next) + (size_t)pre * 4 * 64;
#pragma unroll
                    for (int cg = 0; cg < 4; ++cg) wb[(ch + 3) & 3][cg] = src[cg * 64];
                }
#pragma unroll
                for (int qd = 0; qd < PC_GROUPS / 2; ++qd) {
                    if (DENSE || ((qm >> qd) & 1u)) {
#pragma unroll
                        for (int g = 2 * qd; g < 2 * qd + 2; ++g) {
#pragma unroll
                            for (int cg = 0; cg < 4; ++cg) mfma_16x16x32_acc(acc[g][cg], piece[g], wb[ch & 3][cg]);
                            if (ch + 1 < NC32) piece[g] = *reinterpret_cast<const v4u *>(Sb + g * GROW + (ch + 1) * 64);
                        }
                    }
                }
            }
        };
        cell(std::false_type{});
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
    const size_t lds = (size_t)2 * PC_ROWS * (64 * NCH * 2 + 16) + PC_PROD * PC_ROWS * sizeof(uint32_t) +
                       (MAX_K + 1) * sizeof(int) + 12 + PC_PROD * 64 * NCH * 2;
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
