// Weight gradient (VVOR), Eq. (5) of Sec. 3.3.3, on the matrix cores: dW[k] = sum over cell k's run of
// dy[o] (x) x[i].  The (k, o, i) ordered triplet list is cut into equal chunks, one per wave (per
// sub-block of dW for wide layers); the reduction index of the MFMA is the triplet, both operands are
// rows read straight from memory (lane <-> channel), chunk partial sums go to the workspace and are
// added in a fixed order by a second kernel: no atomics, reproducible.
#include <stdlib.h>

#include <type_traits>

#include "pcpp_internal.h"

namespace pcpp {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int WAVES = 4;


// MFMA register layout used by the fp32 kernel (wave64):
//   v_mfma_f32_32x32x2_f32: A: lane (m = l%32, h = l/32) gives A[m][h];  B: lane (n, h) gives B[h][n];
//   D: lane l, register j -> row 8*(j/4) + 4*(l/32) + j%4, column l%32.

// ---------------------------------------------------------------------------------------------
// Weight gradient (VVOR), Eq. (5).  Wave c owns triplets [c*chunk, (c+1)*chunk) of the (k, o, i)
// ordered list.  A chunk usually lies inside one cell's run; where a run starts inside the chunk the
// accumulator is flushed and restarted.  Slots of the partial buffer:
//   slot c               sum for the cell of the chunk's first triplet
//   slot n_chunks + k    sum for cell k over the part of its run that starts inside a chunk
// fp32 layers (this kernel): one MFMA step consumes 2 triplets: lane (c, h) supplies channel c of dy[o] and
// of x[i] of triplet 2 s + h.  bf16 layers use weight_wide_kernel below.
// Layers wider than one wave's accumulators: a wave owns a SUB_OUT x SUB_IN block of dW[k]; the waves that
// share a chunk are consecutive, so their re-reads of the same rows are served by the L1 / L2 caches.
// ---------------------------------------------------------------------------------------------
template <bool BF16, int C_IN, int C_OUT, int SUB_IN, int SUB_OUT>
__global__ __launch_bounds__(WAVES * 64, (!BF16 && C_IN == 32 && C_OUT == 32) ? 5 : 1) void weight_kernel(const void *__restrict__ x_, const void *__restrict__ dy_,
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
            static_assert(!BF16, "bf16 layers use weight_wide_kernel");
            {
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
                    const int co = co0 + bo * 32 + r, ci = ci0 + bi * 32 + c;
                    dstp[(size_t)co * C_IN + ci] = acc[bo][bi][j];
                }
        first = false;
        p = q;
        ++k;
    }
}

// ---------------------------------------------------------------------------------------------
// fp32 layers, second form: v_mfma_f32_16x16x4_f32 (A: lane (M = l%16, g = l/16) gives A[M][g]; B: lane
// (N = l%16, g) gives B[g][N]; D: lane l, register j -> M = 4g + j, N = l%16).  Lane (m, g) reads 8 bytes =
// channels 2m, 2m+1 (+ 32 per 32-channel group) of the rows of triplets g, 4 + g, ..., 28 + g of a batch of 32:
// one load instruction covers four rows, half the address-unit work of one channel per lane, and the loaded
// values are MFMA operands as they are (row / column m of operand (group, q) is channel 32 group + 2m + q).
// ---------------------------------------------------------------------------------------------
typedef float v2f __attribute__((ext_vector_type(2)));

template <int C_IN, int C_OUT>
__global__ __launch_bounds__(WAVES * 64) void weight_f32_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                                float *__restrict__ part,
                                                                const int32_t *__restrict__ tri_o,
                                                                const int32_t *__restrict__ tri_i,
                                                                const int64_t *__restrict__ seg, int K,
                                                                int64_t n_triplets, int chunk, int64_t n_chunks)
{
    constexpr int QO = C_OUT / 32, QI = C_IN / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int64_t chunk_id = (int64_t)blockIdx.x * WAVES + wave;
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

    v4f acc[QO][2][QI][2];
    bool first = true;
    // o (lanes 0..31) and i (lanes 32..63) of the 32 triplets from `pos` on, clamped to the list
    auto load_oi = [&](int64_t pos) -> int32_t {
        int64_t t = pos + (lane & 31);
        t = t < n_triplets ? t : n_triplets - 1;
        return lane < 32 ? tri_o[t] : tri_i[t];
    };
    int64_t pf_pos = p;
    int32_t oi_pf = load_oi(p);
    while (p < p_end) {
        int64_t q_end = seg[k + 1];
        if (q_end > p_end) q_end = p_end;
        if (q_end <= p) { ++k; continue; }   // empty run
#pragma unroll
        for (int a = 0; a < QO; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int c = 0; c < QI; ++c)
#pragma unroll
                    for (int d = 0; d < 2; ++d) acc[a][b][c][d] = v4f{0.f, 0.f, 0.f, 0.f};

        for (int64_t b0 = p; b0 < q_end; b0 += 32) {
            const int n = (int)(q_end - b0 < 32 ? q_end - b0 : 32);
            // lanes 0..31 hold o of triplet b0 + lane, lanes 32..63 hold i of triplet b0 + lane - 32: asked for one step
            // ahead (the next step starts 32 triplets on, or where the next cell's run starts), so that a step's rows
            // wait for one memory round trip, not for two in a row
            const int32_t oi = pf_pos == b0 ? oi_pf : load_oi(b0);                 // wave-uniform
            pf_pos = b0 + 32 < q_end ? b0 + 32 : q_end;
            oi_pf = load_oi(pf_pos);
            v2f dyw[QO][8], xw[QI][8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int t = 4 * e + g;
                const int32_t o = __shfl(oi, t, 64), i = __shfl(oi, 32 + t, 64);
                const v2f *dyr = reinterpret_cast<const v2f *>(dy + (size_t)o * C_OUT) + m;
                const v2f *xr = reinterpret_cast<const v2f *>(x + (size_t)i * C_IN) + m;
#pragma unroll
                for (int qo = 0; qo < QO; ++qo) dyw[qo][e] = t < n ? dyr[qo * 16] : v2f{0.f, 0.f};
#pragma unroll
                for (int qi = 0; qi < QI; ++qi) xw[qi][e] = t < n ? xr[qi * 16] : v2f{0.f, 0.f};
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int qo = 0; qo < QO; ++qo)
#pragma unroll
                    for (int qd = 0; qd < 2; ++qd)
#pragma unroll
                        for (int qi = 0; qi < QI; ++qi)
#pragma unroll
                            for (int qs = 0; qs < 2; ++qs)
                                acc[qo][qd][qi][qs] = __builtin_amdgcn_mfma_f32_16x16x4f32(dyw[qo][e][qd], xw[qi][e][qs],
                                                                                           acc[qo][qd][qi][qs], 0, 0, 0);
        }
        // flush: lane (m, g), register j of acc[qo][qd][qi][qs] is dW[32 qo + 2 (4g + j) + qd][32 qi + 2m + qs]
        float *dstp = part + (size_t)(first ? chunk_id : n_chunks + k) * C_OUT * C_IN;
#pragma unroll
        for (int qo = 0; qo < QO; ++qo)
#pragma unroll
            for (int qd = 0; qd < 2; ++qd)
#pragma unroll
                for (int qi = 0; qi < QI; ++qi)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int co = 32 * qo + 2 * (4 * g + j) + qd, ci = 32 * qi + 2 * m;
                        *reinterpret_cast<v2f *>(dstp + (size_t)co * C_IN + ci) = v2f{acc[qo][qd][qi][0][j], acc[qo][qd][qi][1][j]};
                    }
        first = false;
        p = q_end;
        ++k;
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 layers: the same chunking, with v_mfma_f32_16x16x32_bf16 (A: lane (M = l%16, g = l/16) holds
// A[M][8g .. 8g+7]; B: lane (N = l%16, g) holds B[8g .. 8g+7][N]; D: lane l, register j -> M = 4g + j,
// N = l%16).  One step consumes 32 triplets; lane (m, g) reads 8 bytes = channels 4m .. 4m+3 (+ 64 per
// 64-channel group) of the rows of triplets 8g .. 8g+7, so one load instruction covers four rows and the
// address units do half the work of dword reads.  Element q of those four channels of the eight triplets is
// one MFMA operand: row / column m of operand (group, q) is channel 64 group + 4m + q.
// ---------------------------------------------------------------------------------------------
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

template <int C_IN, int C_OUT, int SUB_IN, int SUB_OUT>
__global__ __launch_bounds__(WAVES * 64) void weight_wide_kernel(const void *__restrict__ x_, const void *__restrict__ dy_,
                                                                 float *__restrict__ part,
                                                                 const int32_t *__restrict__ tri_o,
                                                                 const int32_t *__restrict__ tri_i,
                                                                 const int64_t *__restrict__ seg, int K,
                                                                 int64_t n_triplets, int chunk, int64_t n_chunks)
{
    constexpr int QO = SUB_OUT / 64, QI = SUB_IN / 64;     // 64-channel groups of the sub-block
    constexpr int N_SUB_IN = C_IN / SUB_IN, N_SUB = N_SUB_IN * (C_OUT / SUB_OUT);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, g = lane >> 4;
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

    v4f acc[QO][4][QI][4];
    bool first = true;
    // o (lanes 0..31) and i (lanes 32..63) of the 32 triplets from `pos` on, clamped to the list
    auto load_oi = [&](int64_t pos) -> int32_t {
        int64_t t = pos + (lane & 31);
        t = t < n_triplets ? t : n_triplets - 1;
        return lane < 32 ? tri_o[t] : tri_i[t];
    };
    int64_t pf_pos = p;
    int32_t oi_pf = load_oi(p);
    while (p < p_end) {
        int64_t q_end = seg[k + 1];
        if (q_end > p_end) q_end = p_end;
        if (q_end <= p) { ++k; continue; }   // empty run
#pragma unroll
        for (int a = 0; a < QO; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int c = 0; c < QI; ++c)
#pragma unroll
                    for (int d = 0; d < 4; ++d) acc[a][b][c][d] = v4f{0.f, 0.f, 0.f, 0.f};

        for (int64_t b0 = p; b0 < q_end; b0 += 32) {
            const int n = (int)(q_end - b0 < 32 ? q_end - b0 : 32);
            // lanes 0..31 hold o of triplet b0 + lane, lanes 32..63 hold i of triplet b0 + lane - 32: asked for one step
            // ahead (the next step starts 32 triplets on, or where the next cell's run starts), so that a step's rows
            // wait for one memory round trip, not for two in a row
            const int32_t oi = pf_pos == b0 ? oi_pf : load_oi(b0);                 // wave-uniform
            pf_pos = b0 + 32 < q_end ? b0 + 32 : q_end;
            oi_pf = load_oi(pf_pos);
            v2u dyw[QO][8], xw[QI][8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int t = 8 * g + e;
                const int32_t o = __shfl(oi, t, 64), i = __shfl(oi, 32 + t, 64);
                const v2u *dyr = reinterpret_cast<const v2u *>(static_cast<const uint16_t *>(dy_) + (size_t)o * C_OUT + co0) + m;
                const v2u *xr = reinterpret_cast<const v2u *>(static_cast<const uint16_t *>(x_) + (size_t)i * C_IN + ci0) + m;
#pragma unroll
                for (int qo = 0; qo < QO; ++qo) dyw[qo][e] = t < n ? dyr[qo * 16] : v2u{0u, 0u};
#pragma unroll
                for (int qi = 0; qi < QI; ++qi) xw[qi][e] = t < n ? xr[qi * 16] : v2u{0u, 0u};
            }
            v4u bv[QI][4];
#pragma unroll
            for (int qi = 0; qi < QI; ++qi)
#pragma unroll
                for (int qs = 0; qs < 4; ++qs)
#pragma unroll
                    for (int wd = 0; wd < 4; ++wd)
                        bv[qi][qs][wd] = __builtin_amdgcn_perm(xw[qi][2 * wd + 1][qs >> 1], xw[qi][2 * wd][qs >> 1],
                                                               (qs & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
            for (int qo = 0; qo < QO; ++qo)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    v4u av;
#pragma unroll
                    for (int wd = 0; wd < 4; ++wd)
                        av[wd] = __builtin_amdgcn_perm(dyw[qo][2 * wd + 1][qd >> 1], dyw[qo][2 * wd][qd >> 1],
                                                       (qd & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
                    for (int qi = 0; qi < QI; ++qi)
#pragma unroll
                        for (int qs = 0; qs < 4; ++qs)
                            acc[qo][qd][qi][qs] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(v8bf, av), __builtin_bit_cast(v8bf, bv[qi][qs]), acc[qo][qd][qi][qs], 0, 0, 0);
                }
        }
        // flush: lane (m, g), register j of acc[qo][qd][qi][qs] is dW[co0 + 64 qo + 4 (4g + j) + qd][ci0 + 64 qi + 4m + qs]
        float *dstp = part + (size_t)(first ? chunk_id : n_chunks + k) * C_OUT * C_IN;
#pragma unroll
        for (int qo = 0; qo < QO; ++qo)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
#pragma unroll
                for (int qi = 0; qi < QI; ++qi)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int co = co0 + 64 * qo + 4 * (4 * g + j) + qd;
                        const int ci = ci0 + 64 * qi + 4 * m;
                        *reinterpret_cast<v4f *>(dstp + (size_t)co * C_IN + ci) =
                            v4f{acc[qo][qd][qi][0][j], acc[qo][qd][qi][1][j], acc[qo][qd][qi][2][j], acc[qo][qd][qi][3][j]};
                    }
        first = false;
        p = q_end;
        ++k;
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 256 -> 256: one block of eight waves per chunk, wave w owning the 128 x 64 sub-block (output channels
// 128 (w / 4) .., input channels 64 (w % 4) ..) of dW[k].  With 128 accumulator registers a wave has no room
// to keep rows in flight, and two waves per SIMD hide little of a gather's latency.  Here the block fetches every
// row of a batch of 32 triplets once (x[i] and dy[o]: 32 x 1 KB) with loads that write straight into LDS
// (global_load_lds_dwordx4: lane l of the wave writes bytes 16 l .. 16 l + 15 behind the address in M0, so one
// instruction moves two rows), into a ring of four batch buffers: rows in flight cost no registers, and the
// batches s + 1 .. s + 4 are on their way while batch s is multiplied.  The triplets' indices travel the same way
// (global_load_lds_dword into a small ring per wave), two batches ahead of their rows.
//   step s:  request the indices of batch s + 6 | first half of batch s (output channels co0 .. co0 + 63, operands
//            read during step s - 1), the LDS reads for the second half under way | wait for the rows of batch
//            s + 1, zero its dy rows past the batch's end | barrier | read the first operands of batch s + 1; second
//            half of batch s meanwhile, with one request for rows of batch s + 4 behind every four MFMAs (into the
//            buffer that batch s has just left: every wave read its last operands of it before the barrier) |
//            wait for the indices of batch s + 5, read them into registers
// The requests are spread between the MFMAs because a request can wait hundreds of cycles for room in the memory
// pipeline and the wave issues in order: bunched at the head of the step they kept the matrix pipe idle (5.1 ->
// 4.7 ms on a million-point cloud); with the operands of the next batch read during the second half, LDS reads and
// MFMAs of the block's lock-stepped waves overlap.  The rows' time in flight matters as well: requested in the second
// half of a step for the batch four ahead they have two and a half steps (4.55 ms), half a step less costs 6 %.
// Wave w moves rows 4 w .. 4 w + 3 of x and of dy.  The compiler does not see these loads, so the waits are written
// by hand; they are exact because every step issues the same five memory instructions per wave, in the same order
// (one for indices, four for rows; a batch that is short or empty re-reads its last triplet, or triplet 0): behind
// the rows to wait for, eleven younger instructions may still be outstanding, behind the indices nine.  (The partial
// sums' stores and the rare reads of a cell's bounds, which the compiler does see, only make these waits stricter.)
// A batch never crosses the end of a cell's run.  The operands are read from LDS in the layout weight_wide_kernel
// reads from memory.
// ---------------------------------------------------------------------------------------------
constexpr int LDS_WAVES = 8;
constexpr int LDS_GROUP_PITCH = 8 * 512 + 128;    // eight rows of 512 B, then 128 B: the rows r, r + 8, r + 16, r + 24 that
                                                  // one LDS read touches start in different banks
constexpr int LDS_BATCH_BYTES = 8 * LDS_GROUP_PITCH;   // 32 rows of x (four groups) then 32 rows of dy
constexpr int LDS_NBUF = 4;                        // batch buffers: batch s in s % 4
constexpr int LDS_INDEX_BYTES = LDS_WAVES * LDS_NBUF * 256;   // per wave and batch: 64 words, word 4 a + r = index of
                                                              // row 4 w + r in tri_i (a = 0) or tri_o (a = 1)
constexpr int LDS_WEIGHT_BYTES = LDS_NBUF * LDS_BATCH_BYTES + LDS_INDEX_BYTES;

// 16 bytes per lane from `src` (per lane) to LDS byte address `lds` + 16 lane (`lds` wave-uniform).  The address
// travels in M0, which the statement overwrites without saying so (the compiler reserves the register and refuses it
// as a clobber); nothing else in a compute kernel for this target lives in M0 (LDS instructions need none here).
__device__ inline void load_to_lds_b128(const void *src, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds) : "memory");
}
// 4 bytes per lane to `lds` + 4 lane
__device__ inline void load_to_lds_b32(const void *src, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(src), "s"(lds) : "memory");
}

__global__ __launch_bounds__(LDS_WAVES * 64, 2) void weight_lds_kernel(const uint16_t *__restrict__ x,
                                                                        const uint16_t *__restrict__ dy,
                                                                        float *__restrict__ part,
                                                                        const int32_t *__restrict__ tri_o,
                                                                        const int32_t *__restrict__ tri_i,
                                                                        const int64_t *__restrict__ seg, int K,
                                                                        int64_t n_triplets, int chunk, int64_t n_chunks)
{
    constexpr int C = 256, ROW = C * 2, GP = LDS_GROUP_PITCH, X_OFF = 0, DY_OFF = 4 * GP;   // row r: (r / 8) GP + (r % 8) ROW
    extern __shared__ __attribute__((aligned(16))) unsigned char stage[];        // four batches, then the index rings
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int ci0 = (wave & 3) * 64, co0 = (wave >> 2) * 128;
    const int64_t chunk_id = blockIdx.x;
    const int64_t p0 = chunk_id * chunk;                                          // positions below are relative to it
    const uint32_t q_end = (uint32_t)((p0 + chunk < n_triplets ? p0 + chunk : n_triplets) - p0);

    // cell of the first triplet: the k with seg[k] <= p0 < seg[k+1]
    int k = 0;
    for (int kb = 0; kb < K; kb += 64) {
        const int kk = kb + lane;
        const bool hit = kk < K && seg[kk] <= p0 && p0 < seg[kk + 1];
        const unsigned long long msk = __ballot(hit);
        if (msk) { k = kb + __ffsll((long long)msk) - 1; break; }
    }
    k = __builtin_amdgcn_readfirstlane(k);
    // A batch travels through the steps as one word: triplets | ends its run << 8 | cell << 16 (0: no batch).  run_end:
    // end of cell k's run inside the chunk, read from seg only when the cell changes.
    auto end_of = [&](int kk) -> uint32_t {
        const int64_t e = seg[kk + 1] - p0;
        return e < (int64_t)q_end ? (uint32_t)e : q_end;
    };
    uint32_t q = 0, run_end = end_of(k);
    uint32_t q5 = 0;                              // first triplet of the batch that next_batch returned last
    auto next_batch = [&]() -> uint32_t {
        while (q < q_end) {
            if (run_end <= q) {                       // next cell (empty runs are passed over)
                ++k;
                run_end = end_of(k);
                continue;
            }
            const uint32_t n = run_end - q < 32u ? run_end - q : 32u;
            q5 = q;
            q += n;
            return n | (q == run_end ? 256u : 0u) | ((uint32_t)k << 16);
        }
        q5 = 0;
        return 0u;
    };

    // mover role of this lane: rows 4 wave + 2 j + half (j = 0, 1), bytes 16 piece .. of the row
    const int half = lane >> 5, piece = lane & 31;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)(stage);
    const uint32_t ring0 = lds0 + LDS_NBUF * LDS_BATCH_BYTES + wave * (LDS_NBUF * 256);
    const unsigned char *ring = stage + LDS_NBUF * LDS_BATCH_BYTES + wave * (LDS_NBUF * 256);
    const unsigned char *xb = reinterpret_cast<const unsigned char *>(x) + piece * 16;
    const unsigned char *dyb = reinterpret_cast<const unsigned char *>(dy) + piece * 16;
    // index requests: lane -> (array, row lane % 4)
    const int32_t *tri_lane = (((lane >> 2) & 1) ? tri_o : tri_i) + p0;
    const int r_lane = 4 * wave + (lane & 3);

    // the first steps request rows before any index has arrived: they read zeros (row 0) from the ring
    *reinterpret_cast<v4u *>(stage + LDS_NBUF * LDS_BATCH_BYTES + wave * (LDS_NBUF * 256) + lane * 16) = v4u{0u, 0u, 0u, 0u};
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

    uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0, w4 = 0, w5 = 0, w6 = next_batch();      // batches s .. s + 6
    int cur = 0;                                  // buffer of batch s

    v4f acc[2][4][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int d = 0; d < 4; ++d) acc[a][b][d] = v4f{0.f, 0.f, 0.f, 0.f};
    bool first = true;

    // operands of batch s that are read during step s - 1: the x side as MFMA operands, the dy rows of the first half
    v4u bv[4];
    v2u dyw0[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) bv[e] = v4u{0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e) dyw0[e] = v2u{0u, 0u};
    int32_t ix[2] = {0, 0}, io[2] = {0, 0};     // rows 4 wave + 2 j + half of the batch whose rows are requested next
    // acc[qo][qd] += dy(16 channels)^T . x over the batch's 32 triplets; dyw: this lane's words of the dy rows
    auto multiply = [&](int qo, int qd, const v2u (&dyw)[8]) __attribute__((always_inline)) {
        v4u av;
#pragma unroll
        for (int wd = 0; wd < 4; ++wd)
            av[wd] = __builtin_amdgcn_perm(dyw[2 * wd + 1][qd >> 1], dyw[2 * wd][qd >> 1],
                                           (qd & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
        for (int qs = 0; qs < 4; ++qs)
            acc[qo][qd][qs] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(v8bf, av), __builtin_bit_cast(v8bf, bv[qs]), acc[qo][qd][qs], 0, 0, 0);
    };

    // one step; COMPUTE = false for the six steps that fill the pipeline (no batch s yet).  Once a batch has reached
    // the front, every step has one until the chunk is used up, and nothing is left behind the last one.
    auto step = [&](auto compute) __attribute__((always_inline)) {
        constexpr bool COMPUTE = decltype(compute)::value;
        // indices of batch s + 6
        {
            const int n6 = (int)(w6 & 255u);
            int t = (int)q5 + (r_lane < n6 ? r_lane : n6 - 1);
            if (t < 0) t = 0;
            load_to_lds_b32(tri_lane + t, (uint32_t)__builtin_amdgcn_readfirstlane((int)(ring0 + ((cur + 6) & 3) * 256)));
        }
        // rows of batch s + 3, one request behind every four MFMAs of the first half of batch s (output channels
        // co0 .. co0 + 63; its operands were read one step ago): a request can wait long for room in the memory
        // pipeline, and the matrix pipe should have work meanwhile.  The reads for the second half go first.
        const unsigned char *buf = stage + cur * LDS_BATCH_BYTES;
        v2u dyw1[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            dyw1[e] = *reinterpret_cast<const v2u *>(buf + DY_OFF + g * GP + e * ROW + (co0 + 64 + 4 * m) * 2);
        if constexpr (COMPUTE) {
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) multiply(0, qd, dyw0);
        }
        // the rows of batch s + 1 have arrived; past its end the dy rows become zeros (the x rows there repeat the
        // batch's last triplet)
        asm volatile("s_waitcnt vmcnt(11)" ::: "memory");
        {
            const int n1 = (int)(w1 & 255u);
            if (n1 > 0 && n1 < 32) {
                unsigned char *dst = stage + ((cur + 1) & 3) * LDS_BATCH_BYTES + DY_OFF + piece * 16;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int r = 4 * wave + 2 * j + half;
                    if (r >= n1) *reinterpret_cast<v4u *>(dst + (r >> 3) * GP + (r & 7) * ROW) = v4u{0u, 0u, 0u, 0u};
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        // batch s + 1 is complete in LDS: ask for its first operands, multiply the second half of batch s meanwhile
        const unsigned char *nbuf = stage + ((cur + 1) & 3) * LDS_BATCH_BYTES;
        v2u xw[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            xw[e] = *reinterpret_cast<const v2u *>(nbuf + X_OFF + g * GP + e * ROW + (ci0 + 4 * m) * 2);
        v2u dyn[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            dyn[e] = *reinterpret_cast<const v2u *>(nbuf + DY_OFF + g * GP + e * ROW + (co0 + 4 * m) * 2);
        {
            // rows of batch s + 4 into the buffer that batch s has just left (every wave has read its last operands
            // of it before the barrier), one request behind every four MFMAs of the second half
            const uint32_t dst = lds0 + (uint32_t)cur * LDS_BATCH_BYTES + (uint32_t)((wave >> 1) * GP + 4 * (wave & 1) * ROW);
            auto request = [&](int i) __attribute__((always_inline)) {
                const int j = i >> 1;
                if (i & 1)
                    load_to_lds_b128(dyb + (size_t)io[j] * ROW,
                                     (uint32_t)__builtin_amdgcn_readfirstlane((int)(dst + DY_OFF + 2 * j * ROW)));
                else
                    load_to_lds_b128(xb + (size_t)ix[j] * ROW,
                                     (uint32_t)__builtin_amdgcn_readfirstlane((int)(dst + X_OFF + 2 * j * ROW)));
            };
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                if constexpr (COMPUTE) multiply(1, qd, dyw1);
                request(qd);
            }
        }
        if constexpr (COMPUTE) {
            if (w0 & 256u) {
                // flush: lane (m, g), register j of acc[qo][qd][qs] is dW[co0 + 64 qo + 4 (4g + j) + qd][ci0 + 4m + qs]
                float *dstp = part + (size_t)(first ? chunk_id : n_chunks + (w0 >> 16)) * C * C;
#pragma unroll
                for (int qo = 0; qo < 2; ++qo)
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int co = co0 + 64 * qo + 4 * (4 * g + j) + qd;
                            const int ci = ci0 + 4 * m;
                            *reinterpret_cast<v4f *>(dstp + (size_t)co * C + ci) =
                                v4f{acc[qo][qd][0][j], acc[qo][qd][1][j], acc[qo][qd][2][j], acc[qo][qd][3][j]};
                            acc[qo][qd][0][j] = acc[qo][qd][1][j] = acc[qo][qd][2][j] = acc[qo][qd][3][j] = 0.f;
                        }
                first = false;
            }
        }
#pragma unroll
        for (int qs = 0; qs < 4; ++qs)
#pragma unroll
            for (int wd = 0; wd < 4; ++wd)
                bv[qs][wd] = __builtin_amdgcn_perm(xw[2 * wd + 1][qs >> 1], xw[2 * wd][qs >> 1],
                                                   (qs & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
        for (int e = 0; e < 8; ++e) dyw0[e] = dyn[e];
        // the indices of batch s + 5 (asked for at the head of the step before) into registers for the next step's row
        // requests
        asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
        {
            const unsigned char *words = ring + ((cur + 5) & 3) * 256;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                ix[j] = *reinterpret_cast<const int32_t *>(words + 4 * (2 * j + half));
                io[j] = *reinterpret_cast<const int32_t *>(words + 4 * (4 + 2 * j + half));
            }
        }
        w0 = w1; w1 = w2; w2 = w3; w3 = w4; w4 = w5; w5 = w6; w6 = next_batch();
        cur = (cur + 1) & 3;
    };
    for (int f = 0; f < 6; ++f) step(std::false_type{});
    while (w0) step(std::true_type{});
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // nothing of this wave is still on its way into LDS
}

// dw[k][e] = (partial of the run's head, if it starts inside a chunk) + partials of the chunks whose first
// triplet lies in run k.  A block of four waves owns 64 consecutive elements of one cell: wave w adds chunks
// c0 + w, c0 + w + 4, ... in ascending order (each read is 256 contiguous bytes) and the four sums are then
// added in order of w, so the result is reproducible.  grid = (ceil(c_out*c_in / 64), K), block = 256
constexpr int REDUCE_WAVES = 4;

__global__ __launch_bounds__(REDUCE_WAVES * 64) void weight_reduce(const float *__restrict__ part, float *__restrict__ dw,
                                                                   const int64_t *__restrict__ seg, int n_elem, int chunk,
                                                                   int64_t n_chunks)
{
    __shared__ float sums[REDUCE_WAVES][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + lane;
    const int k = blockIdx.y;
    const int64_t s = seg[k], t = seg[k + 1];
    float v = 0.f;
    if (t > s && e < n_elem) {
        const int64_t c0 = (s + chunk - 1) / chunk, c1 = (t + chunk - 1) / chunk;
        const float *src = part + (size_t)e;
        int64_t c = c0 + wave;
        for (; c + 3 * REDUCE_WAVES < c1; c += 4 * REDUCE_WAVES) {      // four independent reads in flight
            const float v0 = src[(size_t)c * n_elem], v1 = src[(size_t)(c + REDUCE_WAVES) * n_elem];
            const float v2 = src[(size_t)(c + 2 * REDUCE_WAVES) * n_elem], v3 = src[(size_t)(c + 3 * REDUCE_WAVES) * n_elem];
            v = (((v + v0) + v1) + v2) + v3;
        }
        for (; c < c1; c += REDUCE_WAVES) v += src[(size_t)c * n_elem];
    }
    sums[wave][lane] = v;
    __syncthreads();
    if (wave == 0 && e < n_elem) {
        float r = (t > s && s % chunk != 0) ? part[(size_t)(n_chunks + k) * n_elem + e] : 0.f;
#pragma unroll
        for (int w = 0; w < REDUCE_WAVES; ++w) r += sums[w][lane];
        dw[(size_t)k * n_elem + e] = r;
    }
}

// Triplets per chunk.  The blocks of a launch (`per_block` chunks each) are spread evenly over the CUs, and the
// kernels run at a fixed rate per CU, so a launch takes as long as the CU with the most blocks: the chunk length
// is chosen so that the number of blocks is a whole multiple m of the CU count, with about a thousand triplets
// per chunk and at most 8192 chunks (2048 for wide layers, whose partial sums are large).  Clouds too small for
// one block per CU keep chunks of 512.
constexpr int64_t DEVICE_CUS = 256;           // MI355X

int weight_chunk(int64_t n_triplets, int c_in, int c_out, int per_block)
{
    const int64_t max_chunks = (int64_t)c_in * c_out >= 128 * 128 ? 2048 : 8192;
    const int64_t per_round = DEVICE_CUS * per_block;                  // chunks of one block on every CU
    int64_t m = (n_triplets + per_round * 500) / (per_round * 1000);     // nearest whole number of rounds
    if (m > max_chunks / per_round) m = max_chunks / per_round;
    if (m < 1 || n_triplets < per_round * 512) {
        int chunk = 512;
        while ((n_triplets + chunk - 1) / chunk > max_chunks) chunk *= 2;
        return chunk;
    }
    const int64_t chunk = ceil_div(n_triplets, per_round * m);
    return (int)((chunk + 31) / 32 * 32);
}

// chunks handled by one block of the kernel that serves the shape
int weight_chunks_per_block(bool bf16, int c_in, int c_out)
{
    if (bf16 && c_in == 256 && c_out == 256) return 1;                 // weight_lds_kernel
    if (bf16 && c_in >= 128 && c_out >= 128) return WAVES / 2;          // two sub-block waves per chunk
    return WAVES;                                                       // one wave per chunk
}

template <bool BF16, int C_IN, int C_OUT, int SUB_IN = C_IN, int SUB_OUT = C_OUT>
int launch_weight(const MvmrArgs &a, float *dw, const int32_t *tri_o, const int64_t *seg, void *workspace,
                  size_t workspace_bytes, hipStream_t stream)
{
    const int n_elem = C_IN * C_OUT;
    const int chunk = weight_chunk(a.n_triplets, C_IN, C_OUT, weight_chunks_per_block(BF16, C_IN, C_OUT));
    const int64_t n_chunks = ceil_div(a.n_triplets, chunk);
    constexpr int N_SUB = (C_IN / SUB_IN) * (C_OUT / SUB_OUT);
    const size_t need = (size_t)(n_chunks + a.K) * n_elem * sizeof(float);
    if (workspace_bytes < need) {
        set_error("pcpp_mvmr_bwd_weight: workspace has %zu bytes, needs %zu", workspace_bytes, need);
        return PCPP_ERR_WORKSPACE;
    }
    float *part = static_cast<float *>(workspace);
    if (n_chunks > 0) {
        // (16-byte row reads: the entry point has checked that x and dy are 16-byte aligned, and rows are 512 bytes)
        if constexpr (BF16 && C_IN == 256 && C_OUT == 256) {
            if (int rc = raise_lds_limit(reinterpret_cast<const void *>(&weight_lds_kernel), LDS_WEIGHT_BYTES)) return rc;
            weight_lds_kernel<<<(unsigned)n_chunks, LDS_WAVES * 64, LDS_WEIGHT_BYTES, stream>>>(
                static_cast<const uint16_t *>(a.feat), static_cast<const uint16_t *>(a.dense), part, tri_o, a.gather, seg,
                a.K, a.n_triplets, chunk, n_chunks);
        } else if constexpr (!BF16 && SUB_IN == C_IN && SUB_OUT == C_OUT)
            weight_f32_kernel<C_IN, C_OUT><<<(unsigned)ceil_div(n_chunks, WAVES), WAVES * 64, 0, stream>>>(
                static_cast<const float *>(a.feat), static_cast<const float *>(a.dense), part, tri_o, a.gather, seg, a.K,
                a.n_triplets, chunk, n_chunks);
        else if constexpr (BF16)
            weight_wide_kernel<C_IN, C_OUT, SUB_IN, SUB_OUT><<<(unsigned)ceil_div(n_chunks * N_SUB, WAVES), WAVES * 64, 0, stream>>>(
                a.feat, a.dense, part, tri_o, a.gather, seg, a.K, a.n_triplets, chunk, n_chunks);
        else
            weight_kernel<BF16, C_IN, C_OUT, SUB_IN, SUB_OUT><<<(unsigned)ceil_div(n_chunks * N_SUB, WAVES), WAVES * 64, 0, stream>>>(
                a.feat, a.dense, part, tri_o, a.gather, seg, a.K, a.n_triplets, chunk, n_chunks);
        PCPP_HIP_CHECK(hipGetLastError());
    }
    dim3 grid((unsigned)ceil_div(n_elem, 64), (unsigned)a.K);
    weight_reduce<<<grid, REDUCE_WAVES * 64, 0, stream>>>(part, dw, seg, n_elem, chunk, n_chunks);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

bool weight_shape_supported(int in_dtype, int c_in, int c_out)
{
    if (in_dtype == PCPP_F32) return (c_in == 32 && c_out == 32) || (c_in == 64 && c_out == 64);
    return (c_in == 64 && c_out == 64) || (c_in == 64 && c_out == 128) || (c_in == 128 && c_out == 128) ||
           (c_in == 256 && c_out == 256);
}

}  // namespace

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
    const int chunk = weight_chunk(n_triplets, c_in, c_out, weight_chunks_per_block(in_dtype == PCPP_BF16, c_in, c_out));
    return align_up((size_t)(ceil_div(n_triplets, chunk) + K) * c_in * c_out * sizeof(float));
}

}  // namespace pcpp
