// Matrix-core (MFMA) MVMR kernels for gfx950.
//
// Rows kernel (Eq. (1) forward; Sec. 3.3.3 input gradient with W^T): one wave owns 32 consecutive
// centres and every destination channel.  For each kernel cell k it
//   1. sums the source rows of each (k, centre) run in fp32 registers -- the lanes are laid out so that
//      the summed tile already is the MFMA A operand: lane (m = lane % 32, h = lane / 32) holds
//      channels [h*C/2, (h+1)*C/2) of centre m -- no LDS, no barrier, waves run independently;
//   2. multiplies the 32 x C_SRC tile by W[k]^T on the matrix cores into fp32 accumulators that stay
//      in registers for the whole cell loop.
// The reduction index of the MFMA is permuted (step s of half h <-> channel h*C/2 + s, or the s-th
// group of 8 for bf16) identically for both operands, so every lane reads contiguous memory.
// Each destination row is written once by its owner: no atomics, fixed summation order.
#include "pcpp_internal.h"

namespace pcpp {

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int WAVES = 4;
constexpr int ROWS = 32;   // centres per wave

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

// ---------------------------------------------------------------------------------------------
// fp32: v_mfma_f32_32x32x2_f32.  A: lane (m, h) gives A[m][h]; B: lane (n, h) gives B[h][n];
// D: lane l, register j -> row 8*(j/4) + 4*(l/32) + j%4, column l%32.
// ---------------------------------------------------------------------------------------------
template <int C_SRC, int C_DST>
__global__ __launch_bounds__(WAVES * 64) void rows_f32_kernel(const float *__restrict__ feat,
                                                              const float *__restrict__ w, float *__restrict__ dst,
                                                              int64_t n_centres, int K,
                                                              const int32_t *__restrict__ gather, PlanSideView side)
{
    constexpr int HALF = C_SRC / 2;       // channels per lane
    constexpr int NV = HALF / 4;          // float4 loads per source row per lane
    constexpr int NB = C_DST / 32;        // 32-wide destination blocks
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int64_t blk = (int64_t)blockIdx.x * WAVES + wave;   // 32-row block
    const int64_t row0 = blk * ROWS;
    if (row0 >= n_centres) return;
    const int64_t tile = blk >> 1;
    const int sub = (int)(blk & 1) * ROWS;                     // offset of this block inside its 64-tile
    const bool last_in_tile = (sub + m) == TILE - 1;

    v16f acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[b][j] = 0.f;

    for (int k = 0; k < K; ++k) {
        const uint32_t *rs = side.run_start + ((size_t)tile * K + k) * TILE + sub + m;
        const uint32_t st = rs[0];
        const uint32_t en = last_in_tile ? side.tile_ptr[(size_t)k * side.n_tiles + tile + 1] : rs[1];
        const uint32_t cnt = en - st;
        if (__ballot(cnt != 0) == 0) continue;                 // no neighbour in this cell for these 32 centres

        // W[k] fragments: lane (n, h) reads W[k][b*32 + n][h*HALF .. +HALF)
        v4f bw[NB][NV];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const v4f *wp = reinterpret_cast<const v4f *>(w + ((size_t)k * C_DST + b * 32 + m) * C_SRC + h * HALF);
#pragma unroll
            for (int v = 0; v < NV; ++v) bw[b][v] = wp[v];
        }

        // sum of the source rows of centre m in cell k, this lane's half of the channels
        v4f xs[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) xs[v] = v4f{0.f, 0.f, 0.f, 0.f};
        for (uint32_t j = 0; j < cnt; ++j) {
            const int32_t src = gather[st + j];
            const v4f *xp = reinterpret_cast<const v4f *>(feat + (size_t)src * C_SRC + h * HALF);
#pragma unroll
            for (int v = 0; v < NV; ++v) xs[v] += xp[v];
        }

#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[v][e], bw[b][v][e], acc[b], 0, 0, 0);
    }

#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t row = row0 + 8 * (j / 4) + 4 * h + (j % 4);
            if (row < n_centres) dst[(size_t)row * C_DST + b * 32 + m] = acc[b][j];
        }
}

// ---------------------------------------------------------------------------------------------
// bf16: v_mfma_f32_32x32x16_bf16.  A: lane (m, h) gives A[m][8h .. 8h+7]; B likewise; D as above.
// The summed rows are rounded to bf16 once (the inputs carry the same precision).
// ---------------------------------------------------------------------------------------------
template <int C_SRC, int C_DST, typename TOut>
__global__ __launch_bounds__(WAVES * 64) void rows_bf16_kernel(const uint16_t *__restrict__ feat,
                                                               const uint16_t *__restrict__ w,
                                                               TOut *__restrict__ dst, int64_t n_centres, int K,
                                                               const int32_t *__restrict__ gather, PlanSideView side)
{
    constexpr int HALF = C_SRC / 2;       // channels per lane
    constexpr int NV = HALF / 8;          // 16-byte loads per source row per lane = MFMA steps
    constexpr int NB = C_DST / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int64_t blk = (int64_t)blockIdx.x * WAVES + wave;
    const int64_t row0 = blk * ROWS;
    if (row0 >= n_centres) return;
    const int64_t tile = blk >> 1;
    const int sub = (int)(blk & 1) * ROWS;
    const bool last_in_tile = (sub + m) == TILE - 1;

    v16f acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[b][j] = 0.f;

    for (int k = 0; k < K; ++k) {
        const uint32_t *rs = side.run_start + ((size_t)tile * K + k) * TILE + sub + m;
        const uint32_t st = rs[0];
        const uint32_t en = last_in_tile ? side.tile_ptr[(size_t)k * side.n_tiles + tile + 1] : rs[1];
        const uint32_t cnt = en - st;
        if (__ballot(cnt != 0) == 0) continue;

        v4u bw[NB][NV];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const v4u *wp = reinterpret_cast<const v4u *>(w + ((size_t)k * C_DST + b * 32 + m) * C_SRC + h * HALF);
#pragma unroll
            for (int v = 0; v < NV; ++v) bw[b][v] = wp[v];
        }

        float xs[NV][8];
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int e = 0; e < 8; ++e) xs[v][e] = 0.f;
        for (uint32_t j = 0; j < cnt; ++j) {
            const int32_t src = gather[st + j];
            const v4u *xp = reinterpret_cast<const v4u *>(feat + (size_t)src * C_SRC + h * HALF);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const v4u q = xp[v];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    xs[v][2 * e] += __uint_as_float(q[e] << 16);
                    xs[v][2 * e + 1] += __uint_as_float(q[e] & 0xffff0000u);
                }
            }
        }

#pragma unroll
        for (int v = 0; v < NV; ++v) {
            v4u a;
#pragma unroll
            for (int e = 0; e < 4; ++e) a[e] = pack_bf16x2(xs[v][2 * e], xs[v][2 * e + 1]);
            const v8bf av = __builtin_bit_cast(v8bf, a);
#pragma unroll
            for (int b = 0; b < NB; ++b)
                acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(v8bf, bw[b][v]), acc[b], 0, 0, 0);
        }
    }

#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int64_t row = row0 + 8 * (j / 4) + 4 * h + (j % 4);
            if (row < n_centres) {
                if constexpr (sizeof(TOut) == 4) {
                    dst[(size_t)row * C_DST + b * 32 + m] = acc[b][j];
                } else {
                    dst[(size_t)row * C_DST + b * 32 + m] = (uint16_t)(pack_bf16x2(acc[b][j], 0.f) & 0xffffu);
                }
            }
        }
}

template <int C_SRC, int C_DST>
int launch_f32(const MvmrArgs &a, hipStream_t stream)
{
    const int64_t blocks = ceil_div(ceil_div(a.n_centres, ROWS), WAVES);
    rows_f32_kernel<C_SRC, C_DST><<<(unsigned)blocks, WAVES * 64, 0, stream>>>(
        static_cast<const float *>(a.feat), static_cast<const float *>(a.w), static_cast<float *>(a.dst),
        a.n_centres, a.K, a.gather, a.side);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

template <int C_SRC, int C_DST>
int launch_bf16(const MvmrArgs &a, hipStream_t stream)
{
    const int64_t blocks = ceil_div(ceil_div(a.n_centres, ROWS), WAVES);
    if (a.out_dtype == PCPP_F32)
        rows_bf16_kernel<C_SRC, C_DST, float><<<(unsigned)blocks, WAVES * 64, 0, stream>>>(
            static_cast<const uint16_t *>(a.feat), static_cast<const uint16_t *>(a.w), static_cast<float *>(a.dst),
            a.n_centres, a.K, a.gather, a.side);
    else
        rows_bf16_kernel<C_SRC, C_DST, uint16_t><<<(unsigned)blocks, WAVES * 64, 0, stream>>>(
            static_cast<const uint16_t *>(a.feat), static_cast<const uint16_t *>(a.w),
            static_cast<uint16_t *>(a.dst), a.n_centres, a.K, a.gather, a.side);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

}  // namespace

int mvmr_rows_mfma(const MvmrArgs &a, hipStream_t stream, bool *handled)
{
    *handled = true;
    if (a.in_dtype == PCPP_F32) {
        if (a.c_src == 32 && a.c_dst == 32) return launch_f32<32, 32>(a, stream);
        if (a.c_src == 16 && a.c_dst == 32) return launch_f32<16, 32>(a, stream);
        if (a.c_src == 64 && a.c_dst == 64) return launch_f32<64, 64>(a, stream);
    } else {
        if (a.c_src == 64 && a.c_dst == 64) return launch_bf16<64, 64>(a, stream);
        if (a.c_src == 64 && a.c_dst == 128) return launch_bf16<64, 128>(a, stream);
        if (a.c_src == 128 && a.c_dst == 64) return launch_bf16<128, 64>(a, stream);
        if (a.c_src == 32 && a.c_dst == 32) return launch_bf16<32, 32>(a, stream);
    }
    *handled = false;
    return PCPP_OK;
}

}  // namespace pcpp
