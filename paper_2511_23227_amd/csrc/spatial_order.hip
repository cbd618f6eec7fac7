// Order of a point set along a space-filling curve, for plans built with PCPP_PLAN_SPATIAL.
//
// The rows kernels give every block a tile of consecutive centres (Sec. 3.3.2 groups consecutive triplets the
// same way); when consecutive centres are also neighbours in space the block's source rows and weight slices
// are shared through the caches and whole kernel cells are empty for the block.  This file computes that order
// inside the library so that it does not depend on the caller's point order: Morton code (10 bits per axis) of
// the point's cell in a grid of the given pitch, counted from the cloud's lowest cell, then a stable
// least-significant-digit radix sort of (code, index) in three passes of 10 bits.  Equal codes keep index order,
// so the result is a pure function of the coordinates.
#include <limits.h>
#include <math.h>

#include "pcpp_internal.h"

namespace pcpp {

namespace {

constexpr int SO_THREADS = 256;
constexpr int SO_WAVES = SO_THREADS / 64;
constexpr int SO_ITEMS = 16;                         // per thread
constexpr int SO_BLOCK = SO_THREADS * SO_ITEMS;      // keys per block
constexpr int SO_BITS = 10;                          // per pass and per axis
constexpr int SO_BINS = 1 << SO_BITS;
constexpr int SO_PASSES = 3;
constexpr double SO_CLAMP = 1048574.0;

__device__ inline int so_coord(float p, double inv_pitch)
{
    double u = floor((double)p * inv_pitch);
    u = fmin(fmax(u, -SO_CLAMP), SO_CLAMP);          // NaN falls to a bound
    return (int)u;
}

__global__ void so_init(int *mins)
{
    if (threadIdx.x < 3) mins[threadIdx.x] = INT_MAX;
}

// Lowest grid coordinate per axis.  so_coord never decreases with the coordinate, so the minimum is taken over the
// floats and converted once per block; one atomic per block and axis.
__global__ __launch_bounds__(SO_THREADS) void so_min(const float *__restrict__ xyz, int64_t n, double inv_pitch,
                                                     int *__restrict__ mins)
{
    __shared__ float part[SO_WAVES][3];
    float m[3] = {INFINITY, INFINITY, INFINITY};
    const int64_t stride = (int64_t)gridDim.x * SO_THREADS;
    for (int64_t p = (int64_t)blockIdx.x * SO_THREADS + threadIdx.x; p < n; p += stride)
#pragma unroll
        for (int a = 0; a < 3; ++a) m[a] = fminf(m[a], xyz[3 * p + a]);     // a NaN is passed over
#pragma unroll
    for (int a = 0; a < 3; ++a) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) m[a] = fminf(m[a], __shfl_xor(m[a], d, 64));
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6][a] = m[a];
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        float v = part[0][threadIdx.x];
        for (int w = 1; w < SO_WAVES; ++w) v = fminf(v, part[w][threadIdx.x]);
        atomicMin(&mins[threadIdx.x], so_coord(v, inv_pitch));
    }
}

__device__ inline uint32_t spread3(uint32_t v)       // bit b of v -> bit 3 b
{
    v &= 0x3ffu;
    v = (v | (v << 16)) & 0x030000ffu;
    v = (v | (v << 8)) & 0x0300f00fu;
    v = (v | (v << 4)) & 0x030c30c3u;
    v = (v | (v << 2)) & 0x09249249u;
    return v;
}

__global__ __launch_bounds__(SO_THREADS) void so_keys(const float *__restrict__ xyz, int64_t n, double inv_pitch,
                                                      const int *__restrict__ mins, uint32_t *__restrict__ keys,
                                                      uint32_t *__restrict__ vals)
{
    const int64_t p = (int64_t)blockIdx.x * SO_THREADS + threadIdx.x;
    if (p >= n) return;
    uint32_t q[3];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        const long long d = (long long)so_coord(xyz[3 * p + a], inv_pitch) - (long long)mins[a];
        q[a] = (uint32_t)(d < 0 ? 0 : (d > SO_BINS - 1 ? SO_BINS - 1 : d));
    }
    keys[p] = (spread3(q[0]) << 2) | (spread3(q[1]) << 1) | spread3(q[2]);
    vals[p] = (uint32_t)p;
}

// table[d * n_blocks + block] = number of keys of the block whose digit is d
__global__ __launch_bounds__(SO_THREADS) void so_hist(const uint32_t *__restrict__ keys, int64_t n, int shift,
                                                      uint32_t *__restrict__ table, int64_t n_blocks)
{
    __shared__ uint32_t h[SO_BINS];
    for (int d = threadIdx.x; d < SO_BINS; d += SO_THREADS) h[d] = 0u;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * SO_BLOCK;
    for (int r = 0; r < SO_ITEMS; ++r) {
        const int64_t idx = base + (int64_t)r * SO_THREADS + threadIdx.x;
        if (idx < n) atomicAdd(&h[(keys[idx] >> shift) & (SO_BINS - 1)], 1u);
    }
    __syncthreads();
    for (int d = threadIdx.x; d < SO_BINS; d += SO_THREADS) table[(size_t)d * n_blocks + blockIdx.x] = h[d];
}

// Stable scatter of one pass.  Item order inside a block: wave-major, then round, then lane; an item's place is
// (start of its digit for this block, from the scanned table) + (items with the same digit before it in the block).
__global__ __launch_bounds__(SO_THREADS) void so_scatter(const uint32_t *__restrict__ keys,
                                                         const uint32_t *__restrict__ vals, int64_t n, int shift,
                                                         const uint32_t *__restrict__ table, int64_t n_blocks,
                                                         uint32_t *__restrict__ keys_out, uint32_t *__restrict__ vals_out,
                                                         const uint32_t *__restrict__ err)
{
    __shared__ uint32_t cnt[SO_WAVES][SO_BINS];
    if (err && *err) return;                         // the offsets come from a prefix sum that did not finish
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int d = threadIdx.x; d < SO_WAVES * SO_BINS; d += SO_THREADS) (&cnt[0][0])[d] = 0u;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * SO_BLOCK + (int64_t)wave * (SO_ITEMS * 64);
    const unsigned long long lane_lt = (1ull << lane) - 1ull;
    uint32_t key[SO_ITEMS], val[SO_ITEMS], local[SO_ITEMS];
#pragma unroll
    for (int r = 0; r < SO_ITEMS; ++r) {
        const int64_t idx = base + r * 64 + lane;
        const bool valid = idx < n;
        key[r] = valid ? keys[idx] : 0xffffffffu;    // padding sorts behind everything and is never written
        val[r] = valid ? vals[idx] : 0u;
    }
#pragma unroll
    for (int r = 0; r < SO_ITEMS; ++r) {
        const uint32_t d = (key[r] >> shift) & (SO_BINS - 1);
        unsigned long long same = ~0ull;
#pragma unroll
        for (int b = 0; b < SO_BITS; ++b) {
            const unsigned long long m = __ballot((d >> b) & 1u);
            same &= ((d >> b) & 1u) ? m : ~m;
        }
        const uint32_t before = (uint32_t)__popcll(same & lane_lt);
        const uint32_t prev = cnt[wave][d];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (before == 0) cnt[wave][d] = prev + (uint32_t)__popcll(same);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        local[r] = prev + before;
    }
    __syncthreads();
    for (int d = threadIdx.x; d < SO_BINS; d += SO_THREADS) {
        uint32_t run = table[(size_t)d * n_blocks + blockIdx.x];
#pragma unroll
        for (int w = 0; w < SO_WAVES; ++w) {
            const uint32_t c = cnt[w][d];
            cnt[w][d] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < SO_ITEMS; ++r) {
        const int64_t idx = base + r * 64 + lane;
        if (idx < n) {
            const uint32_t pos = cnt[wave][(key[r] >> shift) & (SO_BINS - 1)] + local[r];
            if (pos < (uint64_t)n) {
                if (keys_out) keys_out[pos] = key[r];
                vals_out[pos] = val[r];
            }
        }
    }
}

struct SoScratch {
    size_t mins_off, keys_off[2], vals_off[2], table_off, end;
    int64_t n_blocks;
};

SoScratch so_scratch(int64_t n)
{
    SoScratch s;
    const size_t m = (size_t)(n > 0 ? n : 1);
    s.n_blocks = ceil_div((int64_t)m, SO_BLOCK);
    size_t off = 0;
    s.mins_off = off; off += 256;
    for (int i = 0; i < 2; ++i) { s.keys_off[i] = off; off += align_up(m * 4); }
    for (int i = 0; i < 2; ++i) { s.vals_off[i] = off; off += align_up(m * 4); }
    s.table_off = off; off += align_up(((size_t)SO_BINS * s.n_blocks + 1) * 4);
    s.end = off;
    return s;
}

}  // namespace

size_t spatial_order_scratch_bytes(int64_t n) { return so_scratch(n).end; }

int64_t spatial_order_scan_items(int64_t n) { return (int64_t)SO_BINS * so_scratch(n).n_blocks; }

int spatial_order(const float *xyz, int64_t n, double pitch, int32_t *perm, void *scratch, void *scan_status,
                  size_t scan_stride, uint32_t *err, hipStream_t stream)
{
    static_assert(SO_PASSES <= SPATIAL_ORDER_SCANS, "one set of status words per pass");
    if (n <= 0) return PCPP_OK;
    const SoScratch s = so_scratch(n);
    char *ws = static_cast<char *>(scratch);
    int *mins = reinterpret_cast<int *>(ws + s.mins_off);
    uint32_t *keys[2] = {reinterpret_cast<uint32_t *>(ws + s.keys_off[0]), reinterpret_cast<uint32_t *>(ws + s.keys_off[1])};
    uint32_t *vals[2] = {reinterpret_cast<uint32_t *>(ws + s.vals_off[0]), reinterpret_cast<uint32_t *>(ws + s.vals_off[1])};
    uint32_t *table = reinterpret_cast<uint32_t *>(ws + s.table_off);
    const double inv_pitch = 1.0 / pitch;
    int64_t rb = ceil_div(n, SO_THREADS);
    if (rb > 512) rb = 512;
    so_init<<<1, 64, 0, stream>>>(mins);
    so_min<<<(unsigned)rb, SO_THREADS, 0, stream>>>(xyz, n, inv_pitch, mins);
    so_keys<<<(unsigned)ceil_div(n, SO_THREADS), SO_THREADS, 0, stream>>>(xyz, n, inv_pitch, mins, keys[0], vals[0]);
    PCPP_HIP_CHECK(hipGetLastError());
    int rc;
    for (int p = 0; p < SO_PASSES; ++p) {
        const int src = p & 1, dst = src ^ 1;
        const bool last = p == SO_PASSES - 1;
        so_hist<<<(unsigned)s.n_blocks, SO_THREADS, 0, stream>>>(keys[src], n, p * SO_BITS, table, s.n_blocks);
        PCPP_HIP_CHECK(hipGetLastError());
        if ((rc = scan_exclusive_u32(table, table, (int64_t)SO_BINS * s.n_blocks,
                                     static_cast<char *>(scan_status) + (size_t)p * scan_stride, nullptr, err,
                                     stream)) != PCPP_OK)
            return rc;
        so_scatter<<<(unsigned)s.n_blocks, SO_THREADS, 0, stream>>>(
            keys[src], vals[src], n, p * SO_BITS, table, s.n_blocks, last ? nullptr : keys[dst],
            last ? reinterpret_cast<uint32_t *>(perm) : vals[dst], err);
        PCPP_HIP_CHECK(hipGetLastError());
    }
    return PCPP_OK;
}

}  // namespace pcpp
