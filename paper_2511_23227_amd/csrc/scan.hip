// Device-wide exclusive prefix sum of uint32 counts (three launches: block sums, scan of the
// block sums, block-local scan plus offset) and small fill kernels.  Used by the triplet
// construction (Sec. 3.3.2: the reordering is a counting sort, whose offsets are a prefix sum).
#include "pcpp_internal.h"

namespace pcpp {

namespace {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;                       // per thread
constexpr int SCAN_BLOCK = SCAN_THREADS * SCAN_ITEMS;

__device__ inline unsigned long long wave_incl_scan_u64(unsigned long long v, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        unsigned long long u = __shfl_up(v, d, 64);
        if (lane >= d) v += u;
    }
    return v;
}

// inclusive scan across the 256 threads of a block; returns this thread's inclusive value,
// *block_total gets the sum of all threads
__device__ inline unsigned long long block_incl_scan_u64(unsigned long long v, unsigned long long *block_total)
{
    __shared__ unsigned long long wave_sum[SCAN_THREADS / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long inc = wave_incl_scan_u64(v, lane);
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    unsigned long long off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SCAN_THREADS / 64; ++w) {
        unsigned long long s = wave_sum[w];
        if (w < wave) off += s;
        tot += s;
    }
    __syncthreads();
    *block_total = tot;
    return inc + off;
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_block_sums(const uint32_t *__restrict__ in, int64_t n,
                                                                unsigned long long *__restrict__ sums)
{
    const int64_t base = (int64_t)blockIdx.x * SCAN_BLOCK;
    unsigned long long s = 0;
#pragma unroll
    for (int j = 0; j < SCAN_ITEMS; ++j) {
        int64_t idx = base + (int64_t)j * SCAN_THREADS + threadIdx.x;
        if (idx < n) s += in[idx];
    }
    unsigned long long tot;
    block_incl_scan_u64(s, &tot);
    if (threadIdx.x == 0) sums[blockIdx.x] = tot;
}

// single block: exclusive scan of the block sums in place, total written to sums[n_blocks]
__global__ __launch_bounds__(SCAN_THREADS) void scan_of_sums(unsigned long long *__restrict__ sums, int64_t n_blocks,
                                                             unsigned long long *__restrict__ total64)
{
    unsigned long long carry = 0;
    for (int64_t base = 0; base < n_blocks; base += SCAN_THREADS) {
        int64_t idx = base + threadIdx.x;
        unsigned long long v = idx < n_blocks ? sums[idx] : 0ull;
        unsigned long long tot;
        unsigned long long inc = block_incl_scan_u64(v, &tot);
        if (idx < n_blocks) sums[idx] = carry + inc - v;
        carry += tot;
    }
    if (threadIdx.x == 0) {
        sums[n_blocks] = carry;
        if (total64) *total64 = carry;
    }
}

__global__ __launch_bounds__(SCAN_THREADS) void scan_apply(const uint32_t *__restrict__ in, uint32_t *__restrict__ out,
                                                           int64_t n, const unsigned long long *__restrict__ sums,
                                                           int64_t n_blocks)
{
    const int64_t base = (int64_t)blockIdx.x * SCAN_BLOCK + (int64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t v[SCAN_ITEMS];
    unsigned long long s = 0;
#pragma unroll
    for (int j = 0; j < SCAN_ITEMS; ++j) {
        int64_t idx = base + j;
        v[j] = idx < n ? in[idx] : 0u;
        s += v[j];
    }
    unsigned long long tot;
    unsigned long long inc = block_incl_scan_u64(s, &tot);
    unsigned long long run = sums[blockIdx.x] + inc - s;
    __syncthreads();     // every read of `in` in this block happens before any write (out may alias in)
#pragma unroll
    for (int j = 0; j < SCAN_ITEMS; ++j) {
        int64_t idx = base + j;
        if (idx < n) out[idx] = (uint32_t)run;
        run += v[j];
    }
    if (blockIdx.x == n_blocks - 1 && threadIdx.x == 0) out[n] = (uint32_t)sums[n_blocks];
}

__global__ void fill_u32_kernel(uint32_t *p, uint32_t v, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

__global__ void fill_u64_kernel(unsigned long long *p, unsigned long long v, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

}  // namespace

size_t scan_scratch_bytes(int64_t n)
{
    return align_up((size_t)(ceil_div(n > 0 ? n : 1, SCAN_BLOCK) + 1) * sizeof(unsigned long long));
}

int scan_exclusive_u32(const uint32_t *in, uint32_t *out, int64_t n, void *scratch,
                       unsigned long long *total64, hipStream_t stream)
{
    auto *sums = static_cast<unsigned long long *>(scratch);
    if (n <= 0) {
        // out[0] = 0, total = 0
        fill_u32_kernel<<<1, 64, 0, stream>>>(out, 0u, 1);
        if (total64) fill_u64_kernel<<<1, 64, 0, stream>>>(total64, 0ull, 1);
        PCPP_HIP_CHECK(hipGetLastError());
        return PCPP_OK;
    }
    const int64_t n_blocks = ceil_div(n, SCAN_BLOCK);
    scan_block_sums<<<(unsigned)n_blocks, SCAN_THREADS, 0, stream>>>(in, n, sums);
    scan_of_sums<<<1, SCAN_THREADS, 0, stream>>>(sums, n_blocks, total64);
    scan_apply<<<(unsigned)n_blocks, SCAN_THREADS, 0, stream>>>(in, out, n, sums, n_blocks);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

int fill_u32(uint32_t *p, uint32_t v, int64_t n, hipStream_t stream)
{
    if (n <= 0) return PCPP_OK;
    int64_t blocks = ceil_div(n, 256);
    if (blocks > 4096) blocks = 4096;
    fill_u32_kernel<<<(unsigned)blocks, 256, 0, stream>>>(p, v, n);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

int fill_u64(unsigned long long *p, unsigned long long v, int64_t n, hipStream_t stream)
{
    if (n <= 0) return PCPP_OK;
    int64_t blocks = ceil_div(n, 256);
    if (blocks > 4096) blocks = 4096;
    fill_u64_kernel<<<(unsigned)blocks, 256, 0, stream>>>(p, v, n);
    PCPP_HIP_CHECK(hipGetLastError());
    return PCPP_OK;
}

}  // namespace pcpp
