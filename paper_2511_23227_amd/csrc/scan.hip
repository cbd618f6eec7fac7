// Device-wide exclusive prefix sum of uint32 counts in one launch (chained scan: every block publishes
// the sum of its items, then adds up what the blocks before it have published) and small fill kernels.
// Used by the triplet construction (Sec. 3.3.2: the reordering is a counting sort, whose offsets are a
// prefix sum).
#include "pcpp_internal.h"

namespace pcpp {

namespace {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;                       // per thread
constexpr int SCAN_BLOCK = SCAN_THREADS * SCAN_ITEMS;

// status word of a block: two flag bits over a 62-bit value
constexpr unsigned long long STATUS_SUM = 1ull << 62;        // value = sum of the block's own items
constexpr unsigned long long STATUS_PREFIX = 2ull << 62;     // value = sum of all items up to the block's last
constexpr unsigned long long STATUS_VALUE = (1ull << 62) - 1;
constexpr int SCAN_SPIN_LIMIT = 1 << 20;

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

// status[0 .. n_blocks-1]: one word per block, status[n_blocks]: ticket counter; all zero at launch.
// A block takes its position from the ticket counter, so every block before it has already started and
// will publish without waiting for a later one: each wait below ends.  The first wave looks back 64
// blocks at a time: it adds the published sums down to the nearest block whose whole prefix is known
// (the position before block 0 counts as a known prefix of 0).  Value and flag share one 64-bit word,
// written and read with single agent-scope accesses, so no ordering between two words is relied on.
__global__ __launch_bounds__(SCAN_THREADS) void scan_chained(const uint32_t *in, uint32_t *out,
                                                             int64_t n, unsigned long long *__restrict__ status,
                                                             int64_t n_blocks, unsigned long long *__restrict__ total64,
                                                             uint32_t *__restrict__ err)
{
    __shared__ unsigned long long shared_word[2];       // ticket, then the block's exclusive prefix
    const int lane = threadIdx.x & 63;
    if (threadIdx.x == 0) shared_word[0] = atomicAdd(&status[n_blocks], 1ull);
    __syncthreads();
    const int64_t bid = (int64_t)shared_word[0];
    const int64_t base = bid * SCAN_BLOCK + (int64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t v[SCAN_ITEMS];
    unsigned long long s = 0;
#pragma unroll
    for (int j = 0; j < SCAN_ITEMS; ++j) {
        const int64_t idx = base + j;
        v[j] = idx < n ? in[idx] : 0u;
        s += v[j];
    }
    unsigned long long tot;
    const unsigned long long inc = block_incl_scan_u64(s, &tot);    // its barriers also order every read of
                                                                    // `in` before any write (out may alias in)
    if (threadIdx.x < 64) {
        unsigned long long excl = 0;
        if (bid > 0) {
            if (lane == 0) __hip_atomic_store(&status[bid], STATUS_SUM | tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int64_t newest = bid - 1;; newest -= 64) {
                const int64_t j = newest - lane;
                unsigned long long w = STATUS_PREFIX, take = 0;
                bool found = false;
                for (int spin = 0;; ++spin) {
                    if (j >= 0) w = __hip_atomic_load(&status[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const unsigned long long known = __ballot((w >> 62) == 2);
                    const unsigned long long empty = __ballot((w >> 62) == 0);
                    // the lanes down to (and including) the newest block with a known prefix
                    const unsigned long long lowest = known & (~known + 1);
                    take = known ? (lowest | (lowest - 1)) : ~0ull;
                    found = known != 0;
                    if (!(empty & take)) break;
                    if (spin >= SCAN_SPIN_LIMIT) {      // cannot happen on a working device: raise the error word
                        if (empty >> lane & 1) w = 0;   // (every later kernel of the build and the host look at it)
                        if (err && lane == 0) {
                            __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            __threadfence();
                        }
                        found = true;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
                unsigned long long part = (take >> lane & 1) ? (w & STATUS_VALUE) : 0ull;
#pragma unroll
                for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d, 64);
                excl += part;
                if (found) break;
            }
            excl = __shfl(excl, 0, 64);
        }
        if (lane == 0) {
            __hip_atomic_store(&status[bid], STATUS_PREFIX | ((excl + tot) & STATUS_VALUE), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            shared_word[1] = excl;
        }
    }
    __syncthreads();
    const unsigned long long before = shared_word[1];
    unsigned long long run = before + inc - s;
#pragma unroll
    for (int j = 0; j < SCAN_ITEMS; ++j) {
        const int64_t idx = base + j;
        if (idx < n) out[idx] = (uint32_t)run;
        run += v[j];
    }
    if (bid == n_blocks - 1 && threadIdx.x == 0) {
        out[n] = (uint32_t)(before + tot);
        // every earlier block has published by now, and a block raises the error word before it publishes
        const bool bad = err && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
        if (total64) *total64 = bad ? ~0ull : before + tot;
    }
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
                       unsigned long long *total64, uint32_t *err, hipStream_t stream)
{
    auto *status = static_cast<unsigned long long *>(scratch);
    if (n <= 0) {
        // out[0] = 0, total = 0
        fill_u32_kernel<<<1, 64, 0, stream>>>(out, 0u, 1);
        if (total64) fill_u64_kernel<<<1, 64, 0, stream>>>(total64, 0ull, 1);
        PCPP_HIP_CHECK(hipGetLastError());
        return PCPP_OK;
    }
    const int64_t n_blocks = ceil_div(n, SCAN_BLOCK);
    scan_chained<<<(unsigned)n_blocks, SCAN_THREADS, 0, stream>>>(in, out, n, status, n_blocks, total64, err);
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
