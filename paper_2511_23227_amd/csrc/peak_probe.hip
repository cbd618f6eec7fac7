// Measurement aid, not part of the library's interface: a loop that does nothing but issue
// v_mfma_f32_16x16x32_bf16 on registers, to show what the matrix cores of the device sustain when nothing else
// is in the way.  Built into its own shared object (libpcpp_probe.so); only the benchmark loads it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int PROBE_CHAINS = 16;      // independent accumulators per wave: no MFMA waits for the one before it

__global__ __launch_bounds__(256) void mfma_issue_loop(int iters, float *sink)
{
    // operands that the compiler cannot fold: small bf16 values derived from the lane
    const uint32_t seed = 0x3c003c00u + ((threadIdx.x & 7u) << 16) + (threadIdx.x & 3u);
    const v8bf a = __builtin_bit_cast(v8bf, v4u{seed, seed + 1u, seed + 2u, seed + 3u});
    const v8bf b = __builtin_bit_cast(v8bf, v4u{seed + 4u, seed + 5u, seed + 6u, seed + 7u});
    v4f acc[PROBE_CHAINS];
#pragma unroll
    for (int j = 0; j < PROBE_CHAINS; ++j) acc[j] = v4f{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < PROBE_CHAINS; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < PROBE_CHAINS; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (s == -1.0f) sink[threadIdx.x] = s;      // never true for these operands; keeps the loop alive
}

}  // namespace

extern "C" {

// Launches `blocks` blocks of four waves, each wave issuing iters * 16 MFMAs; returns the number of floating-point
// operations launched (2 * 16 * 16 * 32 per MFMA), or a negative HIP error code.  sink: at least 256 floats (device).
__attribute__((visibility("default"))) double pcpp_probe_mfma_bf16(int blocks, int iters, float *sink, void *stream)
{
    if (blocks < 1 || iters < 1 || !sink) return -1.0;
    mfma_issue_loop<<<(unsigned)blocks, 256, 0, static_cast<hipStream_t>(stream)>>>(iters, sink);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return -(double)(int)e - 1.0;
    return (double)blocks * 4.0 * (double)iters * PROBE_CHAINS * 2.0 * 16 * 16 * 32;
}

}  // extern "C"
