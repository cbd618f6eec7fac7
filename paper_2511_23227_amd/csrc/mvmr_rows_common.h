// Helpers shared by the rows kernels (mvmr_rows.hip, mvmr_rows_wide.hip); not part of the C ABI.
#pragma once

#include "pcpp_internal.h"

namespace pcpp {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int ROWS = 32;                         // centres per block
constexpr uint32_t OOB_OFFSET = 0xfffff000u;     // buffer offset past any descriptor, also after adding a
                                                 // position inside a row (< 4096): reads zero, no traffic
constexpr size_t MAX_BUFFER_BYTES = 0xfffff000u;

static __device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

static __device__ inline uint32_t cvt_pk_bf16(float lo, float hi)
{
    const v2f v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, v2bf));   // round to nearest even
}


// wide layers (mvmr_rows_wide.hip): a.w of mvmr_rows_wide must have been packed by mvmr_rows_wide_pack_w
bool mvmr_rows_wide_shape(const MvmrArgs &a);
int mvmr_rows_wide_pack_w(const void *w, void *packed, int K, int c_src, int c_dst, int stride_d, int stride_s,
                          hipStream_t stream);
int mvmr_rows_wide(const MvmrArgs &a, hipStream_t stream);

}  // namespace pcpp
