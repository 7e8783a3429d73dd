// Definitions shared by the attention kernels (vector path and GQA matrix-core path).
#pragma once
#include "alise_kernels.h"

#include <hip/hip_fp16.h>

#include <type_traits>

namespace alise {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));

constexpr float kNegInf = -__builtin_inff();
constexpr float kLazy = 8.0f;   // the running maximum is raised only past this slack (log2 units)
constexpr float kFloor = -1.0e30f;   // finite stand-in for "no token seen yet": -inf - kFloor stays -inf

struct AttnParams {
    CacheView c;
    const _Float16 *q;
    _Float16 *out;
    const int32_t *block_tables;
    const int32_t *context_lens;
    int32_t max_blocks, B, H, qper, max_len;
    float scale_log2e;
    int32_t zero_empty;         // the merge kernel writes the zero rows of empty requests (the plan kernel had no output to write to)
    AttnWorkspace ws;
};

__device__ __forceinline__ h2_t as_h2(uint32_t u) { return __builtin_bit_cast(h2_t, u); }
__device__ __forceinline__ uint32_t as_u32(h2_t h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ float half_lo(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xffffu)); }
__device__ __forceinline__ float half_hi(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u >> 16)); }

// The cache is read once per step and is far larger than the L2, so its loads carry the
// non-temporal hint: the lines are not kept at the expense of the small data that is
// reused (queries, descriptors, page ids, partial results).  Measured on the INT4 workload
// this alone takes the attention kernel from 5.4 to 5.8 TB/s.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load16(const void *p) {
    const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
}
__device__ __forceinline__ uint32_t stream_load4(const void *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p));
}

// The matrix-core kernel for grouped-query attention: one wave serves all query heads of a
// KV head, so a tile's items are its KV heads.  Defined in decode_attn_gqa.hip.
hipError_t launch_gqa_mfma(const AttnParams &p, int32_t num_cus, int32_t waves_per_cu, int32_t stages, hipStream_t s);

}  // namespace alise
