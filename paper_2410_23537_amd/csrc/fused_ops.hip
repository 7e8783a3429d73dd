// Residual add + LayerNorm and bias + ReLU for gfx950, and their C-ABI entry points.
//
// ALISE Sec. 3.3 "Implementation" names fused kernels for LayerNorm and ReLU next to the
// attention kernel, applied to the flat token batch of an iteration; Sec. 2 "Transformer
// Architecture" has LayerNorm and the residual connection around the attention and FFN
// modules.  Both operators stream fp16 rows through the chip once -- the bound is HBM -- so
// the kernels are about 16-byte accesses, enough rows in flight and no second pass:
//
//   add + LayerNorm: a row lives in the registers of the threads that own it (256 threads, or
//   one wave for rows up to 1024 wide): h = x + residual as packed fp16 adds (IEEE, one
//   rounding), widened to fp32; the mean, then the squared deviations from it, each reduced
//   over the row with wave shuffles (and four LDS words across the waves of a workgroup);
//   normalise, scale, shift, round once, store.  8 bytes of HBM traffic per element.
//
//   bias + ReLU: the matrix in memory order, 16 bytes per thread and four 4 KiB runs per
//   workgroup; packed fp16 add, then a signed 16-bit integer maximum with 0, which turns
//   every negative pattern (-0 included) into +0 and leaves the positive ones alone.
#include "../../include/alise_ops.h"

#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>

namespace alise {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef short short8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ half8_t load8_stream(const _Float16 *p)
{
    return __builtin_bit_cast(half8_t, __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p)));
}
__device__ __forceinline__ half8_t load8(const _Float16 *p) { return *reinterpret_cast<const half8_t *>(p); }
__device__ __forceinline__ void store8(_Float16 *p, half8_t v) { *reinterpret_cast<half8_t *>(p) = v; }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
    return v;
}

// Sum over the TPR threads of a row: TPR = 64 (one wave per row) or 256 (the workgroup).
template <int TPR>
__device__ __forceinline__ float row_sum(float v, float *s_part)
{
    v = wave_sum(v);
    if constexpr (TPR == 256) {
        const int wave = threadIdx.x >> 6;
        __syncthreads();                                // the previous reduction's readers are done
        if ((threadIdx.x & 63) == 0) s_part[wave] = v;
        __syncthreads();
        v = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
    }
    return v;
}

// CH: 16-byte pieces per thread (the row has at most CH * TPR of them).
template <int TPR, int CH>
__global__ __launch_bounds__(256) void add_layernorm_kernel(const _Float16 *x, const _Float16 *residual,
                                                            const _Float16 *__restrict__ gamma, const _Float16 *__restrict__ beta,
                                                            float eps, _Float16 *h_out, _Float16 *y_out, int64_t rows, int32_t hidden)
{
    __shared__ float s_part[4];
    constexpr int ROWS_PER_WG = 256 / TPR;
    const int t = threadIdx.x % TPR;
    const int64_t row = (int64_t)blockIdx.x * ROWS_PER_WG + threadIdx.x / TPR;
    const bool live = row < rows;                        // whole waves: a wave owns one row or a quarter of one
    const int pieces = hidden >> 3;
    const int64_t base = (live ? row : 0) * (int64_t)hidden;

    float h[CH][8];
    float sum = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int piece = c * TPR + t;
        const bool in = live && piece < pieces;
        half8_t v = (half8_t)(_Float16)0.0f;
        if (in) {
            v = load8_stream(x + base + piece * 8);
            if (residual) v = v + load8_stream(residual + base + piece * 8);      // packed fp16 adds: the exact sum, rounded once
            if (h_out) store8(h_out + base + piece * 8, v);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            h[c][e] = (float)v[e];
            sum += h[c][e];
        }
    }
    const float inv_n = 1.0f / (float)hidden;
    const float mean = row_sum<TPR>(sum, s_part) * inv_n;
    float sq = 0.0f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const bool in = c * TPR + t < pieces;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float d = h[c][e] - mean;
            sq = in ? __builtin_fmaf(d, d, sq) : sq;
        }
    }
    const float var = row_sum<TPR>(sq, s_part) * inv_n;
    const float rstd = 1.0f / sqrtf(var + eps);
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int piece = c * TPR + t;
        if (live && piece < pieces) {
            const half8_t gm = load8(gamma + piece * 8), bt = load8(beta + piece * 8);
            half8_t y;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                y[e] = (_Float16)__builtin_fmaf((h[c][e] - mean) * rstd, (float)gm[e], (float)bt[e]);
            store8(y_out + base + piece * 8, y);
        }
    }
}

template <int TPR, int CH>
hipError_t launch_ln(const void *x, const void *residual, const void *gamma, const void *beta, float eps, void *h_out,
                     void *y_out, int64_t rows, int32_t hidden, hipStream_t s)
{
    constexpr int ROWS_PER_WG = 256 / TPR;
    const int64_t wgs = (rows + ROWS_PER_WG - 1) / ROWS_PER_WG;
    hipLaunchKernelGGL((add_layernorm_kernel<TPR, CH>), dim3((unsigned)wgs), dim3(256), 0, s,
                       static_cast<const _Float16 *>(x), static_cast<const _Float16 *>(residual),
                       static_cast<const _Float16 *>(gamma), static_cast<const _Float16 *>(beta), eps,
                       static_cast<_Float16 *>(h_out), static_cast<_Float16 *>(y_out), rows, hidden);
    return hipGetLastError();
}

// The matrix is walked in memory order, 16-byte pieces, a workgroup taking UNROLL consecutive 4 KiB runs: long
// sequential bursts are what HBM likes best.  The bias piece of a run comes out of the cache.
template <bool BIAS>
__global__ __launch_bounds__(256) void bias_relu_kernel(const _Float16 *x, const _Float16 *__restrict__ bias, _Float16 *y,
                                                        uint32_t n_pieces, uint32_t pieces_per_row)
{
    constexpr int UNROLL = 4;
    const uint32_t first = blockIdx.x * (256u * UNROLL) + threadIdx.x;
    uint32_t col = 0;
    if constexpr (BIAS) col = first % pieces_per_row;
    const uint32_t hop = 256u % pieces_per_row;          // how far the column moves from one run to the next
    const short8_t zero = (short8_t)(short)0;
    half8_t v[UNROLL], b[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint32_t id = first + u * 256u;
        if (id < n_pieces) {
            v[u] = load8_stream(x + (uint64_t)id * 8);
            if constexpr (BIAS) b[u] = load8(bias + col * 8);
        }
        if constexpr (BIAS) {
            col += hop;
            col = col >= pieces_per_row ? col - pieces_per_row : col;
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint32_t id = first + u * 256u;
        if (id < n_pieces) {
            half8_t s = v[u];
            if constexpr (BIAS) s = s + b[u];               // packed fp16 adds: the exact sum, rounded once
            // as 16-bit integers every negative fp16 (and -0) is negative and every positive one keeps its order
            const short8_t m = __builtin_elementwise_max(__builtin_bit_cast(short8_t, s), zero);
            store8(y + (uint64_t)id * 8, __builtin_bit_cast(half8_t, m));
        }
    }
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace alise

extern "C" {

int alise_add_layernorm(const void *x, const void *residual, const void *gamma, const void *beta, float eps, void *h_out,
                        void *y_out, int64_t rows, int32_t hidden, void *hip_stream)
{
    using namespace alise;
    if (rows < 0 || !(eps >= 0.0f) || !std::isfinite(eps)) return ALISE_INVALID_ARGUMENT;
    if (hidden < 8 || hidden > 16384 || (hidden & 7)) return ALISE_UNSUPPORTED;
    if (rows == 0) return ALISE_OK;                     // an empty batch has no buffers to speak of
    if (!x || !gamma || !beta || !y_out || y_out == h_out) return ALISE_INVALID_ARGUMENT;
    if (!aligned16(x) || !aligned16(residual) || !aligned16(gamma) || !aligned16(beta) || !aligned16(h_out) || !aligned16(y_out))
        return ALISE_MISALIGNED;
    if ((rows + 3) / 4 > 0x7fffffffLL && hidden <= 1024) return ALISE_UNSUPPORTED;
    if (rows > 0x7fffffffLL && hidden > 1024) return ALISE_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int pieces = hidden >> 3;
    hipError_t e;
#define ALISE_LN(TPR, CH) e = launch_ln<TPR, CH>(x, residual, gamma, beta, eps, h_out, y_out, rows, hidden, s)
    if (pieces <= 64) ALISE_LN(64, 1);
    else if (pieces <= 128) ALISE_LN(64, 2);
    else if (pieces <= 256) ALISE_LN(256, 1);
    else if (pieces <= 512) ALISE_LN(256, 2);
    else if (pieces <= 768) ALISE_LN(256, 3);
    else if (pieces <= 1024) ALISE_LN(256, 4);
    else if (pieces <= 1536) ALISE_LN(256, 6);
    else ALISE_LN(256, 8);
#undef ALISE_LN
    return e == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

int alise_bias_relu(const void *x, const void *bias, void *y_out, int64_t rows, int32_t cols, void *hip_stream)
{
    using namespace alise;
    if (rows < 0) return ALISE_INVALID_ARGUMENT;
    if (cols < 8 || (cols & 7)) return ALISE_UNSUPPORTED;
    if (rows == 0) return ALISE_OK;
    if (!x || !y_out) return ALISE_INVALID_ARGUMENT;
    if (!aligned16(x) || !aligned16(bias) || !aligned16(y_out)) return ALISE_MISALIGNED;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint32_t ppr = (uint32_t)(cols >> 3);
    const uint64_t total = (uint64_t)rows * ppr;
    if (total > 0xffffffffull - 1024u) return ALISE_UNSUPPORTED;      // the piece index is 32 bits wide (64 GiB of fp16)
    const dim3 grid((unsigned)((total + 1023u) / 1024u));
    if (bias)
        hipLaunchKernelGGL(bias_relu_kernel<true>, grid, dim3(256), 0, s, static_cast<const _Float16 *>(x),
                           static_cast<const _Float16 *>(bias), static_cast<_Float16 *>(y_out), (uint32_t)total, ppr);
    else
        hipLaunchKernelGGL(bias_relu_kernel<false>, grid, dim3(256), 0, s, static_cast<const _Float16 *>(x),
                           static_cast<const _Float16 *>(bias), static_cast<_Float16 *>(y_out), (uint32_t)total, ppr);
    return hipGetLastError() == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

}  // extern "C"
