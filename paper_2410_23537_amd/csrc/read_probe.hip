// Streaming-read probe for gfx950: the rate at which the chip can read HBM with nothing else to do.
//
// The decode path is bound by HBM reads; the published peak (8 TB/s) is a pin rate that no kernel
// reaches.  This kernel reads a buffer once with 16-byte non-temporal loads, as many in flight as a
// persistent grid of full workgroups can keep, and folds what it read into one 32-bit word (the
// exclusive-or of all dwords), which makes the read observable and the call testable.  Its rate
// on a buffer larger than the last-level cache is the second denominator of the measurements.
#include "alise_kernels.h"
#include "../../include/alise_ops.h"

namespace alise {
namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// A wave reads blocks of kProbeLoads KiB (one load instruction = 1 KiB of consecutive addresses), the
// waves of the persistent grid take the blocks in turn, and a wave keeps two blocks in flight: the loads of
// the next block are issued before the last one is folded.  The tail (less than a block) goes to the first
// waves, 16 bytes per lane.  The sink is cleared by sink_clear_kernel first; one atomic per wave at the end.
constexpr int kProbeLoads = 8;

__global__ void sink_clear_kernel(uint32_t *sink) { *sink = 0u; }

__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4_t *__restrict__ src, uint64_t n16, uint32_t *sink)
{
    const int lane = threadIdx.x & 63;
    const uint64_t wave = ((uint64_t)blockIdx.x * 256u + threadIdx.x) >> 6, n_waves = ((uint64_t)gridDim.x * 256u) >> 6;
    constexpr uint64_t kBlock = (uint64_t)kProbeLoads * 64u;       // 16-byte units per block
    const uint64_t n_blocks = n16 / kBlock;
    uint32_t acc = 0u;
    u32x4_t a[kProbeLoads], b[kProbeLoads];
    auto issue = [&](u32x4_t (&v)[kProbeLoads], uint64_t blk) {
#pragma unroll
        for (int u = 0; u < kProbeLoads; ++u) v[u] = __builtin_nontemporal_load(src + blk * kBlock + (uint64_t)u * 64u + lane);
    };
    auto fold = [&](const u32x4_t (&v)[kProbeLoads]) {
#pragma unroll
        for (int u = 0; u < kProbeLoads; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    };
    // A wave steps its priority down with every 16 blocks it has read (wrapping after four steps), so that the waves of
    // a SIMD stay together: left alone the oldest one is served first and finishes long before the youngest, and the
    // end of the kernel runs with too few waves to keep the memory system busy (the same device as in the attention kernels).
    uint64_t blk = wave;
    uint32_t pairs = 0;
    __builtin_amdgcn_s_setprio(3);
    if (blk < n_blocks) {
        issue(a, blk);
        for (;;) {
            blk += n_waves;
            if (blk >= n_blocks) { fold(a); break; }
            issue(b, blk);
            fold(a);
            blk += n_waves;
            if (blk >= n_blocks) { fold(b); break; }
            issue(a, blk);
            fold(b);
            ++pairs;
            if ((pairs & 7u) == 0u) {
                switch ((pairs >> 3) & 3u) {
                case 0: __builtin_amdgcn_s_setprio(3); break;
                case 1: __builtin_amdgcn_s_setprio(2); break;
                case 2: __builtin_amdgcn_s_setprio(1); break;
                default: __builtin_amdgcn_s_setprio(0); break;
                }
            }
        }
    }
    for (uint64_t i = n_blocks * kBlock + wave * 64u + lane; i < n16; i += n_waves * 64u) {
        const u32x4_t v = __builtin_nontemporal_load(src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc ^= __shfl_xor(acc, d);
    if (lane == 0 && acc != 0u) atomicXor(sink, acc);
}

// Issue probe: do the matrix instructions and the ordinary vector instructions of a SIMD's waves run side by side?
// Every wave runs `iters` rounds of 16 independent v_mfma_f32_16x16x32_f16 (four accumulator chains; 16 x 16 cycles
// at the published rate) and/or 64 independent v_fma_f32 (eight chains; 64 x 4 cycles): about equal times when run
// alone.  The launch gives every SIMD two waves.  If the two kinds overlapped, both together would take as long as
// the longer one; the matrix-core attention kernels' roofline is derived from what this measures instead.
typedef _Float16 probe_h8_t __attribute__((ext_vector_type(8)));
typedef float probe_f4_t __attribute__((ext_vector_type(4)));

template <int MODE>
__global__ __launch_bounds__(256) void issue_probe_kernel(float *sink, int iters)
{
    probe_h8_t a = (probe_h8_t)(_Float16)(threadIdx.x * 0.001f), b = (probe_h8_t)(_Float16)1.0f;
    probe_f4_t c0 = (probe_f4_t)0.0f, c1 = c0, c2 = c0, c3 = c0;
    float x0 = threadIdx.x, x1 = 1.0f, x2 = 2.0f, x3 = 3.0f, x4 = 4.0f, x5 = 5.0f, x6 = 6.0f, x7 = 7.0f;
    const float m = 1.0001f, d = 0.5f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (MODE & 1) {
                c0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c1, 0, 0, 0);
                c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c2, 0, 0, 0);
                c3 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c3, 0, 0, 0);
            }
            if (MODE & 2) {
#pragma unroll
                for (int v = 0; v < 2; ++v) {
                    x0 = __builtin_fmaf(x0, m, d); x1 = __builtin_fmaf(x1, m, d); x2 = __builtin_fmaf(x2, m, d); x3 = __builtin_fmaf(x3, m, d);
                    x4 = __builtin_fmaf(x4, m, d); x5 = __builtin_fmaf(x5, m, d); x6 = __builtin_fmaf(x6, m, d); x7 = __builtin_fmaf(x7, m, d);
                }
            }
        }
    }
    const float r = x0 + x1 + x2 + x3 + x4 + x5 + x6 + x7 + c0[0] + c1[1] + c2[2] + c3[3];
    if (r == 12345.678f) sink[0] = r;           // never true for these inputs; keeps the chains alive
}

}  // namespace
}  // namespace alise

extern "C" int alise_issue_overlap_probe(int32_t mode, int32_t iters, void *sink, void *hip_stream)
{
    using namespace alise;
    if (!sink || iters < 0 || iters > (1 << 24)) return ALISE_INVALID_ARGUMENT;
    if (mode < 1 || mode > 3) return ALISE_UNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(sink) & 3u) return ALISE_MISALIGNED;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return ALISE_HIP_ERROR;
    const dim3 grid((unsigned)cus * 2u), block(256);        // two workgroups of four waves per compute unit: two waves per SIMD
    if (mode == 1) hipLaunchKernelGGL(issue_probe_kernel<1>, grid, block, 0, s, static_cast<float *>(sink), iters);
    else if (mode == 2) hipLaunchKernelGGL(issue_probe_kernel<2>, grid, block, 0, s, static_cast<float *>(sink), iters);
    else hipLaunchKernelGGL(issue_probe_kernel<3>, grid, block, 0, s, static_cast<float *>(sink), iters);
    return hipGetLastError() == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

extern "C" int alise_hbm_read_probe(const void *src, size_t bytes, void *xor_out, void *hip_stream)
{
    using namespace alise;
    if (!xor_out || (bytes && !src)) return ALISE_INVALID_ARGUMENT;
    if (bytes & 15u) return ALISE_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(xor_out) & 3u)) return ALISE_MISALIGNED;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return ALISE_HIP_ERROR;
    hipLaunchKernelGGL(sink_clear_kernel, dim3(1), dim3(1), 0, s, static_cast<uint32_t *>(xor_out));
    if (hipGetLastError() != hipSuccess) return ALISE_HIP_ERROR;
    const uint64_t n16 = bytes >> 4;
    if (n16 == 0) return ALISE_OK;
    uint64_t blocks = (n16 + 255u) / 256u;
    const uint64_t resident = (uint64_t)cus * 4u;               // four workgroups of four waves per compute unit
    if (blocks > resident) blocks = resident;
    hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x4_t *>(src), n16,
                       static_cast<uint32_t *>(xor_out));
    return hipGetLastError() == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}
