// Offload / upload of one request's compressed pages for gfx950.
//
// ALISE Sec. 3.2 "Dynamic Swapping", Alg. 2: the KV cache of a preempted job moves between GPU
// memory and CPU memory at the request level.  These kernels are the data movement only: gather
// the request's (page, head) blocks through its block table into one contiguous buffer, or
// scatter such a buffer into the pages the block table names now.  The buffer may be device
// memory or pinned host memory mapped into the device's address space.
//
// One wave moves one (page, head) block at a time -- [K codes | V codes | K meta | V meta],
// every piece a whole number of 16-byte units -- with 16-byte non-temporal loads and stores;
// the waves of a persistent grid stride over the blocks.  Pure streaming: the bound is the
// slower of HBM and the link the buffer sits behind.
#include "alise_kernels.h"

namespace alise {
namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

struct SwapParams {
    CacheView c;
    const int32_t *block_table;
    uint8_t *packed;
    int32_t n_blocks;           // logical blocks * Hkv
    int32_t code_units;         // 16-byte units of one block's K (or V) codes: P * row_code_bytes / 16
    int32_t meta_units;         // 16-byte units of one block's K (or V) meta:  P * NG * 4 / 16
};

template <bool UPLOAD>
__global__ __launch_bounds__(256) void swap_kernel(SwapParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = gridDim.x * 4;
    const int units = 2 * p.code_units + 2 * p.meta_units;
    for (int b = wave; b < p.n_blocks; b += n_waves) {           // wave-uniform
        const int j = b / p.c.Hkv, h = b - j * p.c.Hkv;
        const int64_t blk = (int64_t)p.block_table[j] * p.c.Hkv + h;
        uint8_t *kc = p.c.k_codes + blk * p.c.cstride;
        uint8_t *vc = p.c.v_codes + blk * p.c.cstride;
        uint8_t *km = reinterpret_cast<uint8_t *>(p.c.k_meta) + blk * p.c.mstride;
        uint8_t *vm = reinterpret_cast<uint8_t *>(p.c.v_meta) + blk * p.c.mstride;
        uint8_t *pk = p.packed + (int64_t)b * units * 16;
        for (int u = lane; u < units; u += 64) {
            uint8_t *cell;
            if (u < p.code_units) cell = kc + u * 16;
            else if (u < 2 * p.code_units) cell = vc + (u - p.code_units) * 16;
            else if (u < 2 * p.code_units + p.meta_units) cell = km + (u - 2 * p.code_units) * 16;
            else cell = vm + (u - 2 * p.code_units - p.meta_units) * 16;
            u32x4_t *src = reinterpret_cast<u32x4_t *>(UPLOAD ? pk + u * 16 : cell);
            u32x4_t *dst = reinterpret_cast<u32x4_t *>(UPLOAD ? cell : pk + u * 16);
            __builtin_nontemporal_store(__builtin_nontemporal_load(src), dst);
        }
    }
}

}  // namespace

int64_t swap_block_bytes(const CacheView &c)
{
    return 2 * (int64_t)c.P * c.row_code_bytes + 2 * (int64_t)c.P * c.NG * 4;
}

hipError_t launch_swap(const CacheView &c, const int32_t *block_table, int32_t num_tokens, void *packed,
                       bool upload, int32_t num_cus, hipStream_t s)
{
    if (num_tokens <= 0) return hipSuccess;
    SwapParams p;
    p.c = c;
    p.block_table = block_table;
    p.packed = static_cast<uint8_t *>(packed);
    p.n_blocks = ((num_tokens + c.P - 1) / c.P) * c.Hkv;
    p.code_units = c.P * c.row_code_bytes / 16;
    p.meta_units = c.P * c.NG * 4 / 16;
    int blocks = (p.n_blocks + 3) / 4;
    if (blocks > num_cus * 8) blocks = num_cus * 8;
    if (upload)
        hipLaunchKernelGGL(swap_kernel<true>, dim3(blocks), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL(swap_kernel<false>, dim3(blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace alise
