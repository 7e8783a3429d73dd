// Quantize-and-write and page dequantize kernels for gfx950.
//
// Quantizer: ALISE Sec. 3.2 ("KV Compression"): x_q = round(x/lambda + z),
// x = lambda (x_q - z), lambda = (max - min)/(2^b - 1).  The exact sequence of
// single-rounding fp32 operations is the one stated in include/alise_kv.h; it
// must be followed to the letter because codes and meta are compared bit for bit.
//
// Mapping: one lane owns 8 consecutive channels of one (token, kv-head, K|V) row
// (one 16-byte load).  A row is D/8 lanes, a group G/8 lanes; min/max travel over
// the lanes of a group with xor-shuffles.  Rows are numbered token-major for small
// writes and head-major inside blocks of 16 tokens for large ones (BY_HEAD).  Both kernels are pure streaming:
// 16-byte loads, 8- or 4-byte code stores (16-byte stores for dequantize).
#include "alise_kernels.h"

#include <hip/hip_fp16.h>

namespace alise {
namespace {

typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef _Float16 h2_t __attribute__((ext_vector_type(2)));

struct QuantParams {
    CacheView c;
    const _Float16 *k, *v;
    const int64_t *slots;
    int32_t log_lanes_per_row;  // log2(D / 8)
    int32_t lanes_per_group;    // G / 8
    uint32_t total_lanes;       // T * Hkv * 2 * lanes_per_row, below 2^31
    uint32_t hkv_magic;         // row / Hkv == mul_hi(row, hkv_magic) >> hkv_shift for row < 2^31
    uint32_t hkv_shift;
    int32_t T;                  // tokens of this launch
};

__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// BITS = code width; LPG = lanes per group (G / 8): 2, 4, 8 or 16, so a group never leaves a row of 16 lanes.
template <int BITS, int LPG, bool BY_HEAD>
__global__ __launch_bounds__(256) void quant_write_kernel(QuantParams p)
{
    const uint32_t gl = blockIdx.x * 256u + threadIdx.x;
    bool live = gl < p.total_lanes;
    const uint32_t g = live ? gl : p.total_lanes - 1;
    const int lane_in_row = (int)(g & ((1u << p.log_lanes_per_row) - 1u));
    const uint32_t row = g >> p.log_lanes_per_row;
    int head, which;
    int64_t t;
    if constexpr (!BY_HEAD) {
        // Rows are ordered (token, K|V, head): the lanes of a wave stay inside one
        // tensor's contiguous [Hkv][D] slab of one token as long as possible.
        const uint32_t tw = p.c.Hkv == 1 ? row : (__umulhi(row, p.hkv_magic) >> p.hkv_shift);
        head = (int)(row - tw * (uint32_t)p.c.Hkv);
        which = (int)(tw & 1u);
        t = tw >> 1;
    } else {
        // Rows are ordered (16 tokens, K|V, head, token of the 16): consecutive rows are the same head of
        // consecutive tokens, which a prompt's chunk puts side by side in a page.
        const uint32_t t_lo = row & 15u, r2 = row >> 4;
        const uint32_t r3 = p.c.Hkv == 1 ? r2 : (__umulhi(r2, p.hkv_magic) >> p.hkv_shift);
        head = (int)(r2 - r3 * (uint32_t)p.c.Hkv);
        which = (int)(r3 & 1u);
        int64_t tt = (int64_t)(r3 >> 1) * 16 + t_lo;
        live = live && tt < p.T;
        t = tt < p.T ? tt : p.T - 1;
    }

    const _Float16 *src = (which ? p.v : p.k) + (t * p.c.Hkv + head) * p.c.D + lane_in_row * 8;
    const h8_t x = __builtin_nontemporal_load(reinterpret_cast<const h8_t *>(src));    // read once
    const int64_t slot = p.slots[t];

    float xf[8];
    float mn = 0.0f, mx = 0.0f;          // the range always includes 0
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        xf[i] = (float)x[i];
        mn = fminf(mn, xf[i]);
        mx = fmaxf(mx, xf[i]);
    }
    // minimum and maximum over the lanes of the group, every lane gets both
    mn = fminf(mn, dpp_f<0xB1>(mn));  mx = fmaxf(mx, dpp_f<0xB1>(mx));                    // quad_perm [1,0,3,2]
    if constexpr (LPG >= 4) { mn = fminf(mn, dpp_f<0x4E>(mn)); mx = fmaxf(mx, dpp_f<0x4E>(mx)); }     // quad_perm [2,3,0,1]
    if constexpr (LPG >= 8) { mn = fminf(mn, dpp_f<0x141>(mn)); mx = fmaxf(mx, dpp_f<0x141>(mx)); }   // row_half_mirror
    if constexpr (LPG >= 16) { mn = fminf(mn, dpp_f<0x140>(mn)); mx = fmaxf(mx, dpp_f<0x140>(mx)); }  // row_mirror
    const float qmax = (float)((1 << BITS) - 1);
    const float r = mx - mn;
    const float l32 = r / qmax;
    _Float16 h = (_Float16)l32;                       // round to nearest even
    uint16_t hb = __builtin_bit_cast(uint16_t, h);
    if ((float)h < l32) hb = (uint16_t)(hb + 1);      // scale is rounded up
    if (hb < 0x0400u) hb = 0x0400u;                   // floor at 2^-14
    const float lam = (float)__builtin_bit_cast(_Float16, hb);
    const float inv = 1.0f / lam;
    float zf = __builtin_rintf((-mn) * inv);
    zf = fminf(fmaxf(zf, 0.0f), qmax);
    const int zi = (int)zf;
    zf = (float)zi;
    uint32_t code[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float u = __builtin_fmaf(xf[i], inv, zf);     // one rounding
        float qv = __builtin_rintf(u);
        qv = fminf(fmaxf(qv, 0.0f), qmax);
        code[i] = (uint32_t)(int)qv;
    }
    if (!live || slot < 0) return;

    const int64_t page = slot >> p.c.logP;
    const int off = (int)(slot & (p.c.P - 1));
    const int64_t blk = page * p.c.Hkv + head;
    uint8_t *codes = (which ? p.c.v_codes : p.c.k_codes) + blk * p.c.cstride + (int64_t)off * p.c.row_code_bytes;
    uint32_t *meta = reinterpret_cast<uint32_t *>(reinterpret_cast<uint8_t *>(which ? p.c.v_meta : p.c.k_meta) +
                                                  blk * p.c.mstride) + off * p.c.NG;
    if constexpr (BITS == 8) {
        uint2 w;
        w.x = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
        w.y = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        const u32x2_t wv = {w.x, w.y};
        __builtin_nontemporal_store(wv, reinterpret_cast<u32x2_t *>(codes + lane_in_row * 8));
    } else {
        uint32_t w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) w |= code[i] << (4 * i);   // channel 2i low nibble, 2i+1 high
        __builtin_nontemporal_store(w, reinterpret_cast<uint32_t *>(codes + lane_in_row * 4));
    }
    if ((lane_in_row % LPG) == 0) {
        const int grp = lane_in_row / LPG;
        const uint16_t zb = __builtin_bit_cast(uint16_t, (_Float16)zf);
        __builtin_nontemporal_store((uint32_t)hb | ((uint32_t)zb << 16), meta + grp);
    }
}

struct DequantParams {
    CacheView c;
    int32_t page;
    _Float16 *k_out, *v_out;
    int32_t lanes_per_row;      // D / 8
    int32_t total_lanes;        // P * Hkv * 2 * lanes_per_row
};

__global__ __launch_bounds__(256) void dequant_page_kernel(DequantParams p)
{
    const int gl = blockIdx.x * 256 + threadIdx.x;
    if (gl >= p.total_lanes) return;
    const int lpr = p.lanes_per_row;
    const int lane_in_row = gl % lpr;
    int row = gl / lpr;                     // (which, head, off): follows the cache's own order
    const int off = row % p.c.P;
    row /= p.c.P;
    const int head = row % p.c.Hkv;
    const int which = row / p.c.Hkv;

    const int64_t blk = (int64_t)p.page * p.c.Hkv + head;
    const uint8_t *codes = (which ? p.c.v_codes : p.c.k_codes) + blk * p.c.cstride + (int64_t)off * p.c.row_code_bytes;
    const uint32_t *meta = reinterpret_cast<const uint32_t *>(
                               reinterpret_cast<const uint8_t *>(which ? p.c.v_meta : p.c.k_meta) + blk * p.c.mstride) +
                           off * p.c.NG;
    const int grp = (lane_in_row * 8) / p.c.G;
    const uint32_t m = meta[grp];
    const float lam = (float)__builtin_bit_cast(_Float16, (uint16_t)(m & 0xffffu));
    const float z = (float)__builtin_bit_cast(_Float16, (uint16_t)(m >> 16));
    uint32_t code[8];
    if (p.c.bits == 8) {
        const uint2 w = *reinterpret_cast<const uint2 *>(codes + lane_in_row * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            code[i] = (w.x >> (8 * i)) & 0xffu;
            code[4 + i] = (w.y >> (8 * i)) & 0xffu;
        }
    } else {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(codes + lane_in_row * 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) code[i] = (w >> (4 * i)) & 0xfu;
    }
    h8_t o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (_Float16)(lam * ((float)code[i] - z));   // product is exact in fp32
    _Float16 *dst = (which ? p.v_out : p.k_out) + ((int64_t)off * p.c.Hkv + head) * p.c.D + lane_in_row * 8;
    *reinterpret_cast<h8_t *>(dst) = o;
}

}  // namespace

hipError_t launch_quant_write(const CacheView &c, const void *k, const void *v,
                              const int64_t *slot_mapping, int32_t T, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    QuantParams p;
    p.c = c;
    const int lanes_per_row = c.D / 8;
    p.log_lanes_per_row = lanes_per_row == 16 ? 4 : 3;      // D is 128 or 64
    p.lanes_per_group = c.G / 8;
    // division by Hkv as a multiplication: with L = ceil(log2 Hkv), M = ceil(2^(31+L) / Hkv) fits
    // 32 bits and floor(n / Hkv) == (n * M) >> (31 + L) for every n < 2^31
    int L = 0;
    while ((1 << L) < c.Hkv) ++L;
    p.hkv_magic = (uint32_t)((((uint64_t)1 << (31 + L)) + (uint64_t)c.Hkv - 1) / (uint64_t)c.Hkv);
    p.hkv_shift = (uint32_t)(L > 0 ? L - 1 : 0);
    // a launch covers at most 2^30 lanes (16 GiB of input), so that lane indices fit 31 bits
    const int64_t lanes_per_token = (int64_t)c.Hkv * 2 * lanes_per_row;
    const int64_t tokens_per_launch = (((int64_t)1 << 30) / lanes_per_token) & ~(int64_t)15;
    // Large writes are mostly prompt chunks, whose tokens sit side by side in their pages: with the rows of 16
    // consecutive tokens of one head next to each other a workgroup writes 2 KiB of codes and 128 bytes of
    // scales in one piece instead of sixteen (7 % on a 7 650-token batch).  Small ones are decode steps, one
    // token per request, where the token-major order reads whole tokens and nothing is adjacent anyway.
    const bool by_head = T >= 1024;
    for (int64_t t0 = 0; t0 < T; t0 += tokens_per_launch) {
        const int64_t n = T - t0 < tokens_per_launch ? T - t0 : tokens_per_launch;
        p.k = static_cast<const _Float16 *>(k) + t0 * c.Hkv * c.D;
        p.v = static_cast<const _Float16 *>(v) + t0 * c.Hkv * c.D;
        p.slots = slot_mapping + t0;
        p.T = (int32_t)n;
        p.total_lanes = (uint32_t)((by_head ? (n + 15) / 16 * 16 : n) * lanes_per_token);
        const dim3 grid((p.total_lanes + 255u) / 256u), block(256);
        const int lpg = p.lanes_per_group;
#define ALISE_QW(BITSV, BH)                                                                              \
    do {                                                                                                 \
        if (lpg == 16) hipLaunchKernelGGL((quant_write_kernel<BITSV, 16, BH>), grid, block, 0, s, p);    \
        else if (lpg == 8) hipLaunchKernelGGL((quant_write_kernel<BITSV, 8, BH>), grid, block, 0, s, p); \
        else if (lpg == 4) hipLaunchKernelGGL((quant_write_kernel<BITSV, 4, BH>), grid, block, 0, s, p); \
        else if (lpg == 2) hipLaunchKernelGGL((quant_write_kernel<BITSV, 2, BH>), grid, block, 0, s, p); \
        else return hipErrorInvalidValue;                                                                \
    } while (0)
        if (c.bits == 8) { if (by_head) ALISE_QW(8, true); else ALISE_QW(8, false); }
        else { if (by_head) ALISE_QW(4, true); else ALISE_QW(4, false); }
#undef ALISE_QW
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_dequant_page(const CacheView &c, int32_t page, void *k_out, void *v_out, hipStream_t s)
{
    DequantParams p;
    p.c = c;
    p.page = page;
    p.k_out = static_cast<_Float16 *>(k_out);
    p.v_out = static_cast<_Float16 *>(v_out);
    p.lanes_per_row = c.D / 8;
    p.total_lanes = c.P * c.Hkv * 2 * p.lanes_per_row;
    const int blocks = (p.total_lanes + 255) / 256;
    hipLaunchKernelGGL(dequant_page_kernel, dim3(blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace alise
