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
__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}

// The quantizer of one lane's 8 channels (the arithmetic stated in include/alise_kv.h, operation by operation).
// Returns the packed codes in w0 (and w1 for 8 bits) and the group's meta dword (fp16 scale | fp16 zero << 16).
//
// The kernel is bound by vector instructions, not by memory, so every step is written in the cheapest form that
// still gives the stated result bit for bit:
//   - range: inside the lane with float min/max (which start from 0, so the results are never NaN and
//     mn <= 0 <= mx); across the lanes of the group on the bit patterns, where "larger unsigned pattern" is
//     "larger" for the non-negative mx and "more negative" for the non-positive mn -- one DPP instruction each
//     per step, no NaN canonicalisation;
//   - r / qmax, correctly rounded, as q0 = r * c, q1 = fma(fma(-qmax, q0, r), c, q0) with c = RN(1 / qmax): r is
//     a difference of two fp16 numbers, so 2^-24 <= r <= 131008 or r = 0 and nothing under- or overflows; that
//     q1 equals the IEEE quotient for qmax = 255 and 15 has been checked for every binary32 r in [0, 131008]
//     (tests/divcheck/);
//   - 1 / scale, correctly rounded, as one Newton step on the hardware reciprocal (1 ulp): the scale is an
//     fp16 number, 11 significant bits, so 1 / scale is at least 2^-36 (relative) away from every rounding
//     boundary of binary32 while the step's result before rounding is off by less than 2^-45;
//   - codes: v_cvt_pk_u8_f32 rounds to nearest even and saturates to [0, 255], which is rint + clamp for 8 bits
//     (for 4 bits the upper clamp is a float minimum first; the lower one cannot be hit by more than -0.5,
//     which rounds to 0).
template <int BITS, int LPG>
__device__ __forceinline__ void quantize8(const h8_t x, uint32_t &w0, uint32_t &w1, uint32_t &meta)
{
    float xf[8];
    float mn = 0.0f, mx = 0.0f;          // the range always includes 0
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        xf[i] = (float)x[i];
        mn = fminf(mn, xf[i]);
        mx = fmaxf(mx, xf[i]);
    }
    uint32_t un = as_u32(mn), ux = as_u32(mx);
    un = max(un, dpp_u<0xB1>(un));  ux = max(ux, dpp_u<0xB1>(ux));                                  // quad_perm [1,0,3,2]
    if constexpr (LPG >= 4) { un = max(un, dpp_u<0x4E>(un)); ux = max(ux, dpp_u<0x4E>(ux)); }       // quad_perm [2,3,0,1]
    if constexpr (LPG >= 8) { un = max(un, dpp_u<0x141>(un)); ux = max(ux, dpp_u<0x141>(ux)); }     // row_half_mirror
    if constexpr (LPG >= 16) { un = max(un, dpp_u<0x140>(un)); ux = max(ux, dpp_u<0x140>(ux)); }    // row_mirror
    mn = as_f32(un);
    mx = as_f32(ux);
    constexpr float qmax = (float)((1 << BITS) - 1);
    constexpr float c = 1.0f / qmax;                  // correctly rounded at compile time
    const float r = mx - mn;
    const float q0 = r * c;
    const float l32 = __builtin_fmaf(__builtin_fmaf(-qmax, q0, r), c, q0);
    _Float16 h = (_Float16)l32;                       // round to nearest even
    uint32_t hb = __builtin_bit_cast(uint16_t, h);
    if ((float)h < l32) hb = hb + 1;                  // scale is rounded up
    if (hb < 0x0400u) hb = 0x0400u;                   // floor at 2^-14
    const float lam = (float)__builtin_bit_cast(_Float16, (uint16_t)hb);
    const float y0 = __builtin_amdgcn_rcpf(lam);
    const float inv = __builtin_fmaf(__builtin_fmaf(-lam, y0, 1.0f), y0, y0);
    float zs = (-mn) * inv;
    if constexpr (BITS == 4) zs = fminf(zs, qmax);
    const uint32_t zi = __builtin_amdgcn_cvt_pk_u8_f32(zs, 0, 0u);       // rint, clamped to [0, qmax]
    const float zf = (float)zi;
    float u[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        u[i] = __builtin_fmaf(xf[i], inv, zf);        // one rounding
        if constexpr (BITS == 4) u[i] = fminf(u[i], qmax);
    }
    uint32_t a = 0, b = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a = __builtin_amdgcn_cvt_pk_u8_f32(u[i], i, a);
        b = __builtin_amdgcn_cvt_pk_u8_f32(u[4 + i], i, b);
    }
    if constexpr (BITS == 8) {
        w0 = a;
        w1 = b;
    } else {
        a |= a >> 4;                                  // byte 0: codes 0, 1; byte 2: codes 2, 3
        b |= b >> 4;
        w0 = __builtin_amdgcn_perm(b, a, 0x06040200u);
        w1 = 0;
    }
    const uint32_t zb = __builtin_bit_cast(uint16_t, (_Float16)zf);
    meta = hb | (zb << 16);
}

// BITS = code width; LPG = lanes per group (G / 8): 2, 4, 8 or 16, so a group never leaves a row of 16 lanes.
template <int BITS, int LPG, bool BY_HEAD>
__global__ __launch_bounds__(256) void quant_write_kernel(QuantParams p)
{
    const uint32_t gl = blockIdx.x * 256u + threadIdx.x;
    const int lane_in_row = (int)(gl & ((1u << p.log_lanes_per_row) - 1u));
    bool live;
    int head, which;
    const _Float16 *src;
    const int64_t *slot_at;
    if constexpr (!BY_HEAD) {
        // Rows are ordered (token, K|V, head): the lanes of a wave stay inside one
        // tensor's contiguous [Hkv][D] slab of one token as long as possible.
        live = gl < p.total_lanes;
        const uint32_t g = live ? gl : p.total_lanes - 1;
        const uint32_t row = g >> p.log_lanes_per_row;
        const uint32_t tw = p.c.Hkv == 1 ? row : (__umulhi(row, p.hkv_magic) >> p.hkv_shift);
        head = (int)(row - tw * (uint32_t)p.c.Hkv);
        which = (int)(tw & 1u);
        const int64_t t = tw >> 1;
        src = (which ? p.v : p.k) + (t * p.c.Hkv + head) * p.c.D + (int)(g & ((1u << p.log_lanes_per_row) - 1u)) * 8;
        slot_at = p.slots + t;
    } else {
        // Rows are ordered (16 tokens, K|V, head, token of the 16): consecutive rows are the same head of
        // consecutive tokens, which a prompt's chunk puts side by side in a page.  The launch covers whole blocks of
        // 16 tokens, so every lane index is in range, and a wave (4 or 8 rows) lies inside one (block, K|V, head):
        // those three and every base address are computed once per wave on the scalar unit, the lanes add small
        // 32-bit offsets.
        const uint32_t row = gl >> p.log_lanes_per_row;
        const uint32_t r2 = __builtin_amdgcn_readfirstlane(row >> 4);
        const uint32_t r3 = p.c.Hkv == 1 ? r2 : (__umulhi(r2, p.hkv_magic) >> p.hkv_shift);
        head = (int)(r2 - r3 * (uint32_t)p.c.Hkv);
        which = (int)(r3 & 1u);
        const int32_t t16 = (int32_t)(r3 >> 1) * 16;              // below T: the block has a token
        const int32_t t_lo = (int32_t)(row & 15u);
        live = t16 + t_lo < p.T;
        const uint32_t dt = (uint32_t)(live ? t_lo : p.T - 1 - t16);
        const _Float16 *base = (which ? p.v : p.k) + ((int64_t)t16 * p.c.Hkv + head) * p.c.D;
        src = base + (__umul24(dt, (uint32_t)(p.c.Hkv * p.c.D)) + (uint32_t)lane_in_row * 8u);
        slot_at = p.slots + t16 + dt;
    }
    const h8_t x = __builtin_nontemporal_load(reinterpret_cast<const h8_t *>(src));    // read once
    const int64_t slot = *slot_at;

    uint32_t w0, w1, m;
    quantize8<BITS, LPG>(x, w0, w1, m);
    if (!live || slot < 0) return;

    // a valid slot is below num_pages * page_size < 2^31, and num_pages * Hkv < 2^31
    const uint32_t s32 = (uint32_t)slot;
    const uint32_t page = s32 >> p.c.logP, off = s32 & (uint32_t)(p.c.P - 1);
    const uint32_t blk = page * (uint32_t)p.c.Hkv + (uint32_t)head;
    uint8_t *codes = (which ? p.c.v_codes : p.c.k_codes) + (uint64_t)blk * (uint32_t)p.c.cstride +
                     (off * (uint32_t)p.c.row_code_bytes + (uint32_t)lane_in_row * BITS);
    if constexpr (BITS == 8) {
        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
        const u32x2_t wv = {w0, w1};
        __builtin_nontemporal_store(wv, reinterpret_cast<u32x2_t *>(codes));
    } else {
        __builtin_nontemporal_store(w0, reinterpret_cast<uint32_t *>(codes));     // channel 2i low nibble, 2i+1 high
    }
    if ((lane_in_row % LPG) == 0) {
        uint8_t *meta = reinterpret_cast<uint8_t *>(which ? p.c.v_meta : p.c.k_meta) + (uint64_t)blk * (uint32_t)p.c.mstride +
                        (off * (uint32_t)p.c.NG + (uint32_t)(lane_in_row / LPG)) * 4u;
        __builtin_nontemporal_store(m, reinterpret_cast<uint32_t *>(meta));
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
    const bool by_head = T >= 1024 && (int64_t)c.Hkv * c.D < (1 << 24);     // the kernel multiplies by Hkv * D in 24 bits
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
