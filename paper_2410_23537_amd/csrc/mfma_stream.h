// Pieces shared by the matrix-core attention kernels (decode for grouped-query layouts, chunked
// prefill): direct global -> LDS loads, the hand-placed waits that go with them, LDS reads in
// assembly, operand packing.
#pragma once
#include "attn_common.h"

namespace alise {
namespace {

typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef float f4_t __attribute__((ext_vector_type(4)));

constexpr int kStep = 32;       // tokens per step: two 16-token tiles

typedef const void __attribute__((address_space(1))) *gptr_t;
typedef uint8_t __attribute__((address_space(3))) *lptr_t;
typedef void __attribute__((address_space(3))) *lvoid_t;

// Direct global -> LDS loads: lane l's bytes land at the LDS base + l * size, wherever the
// lane's global address points.  The cache is streamed (non-temporal); the bookkeeping is not.
__device__ __forceinline__ void dma16_stream(const void *g, lptr_t l) { __builtin_amdgcn_global_load_lds((gptr_t)g, (lvoid_t)l, 16, 0, 2); }
__device__ __forceinline__ void dma4_stream(const void *g, lptr_t l) { __builtin_amdgcn_global_load_lds((gptr_t)g, (lvoid_t)l, 4, 0, 2); }
__device__ __forceinline__ void dma16(const void *g, lptr_t l) { __builtin_amdgcn_global_load_lds((gptr_t)g, (lvoid_t)l, 16, 0, 0); }
__device__ __forceinline__ void dma4(const void *g, lptr_t l) { __builtin_amdgcn_global_load_lds((gptr_t)g, (lvoid_t)l, 4, 0, 0); }

#define ALISE_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xf) | (((n) >> 4) << 14) | (0x7 << 4) | (0xf << 8))

// Wait until the load that has `newer` loads issued after it has landed.  Loads complete in
// the order they were issued, so it is enough that at most `newer` stay in flight; the count
// is rounded down to a multiple of four (the menu of immediates), which only waits longer.
// Stores are never counted: they may complete out of order with the loads.
__device__ __forceinline__ void wait_newer(int newer)       // wave-uniform
{
    const int k = newer >> 2;
    if (k >= 12) ALISE_VMCNT(48);
    else if (k >= 9) ALISE_VMCNT(36);
    else if (k >= 6) ALISE_VMCNT(24);
    else if (k >= 4) ALISE_VMCNT(16);
    else if (k == 3) ALISE_VMCNT(12);
    else if (k == 2) ALISE_VMCNT(8);
    else if (k == 1) ALISE_VMCNT(4);
    else ALISE_VMCNT(0);
}

// LDS reads of data that arrived by direct loads are written in assembly: the compiler does
// not see them, so it never orders them against the loads in flight -- the waits above do.
__device__ __forceinline__ uint4 lds_read16(uint32_t addr)
{
    uint4 r;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(r) : "v"(addr) : "memory");
    return r;
}
__device__ __forceinline__ uint32_t lds_read4(uint32_t addr)
{
    uint32_t r;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(r) : "v"(addr) : "memory");
    return r;
}
// four 16-byte reads, one wait
__device__ __forceinline__ void lds_read16x4(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3,
                                             uint4 &r0, uint4 &r1, uint4 &r2, uint4 &r3)
{
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3) : "v"(a0), "v"(a1), "v"(a2), "v"(a3) : "memory");
}
// eight dword reads at eight addresses, one wait
__device__ __forceinline__ void lds_read4x8(const uint32_t (&a)[8], uint32_t off, uint32_t (&r)[8])
{
    asm volatile("ds_read_b32 %0, %8\n\tds_read_b32 %1, %9\n\tds_read_b32 %2, %10\n\tds_read_b32 %3, %11\n\t"
                 "ds_read_b32 %4, %12\n\tds_read_b32 %5, %13\n\tds_read_b32 %6, %14\n\tds_read_b32 %7, %15\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7])
                 : "v"(a[0] + off), "v"(a[1] + off), "v"(a[2] + off), "v"(a[3] + off),
                   "v"(a[4] + off), "v"(a[5] + off), "v"(a[6] + off), "v"(a[7] + off)
                 : "memory");
}

// The same with one address register per read and compile-time byte offsets in the instructions.
template <int O0, int O1, int O2, int O3>
__device__ __forceinline__ void lds_read16x4_at(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3,
                                                uint4 &r0, uint4 &r1, uint4 &r2, uint4 &r3)
{
    asm volatile("ds_read_b128 %0, %4 offset:%8\n\tds_read_b128 %1, %5 offset:%9\n\t"
                 "ds_read_b128 %2, %6 offset:%10\n\tds_read_b128 %3, %7 offset:%11\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3)
                 : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "n"(O0), "n"(O1), "n"(O2), "n"(O3) : "memory");
}
// two 16-byte reads with compile-time byte offsets, one wait
template <int O0, int O1>
__device__ __forceinline__ void lds_read16x2_at(uint32_t a0, uint32_t a1, uint4 &r0, uint4 &r1)
{
    asm volatile("ds_read_b128 %0, %2 offset:%4\n\tds_read_b128 %1, %3 offset:%5\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(r0), "=&v"(r1) : "v"(a0), "v"(a1), "n"(O0), "n"(O1) : "memory");
}
// eight addresses a[set * 4 + r], each read at + r * ROW and at + r * ROW + OFF: r0[i] and r1[i]; one wait
template <int ROW, int OFF>
__device__ __forceinline__ void lds_read4x8x2(const uint32_t (&a)[8], uint32_t (&r0)[8], uint32_t (&r1)[8])
{
    asm volatile("ds_read_b32 %0, %16\n\tds_read_b32 %1, %17 offset:%24\n\tds_read_b32 %2, %18 offset:%25\n\tds_read_b32 %3, %19 offset:%26\n\t"
                 "ds_read_b32 %4, %20\n\tds_read_b32 %5, %21 offset:%24\n\tds_read_b32 %6, %22 offset:%25\n\tds_read_b32 %7, %23 offset:%26\n\t"
                 "ds_read_b32 %8, %16 offset:%27\n\tds_read_b32 %9, %17 offset:%28\n\t"
                 "ds_read_b32 %10, %18 offset:%29\n\tds_read_b32 %11, %19 offset:%30\n\t"
                 "ds_read_b32 %12, %20 offset:%27\n\tds_read_b32 %13, %21 offset:%28\n\t"
                 "ds_read_b32 %14, %22 offset:%29\n\tds_read_b32 %15, %23 offset:%30\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r0[0]), "=&v"(r0[1]), "=&v"(r0[2]), "=&v"(r0[3]), "=&v"(r0[4]), "=&v"(r0[5]), "=&v"(r0[6]), "=&v"(r0[7]),
                   "=&v"(r1[0]), "=&v"(r1[1]), "=&v"(r1[2]), "=&v"(r1[3]), "=&v"(r1[4]), "=&v"(r1[5]), "=&v"(r1[6]), "=&v"(r1[7])
                 : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]),
                   "n"(ROW), "n"(2 * ROW), "n"(3 * ROW), "n"(OFF), "n"(OFF + ROW), "n"(OFF + 2 * ROW), "n"(OFF + 3 * ROW)
                 : "memory");
}

// four addresses, each read at +0 and at +OFF: r0[i] = [a[i]], r1[i] = [a[i] + OFF]; one wait
template <int OFF>
__device__ __forceinline__ void lds_read4x4x2(const uint32_t (&a)[4], uint32_t (&r0)[4], uint32_t (&r1)[4])
{
    asm volatile("ds_read_b32 %0, %8\n\tds_read_b32 %1, %9\n\tds_read_b32 %2, %10\n\tds_read_b32 %3, %11\n\t"
                 "ds_read_b32 %4, %8 offset:%12\n\tds_read_b32 %5, %9 offset:%12\n\t"
                 "ds_read_b32 %6, %10 offset:%12\n\tds_read_b32 %7, %11 offset:%12\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r0[0]), "=&v"(r0[1]), "=&v"(r0[2]), "=&v"(r0[3]), "=&v"(r1[0]), "=&v"(r1[1]), "=&v"(r1[2]), "=&v"(r1[3])
                 : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "n"(OFF)
                 : "memory");
}
// four addresses, the dwords at +0 and +8 of each (one two-dword read per address): r[i][0] = [a[i]], r[i][1] = [a[i] + 8]; one wait
__device__ __forceinline__ void lds_read2x4(const uint32_t (&a)[4], uint32_t (&r)[4][2])
{
    typedef uint32_t u2_t __attribute__((ext_vector_type(2)));
    u2_t r0, r1, r2, r3;
    asm volatile("ds_read2_b32 %0, %4 offset1:2\n\tds_read2_b32 %1, %5 offset1:2\n\t"
                 "ds_read2_b32 %2, %6 offset1:2\n\tds_read2_b32 %3, %7 offset1:2\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3) : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]) : "memory");
    r[0][0] = r0.x; r[0][1] = r0.y; r[1][0] = r1.x; r[1][1] = r1.y;
    r[2][0] = r2.x; r[2][1] = r2.y; r[3][0] = r3.x; r[3][1] = r3.y;
}
// two addresses, each read at + r * ROW (r = 0..3) and at + r * ROW + OFF: a0 -> (p0, p1), a1 -> (q0, q1); one wait
template <int ROW, int OFF>
__device__ __forceinline__ void lds_read4_rows2x2(uint32_t a0, uint32_t a1, uint32_t (&p0)[4], uint32_t (&p1)[4],
                                                  uint32_t (&q0)[4], uint32_t (&q1)[4])
{
    asm volatile("ds_read_b32 %0, %16\n\tds_read_b32 %1, %16 offset:%18\n\tds_read_b32 %2, %16 offset:%19\n\tds_read_b32 %3, %16 offset:%20\n\t"
                 "ds_read_b32 %4, %16 offset:%21\n\tds_read_b32 %5, %16 offset:%22\n\tds_read_b32 %6, %16 offset:%23\n\tds_read_b32 %7, %16 offset:%24\n\t"
                 "ds_read_b32 %8, %17\n\tds_read_b32 %9, %17 offset:%18\n\tds_read_b32 %10, %17 offset:%19\n\tds_read_b32 %11, %17 offset:%20\n\t"
                 "ds_read_b32 %12, %17 offset:%21\n\tds_read_b32 %13, %17 offset:%22\n\tds_read_b32 %14, %17 offset:%23\n\tds_read_b32 %15, %17 offset:%24\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(p0[0]), "=&v"(p0[1]), "=&v"(p0[2]), "=&v"(p0[3]), "=&v"(p1[0]), "=&v"(p1[1]), "=&v"(p1[2]), "=&v"(p1[3]),
                   "=&v"(q0[0]), "=&v"(q0[1]), "=&v"(q0[2]), "=&v"(q0[3]), "=&v"(q1[0]), "=&v"(q1[1]), "=&v"(q1[2]), "=&v"(q1[3])
                 : "v"(a0), "v"(a1), "n"(ROW), "n"(2 * ROW), "n"(3 * ROW), "n"(OFF), "n"(OFF + ROW), "n"(OFF + 2 * ROW), "n"(OFF + 3 * ROW)
                 : "memory");
}

// The weights p * lambda_v enter the second product as fp16 (high + low part).  With the
// running maximum as the reference, p <= 2^kLazy and the largest weight of a row may be as
// small as lambda_v itself, so that weights a million times smaller already fall under the
// fp16 subnormal spacing of 2^-24 -- and thousands of such tokens add up to 1e-3 of the
// result on peaked rows.  The reference is therefore lowered by kWeightBias: every weight,
// the denominator and the weighted zero-points carry the same extra factor 2^kWeightBias,
// which cancels in the quotient and moves the floor 64 times further down.  Weights then
// reach 2^(kLazy + kWeightBias) * lambda_v, inside the fp16 range while lambda_v < 2; a step
// that holds a larger V scale drops the bias for the rest of the item (rescaling what has
// been accumulated), after which the range suffices up to lambda_v = 256.
constexpr float kWeightBias = 6.0f;

// Largest fp16 bit pattern in the low halves of `n` dwords (positive fp16: integer order is value order).
template <int N>
__device__ __forceinline__ uint32_t max_low_half(const uint32_t *v)
{
    typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));
    u16x2_t m = {0, 0};
#pragma unroll
    for (int k = 0; k < N; ++k) m = __builtin_elementwise_max(m, __builtin_bit_cast(u16x2_t, v[k]));
    return m.x;
}

template <int NGRP>
__device__ __forceinline__ uint32_t meta_of(const uint4 (&m)[NGRP], int r, int grp)
{
    const int idx = r * NGRP + grp;
    const uint4 u = m[idx / 4];
    const int c = idx % 4;
    return c == 0 ? u.x : c == 1 ? u.y : c == 2 ? u.z : u.w;
}

// Mixed-precision multiply-adds that read an fp16 factor in place out of a dword (v_fma_mix_*), written
// out because the compiler mostly converts the half to fp32 first and then spends a plain fp32
// multiply-add on it all the same: one instruction more per half.  The compiler does not see into these
// statements, so it inserts none of the wait states that an operand just written by a matrix or a
// transcendental instruction needs: no operand may come straight from a matrix instruction (use them
// on values that ordinary vector instructions or LDS reads produced), and the ones that take the
// softmax weights (fresh from v_exp_f32) bring their own wait state.
// lo(h) * b + c in fp32:
__device__ __forceinline__ float fma_lo_half(uint32_t h, float b, float c)
{
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(h), "v"(b), "v"(c));
    return d;
}
// hi(a) * (half E of b) + c in fp32, both factors fp16:
template <int E>
__device__ __forceinline__ float fma_hi_by_half(uint32_t a, uint32_t b, float c)
{
    float d;
    if constexpr (E == 0) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,1,0]" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
// (lo(h0) * p0, lo(h1) * p1), each rounded to fp16 (nearest even), as one dword; p0 and p1 may be
// results of a transcendental instruction issued just before (one wait state, spent here).
__device__ __forceinline__ uint32_t mul_lo_halves_to_h2(uint32_t h0, float p0, uint32_t h1, float p1)
{
    uint32_t d;
    asm("s_nop 0\n\tv_fma_mixlo_f16 %0, %1, %2, 0 op_sel_hi:[1,0,0]\n\tv_fma_mixhi_f16 %0, %3, %4, 0 op_sel_hi:[1,0,0]"
        : "=&v"(d) : "v"(h0), "v"(p0), "v"(h1), "v"(p1));
    return d;
}
// lo(h) * p in fp32, p possibly fresh from a transcendental instruction (one wait state, spent here)
__device__ __forceinline__ float mul_lo_half_f32(uint32_t h, float p)
{
    float d;
    asm("s_nop 0\n\tv_fma_mix_f32 %0, %1, %2, 0 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(h), "v"(p));
    return d;
}
// hi(h) * b + c in fp32, b and c fp32 values that an ordinary vector instruction produced
__device__ __forceinline__ float fma_hi_half(uint32_t h, float b, float c)
{
    float d;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(h), "v"(b), "v"(c));
    return d;
}
// What the fp16 pair w lacks of the exact products (w: the products rounded to fp16, made from the same operands):
// (lo(h0) * p0 - lo(w), lo(h1) * p1 - hi(w)), each computed with one rounding, as one dword.
__device__ __forceinline__ uint32_t residual_of_h2(uint32_t h0, float p0, uint32_t h1, float p1, uint32_t w)
{
    uint32_t d;
    asm("v_fma_mixlo_f16 %0, %1, %2, -%5 op_sel_hi:[1,0,1]\n\tv_fma_mixhi_f16 %0, %3, %4, -%5 op_sel:[0,0,1] op_sel_hi:[1,0,1]"
        : "=&v"(d) : "v"(h0), "v"(p0), "v"(h1), "v"(p1), "v"(w));
    return d;
}

__device__ __forceinline__ h8_t pack8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
    const u4_t u = {a, b, c, d};
    return __builtin_bit_cast(h8_t, u);
}

}  // namespace
}  // namespace alise
