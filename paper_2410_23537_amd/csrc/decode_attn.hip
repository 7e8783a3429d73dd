// Paged single-query attention over b-bit KV codes for gfx950 (vector-ALU path).
//
// Computes, per request i and query head h (ALISE Sec. 2, Eq. 1-2, over the cache
// of Sec. 3.2):   out = sum_t softmax_t(scale * q . k^_t) v^_t,  t < L_i,
// with k^ = lambda_k (code - z_k), v^ = lambda_v (code - z_v) dequantized in registers.
//
// Work decomposition (this build's, not the paper's):
//   plan kernel   : context_lens -> list of tiles (request, split of C tokens)
//   attn kernel   : persistent waves pull (tile, head) items from an atomic counter;
//                   one wave = one item, no workgroup barrier anywhere
//   merge kernel  : log-sum-exp combination of the splits of long requests
//
// Inside a wave every load instruction reads 1 KiB of contiguous codes: a token's
// row of D*bits/8 bytes is split over LPT lanes of 16 bytes, so a wave-load covers
// TPW = 64/LPT consecutive tokens ("slots").  A lane keeps its 16 bytes' worth of
// channels for both K and V, so the scalar product needs a reduction over the LPT
// lanes of a slot (DPP) and the weighted sum needs one reduction over the TPW slots
// at the end of the tile (through LDS).
//
// Dequantization never materialises k^: with the group's (lambda, z),
//   q . k^ = lambda * (sum_c q_c code_c - z * sum_c q_c)
// and the codes are turned into fp16 by bit tricks (1024 + code has the bit pattern
// 0x6400 | code), two at a time, and fed to the packed fp16 dot product with fp32
// accumulation.  The offset 1024 * sum q is subtracted with the zero-point.
#include "alise_kernels.h"

#include <hip/hip_fp16.h>

namespace alise {
namespace {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));

constexpr float kNegInf = -__builtin_inff();
constexpr float kLazy = 8.0f;   // the running maximum is raised only past this slack (log2 units)

struct AttnParams {
    CacheView c;
    const _Float16 *q;
    _Float16 *out;
    const int32_t *block_tables;
    const int32_t *context_lens;
    int32_t max_blocks, B, H, qper, max_len;
    float scale_log2e;
    AttnWorkspace ws;
};

__device__ __forceinline__ h2_t as_h2(uint32_t u) { return __builtin_bit_cast(h2_t, u); }
__device__ __forceinline__ uint32_t as_u32(h2_t h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ float half_lo(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xffffu)); }
__device__ __forceinline__ float half_hi(uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u >> 16)); }

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over the LPT (2, 4 or 8) adjacent lanes that share a token; every lane gets the sum.
template <int LPT>
__device__ __forceinline__ float slot_sum(float v)
{
    v += dpp_f<0xB1>(v);                           // quad_perm [1,0,3,2]
    if constexpr (LPT >= 4) v += dpp_f<0x4E>(v);   // quad_perm [2,3,0,1]
    if constexpr (LPT >= 8) v += dpp_f<0x141>(v);  // row_half_mirror: the other quad of the 8
    return v;
}

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ------------------------------------------------------------------ plan

// One workgroup: chunk counts, their exclusive scan, the tile -> request table.
__global__ __launch_bounds__(1024) void plan_kernel(const int32_t *context_lens, int32_t B, int32_t H,
                                                    int32_t max_len, AttnWorkspace ws)
{
    __shared__ int32_t s_scan[1024];
    __shared__ int32_t s_carry;
    const int tid = threadIdx.x;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    const int C = ws.chunk_tokens;
    for (int base = 0; base < B; base += 1024) {
        const int i = base + tid;
        int n = 0;
        if (i < B) {
            int L = context_lens[i];
            L = L < 0 ? 0 : (L > max_len ? max_len : L);
            n = (L + C - 1) / C;
        }
        s_scan[tid] = n;
        __syncthreads();
        for (int d = 1; d < 1024; d <<= 1) {
            int add = tid >= d ? s_scan[tid - d] : 0;
            __syncthreads();
            s_scan[tid] += add;
            __syncthreads();
        }
        const int carry = s_carry;
        const int first = carry + s_scan[tid] - n;
        if (i < B) {
            ws.tile_base[i] = first;
            for (int c = 0; c < n; ++c)
                if (first + c < ws.max_tiles) ws.tile_req[first + c] = i;
        }
        __syncthreads();
        if (tid == 1023) s_carry = carry + s_scan[1023];
        __syncthreads();
    }
    if (tid == 0) {
        int total = s_carry;
        if (total > ws.max_tiles) total = ws.max_tiles;
        ws.tile_base[B] = total;
        *ws.n_items = total * H;
        *ws.counter = 0u;
    }
}

// ------------------------------------------------------------------ attention

template <int BITS, int D>
struct Geo {
    static constexpr int ROWB = D * BITS / 8;   // code bytes of one token's row
    static constexpr int LPT = ROWB / 16;       // lanes per token
    static constexpr int TPW = 64 / LPT;        // tokens per wave-load
    static constexpr int SL = 128 / BITS;       // channels per lane
    static constexpr int NB = 4;                // wave-loads in flight per block
    static constexpr int LDS_ROW = D + 4;       // floats per slot row in the end-of-tile reduction
};

template <int BITS, int D>
__global__ __launch_bounds__(256) void decode_attn_kernel(AttnParams p)
{
    using G = Geo<BITS, D>;
    constexpr int LPT = G::LPT, TPW = G::TPW, SL = G::SL, NB = G::NB, ROWB = G::ROWB;
    __shared__ float s_red[4][TPW * G::LDS_ROW];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int sub = lane % LPT;         // which 16-byte slice of the row
    const int slot = lane / LPT;        // which token of a wave-load
    const int ch0 = sub * SL;           // first channel of this lane
    const int grp = ch0 / p.c.G;        // the lane's channels lie in one group
    float *red = s_red[wave];
    const int n_items = *p.ws.n_items;
    const int C = p.ws.chunk_tokens;

    for (;;) {
        int it = 0;
        if (lane == 0) it = (int)atomicAdd(p.ws.counter, 1u);
        it = __builtin_amdgcn_readfirstlane(it);
        if (it >= n_items) break;
        const int tile = it / p.H;
        const int h = it - tile * p.H;
        const int i = p.ws.tile_req[tile];
        const int tb_first = p.ws.tile_base[i];
        const int n_split = p.ws.tile_base[i + 1] - tb_first;
        const int split = tile - tb_first;
        int L = p.context_lens[i];
        L = L > p.max_len ? p.max_len : L;
        const int t0 = split * C;
        const int t1 = min(L, t0 + C);
        const int hk = h / p.qper;
        const int32_t *bt = p.block_tables + (int64_t)i * p.max_blocks;

        // ---- this lane's slice of q, arranged to meet the code pairs
        uint32_t qp[SL / 2];
        float qsum = 0.0f;      // sum of q over the slice
        float koff = 0.0f;      // what the 1024 offsets add to the packed dot product
        {
            const uint32_t *qsrc = reinterpret_cast<const uint32_t *>(p.q + ((int64_t)i * p.H + h) * D + ch0);
            uint32_t raw[SL / 2];
#pragma unroll
            for (int k = 0; k < SL / 2; k += 4) {
                const uint4 v4 = *reinterpret_cast<const uint4 *>(qsrc + k);
                raw[k] = v4.x; raw[k + 1] = v4.y; raw[k + 2] = v4.z; raw[k + 3] = v4.w;
            }
            if constexpr (BITS == 8) {
#pragma unroll
                for (int k = 0; k < SL / 2; ++k) {
                    qp[k] = raw[k];
                    qsum += half_lo(raw[k]) + half_hi(raw[k]);
                }
                koff = 1024.0f * qsum;
            } else {
                // a code dword holds channels 8w..8w+7 in nibbles 0..7; the pairs taken from it are
                // (n0,n4) (n1,n5)*16 (n2,n6) (n3,n7)*16, so q is paired the same way and the
                // partners of the *16 pairs are pre-divided by 16.
                float sa = 0.0f, sb = 0.0f;
#pragma unroll
                for (int w = 0; w < SL / 8; ++w) {
                    _Float16 qc[8];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        qc[2 * k] = __builtin_bit_cast(_Float16, (uint16_t)(raw[4 * w + k] & 0xffffu));
                        qc[2 * k + 1] = __builtin_bit_cast(_Float16, (uint16_t)(raw[4 * w + k] >> 16));
                    }
                    const _Float16 sc = (_Float16)0.0625f;
                    h2_t a0 = {qc[0], qc[4]}, b0 = {qc[1] * sc, qc[5] * sc};
                    h2_t a1 = {qc[2], qc[6]}, b1 = {qc[3] * sc, qc[7] * sc};
                    qp[4 * w + 0] = as_u32(a0); qp[4 * w + 1] = as_u32(b0);
                    qp[4 * w + 2] = as_u32(a1); qp[4 * w + 3] = as_u32(b1);
                    sa += (float)a0.x + (float)a0.y + (float)a1.x + (float)a1.y;
                    sb += (float)b0.x + (float)b0.y + (float)b1.x + (float)b1.y;   // already /16
                }
                qsum = sa + 16.0f * sb;
                koff = 1024.0f * (sa + sb);
            }
        }

        float m_ref = kNegInf, l = 0.0f, wz = 0.0f;
        float acc[SL];
#pragma unroll
        for (int k = 0; k < SL; ++k) acc[k] = 0.0f;

        for (int tb = t0; tb < t1; tb += NB * TPW) {
            uint4 kc[NB], vc[NB];
            uint32_t km[NB], vm[NB];
            bool valid[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int tok = tb + j * TPW + slot;
                valid[j] = tok < t1;
                const int tc = valid[j] ? tok : t1 - 1;        // stay on a real token
                const int64_t page = bt[tc >> p.c.logP];
                const int64_t row = (page * p.c.Hkv + hk) * p.c.P + (tc & (p.c.P - 1));
                const int64_t coff = row * ROWB + sub * 16;
                kc[j] = *reinterpret_cast<const uint4 *>(p.c.k_codes + coff);
                vc[j] = *reinterpret_cast<const uint4 *>(p.c.v_codes + coff);
                km[j] = p.c.k_meta[row * p.c.NG + grp];
                vm[j] = p.c.v_meta[row * p.c.NG + grp];
            }

            // ---- scores (log2 domain)
            float s[NB];
            float mx = kNegInf;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const uint32_t kw[4] = {kc[j].x, kc[j].y, kc[j].z, kc[j].w};
                float dot = 0.0f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    if constexpr (BITS == 8) {
                        const uint32_t lo = __builtin_amdgcn_perm(0x64646464u, kw[w], 0x04010400u);
                        const uint32_t hi = __builtin_amdgcn_perm(0x64646464u, kw[w], 0x04030402u);
                        dot = __builtin_amdgcn_fdot2(as_h2(lo), as_h2(qp[2 * w]), dot, false);
                        dot = __builtin_amdgcn_fdot2(as_h2(hi), as_h2(qp[2 * w + 1]), dot, false);
                    } else {
                        const uint32_t x = kw[w], y = kw[w] >> 8;
                        const uint32_t a0 = (x & 0x000F000Fu) | 0x64006400u;
                        const uint32_t b0 = (x & 0x00F000F0u) | 0x64006400u;
                        const uint32_t a1 = (y & 0x000F000Fu) | 0x64006400u;
                        const uint32_t b1 = (y & 0x00F000F0u) | 0x64006400u;
                        dot = __builtin_amdgcn_fdot2(as_h2(a0), as_h2(qp[4 * w + 0]), dot, false);
                        dot = __builtin_amdgcn_fdot2(as_h2(b0), as_h2(qp[4 * w + 1]), dot, false);
                        dot = __builtin_amdgcn_fdot2(as_h2(a1), as_h2(qp[4 * w + 2]), dot, false);
                        dot = __builtin_amdgcn_fdot2(as_h2(b1), as_h2(qp[4 * w + 3]), dot, false);
                    }
                }
                const float lam = half_lo(km[j]) * p.scale_log2e;
                const float z = half_hi(km[j]);
                float part = lam * ((dot - koff) - z * qsum);
                part = slot_sum<LPT>(part);
                s[j] = valid[j] ? part : kNegInf;
                mx = fmaxf(mx, s[j]);
            }

            // ---- running maximum, raised lazily (wave-uniform branch, rarely taken)
            if (__builtin_amdgcn_ballot_w64(mx > m_ref + kLazy) != 0) {
                const float m_new = (mx > m_ref + kLazy) ? mx : m_ref;
                const float f = (m_new == m_ref) ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);
                l *= f;
                wz *= f;
#pragma unroll
                for (int k = 0; k < SL; ++k) acc[k] *= f;
                m_ref = m_new;
            }

            // ---- weights and weighted sum of V codes
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const float pj = valid[j] ? __builtin_amdgcn_exp2f(s[j] - m_ref) : 0.0f;
                l += pj;
                const float w = pj * half_lo(vm[j]);
                const uint32_t vw[4] = {vc[j].x, vc[j].y, vc[j].z, vc[j].w};
                if constexpr (BITS == 8) {
                    wz = __builtin_fmaf(w, 1024.0f + half_hi(vm[j]), wz);
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const h2_t lo = as_h2(__builtin_amdgcn_perm(0x64646464u, vw[d], 0x04010400u));
                        const h2_t hi = as_h2(__builtin_amdgcn_perm(0x64646464u, vw[d], 0x04030402u));
                        acc[4 * d + 0] = __builtin_fmaf((float)lo.x, w, acc[4 * d + 0]);
                        acc[4 * d + 1] = __builtin_fmaf((float)lo.y, w, acc[4 * d + 1]);
                        acc[4 * d + 2] = __builtin_fmaf((float)hi.x, w, acc[4 * d + 2]);
                        acc[4 * d + 3] = __builtin_fmaf((float)hi.y, w, acc[4 * d + 3]);
                    }
                } else {
                    // exact integer (code - z) in fp16, so nothing is left to cancel later
                    const uint32_t zb = vm[j] >> 16;                       // fp16 bits of z
                    const h2_t zz = as_h2(zb | (zb << 16));
                    const h2_t k1 = {(_Float16)-1024.0f, (_Float16)-1024.0f};
                    const h2_t k16 = {(_Float16)-16.0f, (_Float16)-16.0f};
                    const h2_t offa = k1 - zz;                             // -(1024 + z)
                    const h2_t offb = zz * k16 + k1;                       // -(1024 + 16 z)
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const uint32_t x = vw[d], y = vw[d] >> 8;
                        const h2_t a0 = as_h2((x & 0x000F000Fu) | 0x64006400u) + offa;
                        const h2_t b0 = as_h2((x & 0x00F000F0u) | 0x64006400u) + offb;
                        const h2_t a1 = as_h2((y & 0x000F000Fu) | 0x64006400u) + offa;
                        const h2_t b1 = as_h2((y & 0x00F000F0u) | 0x64006400u) + offb;
                        // acc order inside a dword: channels 0,4,1,5,2,6,3,7 (odd ones carry *16)
                        acc[8 * d + 0] = __builtin_fmaf((float)a0.x, w, acc[8 * d + 0]);
                        acc[8 * d + 1] = __builtin_fmaf((float)a0.y, w, acc[8 * d + 1]);
                        acc[8 * d + 2] = __builtin_fmaf((float)b0.x, w, acc[8 * d + 2]);
                        acc[8 * d + 3] = __builtin_fmaf((float)b0.y, w, acc[8 * d + 3]);
                        acc[8 * d + 4] = __builtin_fmaf((float)a1.x, w, acc[8 * d + 4]);
                        acc[8 * d + 5] = __builtin_fmaf((float)a1.y, w, acc[8 * d + 5]);
                        acc[8 * d + 6] = __builtin_fmaf((float)b1.x, w, acc[8 * d + 6]);
                        acc[8 * d + 7] = __builtin_fmaf((float)b1.y, w, acc[8 * d + 7]);
                    }
                }
            }
        }

        // ---- bring the TPW slots to one maximum, then add them up through LDS
        float m_fin = m_ref;
#pragma unroll
        for (int d = LPT; d < 64; d <<= 1) m_fin = fmaxf(m_fin, __shfl_xor(m_fin, d));
        const float f = (m_ref == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(m_ref - m_fin);
        l *= f;
#pragma unroll
        for (int d = LPT; d < 64; d <<= 1) l += __shfl_xor(l, d);
        float *myrow = red + slot * G::LDS_ROW + ch0;
        if constexpr (BITS == 8) {
#pragma unroll
            for (int k = 0; k < SL; ++k) myrow[k] = (acc[k] - wz) * f;
        } else {
            const float f16 = f * 0.0625f;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                myrow[8 * d + 0] = acc[8 * d + 0] * f;
                myrow[8 * d + 4] = acc[8 * d + 1] * f;
                myrow[8 * d + 1] = acc[8 * d + 2] * f16;
                myrow[8 * d + 5] = acc[8 * d + 3] * f16;
                myrow[8 * d + 2] = acc[8 * d + 4] * f;
                myrow[8 * d + 6] = acc[8 * d + 5] * f;
                myrow[8 * d + 3] = acc[8 * d + 6] * f16;
                myrow[8 * d + 7] = acc[8 * d + 7] * f16;
            }
        }
        wave_lds_sync();
        float o[D / 64];
#pragma unroll
        for (int r = 0; r < D / 64; ++r) {
            float sum = 0.0f;
#pragma unroll
            for (int sl = 0; sl < TPW; ++sl) sum += red[sl * G::LDS_ROW + r * 64 + lane];
            o[r] = sum;
        }
        wave_lds_sync();   // the next item overwrites `red`

        if (n_split == 1) {
            const float inv_l = 1.0f / l;
            _Float16 *dst = p.out + ((int64_t)i * p.H + h) * D;
#pragma unroll
            for (int r = 0; r < D / 64; ++r) dst[r * 64 + lane] = (_Float16)(o[r] * inv_l);
        } else {
            float *dst = p.ws.part + ((int64_t)tile * p.H + h) * (D + 2);
            if (lane == 0) { dst[0] = m_fin; dst[1] = l; }
#pragma unroll
            for (int r = 0; r < D / 64; ++r) dst[2 + r * 64 + lane] = o[r];
        }
    }
}

// ------------------------------------------------------------------ merge

// One wave per (request, head): zero rows for empty requests, log-sum-exp combination
// of the splits of requests longer than one split; single-split rows were already written.
template <int D>
__global__ __launch_bounds__(256) void merge_kernel(AttnParams p)
{
    const int lane = threadIdx.x & 63;
    const int ih = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (ih >= p.B * p.H) return;
    const int i = ih / p.H, h = ih - i * p.H;
    const int first = p.ws.tile_base[i];
    const int n = p.ws.tile_base[i + 1] - first;
    if (n == 1) return;
    _Float16 *dst = p.out + (int64_t)ih * D;
    if (n == 0) {
#pragma unroll
        for (int r = 0; r < D / 64; ++r) dst[r * 64 + lane] = (_Float16)0.0f;
        return;
    }
    const float *part = p.ws.part + ((int64_t)first * p.H + h) * (D + 2);
    const int64_t stride = (int64_t)p.H * (D + 2);
    float m = kNegInf;
    for (int c = 0; c < n; ++c) m = fmaxf(m, part[c * stride]);
    float l = 0.0f, o[D / 64];
#pragma unroll
    for (int r = 0; r < D / 64; ++r) o[r] = 0.0f;
    for (int c = 0; c < n; ++c) {
        const float *pc = part + c * stride;
        const float f = __builtin_amdgcn_exp2f(pc[0] - m);
        l = __builtin_fmaf(pc[1], f, l);
#pragma unroll
        for (int r = 0; r < D / 64; ++r) o[r] = __builtin_fmaf(pc[2 + r * 64 + lane], f, o[r]);
    }
    const float inv_l = 1.0f / l;
#pragma unroll
    for (int r = 0; r < D / 64; ++r) dst[r * 64 + lane] = (_Float16)(o[r] * inv_l);
}

template <int BITS, int D>
hipError_t launch_t(const AttnParams &p, int32_t resident_waves, hipStream_t s)
{
    int blocks = resident_waves / 4;
    const int64_t max_items = (int64_t)p.ws.max_tiles * p.H;
    if ((int64_t)blocks * 4 > max_items) blocks = (int)((max_items + 3) / 4);
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((decode_attn_kernel<BITS, D>), dim3(blocks), dim3(256), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int mblocks = (p.B * p.H + 3) / 4;
    hipLaunchKernelGGL((merge_kernel<D>), dim3(mblocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_attn(const CacheView &c, const void *q, void *out,
                              const int32_t *block_tables, int32_t max_blocks,
                              const int32_t *context_lens, int32_t B, int32_t H,
                              int32_t max_context_len, float softmax_scale,
                              const AttnWorkspace &ws, int32_t resident_waves, hipStream_t s)
{
    if (B == 0) return hipSuccess;
    AttnParams p;
    p.c = c;
    p.q = static_cast<const _Float16 *>(q);
    p.out = static_cast<_Float16 *>(out);
    p.block_tables = block_tables;
    p.context_lens = context_lens;
    p.max_blocks = max_blocks;
    p.B = B;
    p.H = H;
    p.qper = H / c.Hkv;
    p.max_len = max_context_len;
    p.scale_log2e = softmax_scale * 1.44269504088896340736f;
    p.ws = ws;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(1024), 0, s, context_lens, B, H, max_context_len, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (c.bits == 8 && c.D == 128) return launch_t<8, 128>(p, resident_waves, s);
    if (c.bits == 8 && c.D == 64) return launch_t<8, 64>(p, resident_waves, s);
    if (c.bits == 4 && c.D == 128) return launch_t<4, 128>(p, resident_waves, s);
    if (c.bits == 4 && c.D == 64) return launch_t<4, 64>(p, resident_waves, s);
    return hipErrorInvalidValue;
}

}  // namespace alise
