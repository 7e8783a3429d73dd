// Paged single-query attention for grouped-query layouts on the gfx950 matrix cores.
//
// With H / Hkv = qper query heads per KV head, every KV byte is used by qper queries, so
// q K^T and P V are real (small) matrix products (ALISE Sec. 2, Eq. 1-2, over the INT8
// cache of Sec. 3.2).  One wave serves all query heads of one KV head for one tile of
// tokens; the work items of a tile are its KV heads.  Per step of 32 tokens:
//
//   S^T = K Q^T   v_mfma_f32_16x16x32_f16, A = K codes as fp16 (16 tokens x 32 channels),
//                 B = Q^T (32 channels x 16 query heads, the heads past qper are zero).
//                 The result has a query head per lane column and 4 tokens per lane, which
//                 is exactly the A-operand layout the second product needs for P.
//   O  += P V     A = p * lambda_v as fp16 (split into high and low parts so that no
//                 weight loses precision), B = V codes (32 tokens x 16 channels).
//
// Operands are built in registers, never through LDS:
//   K: a lane loads 2 x 16 bytes of one token's row; 0x6400 | code is the fp16 1024 + code;
//      the 1024 * sum(q) offset leaves with the zero-point, per group of the row.
//   V: the product contracts over tokens, but a row holds channels.  A lane loads one dword
//      (4 channels) from each of its 8 tokens and a byte permute picks the same channel out
//      of two dwords, leaving the fp16 subnormals code * 2^-24 of two tokens side by side --
//      which is the operand layout.  The matrix cores multiply subnormals exactly.
//
// Softmax state (running maximum, denominator, weighted zero-points) lives in the lanes of
// the S^T layout and is brought to the rows of O only at the end of a tile.
#include "attn_common.h"

namespace alise {
namespace {

typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef float f4_t __attribute__((ext_vector_type(4)));

constexpr int kStep = 32;       // tokens per step: two 16-token tiles

// Loaded data of one step.  NGRP = groups per token row (1 or 2).
template <int NGRP>
struct StepBuf {
    uint4 k[2][2];          // [tile][piece]: 16 code bytes of this lane's token, channels g*16.. and 64+g*16..
    uint4 km[2][NGRP];      // [tile]: (scale, zero) of this lane's 4 tokens, NGRP dwords per token
    uint4 vm[2][NGRP];
    uint32_t v[2][4][2];    // [tile][token r][set]: 4 code bytes, channels 64*set + 4n ..
};

template <int NGRP>
__device__ __forceinline__ uint32_t meta_of(const uint4 (&m)[NGRP], int r, int grp)
{
    const int idx = r * NGRP + grp;
    const uint4 u = m[idx / 4];
    const int c = idx % 4;
    return c == 0 ? u.x : c == 1 ? u.y : c == 2 ? u.z : u.w;
}

__device__ __forceinline__ h8_t pack8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
    const u4_t u = {a, b, c, d};
    return __builtin_bit_cast(h8_t, u);
}

template <int NGRP>
__global__ __launch_bounds__(256) void decode_attn_gqa_kernel(AttnParams p)
{
    constexpr int D = 128, ROWB = 128;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15;        // column of the matrix layouts: token (K), query head (S^T), channel (V, O)
    const int g = lane >> 4;        // quarter of the wave: 8 consecutive k-slots, 4 consecutive rows
    const int logP = p.c.logP, P = p.c.P, Hkv = p.c.Hkv, qper = p.qper;
    const int n_items = *p.ws.n_items;
    const int4 *order = p.ws.order;
    const int C = p.ws.chunk_tokens;
    (void)C;

    // work queues: see the vector kernel; an item is (tile, KV head)
    const int nq = gridDim.x >= kQueues ? kQueues : 1;
    const int qid = blockIdx.x % nq;
    uint32_t *counter = p.ws.counter + qid * kQueueStride;

    int ticket = 0;
    if (lane == 0) ticket = (int)atomicAdd(counter, 1u);
    int it = qid + nq * __builtin_amdgcn_readfirstlane(ticket);

    while (it < n_items) {
        // the next ticket travels while this item is processed
        if (lane == 0) ticket = (int)atomicAdd(counter, 1u);

        const int4 d = order[it / Hkv];
        const int hk = it % Hkv;
        const int i = __builtin_amdgcn_readfirstlane(d.x);
        const int t0 = __builtin_amdgcn_readfirstlane(d.y);
        const int t1 = __builtin_amdgcn_readfirstlane(d.z);
        const int part = __builtin_amdgcn_readfirstlane(d.w);
        const int32_t *bt = p.block_tables + (int64_t)i * p.max_blocks;
        const int win_first = t0 >> logP;
        const int pg = bt[min(win_first + lane, (t1 - 1) >> logP)];    // a tile spans at most 64 pages
        const int nsteps = (t1 - t0 + kStep - 1) / kStep;

        // ---- Q^T as the B operand of the four k-chunks: chunk j, slot g*8+e <-> channel (j/2)*64 + g*16 + (j%2)*8 + e
        h8_t qop[4];
        float qs[NGRP];             // sum of this query head's q over the channels of a group
        {
            const int qh = hk * qper + n;
            const _Float16 *qrow = p.q + ((int64_t)i * p.H + (n < qper ? qh : hk * qper)) * D;
            float part_sum[NGRP];
#pragma unroll
            for (int gr = 0; gr < NGRP; ++gr) part_sum[gr] = 0.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                h8_t v = *reinterpret_cast<const h8_t *>(qrow + (j / 2) * 64 + g * 16 + (j % 2) * 8);
                if (n >= qper) v = (h8_t)(_Float16)0.0f;
                qop[j] = v;
                float sacc = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) sacc += (float)v[e];
                part_sum[NGRP == 2 ? j / 2 : 0] += sacc;
            }
#pragma unroll
            for (int gr = 0; gr < NGRP; ++gr) {
                float v = part_sum[gr];
                v += __shfl_xor(v, 16);
                v += __shfl_xor(v, 32);
                qs[gr] = v;
            }
        }

        float m_ref = kFloor, l_part = 0.0f, z_part[NGRP];
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) z_part[gr] = 0.0f;
        f4_t o[8];                  // [set*4 + nu]: rows = query heads 4g..4g+3, column n <-> channel 64*set + 4n + nu
#pragma unroll
        for (int t = 0; t < 8; ++t) o[t] = (f4_t)0.0f;

        // Issue the loads of step k (clamped to the last step; tiles past the end of the tile
        // re-read its last 16-token tile).  Straight-line code: no branch around a load.
        auto issue = [&](StepBuf<NGRP> &b, int k) {
            const int ks = min(k, nsteps - 1);
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                int tx = t0 + ks * kStep + x * 16;
                if (tx >= t1) tx -= 16;                     // second tile starts past the end: repeat the first
                const int page = __builtin_amdgcn_readlane(pg, (tx >> logP) - win_first);
                const int blk = page * Hkv + hk;
                const int off = tx & (P - 1);
                const int64_t co = (int64_t)blk * p.c.cstride + (int64_t)off * ROWB;
                const int64_t mo = (int64_t)blk * p.c.mstride + (int64_t)(off + g * 4) * NGRP * 4;
                const uint8_t *kb = p.c.k_codes + co + n * ROWB + g * 16;
                b.k[x][0] = stream_load16(kb);
                b.k[x][1] = stream_load16(kb + 64);
                const uint8_t *kmb = reinterpret_cast<const uint8_t *>(p.c.k_meta) + mo;
                const uint8_t *vmb = reinterpret_cast<const uint8_t *>(p.c.v_meta) + mo;
#pragma unroll
                for (int u = 0; u < NGRP; ++u) {
                    b.km[x][u] = stream_load16(kmb + u * 16);
                    b.vm[x][u] = stream_load16(vmb + u * 16);
                }
                const uint8_t *vb = p.c.v_codes + co + (g * 4) * ROWB + n * 4;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    b.v[x][r][0] = stream_load4(vb + r * ROWB);
                    b.v[x][r][1] = stream_load4(vb + r * ROWB + 64);
                }
            }
        };

        auto eat = [&](const StepBuf<NGRP> &b, int k) {
            // ---- S^T = K Q^T for the two 16-token tiles
            float s[2][4];
            float lamv[2][4][NGRP], zv[2][4][NGRP];
            float mx = kNegInf;
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                f4_t acc[NGRP];
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) acc[gr] = (f4_t)0.0f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint4 piece = b.k[x][j / 2];
                    const uint32_t w0 = (j % 2) ? piece.z : piece.x, w1 = (j % 2) ? piece.w : piece.y;
                    const h8_t a = pack8(__builtin_amdgcn_perm(0x64646464u, w0, 0x04010400u),
                                         __builtin_amdgcn_perm(0x64646464u, w0, 0x04030402u),
                                         __builtin_amdgcn_perm(0x64646464u, w1, 0x04010400u),
                                         __builtin_amdgcn_perm(0x64646464u, w1, 0x04030402u));
                    f4_t &dst = acc[NGRP == 2 ? j / 2 : 0];
                    dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, qop[j], dst, 0, 0, 0);
                }
                const int tok0 = t0 + k * kStep + x * 16 + g * 4;       // nominal tokens of this lane's 4 rows
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const bool valid = tok0 + r < t1;
                    float sv = 0.0f;
#pragma unroll
                    for (int gr = 0; gr < NGRP; ++gr) {
                        const uint32_t km = meta_of<NGRP>(b.km[x], r, gr);
                        const uint32_t vm = valid ? meta_of<NGRP>(b.vm[x], r, gr) : 0u;
                        const float lam = half_lo(km) * p.scale_log2e;
                        sv += lam * (acc[gr][r] - (1024.0f + half_hi(km)) * qs[gr]);
                        lamv[x][r][gr] = half_lo(vm);
                        zv[x][r][gr] = half_hi(vm);
                    }
                    s[x][r] = valid ? sv : kNegInf;
                    mx = fmaxf(mx, s[x][r]);
                }
            }

            // ---- running maximum per query head, raised lazily; all four quarters hold the same value
            if (__builtin_amdgcn_ballot_w64(mx > m_ref + kLazy) != 0) {
                float mq = fmaxf(mx, __shfl_xor(mx, 16));
                mq = fmaxf(mq, __shfl_xor(mq, 32));
                const float m_new = (mq > m_ref + kLazy) ? mq : m_ref;
                const float f = __builtin_amdgcn_exp2f(m_ref - m_new);
                l_part *= f;
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) z_part[gr] *= f;
                m_ref = m_new;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float fr = __shfl(f, 4 * g + r);          // factor of the query head in row 4g+r
#pragma unroll
                    for (int t = 0; t < 8; ++t) o[t][r] *= fr;
                }
            }

            // ---- weights p * lambda_v as fp16 high + low parts, in the A-operand order (tile, row)
            h8_t a_hi[NGRP], a_lo[NGRP];
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float pj = __builtin_amdgcn_exp2f(s[x][r] - m_ref);
                    l_part += pj;
#pragma unroll
                    for (int gr = 0; gr < NGRP; ++gr) {
                        const float w = pj * lamv[x][r][gr];
                        z_part[gr] = __builtin_fmaf(w, zv[x][r][gr], z_part[gr]);
                        const _Float16 hi = (_Float16)w;
                        const _Float16 lo = (_Float16)(w - (float)hi);
                        a_hi[gr][x * 4 + r] = hi;
                        a_lo[gr][x * 4 + r] = lo;
                    }
                }

            // ---- O += P V: byte nu of the dwords of two tokens -> two fp16 subnormals
#pragma unroll
            for (int set = 0; set < 2; ++set)
#pragma unroll
                for (int nu = 0; nu < 4; ++nu) {
                    const uint32_t sel = 0x0c000c00u | ((4u + nu) << 16) | (uint32_t)nu;
                    const h8_t bv = pack8(__builtin_amdgcn_perm(b.v[0][1][set], b.v[0][0][set], sel),
                                          __builtin_amdgcn_perm(b.v[0][3][set], b.v[0][2][set], sel),
                                          __builtin_amdgcn_perm(b.v[1][1][set], b.v[1][0][set], sel),
                                          __builtin_amdgcn_perm(b.v[1][3][set], b.v[1][2][set], sel));
                    const int gr = NGRP == 2 ? set : 0;
                    f4_t &dst = o[set * 4 + nu];
                    dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_hi[gr], bv, dst, 0, 0, 0);
                    dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_lo[gr], bv, dst, 0, 0, 0);
                }
        };

        {
            StepBuf<NGRP> bufA, bufB;
            issue(bufA, 0);
            for (int k = 0; k < nsteps; k += 2) {
                issue(bufB, k + 1);
                eat(bufA, k);
                issue(bufA, k + 2);
                if (k + 1 < nsteps) eat(bufB, k + 1);
            }
        }

        // ---- per query head: add the four quarters; then fetch the values of this lane's rows
        float l = l_part + __shfl_xor(l_part, 16);
        l += __shfl_xor(l, 32);
        float zsum[NGRP];
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) {
            float v = z_part[gr] + __shfl_xor(z_part[gr], 16);
            v += __shfl_xor(v, 32);
            zsum[gr] = v;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * g + r;                      // query head of the group
            const float l_row = __shfl(l, row);
            const float m_row = __shfl(m_ref, row);
            float z_row[NGRP];
#pragma unroll
            for (int gr = 0; gr < NGRP; ++gr) z_row[gr] = __shfl(zsum[gr], row);
            if (row < qper) {
                const int qh = hk * qper + row;
                if (part < 0) {
                    const float inv_l = 1.0f / l_row;
                    _Float16 *dst = p.out + ((int64_t)i * p.H + qh) * D + 4 * n;
#pragma unroll
                    for (int set = 0; set < 2; ++set) {
                        const float zr = z_row[NGRP == 2 ? set : 0];
                        typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
                        h4_t v;
#pragma unroll
                        for (int nu = 0; nu < 4; ++nu)
                            v[nu] = (_Float16)(__builtin_fmaf(o[set * 4 + nu][r], 16777216.0f, -zr) * inv_l);
                        *reinterpret_cast<h4_t *>(dst + 64 * set) = v;
                    }
                } else {
                    float *dst = p.ws.part + ((int64_t)part * p.H + qh) * (D + 2);
                    if (n == 0) { dst[0] = m_row; dst[1] = l_row; }
#pragma unroll
                    for (int set = 0; set < 2; ++set) {
                        const float zr = z_row[NGRP == 2 ? set : 0];
                        float2 lo2, hi2;
                        lo2.x = __builtin_fmaf(o[set * 4 + 0][r], 16777216.0f, -zr);
                        lo2.y = __builtin_fmaf(o[set * 4 + 1][r], 16777216.0f, -zr);
                        hi2.x = __builtin_fmaf(o[set * 4 + 2][r], 16777216.0f, -zr);
                        hi2.y = __builtin_fmaf(o[set * 4 + 3][r], 16777216.0f, -zr);
                        float *q4 = dst + 2 + 64 * set + 4 * n;
                        *reinterpret_cast<float2 *>(q4) = lo2;
                        *reinterpret_cast<float2 *>(q4 + 2) = hi2;
                    }
                }
            }
        }

        it = qid + nq * __builtin_amdgcn_readfirstlane(ticket);
    }
}

}  // namespace

bool gqa_mfma_applies(const CacheView &c, int32_t H)
{
    const int qper = H / c.Hkv;
    return c.bits == 8 && c.D == 128 && (c.G == 128 || c.G == 64) && c.P >= 16 && qper >= 2 && qper <= 16;
}

hipError_t launch_gqa_mfma(const AttnParams &p, int32_t num_cus, hipStream_t s)
{
    static int occ[2] = {0, 0};
    const int ngrp = p.c.D / p.c.G;
    int &o = occ[ngrp - 1];
    if (o == 0) {
        int n = 0;
        hipError_t oe = ngrp == 1
            ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, decode_attn_gqa_kernel<1>, 256, 0)
            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, decode_attn_gqa_kernel<2>, 256, 0);
        o = (oe == hipSuccess && n > 0) ? n : 2;
    }
    int blocks = num_cus * o;
    const int64_t max_items = (int64_t)p.ws.max_tiles * p.c.Hkv;
    if ((int64_t)blocks * 4 > max_items) blocks = (int)((max_items + 3) / 4);
    if (blocks < 1) blocks = 1;
    if (ngrp == 1)
        hipLaunchKernelGGL((decode_attn_gqa_kernel<1>), dim3(blocks), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL((decode_attn_gqa_kernel<2>), dim3(blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace alise
