// Paged single-query attention over b-bit KV codes for gfx950 (vector-ALU path).
//
// Computes, per request i and query head h (ALISE Sec. 2, Eq. 1-2, over the cache
// of Sec. 3.2):   out = sum_t softmax_t(scale * q . k^_t) v^_t,  t < L_i,
// with k^ = lambda_k (code - z_k), v^ = lambda_v (code - z_v) dequantized in registers.
//
// Work decomposition (this build's, not the paper's):
//   plan kernel   : context_lens -> tile descriptors (request, token range of at most C
//                   tokens), full tiles first, the shorter remainders last
//   attn kernel   : persistent waves, each with a fixed list of (tile, head) items dealt
//                   out from the longest-first order; one wave = one item at a time, no
//                   workgroup barrier anywhere; the stream of loads runs on across items
//   merge kernel  : log-sum-exp combination of the splits of long requests
//
// Inside a wave every load instruction reads 1 KiB of contiguous codes: a token's
// row of D*bits/8 bytes is split over LPT lanes of 16 bytes, so a wave-load covers
// TPW = 64/LPT consecutive tokens ("slots").  When a wave-load never straddles a page
// (TPW <= page size) its base address is wave-uniform and lives in scalar registers.
// Loads are double buffered: the codes of block n+1 are in flight while block n is
// being consumed.  A lane keeps its 16 bytes' worth of channels for both K and V, so
// the scalar product needs a reduction over the LPT lanes of a slot (DPP) and the
// weighted sum needs one reduction over the TPW slots at the end of the tile (LDS).
//
// Dequantization never materialises k^ or v^:
//   q . k^      = lambda_k (sum_c q_c code_c - z_k sum_c q_c)
//   sum_t p_t v^ = sum_t (p_t lambda_v) code  -  sum_t (p_t lambda_v) z_v
// Codes become fp16 by bit tricks, two at a time: for K, 0x6400 | code is 1024 + code
// and feeds the packed fp16 dot product (fp32 accumulate; the 1024 sum(q) offset leaves
// with the zero-point); for V the bare code bits are the fp16 subnormal code * 2^-24,
// which the mixed-precision FMA multiplies by the fp32 weight exactly.
#include "attn_common.h"

#include <atomic>

namespace alise {
namespace {

// (x & mask) | bits in one instruction; the mask sits in a scalar register.
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t bits)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(bits));
    return r;
}

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

// Inclusive scans of two ints per thread over a 1024-thread workgroup, and their totals:
// a shuffle scan inside each wave, then the 16 wave totals through LDS (two barriers).
__device__ __forceinline__ void block_scan2_1024(int a, int b, int32_t (*wave_tot)[16], int &scan_a, int &scan_b,
                                                 int &total_a, int &total_b)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int ua = __shfl_up(a, d), ub = __shfl_up(b, d);
        if (lane >= d) { a += ua; b += ub; }
    }
    if (lane == 63) { wave_tot[0][wave] = a; wave_tot[1][wave] = b; }
    __syncthreads();
    int pa = 0, pb = 0, ta = 0, tb = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int va = wave_tot[0][k], vb = wave_tot[1][k];
        if (k < wave) { pa += va; pb += vb; }
        ta += va; tb += vb;
    }
    __syncthreads();        // wave_tot may be rewritten by the next call
    scan_a = a + pa; scan_b = b + pb;
    total_a = ta; total_b = tb;
}

constexpr int kRemBuckets = 1024;   // remainder tiles are ordered by length through this many buckets

// Bucket of a remainder of r tokens (0 < r < C): longer remainders get lower buckets.
__device__ __forceinline__ int rem_bucket(int r, int C)
{
    return (int)(((uint32_t)(C - r) * (uint32_t)kRemBuckets) / (uint32_t)C);      // in [0, kRemBuckets); C is at most 2^20: no overflow
}

// Tokens of a request cut into splits of C tokens: full splits and the remainder.  The default splits are powers of two
// (log2C >= 0: a shift); a split fixed through the environment may be any multiple of 64 (log2C < 0: a division).
__device__ __forceinline__ void cut(int L, int C, int log2C, int &nfull, int &r)
{
    if (log2C >= 0) {
        nfull = L >> log2C;
        r = L & (C - 1);
    } else {
        nfull = L / C;
        r = L % C;
    }
}
__device__ __forceinline__ int rem_bucket(int r, int C, int log2C)
{
    return log2C >= 0 ? (int)(((uint32_t)(C - r) * (uint32_t)kRemBuckets) >> log2C) : rem_bucket(r, C);
}

// One workgroup.  Per request: number of full tiles (C tokens) and whether a shorter
// remainder tile exists.  Tiles of a request are numbered consecutively (tile_base) for
// the split buffers.  The work order is longest-first: all full tiles, then the remainder
// tiles by decreasing length (a counting sort over length buckets; the order inside a
// bucket is arbitrary), so that the waves that finish last finish on the shortest items.
// Also counts the requests whose splits need merging and zeroes the rows of empty requests.
__global__ __launch_bounds__(1024) void plan_kernel(const int32_t *context_lens, int32_t B, int32_t H,
                                                    int32_t items_per_tile, int32_t max_len, AttnWorkspace ws,
                                                    _Float16 *out, int32_t D, int32_t keep_negative)
{
    __shared__ int32_t s_wave[2][16];
    __shared__ int32_t s_hist[kRemBuckets];
    __shared__ int32_t s_merge;
    __shared__ int32_t s_first_extra;
    const int tid = threadIdx.x;
    s_hist[tid] = 0;            // kRemBuckets == blockDim.x
    if (tid == 0) s_merge = 0;
    __syncthreads();
    // Split length: the largest allowed, halved while the batch would leave the persistent
    // grid with too few items to balance (small batches, or few items per tile).
    int C = ws.chunk_tokens;
    {
        int64_t sum = 0;
        int nonempty = 0;
        for (int i = tid; i < B; i += 1024) {
            int L = context_lens[i];
            L = L < 0 ? 0 : (L > max_len ? max_len : L);
            sum += L;
            nonempty += L > 0;
        }
        // the token total is counted in units of 64 tokens so that it fits an int
        int sa, sb, total64, total_req;
        block_scan2_1024((int)((sum + 63) >> 6), nonempty, s_wave, sa, sb, total64, total_req);
        // ... and only while the tiles of the shorter split (at most tokens / split + one per request) fit the work
        // order and the split buffers, which are sized for the largest split and for small batches.  A split that may
        // be halved is a power of two (2048, or the page window): the quotients are shifts of the token total.
        int sh = 31 - __builtin_clz(C) - 6;             // tokens / C == total64 >> sh
        while (C > ws.min_chunk_tokens && (int64_t)((total64 >> sh) + total_req) * items_per_tile < ws.min_items &&
               (total64 >> (sh - 1)) + total_req <= ws.max_tiles) {
            C >>= 1;
            --sh;
        }
    }
    const int log2C = (C & (C - 1)) == 0 ? 31 - __builtin_clz(C) : -1;
    int total = 0, total_full = 0;
    int my_L = 0, my_tb = 0, my_fb = 0;     // with B <= 1024 a thread has one request and keeps what it computed for it
    for (int base = 0; base < B; base += 1024) {
        const int i = base + tid;
        int L = 0;
        bool no_request = false;    // a row that is nobody's: not even a zero row is written
        if (i < B) {
            L = context_lens[i];
            no_request = keep_negative && L < 0;
            L = L < 0 ? 0 : (L > max_len ? max_len : L);
        }
        int nfull, r;
        cut(L, C, log2C, nfull, r);
        const int nrem = r != 0;
        int s_all, s_full, t_all, t_full;
        block_scan2_1024(nfull + nrem, nfull, s_wave, s_all, s_full, t_all, t_full);
        if (i < B) {
            my_L = L;
            my_tb = total + s_all - (nfull + nrem);
            my_fb = total_full + s_full - nfull;
            ws.tile_base[i] = my_tb;
            if (B > 1024) ws.req_full_base[i] = my_fb;
            if (nrem) atomicAdd(&s_hist[rem_bucket(r, C, log2C)], 1);
            if (nfull + nrem > 1) atomicAdd(&s_merge, 1);
            if (L == 0 && out && !no_request)           // out == nullptr: a plan made ahead of the calls that use it; they zero these rows
                for (int e = 0; e < H * D; ++e) out[(int64_t)i * H * D + e] = (_Float16)0.0f;
        }
        total += t_all;
        total_full += t_full;
    }
    __syncthreads();            // the histogram is complete
    // exclusive scan of the bucket counts -> first position of each bucket among the remainders
    {
        const int my_count = s_hist[tid];
        // cost of this bucket's tiles in units of 64 tokens: their length (the bucket's upper end) plus what starting
        // and ending an item costs a wave (about 128 tokens' worth)
        const int my_cost = (int)(((int64_t)my_count * (C - ((tid * C) >> 10) + 128)) >> 6);      // kRemBuckets is 1024, C at most 2^20
        int incl, cost_incl, t0, cost_rem;
        block_scan2_1024(my_count, my_cost, s_wave, incl, cost_incl, t0, cost_rem);
        s_hist[tid] = incl - my_count;
        // The shortest tiles, worth ws.skew_permille thousandths of the whole work, are dealt out among the favoured
        // half of the waves only (see the attention kernel): they start at the first bucket whose tiles, with all
        // shorter ones, fit that share.
        if (tid == 0) s_first_extra = total;
        __syncthreads();
        const float cost_all = (float)total_full * (float)(C + 128) * (1.0f / 64.0f) + (float)cost_rem;
        const float share = cost_all * (float)ws.skew_permille * 1.0e-3f;
        const float with_shorter = (float)(cost_rem - (cost_incl - my_cost));
        // only where a wave has enough items for such a shift to be fine-grained: with two or three items per wave it
        // unbalances more than it repairs (measured: +4 % on a 64-request batch)
        const bool many_items = (int64_t)total * items_per_tile >= 3 * (int64_t)ws.min_items;
        if (many_items && my_count > 0 && with_shorter <= share) atomicMin(&s_first_extra, total_full + incl - my_count);
        __syncthreads();
    }
    // The buffers hold max_tiles tiles: enough for every batch whose lengths add up to no more than the cache's
    // capacity.  A batch beyond that (requests that share pages) gets no work at all rather than writes past the end.
    const bool fits = total <= ws.max_tiles;
    for (int i = tid; fits && i < B; i += 1024) {
        int L = my_L, tb = my_tb, fb = my_fb;
        if (B > 1024) {
            L = context_lens[i];
            L = L < 0 ? 0 : (L > max_len ? max_len : L);
            tb = ws.tile_base[i];
            fb = ws.req_full_base[i];
        }
        int nfull, r;
        cut(L, C, log2C, nfull, r);
        const bool split = nfull + (r != 0) > 1;
        for (int s = 0; s < nfull; ++s)
            ws.order[fb + s] = make_int4(i, s * C, (s + 1) * C, split ? tb + s : -1);
        if (r) {
            const int pos = atomicAdd(&s_hist[rem_bucket(r, C, log2C)], 1);
            ws.order[total_full + pos] = make_int4(i, nfull * C, L, split ? tb + nfull : -1);
        }
    }
    if (tid == 0) {
        ws.tile_base[B] = total;
        *ws.n_items = fits ? total * items_per_tile : 0;
        *ws.n_shared = fits ? s_first_extra * items_per_tile : 0;
        *ws.n_merge = fits ? s_merge : 0;
    }
}

// ------------------------------------------------------------------ attention

// Stores of the end of a tile, written in assembly so that the compiler does not count them.
// A store may complete out of order with the loads, so with a store in flight the compiler's
// next wait for a load becomes "wait for everything", which drained the double buffer once
// per item.  Not counting a store only makes the compiler's waits for loads longer than
// needed by at most that store, never shorter: loads still complete in issue order.
__device__ __forceinline__ void stream_store_f32(float *p, float v)
{
    asm volatile("global_store_dword %0, %1, off" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store_f16(_Float16 *p, _Float16 v)
{
    const uint32_t u = __builtin_bit_cast(uint16_t, v);
    asm volatile("global_store_short %0, %1, off" : : "v"(p), "v"(u) : "memory");
}


template <int BITS, int D>
struct Geo {
    static constexpr int ROWB = D * BITS / 8;   // code bytes of one token's row
    static constexpr int LPT = ROWB / 16;       // lanes per token
    static constexpr int TPW = 64 / LPT;        // tokens per wave-load
    static constexpr int SL = 128 / BITS;       // channels per lane
    static constexpr int LDS_ROW = D + 4;       // floats per slot row in the end-of-tile reduction
};

// The codes and meta of N wave-loads, as they arrive.
template <int N>
struct Buf {
    uint4 kc[N], vc[N];
    uint32_t km[N], vm[N];
};

// Running softmax state of one lane: its slot's reference maximum and denominator, the
// weighted code sums of its SL channels, and the weighted zero-point sum.
template <int SL>
struct Acc {
    float m_ref, l, wz;
    float a[SL];
};

// This lane's slice of q, paired the way the code pairs come out of a dword.
template <int BITS>
struct QSlice {
    uint32_t qp[64 / BITS];   // SL / 2 packed fp16 pairs
    float qsum;               // sum of q over the slice
    float koff;               // what the 1024 offsets add to the packed dot product
};

template <int BITS, int D>
__device__ __forceinline__ void make_q(QSlice<BITS> &qs, const uint32_t (&raw)[Geo<BITS, D>::SL / 2])
{
    constexpr int SL = Geo<BITS, D>::SL;
    if constexpr (BITS == 8) {
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < SL / 2; ++k) {
            qs.qp[k] = raw[k];
            s += half_lo(raw[k]) + half_hi(raw[k]);
        }
        qs.qsum = s;
        qs.koff = 1024.0f * s;
    } else {
        // a code dword holds channels 8w..8w+7 in nibbles 0..7; the pairs taken from it are
        // (n0,n4) (n1,n5)*16 (n2,n6) (n3,n7)*16, so q is paired the same way and the
        // partners of the *16 pairs are pre-divided by 16 (exact in fp16 above the subnormals).
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
            const h2_t a0 = {qc[0], qc[4]}, b0 = {qc[1] * sc, qc[5] * sc};
            const h2_t a1 = {qc[2], qc[6]}, b1 = {qc[3] * sc, qc[7] * sc};
            qs.qp[4 * w + 0] = as_u32(a0); qs.qp[4 * w + 1] = as_u32(b0);
            qs.qp[4 * w + 2] = as_u32(a1); qs.qp[4 * w + 3] = as_u32(b1);
            sa += (float)a0.x + (float)a0.y + (float)a1.x + (float)a1.y;
            sb += (float)b0.x + (float)b0.y + (float)b1.x + (float)b1.y;   // already /16
        }
        qs.qsum = sa + 16.0f * sb;
        qs.koff = 1024.0f * (sa + sb);
    }
}

// One wave-load: score of this lane's token, lazy maximum, weight, weighted code sums.
// `valid` is false for a token at or beyond the end of the tile (its slot may hold
// anything, NaN meta included: selected away, never multiplied by zero).
template <int BITS, int D>
__device__ __forceinline__ void consume_one(const uint4 kc, const uint4 vc, const uint32_t km, uint32_t vm,
                                            Acc<Geo<BITS, D>::SL> &st, const QSlice<BITS> &qs,
                                            float scale_log2e, bool valid)
{
    using G = Geo<BITS, D>;
    constexpr int LPT = G::LPT, SL = G::SL;
    const uint32_t kw[4] = {kc.x, kc.y, kc.z, kc.w};
    float dot = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if constexpr (BITS == 8) {
            const uint32_t lo = __builtin_amdgcn_perm(0x64646464u, kw[w], 0x04010400u);
            const uint32_t hi = __builtin_amdgcn_perm(0x64646464u, kw[w], 0x04030402u);
            dot = __builtin_amdgcn_fdot2(as_h2(lo), as_h2(qs.qp[2 * w]), dot, false);
            dot = __builtin_amdgcn_fdot2(as_h2(hi), as_h2(qs.qp[2 * w + 1]), dot, false);
        } else {
            const uint32_t x = kw[w], y = kw[w] >> 8;
            const uint32_t a0 = and_or(x, 0x000F000Fu, 0x64006400u);
            const uint32_t b0 = and_or(x, 0x00F000F0u, 0x64006400u);
            const uint32_t a1 = and_or(y, 0x000F000Fu, 0x64006400u);
            const uint32_t b1 = and_or(y, 0x00F000F0u, 0x64006400u);
            dot = __builtin_amdgcn_fdot2(as_h2(a0), as_h2(qs.qp[4 * w + 0]), dot, false);
            dot = __builtin_amdgcn_fdot2(as_h2(b0), as_h2(qs.qp[4 * w + 1]), dot, false);
            dot = __builtin_amdgcn_fdot2(as_h2(a1), as_h2(qs.qp[4 * w + 2]), dot, false);
            dot = __builtin_amdgcn_fdot2(as_h2(b1), as_h2(qs.qp[4 * w + 3]), dot, false);
        }
    }
    const float lam = half_lo(km) * scale_log2e;
    const float z = half_hi(km);
    float part = lam * ((dot - qs.koff) - z * qs.qsum);
    part = slot_sum<LPT>(part);
    const float s = valid ? part : kNegInf;
    vm = valid ? vm : 0u;                 // scale 0, zero-point 0: the token adds nothing

    // running maximum, raised lazily (wave-uniform branch, rarely taken after the first tokens)
    if (__builtin_amdgcn_ballot_w64(s > st.m_ref + kLazy) != 0) {
        const float m_new = (s > st.m_ref + kLazy) ? s : st.m_ref;
        const float f = __builtin_amdgcn_exp2f(st.m_ref - m_new);     // 1 where unchanged
        st.l *= f;
        st.wz *= f;
#pragma unroll
        for (int k = 0; k < SL; ++k) st.a[k] *= f;
        st.m_ref = m_new;
    }

    const float pj = __builtin_amdgcn_exp2f(s - st.m_ref);            // 0 for a masked token
    st.l += pj;
    const float w = pj * half_lo(vm);
    st.wz = __builtin_fmaf(w, half_hi(vm), st.wz);
    const uint32_t vw[4] = {vc.x, vc.y, vc.z, vc.w};
    if constexpr (BITS == 8) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            // bytes -> fp16 subnormals code * 2^-24 (high byte zero)
            const h2_t lo = as_h2(__builtin_amdgcn_perm(0u, vw[d], 0x0c010c00u));
            const h2_t hi = as_h2(__builtin_amdgcn_perm(0u, vw[d], 0x0c030c02u));
            st.a[4 * d + 0] = __builtin_fmaf((float)lo.x, w, st.a[4 * d + 0]);
            st.a[4 * d + 1] = __builtin_fmaf((float)lo.y, w, st.a[4 * d + 1]);
            st.a[4 * d + 2] = __builtin_fmaf((float)hi.x, w, st.a[4 * d + 2]);
            st.a[4 * d + 3] = __builtin_fmaf((float)hi.y, w, st.a[4 * d + 3]);
        }
    } else {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t x = vw[d], y = vw[d] >> 8;
            const h2_t a0 = as_h2(x & 0x000F000Fu);      // (n0, n4)      * 2^-24
            const h2_t b0 = as_h2(x & 0x00F000F0u);      // (n1, n5) * 16 * 2^-24
            const h2_t a1 = as_h2(y & 0x000F000Fu);      // (n2, n6)
            const h2_t b1 = as_h2(y & 0x00F000F0u);      // (n3, n7) * 16
            st.a[8 * d + 0] = __builtin_fmaf((float)a0.x, w, st.a[8 * d + 0]);
            st.a[8 * d + 1] = __builtin_fmaf((float)a0.y, w, st.a[8 * d + 1]);
            st.a[8 * d + 2] = __builtin_fmaf((float)b0.x, w, st.a[8 * d + 2]);
            st.a[8 * d + 3] = __builtin_fmaf((float)b0.y, w, st.a[8 * d + 3]);
            st.a[8 * d + 4] = __builtin_fmaf((float)a1.x, w, st.a[8 * d + 4]);
            st.a[8 * d + 5] = __builtin_fmaf((float)a1.y, w, st.a[8 * d + 5]);
            st.a[8 * d + 6] = __builtin_fmaf((float)b1.x, w, st.a[8 * d + 6]);
            st.a[8 * d + 7] = __builtin_fmaf((float)b1.y, w, st.a[8 * d + 7]);
        }
    }
}

// The block-table entries of a tile's pages: entry win_first + lane in `lo`, win_first + 64 + lane in `hi`.
struct PageWindow {
    int lo, hi;
};

// One work item: a tile (request, token range) for one query head.  Everything is
// wave-uniform except `pg`, which holds the tile's block-table entries, one per lane.
struct TileCtx {
    int valid;          // item index below n_items
    int i, h, hk;       // request, query head, KV head
    int t0, t1;         // token range
    int part;           // split buffer index, or -1: the tile is the whole request
    int nw, nblk;       // wave-loads, blocks
    int win_first;      // first page index of the tile
};

// NB = wave-loads per block; two blocks are in flight per wave.
//
// The kernel is one continuous stream of blocks: the last load slot of a tile already
// fetches the first block of the wave's next tile, and what a tile needs besides the cache
// is there before it starts: its q is fetched at the start of the tile before it, its
// block-table entries (pg) at the end of the tile before it, its descriptor through the
// scalar unit.  Nothing at a tile boundary waits for the vector loads in flight.
template <int BITS, int D, bool UNI, int NB>
__global__ __launch_bounds__(256) void decode_attn_kernel(AttnParams p)
{
    using G = Geo<BITS, D>;
    constexpr int LPT = G::LPT, TPW = G::TPW, SL = G::SL, ROWB = G::ROWB;
    constexpr int BT = NB * TPW;      // tokens per block
    __shared__ float s_red[4][TPW * G::LDS_ROW];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int sub = lane % LPT;         // which 16-byte slice of the row
    const int slot = lane / LPT;        // which token of a wave-load
    const int ch0 = sub * SL;           // first channel of this lane
    const int grp = ch0 / p.c.G;        // the lane's channels lie in one group
    const int NG = p.c.NG, logP = p.c.logP, P = p.c.P, Hkv = p.c.Hkv;
    // per-lane addresses of the first (page, head) block; == slot * ROWB + sub * 16 == lane * 16
    const uint8_t *lane_k = p.c.k_codes + lane * 16;
    const uint8_t *lane_v = p.c.v_codes + lane * 16;
    const uint8_t *lane_km = reinterpret_cast<const uint8_t *>(p.c.k_meta) + (slot * NG + grp) * 4;
    const uint8_t *lane_vm = reinterpret_cast<const uint8_t *>(p.c.v_meta) + (slot * NG + grp) * 4;
    float *red = s_red[wave];
    const int n_items = *p.ws.n_items;
    const int4 *order = p.ws.order;

    // A wave owns a fixed list of items, dealt out by rank in the longest-first order: round r
    // gives wave w item r * W + w, odd rounds in reverse wave order.  That evens out the totals
    // to a few per cent (2 % on the Zipf lengths of the large INT4 batch), and it needs no counter: a ticket fetched with an atomic
    // returns into a register, and waiting for it drained the wave's load pipeline once per
    // item (the whole grid must be resident, which the occupancy-sized launch guarantees).
    const int W = gridDim.x * 4, w_id = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + wave);
    auto item_at = [&](int r) { return r * W + ((r & 1) ? W - 1 - w_id : w_id); };
    // The shortest items (from n_shared on) go to the favoured half of the waves only.  Workgroups are handed to the
    // chip's eight XCDs in turn, and on this chip the even ones get through the same work about 7 % sooner than the
    // odd ones (a timestamp per wave: 1517-1539 us against 1626-1645 us on equal lists, on two machines), so the waves
    // of even workgroups take that much more.
    const int n_shared = min(*p.ws.n_shared, n_items);
    const int shared_rounds = n_shared / W, shared_tail = n_shared - shared_rounds * W;
    const int n_mine = shared_rounds + ((((shared_rounds & 1) ? W - 1 - w_id : w_id) < shared_tail) ? 1 : 0);
    const bool favoured = ((blockIdx.x & 1) == 0) && gridDim.x > 1;
    const int W2 = ((gridDim.x + 1) >> 1) * 4, w2 = (blockIdx.x >> 1) * 4 + (w_id & 3);
    auto item_seq = [&](int k) {                // the k-th item of this wave; n_items: none
        if (k < n_mine) return item_at(k);
        const int r = k - n_mine;
        const int it = n_shared + r * W2 + ((r & 1) ? W2 - 1 - w2 : w2);
        return (favoured && it < n_items) ? it : n_items;
    };
    // The descriptor of an item comes through the scalar unit, at the moment it is needed: a
    // scalar load is counted apart from the vector loads, so waiting for it leaves the wave's
    // prefetched blocks in flight (a vector load here made the compiler wait for all of them).
    auto desc_of = [&](int it) {
        typedef int32_t i32x4_t __attribute__((ext_vector_type(4)));
        const int4 *src = order + (it < n_items ? it : 0) / p.H;
        i32x4_t d;
        asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(d) : "s"(src) : "memory");
        return make_int4(d.x, d.y, d.z, d.w);
    };
    auto make_ctx = [&](int it, const int4 d) {
        TileCtx c;
        c.valid = it < n_items;
        c.h = (it < n_items ? it : 0) % p.H;
        c.hk = c.h / p.qper;
        c.i = __builtin_amdgcn_readfirstlane(d.x);
        c.t0 = __builtin_amdgcn_readfirstlane(d.y);
        c.t1 = __builtin_amdgcn_readfirstlane(d.z);
        c.part = __builtin_amdgcn_readfirstlane(d.w);
        c.nw = (c.t1 - c.t0 + TPW - 1) / TPW;
        c.nblk = (c.nw + NB - 1) / NB;
        c.win_first = c.t0 >> logP;
        return c;
    };
    // a tile spans at most 128 pages, so two entries per lane cover it
    auto load_pg = [&](const TileCtx &c) {
        const int32_t *bt = p.block_tables + (int64_t)c.i * p.max_blocks;
        const int last = (c.t1 - 1) >> logP;
        PageWindow w;
        w.lo = bt[min(c.win_first + lane, last)];
        w.hi = bt[min(c.win_first + 64 + lane, last)];
        return w;
    };
    auto load_q_raw = [&](const TileCtx &c, uint32_t (&raw)[SL / 2]) {
        const uint32_t *qsrc = reinterpret_cast<const uint32_t *>(p.q + ((int64_t)c.i * p.H + c.h) * D + ch0);
#pragma unroll
        for (int k = 0; k < SL / 2; k += 4) {
            const uint4 v4 = *reinterpret_cast<const uint4 *>(qsrc + k);
            raw[k] = v4.x; raw[k + 1] = v4.y; raw[k + 2] = v4.z; raw[k + 3] = v4.w;
        }
    };

    // Issue the NB wave-loads of block k of tile c.  Straight-line code on purpose: a branch
    // around a load would make the compiler wait for every outstanding load at the join,
    // which serialises the two buffers.  Wave-loads past the end of the tile re-read its
    // last wave-load; their tokens are masked when consumed.
    auto issue = [&](Buf<NB> &buf, const TileCtx &c, const PageWindow &pg, int k) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int w = min(k * NB + j, c.nw - 1);
            const int tw = c.t0 + w * TPW;
            if constexpr (UNI) {
                const int idx = (tw >> logP) - c.win_first;             // wave-uniform, 0 .. 127
                const int e_lo = __builtin_amdgcn_readlane(pg.lo, idx & 63), e_hi = __builtin_amdgcn_readlane(pg.hi, idx & 63);
                const int page = idx < 64 ? e_lo : e_hi;
                const int blk = page * Hkv + c.hk;                    // < 2^31, checked on the host
                const int off = tw & (P - 1);
                const int64_t co = (int64_t)blk * p.c.cstride + off * ROWB;
                const int64_t mo = (int64_t)blk * p.c.mstride + off * NG * 4;
                buf.kc[j] = stream_load16(lane_k + co);
                buf.vc[j] = stream_load16(lane_v + co);
                buf.km[j] = stream_load4(lane_km + mo);
                buf.vm[j] = stream_load4(lane_vm + mo);
            } else {
                const int tok = tw + slot;
                const int tc = tok < c.t1 ? tok : c.t1 - 1;        // stay on a real token
                const int idx = (tc >> logP) - c.win_first;
                const int e_lo = __shfl(pg.lo, idx & 63), e_hi = __shfl(pg.hi, idx & 63);
                const int page = idx < 64 ? e_lo : e_hi;
                const int blk = page * Hkv + c.hk;
                const int off = tc & (P - 1);
                const int64_t co = (int64_t)blk * p.c.cstride + off * ROWB + sub * 16;
                const int64_t mo = (int64_t)blk * p.c.mstride + (off * NG + grp) * 4;
                buf.kc[j] = stream_load16(p.c.k_codes + co);
                buf.vc[j] = stream_load16(p.c.v_codes + co);
                buf.km[j] = stream_load4(reinterpret_cast<const uint8_t *>(p.c.k_meta) + mo);
                buf.vm[j] = stream_load4(reinterpret_cast<const uint8_t *>(p.c.v_meta) + mo);
            }
        }
    };

    // The issue arbiter of a SIMD prefers its oldest wave, and the memory system serves whoever asks first: left
    // alone, the three waves of a SIMD get through equal lists in about 57 %, 79 % and 100 % of the kernel's time
    // (measured with a timestamp per wave), and the last fifth of the kernel runs with one wave per SIMD, too few
    // to keep the memory system busy.  So a wave lowers its own priority by one step with every 256 tokens it has
    // done, wrapping around after four steps: of two waves the one that is behind has the higher priority (except
    // just after the one ahead has wrapped), which keeps the waves of a SIMD within a few hundred tokens of each
    // other -- they finish within 10 % of the kernel's time of each other instead of 43 %.
    int done_tokens = 0, prio_bin = 0;
    __builtin_amdgcn_s_setprio(3);
    auto step_priority = [&]() {
        const int bin = done_tokens >> 8;
        if (bin != prio_bin) {                  // wave-uniform; no memory operation inside
            prio_bin = bin;
            switch (bin & 3) {
            case 0: __builtin_amdgcn_s_setprio(3); break;
            case 1: __builtin_amdgcn_s_setprio(2); break;
            case 2: __builtin_amdgcn_s_setprio(1); break;
            default: __builtin_amdgcn_s_setprio(0); break;
            }
        }
    };
    // ---- fill the pipeline
    int round = 0;
    const int it0 = item_seq(0), it1 = item_seq(1);
    TileCtx cur = make_ctx(it0, desc_of(it0));
    if (!cur.valid) return;                     // wave-uniform
    TileCtx nxt = make_ctx(it1, desc_of(it1));
    PageWindow pg_cur = load_pg(cur);
    PageWindow pg_nxt = load_pg(nxt);
    uint32_t qraw[SL / 2];
    load_q_raw(cur, qraw);
    Buf<NB> bufA, bufB;
    issue(bufA, cur, pg_cur, 0);

    for (;;) {
        QSlice<BITS> qs;
        make_q<BITS, D>(qs, qraw);
        // the next tile's q travels during this whole tile, so nothing waits for it later
        load_q_raw(nxt.valid ? nxt : cur, qraw);

        Acc<SL> st;
        st.m_ref = kFloor; st.l = 0.0f; st.wz = 0.0f;
#pragma unroll
        for (int k = 0; k < SL; ++k) st.a[k] = 0.0f;

        auto eat = [&](const Buf<NB> &buf, int k) {
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const bool valid = cur.t0 + k * BT + j * TPW + slot < cur.t1;
                consume_one<BITS, D>(buf.kc[j], buf.vc[j], buf.km[j], buf.vm[j], st, qs, p.scale_log2e, valid);
            }
        };

        // bufA holds block 0 of the tile (in flight).  The slot after the tile's last block
        // fetches block 0 of the next tile, so bufA is ready for it when this tile is done.
        const int nblk = cur.nblk;
        // A tile has at least one block, and the loop says so (do-while): the compiler sizes
        // its waits for the loads issued an item ago (descriptor, page ids, q) by the fewest
        // loads that can follow them, and a loop that might not run counts as none, which
        // turned those waits into "wait for the prefetched block as well".
        int k = 0;
        do {
            issue(bufB, cur, pg_cur, min(k + 1, nblk - 1));
            eat(bufA, k);
            const bool hop = (k + 2 >= nblk) && nxt.valid;      // wave-uniform
            TileCtx src = cur;
            if (hop) src = nxt;
            issue(bufA, src, hop ? pg_nxt : pg_cur, hop ? 0 : min(k + 2, nblk - 1));
            if (k + 1 < nblk) eat(bufB, k + 1);
            k += 2;
            done_tokens += 2 * BT;
            step_priority();
        } while (k < nblk);

        // ---- bring the TPW slots to one maximum, then add them up through LDS
        float m_fin = st.m_ref;
#pragma unroll
        for (int d = LPT; d < 64; d <<= 1) m_fin = fmaxf(m_fin, __shfl_xor(m_fin, d));
        const float f = __builtin_amdgcn_exp2f(st.m_ref - m_fin);     // 0 for a slot that saw no token
        float l = st.l * f;
#pragma unroll
        for (int d = LPT; d < 64; d <<= 1) l += __shfl_xor(l, d);
        float *myrow = red + slot * G::LDS_ROW + ch0;
        const float fz = st.wz * f;
        const float f24 = f * 16777216.0f;      // undo the 2^-24 of the subnormal codes
        if constexpr (BITS == 8) {
#pragma unroll
            for (int k = 0; k < SL; ++k) myrow[k] = __builtin_fmaf(st.a[k], f24, -fz);
        } else {
            const float f20 = f * 1048576.0f;   // ... and the extra *16 of the odd nibbles
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                myrow[8 * d + 0] = __builtin_fmaf(st.a[8 * d + 0], f24, -fz);
                myrow[8 * d + 4] = __builtin_fmaf(st.a[8 * d + 1], f24, -fz);
                myrow[8 * d + 1] = __builtin_fmaf(st.a[8 * d + 2], f20, -fz);
                myrow[8 * d + 5] = __builtin_fmaf(st.a[8 * d + 3], f20, -fz);
                myrow[8 * d + 2] = __builtin_fmaf(st.a[8 * d + 4], f24, -fz);
                myrow[8 * d + 6] = __builtin_fmaf(st.a[8 * d + 5], f24, -fz);
                myrow[8 * d + 3] = __builtin_fmaf(st.a[8 * d + 6], f20, -fz);
                myrow[8 * d + 7] = __builtin_fmaf(st.a[8 * d + 7], f20, -fz);
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

        if (cur.part < 0) {
            const float inv_l = 1.0f / l;
            _Float16 *dst = p.out + ((int64_t)cur.i * p.H + cur.h) * D;
#pragma unroll
            for (int r = 0; r < D / 64; ++r) stream_store_f16(dst + r * 64 + lane, (_Float16)(o[r] * inv_l));
        } else {
            float *dst = p.ws.part + ((int64_t)cur.part * p.H + cur.h) * (D + 2);
            if (lane == 0) { stream_store_f32(dst, m_fin); stream_store_f32(dst + 1, l); }
#pragma unroll
            for (int r = 0; r < D / 64; ++r) stream_store_f32(dst + 2 + r * 64 + lane, o[r]);
        }

        // ---- advance the pipeline (loads below are unconditional; indices are clamped)
        if (!nxt.valid) break;                  // wave-uniform; nothing is in flight that matters
        cur = nxt;
        pg_cur = pg_nxt;
        ++round;
        const int it_nxt = item_seq(round + 1);
        nxt = make_ctx(it_nxt, desc_of(it_nxt));
        pg_nxt = load_pg(nxt);
    }
}

// ------------------------------------------------------------------ merge

// Log-sum-exp combination of the splits of every request that has more than one; a
// fixed grid of waves strides over all (request, head) pairs.  Lane c reads the (m, l)
// header of split c, so the maximum and the denominator are two wave reductions, and the
// weighted rows are then fetched with independent loads.
template <int D>
__global__ __launch_bounds__(256) void merge_kernel(AttnParams p)
{
    const int lane = threadIdx.x & 63;
    const int n_waves = gridDim.x * 4;
    if (p.zero_empty) {                     // the plan was made without an output to write to: empty requests give zero rows
        for (int pair = blockIdx.x * 4 + (threadIdx.x >> 6); pair < p.B * p.H; pair += n_waves)
            if (p.context_lens[pair / p.H] <= 0) {
                _Float16 *dst = p.out + (int64_t)pair * D;
#pragma unroll
                for (int r = 0; r < D / 64; ++r) dst[r * 64 + lane] = (_Float16)0.0f;
            }
    }
    // Every (request, head) pair looks up its own splits: the pair's first load does not wait for a list of the requests
    // that need merging (the count of that list only says whether there is anything to merge at all -- it is 0 too for a
    // batch that did not fit the workspace and got no work).
    const int n_merge = *p.ws.n_merge;
    for (int pair = blockIdx.x * 4 + (threadIdx.x >> 6); pair < p.B * p.H; pair += n_waves) {
        const int i = pair / p.H, h = pair - i * p.H;
        const int first = p.ws.tile_base[i];
        const int n = p.ws.tile_base[i + 1] - first;
        if (n_merge == 0 || n < 2) continue;
        const float *part = p.ws.part + ((int64_t)first * p.H + h) * (D + 2);
        const int64_t stride = (int64_t)p.H * (D + 2);
        float m = kNegInf, l = 0.0f, o[D / 64];
#pragma unroll
        for (int r = 0; r < D / 64; ++r) o[r] = 0.0f;
        for (int c0 = 0; c0 < n; c0 += 64) {            // 64 splits at a time
            const int nc = min(64, n - c0);
            const float *pc = part + (c0 + min(lane, nc - 1)) * stride;
            const float mc = lane < nc ? pc[0] : kNegInf;
            const float lc = lane < nc ? pc[1] : 0.0f;
            float m_new = mc;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) m_new = fmaxf(m_new, __shfl_xor(m_new, d));
            m_new = fmaxf(m_new, m);
            const float fc = __builtin_amdgcn_exp2f(mc - m_new);        // weight of split c0 + lane
            const float fo = __builtin_amdgcn_exp2f(m - m_new);         // rescale what was merged before
            float lsum = lc * fc;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) lsum += __shfl_xor(lsum, d);
            l = l * fo + lsum;
#pragma unroll
            for (int r = 0; r < D / 64; ++r) o[r] *= fo;
            for (int c = 0; c < nc; ++c) {
                const float f = __shfl(fc, c);
                const float *row = part + (c0 + c) * stride + 2;
#pragma unroll
                for (int r = 0; r < D / 64; ++r) o[r] = __builtin_fmaf(row[r * 64 + lane], f, o[r]);
            }
            m = m_new;
        }
        const float inv_l = 1.0f / l;
        _Float16 *dst = p.out + ((int64_t)i * p.H + h) * D;
#pragma unroll
        for (int r = 0; r < D / 64; ++r) dst[r * 64 + lane] = (_Float16)(o[r] * inv_l);
    }
}

template <int BITS, int D, int NB>
hipError_t launch_t(const AttnParams &p, int32_t num_cus, int32_t waves_per_cu, hipStream_t s)
{
    // a wave-load covers TPW consecutive tokens; it has one page if pages are at least that long
    const bool uniform_page = p.c.P >= Geo<BITS, D>::TPW;
    // The grid is persistent: as many workgroups as the kernel's registers and LDS let the
    // chip hold at once (asked once per kernel variant), unless the caller fixes the number.
    // (two threads that ask at the same time store the same number)
    static std::atomic<int> resident_wgs_per_cu[2];
    int occ = resident_wgs_per_cu[uniform_page ? 1 : 0].load(std::memory_order_relaxed);
    if (occ == 0) {
        int n = 0;
        hipError_t oe = uniform_page
            ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, decode_attn_kernel<BITS, D, true, NB>, 256, 0)
            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, decode_attn_kernel<BITS, D, false, NB>, 256, 0);
        occ = (oe == hipSuccess && n > 0) ? n : 2;
        resident_wgs_per_cu[uniform_page ? 1 : 0].store(occ, std::memory_order_relaxed);
    }
    // three workgroups (twelve waves) per compute unit saturate the memory system; a fourth one, where the registers
    // allow it (INT8), only spreads the same work over more lists (llama7b: 307 us with three, 313 us with four)
    int blocks = num_cus * (waves_per_cu > 0 ? waves_per_cu / 4 : (occ < 3 ? occ : 3));
    const int64_t max_items = (int64_t)p.ws.max_tiles * p.H;
    if ((int64_t)blocks * 4 > max_items) blocks = (int)((max_items + 3) / 4);
    if (blocks < 1) blocks = 1;
    if (uniform_page)
        hipLaunchKernelGGL((decode_attn_kernel<BITS, D, true, NB>), dim3(blocks), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL((decode_attn_kernel<BITS, D, false, NB>), dim3(blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_merge(const AttnParams &p, hipStream_t s)
{
    int mblocks = (p.B * p.H + 3) / 4;
    if (mblocks > 1024) mblocks = 1024;
    if (p.c.D == 128)
        hipLaunchKernelGGL((merge_kernel<128>), dim3(mblocks), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL((merge_kernel<64>), dim3(mblocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace

namespace {

// One wave per query row t: the length and the block-table row of the single-query request that stands for it.  The
// row's request is found by bisection in q_start, so every row gets a defined entry whatever q_start holds: a length
// in [1, L] with the entries that length reaches, or -1 (a row that no chunk owns, or one beyond a chunk cut short).
__global__ __launch_bounds__(256) void prefill_expand_kernel(const int32_t *q_start, const int32_t *block_tables, int32_t max_blocks,
                                                             const int32_t *context_lens, int32_t B, int32_t total_q, int32_t max_len,
                                                             int32_t logP, int32_t *lens, int32_t *tables, int32_t blocks_per_row)
{
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= total_q) return;
    int len = -1, i = 0;
    if (t < q_start[B]) {
        int lo = 0, hi = B;                 // the last request whose first row is at or before t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (q_start[mid] <= t) lo = mid; else hi = mid;
        }
        i = lo;
        const int L = min(max(context_lens[i], 0), max_len);
        const int n = min(max(q_start[i + 1] - q_start[i], 0), L);         // a chunk cannot be longer than its request
        const int j = t - q_start[i];
        if (j >= 0 && j < n) len = L - n + j + 1;
    }
    if (len > 0) {
        const int nblk = min(min((len + (1 << logP) - 1) >> logP, blocks_per_row), max_blocks);
        const int32_t *row = block_tables + (int64_t)i * max_blocks;
        int32_t *dst = tables + (int64_t)t * blocks_per_row;
        for (int b = lane; b < nblk; b += 64) dst[b] = row[b];
    }
    if (lane == 0) lens[t] = len;
}

}  // namespace

hipError_t launch_prefill_expand(const CacheView &c, const int32_t *q_start, const int32_t *block_tables, int32_t max_blocks,
                                 const int32_t *context_lens, int32_t B, int32_t total_q, int32_t max_context_len,
                                 int32_t *lens, int32_t *tables, int32_t blocks_per_row, hipStream_t s)
{
    hipLaunchKernelGGL(prefill_expand_kernel, dim3((total_q + 3) / 4), dim3(256), 0, s, q_start, block_tables, max_blocks, context_lens, B,
                       total_q, max_context_len, c.logP, lens, tables, blocks_per_row);
    return hipGetLastError();
}

hipError_t launch_decode_attn(const CacheView &c, const void *q, void *out,
                              const int32_t *block_tables, int32_t max_blocks,
                              const int32_t *context_lens, int32_t B, int32_t H,
                              int32_t max_context_len, float softmax_scale,
                              const AttnWorkspace &ws, int32_t num_cus, int32_t waves_per_cu,
                              int32_t loads_per_block, int32_t phases, hipStream_t s)
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
    const bool gqa = gqa_mfma_applies(c, H);
    // the plan kernel shortens the splits until every wave of a full grid (about eight waves
    // per compute unit) would get this many items; the matrix-core kernel, whose items are
    // heavier to start, asks for one
    p.ws.min_items = plan_min_items(num_cus, gqa);
    p.zero_empty = (phases & kPhasePlan) ? 0 : 1;
    hipError_t e = hipSuccess;
    if (phases & kPhasePlan) {
        const int32_t items_per_tile = gqa ? c.Hkv : H;
        const int32_t keep_negative = (phases & kPhaseKeepNegative) ? 1 : 0;
        // (A one-wave version of the plan for batches of at most 64 requests -- no barriers, no histogram -- was slower, 8.8 us
        // against 7.2 us in the kernel trace: a nearly empty kernel already shows 4-5 us there, the rest is the latency of
        // dependent shuffles, which 1024 threads hide no worse than 64.)
        hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(1024), 0, s, context_lens, B, H, items_per_tile, max_context_len, p.ws,
                           p.out, c.D, keep_negative);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (!(phases & kPhaseRun)) return hipSuccess;
    e = hipErrorInvalidValue;
    if (gqa) {
        e = launch_gqa_mfma(p, num_cus, waves_per_cu, loads_per_block, s);
    } else {
#define ALISE_DISPATCH(NBV)                                                                          \
    do {                                                                                             \
        if (c.bits == 8 && c.D == 128) e = launch_t<8, 128, NBV>(p, num_cus, waves_per_cu, s);        \
        else if (c.bits == 8 && c.D == 64) e = launch_t<8, 64, NBV>(p, num_cus, waves_per_cu, s);     \
        else if (c.bits == 4 && c.D == 128) e = launch_t<4, 128, NBV>(p, num_cus, waves_per_cu, s);   \
        else if (c.bits == 4 && c.D == 64) e = launch_t<4, 64, NBV>(p, num_cus, waves_per_cu, s);     \
    } while (0)
        if (loads_per_block == 0) loads_per_block = 2;      // 3 and 4 measure within 1 % of it
        if (loads_per_block == 2) ALISE_DISPATCH(2);
        else if (loads_per_block == 3) ALISE_DISPATCH(3);
        else if (loads_per_block == 4) ALISE_DISPATCH(4);
#undef ALISE_DISPATCH
    }
    if (e != hipSuccess) return e;
    // No request can have more than one split when the longest context fits the shortest split the plan may choose, and
    // then there is nothing to merge (the zero rows of a run on an earlier plan are the merge kernel's too).
    if (max_context_len <= p.ws.min_chunk_tokens && !p.zero_empty) return hipSuccess;
    return launch_merge(p, s);
}

}  // namespace alise
