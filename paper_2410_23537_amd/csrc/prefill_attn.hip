// Chunked-prefill attention over the quantized, paged cache on the gfx950 matrix cores.
//
// The prompt's tokens are processed in one pass (ALISE Sec. 2 "LLM Inference"); with the cache
// of Sec. 3.2 that means: the chunk's K/V are quantized and written first, then every query
// token of the chunk attends causally (Eq. 1-2) over the cached codes -- positions 0 .. its own.
// Query token j of an n-token chunk of a request with L cached tokens sits at position L - n + j.
//
// Work decomposition.  Rows of the problem are (query token, query head) pairs; the rows that
// share a KV head share every KV byte.  A workgroup of four waves takes 64 or 128 such rows of one
// request and one KV head (one or two 16-row tiles per wave; a tile is 16 / qper tokens x qper
// heads) and walks the cache once from position 0 to the last position any of its rows may see.
// The four waves share the cache through LDS: per step of 32 tokens each wave fetches a quarter
// of the step (K or V codes of one 16-token tile plus its scales and zero-points) with direct
// global -> LDS loads, three stages deep, one workgroup barrier per step.  Per wave the step is
// the one of the grouped-query decode kernel: S^T = K Q^T and O += P V on
// v_mfma_f32_16x16x32_f16, K and V codes as fp16 subnormals code * 2^-24, P * lambda_v split in
// high and low fp16 parts, online softmax with a lazily raised maximum -- except that the mask
// is per row (token <= the row's position), that only the steps on a wave's diagonal are masked
// at all, and that a wave skips the steps none of its rows can see.  Two row tiles of a wave
// share the operands built from the cache.  A second set of kernels (ALISE_PREFILL_WEIGHTS=single)
// takes a weight as ONE fp16 number rounded to nearest even: the kernel is bound by its vector
// instructions, and the second product per weight with the instructions that form the low part
// are a sixth of them.  With the zero-point sum taken over the same rounded weights the rounding
// only perturbs each weight by 2^-12 relative (nothing cancels between a code sum and a zero-point
// sum that were rounded differently), i.e. the output by at most 2^-12 max|v|: invisible where many
// tokens share a row's weight, up to 1e-3 for |v| near 4 where a few tokens carry it -- on top of
// the fp16 rounding of the output that is too much for the 2e-3 bar, hence not the default.
// INT8 caches (one or two scale groups per head) and
// INT4 caches with groups of 32, 64 or 128 channels are taken; the INT4 operand formats are described at the
// top of the kernel body.
// There is no split along the context and therefore nothing to merge: a chunk of a few
// hundred tokens gives thousands of workgroups, handed out longest walk first.
//
// The block-table entries of the 64 pages around the current position sit in a register (one
// entry per lane), refilled every 64 pages from a window fetched ahead of time into LDS.
#include "mfma_stream.h"
#include <cstdlib>
#include <type_traits>

namespace alise {
namespace {

struct PrefillParams {
    CacheView c;
    const _Float16 *q;
    _Float16 *out;
    const int32_t *q_start;
    const int32_t *block_tables;
    const int32_t *context_lens;
    int32_t max_blocks, B, H, qper, max_len;
    float scale_log2e;
    PrefillWorkspace ws;
};

// One workgroup writes the table of (request, row tile) pairs, ordered by decreasing work: a tile
// walks the cache from position 0 to the last position its rows may see, so that position is its
// cost, and the hardware hands out workgroups in table order -- longest first, which keeps the
// tail of the grid short (a counting sort over 1024 length buckets; inside a bucket any order).
__global__ __launch_bounds__(1024) void prefill_plan_kernel(const int32_t *q_start, const int32_t *context_lens, int32_t B,
                                                            int32_t tokens_per_wg, int32_t max_len, PrefillWorkspace ws)
{
    __shared__ int32_t s_hist[1024];
    __shared__ int32_t s_wave[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    s_hist[tid] = 0;
    __syncthreads();
    auto chunk_of = [&](int i, int &n, int &first_pos) {
        const int L = min(max(context_lens[i], 0), max_len);
        n = min(max(q_start[i + 1] - q_start[i], 0), L);       // a chunk cannot be longer than its request
        first_pos = L - n;
    };
    auto bucket_of = [&](int kv_end) {                          // bucket 0 holds the longest walks
        const int b = (int)(((int64_t)(max_len - kv_end) * 1024) / ((int64_t)max_len + 1));
        return min(max(b, 0), 1023);
    };
    for (int i = tid; i < B; i += 1024) {
        int n, first_pos;
        chunk_of(i, n, first_pos);
        const int tiles = (n + tokens_per_wg - 1) / tokens_per_wg;
        for (int t = 0; t < tiles; ++t) atomicAdd(&s_hist[bucket_of(first_pos + min((t + 1) * tokens_per_wg, n))], 1);
    }
    __syncthreads();
    // exclusive scan of the bucket counts: the first table position of every bucket
    const int mine = s_hist[tid];
    int incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int u = __shfl_up(incl, d);
        if (lane >= d) incl += u;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
    for (int k = 0; k < 16; ++k) {
        if (k < wave) before += s_wave[k];
        total += s_wave[k];
    }
    s_hist[tid] = before + incl - mine;
    __syncthreads();
    for (int i = tid; i < B; i += 1024) {
        int n, first_pos;
        chunk_of(i, n, first_pos);
        const int tiles = (n + tokens_per_wg - 1) / tokens_per_wg;
        for (int t = 0; t < tiles; ++t) {
            const int pos = atomicAdd(&s_hist[bucket_of(first_pos + min((t + 1) * tokens_per_wg, n))], 1);
            if (pos < ws.max_tiles) ws.table[pos] = make_int2(i, t);
        }
    }
    if (tid == 0) *ws.n_tiles = total < ws.max_tiles ? total : ws.max_tiles;
}

// RT: 16-row tiles per wave.  Two tiles share every code -> fp16 conversion and every LDS read of a step.
// BITS: 8, or 4 (two channels per byte, channel 2i in the low nibble): see the INT4 notes below.
// SPLIT: a weight enters the second product as a high and a low fp16 part (exact to 22 bits) instead of one
// rounded fp16 number.
template <int BITS, int NGRP, int RT, bool SPLIT>
__device__ __forceinline__ void prefill_attn_body(const PrefillParams &p)
{
    constexpr int D = 128, ROWB = D * BITS / 8, S = 3;
    // one 16-token tile in LDS: K codes | V codes | K meta | V meta (INT8, two groups: 2 KiB | 2 KiB | 128 B | 128 B)
    constexpr int T_V = 16 * ROWB, T_KM = 32 * ROWB, T_VM = T_KM + 64 * NGRP;
    constexpr int TILEB = BITS == 8 ? 4352 : T_VM + 64 * NGRP;
    static_assert(TILEB % 128 == 0 && TILEB >= T_VM + 64 * NGRP, "tile layout");
    constexpr int STEPB = 2 * TILEB;
    constexpr int LOADS_PER_STEP = BITS == 8 ? 3 : 2;       // direct loads a wave issues per step
    // With two row tiles every scale and zero-point has two uses, and the compiler then converts the half to
    // fp32 first instead of reading it in place: the hand-written multiply-adds of mfma_stream.h take over.
    // With one tile it reads them in place by itself and schedules better around its own instructions.
    constexpr bool IN_PLACE = RT > 1 || !SPLIT;
    // INT4.  A token's row is 64 bytes, so one 1 KiB load brings a whole 16-token tile; row r keeps its
    // 16-byte piece c at position c ^ (r / 4 % 4).  K: chunk jj of the first product is the 32 channels
    // of piece jj (one scale group when G = 32, half or a quarter of one when G = 64 or 128); a lane's dword of it holds 8 nibbles, which two masks on
    // the dword and two on the dword shifted by a byte turn into fp16 pairs code * 2^-24 (even
    // channels) and 16 code * 2^-24 (odd channels) -- k-slots in the order 0 4 1 5 2 6 3 7, Q permuted
    // likewise with its odd channels divided by 16.  V: columns of a product are 16 channels of one
    // 32-channel block b: lane n takes the byte n % 4 of dword n / 4 of the block, i.e. channels
    // 32 b + 2 n and 32 b + 2 n + 1 -- the low nibbles go to one product, the high nibbles (times 16,
    // undone at the output) to another.
    __shared__ __attribute__((aligned(128))) uint8_t lds[S * STEPB + 4 * 512];     // stages, then two page-window slots per wave

    // Workgroups start in the order of their number, so the KV head is its fast index: the table is sorted by the
    // length of the walk, and every head's longest tiles must start before anybody's short ones.  (With the head as
    // the slow index the last head's longest walk began when the grid was almost through; on chunk mixes with a few
    // long contexts a fifth to a third of the time went into that tail.  Workgroup w runs on XCD w % 8, so with a
    // multiple of 8 heads all row tiles of one request and head also share an L2.  Runs of 2 or 8 consecutive table
    // entries per head before the next head measured within a few per cent of this, either way.)
    const int f = blockIdx.x / p.c.Hkv;
    const int hk = blockIdx.x - f * p.c.Hkv;
    if (f >= *p.ws.n_tiles) return;             // workgroup-uniform, before any barrier
    const int2 entry = p.ws.table[f];
    const int i = min(max(entry.x, 0), p.B - 1), rt = max(entry.y, 0);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15;        // column of the matrix layouts: token (K), row of the problem (S^T), channel (V, O)
    const int g = lane >> 4;        // quarter of the wave: 8 consecutive k-slots, 4 consecutive rows
    const int logP = p.c.logP, P = p.c.P, Hkv = p.c.Hkv, qper = p.qper, H = p.H;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)lds;
    lptr_t const ldsp = (lptr_t)lds;

    // ---- the request's chunk and this wave's rows
    const int L = min(max(p.context_lens[i], 0), p.max_len);
    const int qs = p.q_start[i];
    int n_q = p.q_start[i + 1] - qs;
    n_q = min(max(n_q, 0), L);
    const int TT = 16 * RT / qper;              // query tokens per wave
    const int first_pos = L - n_q;              // position of the chunk's first token
    const int j0 = (rt * 4 + wave) * TT;        // this wave's first query token
    // row tile t, column n of the matrix layouts <-> row 16 t + n of the wave's 16 RT rows <-> (token, head of the group)
    int j_n[RT], e_n[RT], pos_n[RT];
    bool row_valid[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int row = 16 * t + n;
        j_n[t] = j0 + row / qper;
        e_n[t] = row % qper;
        row_valid[t] = row < TT * qper && j_n[t] < n_q;
        pos_n[t] = row_valid[t] ? first_pos + j_n[t] : -1;          // what the row may see: tokens <= pos_n
    }
    const int wave_last = first_pos + min(j0 + TT, n_q) - 1;         // last position any row of this wave sees (< first_pos + j0: none)
    const bool wave_has_rows = j0 < n_q;
    const int kv_end = first_pos + min((rt + 1) * 4 * TT, n_q);     // the workgroup walks positions [0, kv_end)
    const int nsteps = (kv_end + kStep - 1) / kStep;
    if (n_q <= 0 || nsteps <= 0) return;        // workgroup-uniform

    // ---- per-lane constants of the LDS layout (see the decode kernel): INT8: a 1 KiB load covers 8
    // token rows; row r keeps its 16-byte piece c at position c ^ r.  The array starts on a
    // 128-byte boundary and every stage, tile and row is a multiple of 64 bytes long, so the
    // swizzle of an address is an exclusive-or of address bits with the row number.
    const int src_lane = BITS == 8 ? (lane >> 3) * ROWB + (((lane & 7) ^ (lane >> 3)) * 16)
                                   : (lane >> 2) * ROWB + (((lane & 3) ^ ((lane >> 4) & 3)) * 16);
    // K, INT8: token n of a tile, pieces g and 4 + g (the second: the first with bit 6 flipped);
    // INT4: token n, dword g of piece jj at (k_rd ^ 16 jj)
    const uint32_t k_rd = BITS == 8 ? (n >> 3) * 1024 + ((n & 7) * 8 + (g ^ (n & 7))) * 16
                                    : n * 64 + ((n >> 2) & 3) * 16 + g * 4;
    // V, INT8: token rows 4g + r (r = 0..3), piece 4 * set + n / 4, dword n % 4 of the piece: row r of set `set`
    // sits at (v_rd ^ (16 r + 64 set)) + 128 r;  INT4: rows 4g + r, dword n / 4 of block b at (v_rd ^ 16 b) + 64 r
    const uint32_t v_rd = BITS == 8 ? T_V + (g >> 1) * 1024 + (g & 1) * 512 + (((n >> 2) ^ ((g & 1) * 4)) * 16) + (n & 3) * 4
                                    : T_V + g * 256 + g * 16 + (n >> 2) * 4;
    const uint32_t m_rd = g * 16 * NGRP;
    const uint32_t v_sel = 0x0c000c00u | ((4u + (n & 3)) << 16) | (uint32_t)(n & 3);     // INT4: byte n % 4 of two dwords into the low bytes of two halves

    // ---- Q^T as the B operand of the four k-chunks: chunk jj, slot g*8+e <-> channel (jj/2)*64 + g*16 + (jj%2)*8 + e
    h8_t qop[RT][4];
    float nqs24[RT][NGRP];                  // -sum(q) 2^-24 over the channels of a group
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int jc = min(j_n[t], n_q - 1);
        const _Float16 *qrow = p.q + ((int64_t)(qs + jc) * H + hk * qper + e_n[t]) * D;
        float part_sum[NGRP];
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) part_sum[gr] = 0.0f;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            // INT8: chunk jj, slot g*8+e <-> channel (jj/2)*64 + g*16 + (jj%2)*8 + e;  INT4: channel 32 jj + 8 g + {0 4 1 5 2 6 3 7}[e]
            h8_t v = *reinterpret_cast<const h8_t *>(qrow + (BITS == 8 ? (jj / 2) * 64 + g * 16 + (jj % 2) * 8 : jj * 32 + g * 8));
            if (!row_valid[t]) v = (h8_t)(_Float16)0.0f;
            float sacc = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) sacc += (float)v[e];
            part_sum[jj * NGRP / 4] += sacc;
            if constexpr (BITS == 4) {
                const _Float16 sixteenth = (_Float16)0.0625f;       // the odd nibbles arrive 16 times too large
                const h8_t w = {v[0], v[4], v[1] * sixteenth, v[5] * sixteenth, v[2], v[6], v[3] * sixteenth, v[7] * sixteenth};
                v = w;
            }
            qop[t][jj] = v;
        }
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) {
            float v = part_sum[gr];
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            nqs24[t][gr] = -v * (1.0f / 16777216.0f);
        }
    }
    // Scores are kept in the units of the accumulator: t = sum_g lambda_k (acc_g - z_k sum(q_g) 2^-24), the true
    // score being t * scale24 (the softmax scale, log2 e and the 2^24 that the subnormal K codes lack).
    const float scale24 = p.scale_log2e * 16777216.0f;
    const float inv24 = 1.0f / scale24;
    const float lazy_t = kLazy * inv24;

    // ---- block-table windows: 64 entries, one per lane.  Lookups use window wa in pg_a; the
    // windows come through LDS by direct loads (two slots per wave), fetched one window ahead,
    // so that no vector load ever returns into a register inside the loop.
    const int32_t *bt = p.block_tables + (int64_t)i * p.max_blocks;
    const int last_page = (kv_end - 1) >> logP;
    const int pg_slots = S * STEPB + wave * 512;
    auto fetch_window = [&](int wdw) { dma4(bt + min(wdw * 64 + lane, last_page), ldsp + pg_slots + (wdw & 1) * 256); };
    auto read_window = [&](int wdw) { return (int)lds_read4(lds0 + pg_slots + (wdw & 1) * 256 + lane * 4); };
    int wa = 0;
    fetch_window(0);
    fetch_window(1);
    ALISE_VMCNT(0);
    int pg_a = read_window(0);

    // ---- this wave's quarter of a step: tile x = wave / 2, K (even waves) or V (odd waves)
    const int my_x = wave >> 1;
    const bool my_v = wave & 1;
    auto issue = [&](int k, int stage) {
        int tx = k * kStep + my_x * 16;
        if (tx >= kv_end) tx -= 16;                             // second tile starts past the end: repeat the first
        const int pi = tx >> logP;
        if ((pi >> 6) > wa) {                                   // wave-uniform; once per 64 pages
            ++wa;
            pg_a = read_window(wa);                             // fetched a window ago: landed long since (every step waits for all but three loads)
            fetch_window(wa + 1);                               // into the slot of the window just left
        }
        const int page = min(max(__builtin_amdgcn_readlane(pg_a, pi & 63), 0), p.c.num_pages - 1);
        const int blk = page * Hkv + hk;
        const int off = tx & (P - 1);
        const int64_t co = (int64_t)blk * p.c.cstride + (int64_t)off * ROWB;
        const int64_t mo = (int64_t)blk * p.c.mstride + (int64_t)off * NGRP * 4;
        lptr_t dst = ldsp + stage * STEPB + my_x * TILEB;
        const uint8_t *cb = (my_v ? p.c.v_codes : p.c.k_codes) + co + src_lane;
        const uint8_t *mb = reinterpret_cast<const uint8_t *>(my_v ? p.c.v_meta : p.c.k_meta) + mo + lane * 4;
        // the rows of a head are read again by the workgroups of its other row tiles: keep them in the L2
        dma16(cb, dst + (my_v ? T_V : 0));
        if constexpr (BITS == 8) dma16(cb + 1024, dst + (my_v ? T_V : 0) + 1024);
        if (lane < 16 * NGRP) dma4(mb, dst + (my_v ? T_VM : T_KM));
    };

    // m_ref: the running maximum in the units of t.  c_ref = bias - m_ref scale24: a weight is 2^(t scale24 + c_ref).
    float m_ref[RT], c_ref[RT], l_part[RT], z_part[RT][NGRP];
    float bias = kWeightBias;           // see kWeightBias; wave-uniform, common to the row tiles
    f4_t o[RT][8];              // INT8: [tile][set*4 + nu]: rows 4g..4g+3 of the tile, column n <-> channel 64*set + 4n + nu;  INT4: [tile][2b + m] <-> channel 32b + 2n + m
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        m_ref[t] = kFloor * inv24;
        c_ref[t] = __builtin_fmaf(-m_ref[t], scale24, bias);
        l_part[t] = 0.0f;
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) z_part[t][gr] = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) o[t][c] = (f4_t)0.0f;
    }

    // One step of 32 tokens out of the LDS stage at `base`.  MASKED: some row of this wave must not see
    // some token of the step (the steps on the diagonal); otherwise no comparison and no select is spent.
    auto step = [&](auto masked_c, int k, uint32_t base) {
        constexpr bool MASKED = decltype(masked_c)::value;
        // ---- S^T = K Q^T for the two 16-token tiles, every row tile against the same K operands
        float s[RT][2][4];
        uint32_t vmraw[MASKED ? RT : 1][2][4][NGRP];   // V (scale, zero) dwords of this lane's tokens; 0 where a row tile must not see the token
        float mx[RT];
#pragma unroll
        for (int t = 0; t < RT; ++t) mx[t] = kNegInf;
        uint4 kp[2][2];                // INT8: [tile][piece];  INT4: kp[tile][0] holds the dwords of the four chunks
        const uint32_t ka0 = base + k_rd, ma = base + m_rd;
        if constexpr (BITS == 8) {
            const uint32_t ka1 = ka0 ^ 64u;
            lds_read16x4_at<0, 0, TILEB, TILEB>(ka0, ka1, ka0, ka1, kp[0][0], kp[0][1], kp[1][0], kp[1][1]);
        } else {
            const uint32_t ka[4] = {ka0, ka0 ^ 16u, ka0 ^ 32u, ka0 ^ 48u};
            uint32_t k0[4], k1[4];
            lds_read4x4x2<TILEB>(ka, k0, k1);
            kp[0][0] = make_uint4(k0[0], k0[1], k0[2], k0[3]);
            kp[1][0] = make_uint4(k1[0], k1[1], k1[2], k1[3]);
        }
        uint4 kmeta[2][NGRP], vmeta[2][NGRP];
        if constexpr (NGRP == 4) {
            lds_read16x4_at<T_KM, T_KM + 16, T_KM + 32, T_KM + 48>(ma, ma, ma, ma, kmeta[0][0], kmeta[0][1], kmeta[0][2], kmeta[0][3]);
            lds_read16x4_at<T_VM, T_VM + 16, T_VM + 32, T_VM + 48>(ma, ma, ma, ma, vmeta[0][0], vmeta[0][1], vmeta[0][2], vmeta[0][3]);
            lds_read16x4_at<TILEB + T_KM, TILEB + T_KM + 16, TILEB + T_KM + 32, TILEB + T_KM + 48>(ma, ma, ma, ma, kmeta[1][0], kmeta[1][1],
                                                                                                   kmeta[1][2], kmeta[1][3]);
            lds_read16x4_at<TILEB + T_VM, TILEB + T_VM + 16, TILEB + T_VM + 32, TILEB + T_VM + 48>(ma, ma, ma, ma, vmeta[1][0], vmeta[1][1],
                                                                                                   vmeta[1][2], vmeta[1][3]);
        } else if constexpr (NGRP == 1) {
            lds_read16x4_at<T_KM, T_VM, TILEB + T_KM, TILEB + T_VM>(ma, ma, ma, ma, kmeta[0][0], vmeta[0][0], kmeta[1][0], vmeta[1][0]);
        } else {
            lds_read16x4_at<T_KM, T_KM + 16, T_VM, T_VM + 16>(ma, ma, ma, ma, kmeta[0][0], kmeta[0][1], vmeta[0][0], vmeta[0][1]);
            lds_read16x4_at<TILEB + T_KM, TILEB + T_KM + 16, TILEB + T_VM, TILEB + T_VM + 16>(ma, ma, ma, ma, kmeta[1][0], kmeta[1][1],
                                                                                              vmeta[1][0], vmeta[1][1]);
        }
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            f4_t acc[RT][NGRP];
#pragma unroll
            for (int t = 0; t < RT; ++t)
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) acc[t][gr] = (f4_t)0.0f;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                h8_t a;
                if constexpr (BITS == 8) {
                    const uint4 piece = kp[x][jj / 2];
                    const uint32_t w0 = (jj % 2) ? piece.z : piece.x, w1 = (jj % 2) ? piece.w : piece.y;
                    a = pack8(__builtin_amdgcn_perm(0u, w0, 0x0c010c00u), __builtin_amdgcn_perm(0u, w0, 0x0c030c02u),
                              __builtin_amdgcn_perm(0u, w1, 0x0c010c00u), __builtin_amdgcn_perm(0u, w1, 0x0c030c02u));
                } else {
                    const uint4 d4 = kp[x][0];
                    const uint32_t w0 = jj == 0 ? d4.x : jj == 1 ? d4.y : jj == 2 ? d4.z : d4.w, w1 = w0 >> 8;
                    a = pack8(w0 & 0x000F000Fu, w0 & 0x00F000F0u, w1 & 0x000F000Fu, w1 & 0x00F000F0u);
                }
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    f4_t &dst = acc[t][jj * NGRP / 4];
                    dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, qop[t][jj], dst, 0, 0, 0);
                }
            }
            const int tok0 = k * kStep + x * 16 + g * 4;                // first token of this lane's 4 rows of S^T
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                const int room = pos_n[t] - tok0;                       // row r of the block is visible iff r <= room
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const bool valid = !MASKED || r <= room;            // causal, per row of the problem
                    float sv = 0.0f;
#pragma unroll
                    for (int gr = 0; gr < NGRP; ++gr) {
                        const uint32_t km = meta_of<NGRP>(kmeta[x], r, gr);         // (scale, zero-point)
                        // the reader of the matrix result is left to the compiler (wait states), the scale is read in place
                        const float u = __builtin_fmaf((float)as_h2(km).y, nqs24[t][gr], acc[t][gr][r]);
                        if constexpr (IN_PLACE) sv = fma_lo_half(km, u, sv);
                        else sv = __builtin_fmaf((float)as_h2(km).x, u, sv);
                        if (MASKED || t == 0) {
                            const uint32_t vm = meta_of<NGRP>(vmeta[x], r, gr);
                            vmraw[MASKED ? t : 0][x][r][gr] = valid ? vm : 0u;
                        }
                    }
                    s[t][x][r] = valid ? sv : kNegInf;
                    mx[t] = fmaxf(mx[t], s[t][x][r]);
                }
            }
        }

        // ---- running maximum per row of the problem, raised lazily; all four quarters hold the same value
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            if (__builtin_amdgcn_ballot_w64(mx[t] > m_ref[t] + lazy_t) != 0) {
                float mq = fmaxf(mx[t], __shfl_xor(mx[t], 16));
                mq = fmaxf(mq, __shfl_xor(mq, 32));
                m_ref[t] = (mq > m_ref[t] + lazy_t) ? mq : m_ref[t];
                const float c_new = __builtin_fmaf(-m_ref[t], scale24, bias);
                const float fac = __builtin_amdgcn_exp2f(c_new - c_ref[t]);
                c_ref[t] = c_new;
                l_part[t] *= fac;
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) z_part[t][gr] *= fac;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float fr = __shfl(fac, 4 * g + r);        // factor of the problem row 4g+r
#pragma unroll
                    for (int c = 0; c < 8; ++c) o[t][c][r] *= fr;
                }
            }
        }

        // ---- a V scale of 2 or more in this step: the biased weights could leave the fp16 range (rare, wave-uniform)
        if (bias != 0.0f &&
            __builtin_amdgcn_ballot_w64(max_low_half<(MASKED ? RT : 1) * 8 * NGRP>(&vmraw[0][0][0][0]) >= 0x4000u) != 0) {
            bias = 0.0f;
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                const float c_new = __builtin_fmaf(-m_ref[t], scale24, 0.0f);
                const float fb = __builtin_amdgcn_exp2f(c_new - c_ref[t]);
                c_ref[t] = c_new;
                l_part[t] *= fb;
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) z_part[t][gr] *= fb;
#pragma unroll
                for (int c = 0; c < 8; ++c) o[t][c] *= fb;
            }
        }

        // ---- weights p * lambda_v in the A-operand order (tile, row): the product rounded to fp16 (nearest even)
        // and, with SPLIT, what that lacks of the exact product as a second fp16 number
        h8_t a_w[RT][NGRP], a_lo[SPLIT ? RT : 1][NGRP];
#pragma unroll
        for (int t = 0; t < RT; ++t)
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int rr = 0; rr < 4; rr += 2) {
                    float pj[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        pj[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[t][x][rr + e], scale24, c_ref[t]));
                        l_part[t] += pj[e];
                    }
#pragma unroll
                    for (int gr = 0; gr < NGRP; ++gr) {
                        const uint32_t vm0 = vmraw[MASKED ? t : 0][x][rr][gr], vm1 = vmraw[MASKED ? t : 0][x][rr + 1][gr];
                        uint32_t w16;
                        if constexpr (SPLIT) {
                            // the zero-point sum takes the exact weight, as the two products together do
                            typedef float f2_t __attribute__((ext_vector_type(2)));
                            uint32_t lo16;
                            if constexpr (IN_PLACE) {
                                const float w0 = mul_lo_half_f32(vm0, pj[0]), w1 = mul_lo_half_f32(vm1, pj[1]);
                                z_part[t][gr] = fma_hi_half(vm0, w0, z_part[t][gr]);
                                z_part[t][gr] = fma_hi_half(vm1, w1, z_part[t][gr]);
                                const f2_t wv = {w0, w1};
                                w16 = as_u32(__builtin_convertvector(wv, h2_t));
                                lo16 = residual_of_h2(vm0, pj[0], vm1, pj[1], w16);
                            } else {
                                const h2_t m0 = as_h2(vm0), m1 = as_h2(vm1);
                                const f2_t wv = {__builtin_fmaf((float)m0.x, pj[0], 0.0f), __builtin_fmaf((float)m1.x, pj[1], 0.0f)};
                                z_part[t][gr] = __builtin_fmaf((float)m0.y, wv.x, z_part[t][gr]);
                                z_part[t][gr] = __builtin_fmaf((float)m1.y, wv.y, z_part[t][gr]);
                                const h2_t hi = __builtin_convertvector(wv, h2_t);
                                const h2_t lo = {(_Float16)__builtin_fmaf((float)m0.x, pj[0], -(float)hi.x),
                                                 (_Float16)__builtin_fmaf((float)m1.x, pj[1], -(float)hi.y)};
                                w16 = as_u32(hi);
                                lo16 = as_u32(lo);
                            }
                            a_lo[t][gr][x * 4 + rr] = as_h2(lo16).x;
                            a_lo[t][gr][x * 4 + rr + 1] = as_h2(lo16).y;
                        } else {
                            w16 = mul_lo_halves_to_h2(vm0, pj[0], vm1, pj[1]);
                            // the zero-point sum takes the rounded weight, the one the matrix product multiplies the codes with
                            z_part[t][gr] = fma_hi_by_half<0>(vm0, w16, z_part[t][gr]);
                            z_part[t][gr] = fma_hi_by_half<1>(vm1, w16, z_part[t][gr]);
                        }
                        a_w[t][gr][x * 4 + rr] = as_h2(w16).x;
                        a_w[t][gr][x * 4 + rr + 1] = as_h2(w16).y;
                    }
                }

        // ---- O += P V, the B operands built once for all row tiles
        if constexpr (BITS == 8) {
            // byte nu of the dwords of two tokens -> two fp16 subnormals
            uint32_t va[8], vd[2][8];          // vd[tile][set * 4 + r]
            va[0] = v_rd + base;
#pragma unroll
            for (int c = 1; c < 8; ++c) va[c] = va[0] ^ (uint32_t)((c & 3) * 16 + (c >> 2) * 64);
            lds_read4x8x2<ROWB, TILEB>(va, vd[0], vd[1]);
#pragma unroll
            for (int set = 0; set < 2; ++set)
#pragma unroll
                for (int nu = 0; nu < 4; ++nu) {
                    const uint32_t sel = 0x0c000c00u | ((4u + nu) << 16) | (uint32_t)nu;
                    const h8_t bv = pack8(__builtin_amdgcn_perm(vd[0][set * 4 + 1], vd[0][set * 4 + 0], sel),
                                          __builtin_amdgcn_perm(vd[0][set * 4 + 3], vd[0][set * 4 + 2], sel),
                                          __builtin_amdgcn_perm(vd[1][set * 4 + 1], vd[1][set * 4 + 0], sel),
                                          __builtin_amdgcn_perm(vd[1][set * 4 + 3], vd[1][set * 4 + 2], sel));
                    const int gr = NGRP == 2 ? set : 0;
#pragma unroll
                    for (int t = 0; t < RT; ++t) {
                        f4_t &dst = o[t][set * 4 + nu];
                        dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_w[t][gr], bv, dst, 0, 0, 0);
                        if constexpr (SPLIT) dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_lo[t][gr], bv, dst, 0, 0, 0);
                    }
                }
        } else {
            // byte n % 4 of the block's dword of two tokens -> (low nibbles) and (high nibbles * 16) as fp16 subnormals
            const uint32_t va0 = v_rd + base;
#pragma unroll
            for (int bb = 0; bb < 4; bb += 2) {
                uint32_t vd[2][2][4];          // [block of the pair][tile][r]
                lds_read4_rows2x2<ROWB, TILEB>(va0 ^ (uint32_t)(bb * 16), va0 ^ (uint32_t)((bb + 1) * 16), vd[0][0], vd[0][1], vd[1][0], vd[1][1]);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int b = bb + h;
                    const uint32_t p0 = __builtin_amdgcn_perm(vd[h][0][1], vd[h][0][0], v_sel), p1 = __builtin_amdgcn_perm(vd[h][0][3], vd[h][0][2], v_sel);
                    const uint32_t p2 = __builtin_amdgcn_perm(vd[h][1][1], vd[h][1][0], v_sel), p3 = __builtin_amdgcn_perm(vd[h][1][3], vd[h][1][2], v_sel);
#pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        const uint32_t mask = m ? 0x00F000F0u : 0x000F000Fu;
                        const h8_t bv = pack8(p0 & mask, p1 & mask, p2 & mask, p3 & mask);
                        const int gr = b * NGRP / 4;
#pragma unroll
                        for (int t = 0; t < RT; ++t) {
                            f4_t &dst = o[t][b * 2 + m];
                            dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_w[t][gr], bv, dst, 0, 0, 0);
                            if constexpr (SPLIT) dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_lo[t][gr], bv, dst, 0, 0, 0);
                        }
                    }
                }
            }
        }
    };

    // Every wave passes the same nsteps barriers; what it computes in between is its own business.  The steps
    // that lie wholly before the wave's first row come first and need no mask, then the steps on its diagonal
    // (masked), then steps that none of its rows may see (skipped).
    int stage = 0;                              // k % S, kept as a counter
    auto advance = [&](int k) -> uint32_t {
        // this wave's quarter of step k has landed once at most the three loads of the step after it are in flight
        if (k + 1 < nsteps) ALISE_VMCNT(LOADS_PER_STEP); else ALISE_VMCNT(0);
        // all four quarters have landed, and every wave is done reading the stage that step k + 2 overwrites
        asm volatile("s_barrier" ::: "memory");
        if (k + 2 < nsteps) issue(k + 2, stage == 0 ? 2 : stage - 1);
        const uint32_t base = lds0 + stage * STEPB;
        stage = stage == S - 1 ? 0 : stage + 1;
        return base;
    };
    const int n_open = wave_has_rows ? min(nsteps, (first_pos + j0 + 1) / kStep) : 0;   // steps k with k*32 + 31 <= the wave's first position
    issue(0, 0);
    if (nsteps > 1) issue(1, 1);
    int k = 0;
    for (; k < n_open; ++k) {
        const uint32_t base = advance(k);
        step(std::false_type{}, k, base);
    }
    for (; k < nsteps; ++k) {
        const uint32_t base = advance(k);
        if (!wave_has_rows || k * kStep > wave_last) continue;     // nothing here that a row of this wave may see
        step(std::true_type{}, k, base);
    }

    // ---- per row of the problem: add the four quarters; then fetch the values of this lane's rows
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        float l = l_part[t] + __shfl_xor(l_part[t], 16);
        l += __shfl_xor(l, 32);
        float zsum[NGRP];
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) {
            float v = z_part[t][gr] + __shfl_xor(z_part[t][gr], 16);
            v += __shfl_xor(v, 32);
            zsum[gr] = v;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int col = 4 * g + r;                  // column of the S^T layout that holds the row's l and z
            const float l_row = __shfl(l, col);
            float z_row[NGRP];
#pragma unroll
            for (int gr = 0; gr < NGRP; ++gr) z_row[gr] = __shfl(zsum[gr], col);
            const int row = 16 * t + col;
            const int j_r = j0 + row / qper, e_r = row % qper;
            if (row < TT * qper && j_r < n_q) {
                const float inv_l = 1.0f / l_row;
                _Float16 *orow = p.out + ((int64_t)(qs + j_r) * H + hk * qper + e_r) * D;
                if constexpr (BITS == 8) {
                    _Float16 *dst = orow + 4 * n;
#pragma unroll
                    for (int set = 0; set < 2; ++set) {
                        const float zr = z_row[NGRP == 2 ? set : 0];
                        typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
                        h4_t v;
#pragma unroll
                        for (int nu = 0; nu < 4; ++nu)
                            v[nu] = (_Float16)(__builtin_fmaf(o[t][set * 4 + nu][r], 16777216.0f, -zr) * inv_l);
                        *reinterpret_cast<h4_t *>(dst + 64 * set) = v;
                    }
                } else {
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const float zr = z_row[b * NGRP / 4];
                        h2_t v;
                        v.x = (_Float16)(__builtin_fmaf(o[t][b * 2 + 0][r], 16777216.0f, -zr) * inv_l);
                        v.y = (_Float16)(__builtin_fmaf(o[t][b * 2 + 1][r], 1048576.0f, -zr) * inv_l);      // 2^24 / 16
                        *reinterpret_cast<h2_t *>(orow + 32 * b + 2 * n) = v;
                    }
                }
            }
        }
    }
}

// Register budgets: one 16-row tile per wave with one scale group per head (G = 128) fits four waves per
// SIMD, with two groups three; two row tiles per wave take two waves per SIMD.
#define ALISE_PREFILL_KERNEL(NAME, WAVES, BITSV, NGRPV, RTV)                                                              \
    __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES))) void NAME(PrefillParams p)       \
    {                                                                                                                     \
        prefill_attn_body<BITSV, NGRPV, RTV, true>(p);                                                                    \
    }                                                                                                                     \
    __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES))) void NAME##_w1(PrefillParams p)  \
    {                                                                                                                     \
        prefill_attn_body<BITSV, NGRPV, RTV, false>(p);                                                                   \
    }
ALISE_PREFILL_KERNEL(prefill_attn_kernel_g1, 4, 8, 1, 1)
ALISE_PREFILL_KERNEL(prefill_attn_kernel_g2, 3, 8, 2, 1)
ALISE_PREFILL_KERNEL(prefill_attn_kernel_g1_r2, 2, 8, 1, 2)
ALISE_PREFILL_KERNEL(prefill_attn_kernel_g2_r2, 2, 8, 2, 2)
// INT4 with groups of 32 channels: four scale groups per head, one row tile per wave.
ALISE_PREFILL_KERNEL(prefill_attn_kernel_i4, 3, 4, 4, 1)
// INT4 with groups of 64 and 128 channels: two scale groups per head, or one
ALISE_PREFILL_KERNEL(prefill_attn_kernel_i4_g2, 3, 4, 2, 1)
ALISE_PREFILL_KERNEL(prefill_attn_kernel_i4_g1, 4, 4, 1, 1)
ALISE_PREFILL_KERNEL(prefill_attn_kernel_i4_g2_r2, 2, 4, 2, 2)
ALISE_PREFILL_KERNEL(prefill_attn_kernel_i4_g1_r2, 2, 4, 1, 2)
#undef ALISE_PREFILL_KERNEL

}  // namespace

bool prefill_mfma_applies(const CacheView &c, int32_t H)
{
    const int qper = H / c.Hkv;
    if (c.D != 128 || c.P < 16 || qper < 1 || qper > 16) return false;
    return (c.bits == 8 && (c.G == 128 || c.G == 64)) || (c.bits == 4 && (c.G == 128 || c.G == 64 || c.G == 32));
}

// Query tokens per workgroup: four waves of `row_tiles` 16-row tiles, a row being a (token, head of the group) pair.
int32_t prefill_tokens_per_workgroup(int32_t qper, int32_t row_tiles) { return 4 * (16 * row_tiles / qper); }

// Row tiles per wave: two, unless ALISE_PREFILL_ROW_TILES=1 (for tuning).
static int32_t prefill_row_tiles() { return tuning().prefill_row_tiles; }

// ALISE_PREFILL_WEIGHTS=single: one rounded fp16 number per weight instead of a high and a low part
// (faster; adds up to 2^-12 max|v| to the error of a row that a few tokens dominate).
static bool prefill_split_weights() { return tuning().prefill_split_weights; }

hipError_t launch_prefill_attn(const CacheView &c, const void *q, void *out, const int32_t *q_start,
                               const int32_t *block_tables, int32_t max_blocks, const int32_t *context_lens,
                               int32_t B, int32_t H, int32_t max_context_len, float softmax_scale,
                               const PrefillWorkspace &ws, hipStream_t s)
{
    if (B == 0 || ws.max_tiles == 0) return hipSuccess;
    PrefillParams p;
    p.c = c;
    p.q = static_cast<const _Float16 *>(q);
    p.out = static_cast<_Float16 *>(out);
    p.q_start = q_start;
    p.block_tables = block_tables;
    p.context_lens = context_lens;
    p.max_blocks = max_blocks;
    p.B = B;
    p.H = H;
    p.qper = H / c.Hkv;
    p.max_len = max_context_len;
    p.scale_log2e = softmax_scale * 1.44269504088896340736f;
    p.ws = ws;
    const int32_t rt = (c.bits == 4 && c.D / c.G == 4) ? 1 : prefill_row_tiles();     // four scale groups: one row tile
    hipLaunchKernelGGL(prefill_plan_kernel, dim3(1), dim3(1024), 0, s, q_start, context_lens, B,
                       prefill_tokens_per_workgroup(p.qper, rt), max_context_len, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)ws.max_tiles * (unsigned)c.Hkv);        // sized for one row tile per wave: enough for two
    const bool one_group = c.D / c.G == 1;
    const bool split = prefill_split_weights();
#define ALISE_PREFILL_LAUNCH(NAME)                                                    \
    do {                                                                              \
        if (split) hipLaunchKernelGGL(NAME, grid, dim3(256), 0, s, p);                \
        else hipLaunchKernelGGL(NAME##_w1, grid, dim3(256), 0, s, p);                 \
    } while (0)
    if (c.bits == 4) {
        if (c.D / c.G == 4) ALISE_PREFILL_LAUNCH(prefill_attn_kernel_i4);
        else if (c.D / c.G == 2 && rt == 1) ALISE_PREFILL_LAUNCH(prefill_attn_kernel_i4_g2);
        else if (c.D / c.G == 2) ALISE_PREFILL_LAUNCH(prefill_attn_kernel_i4_g2_r2);
        else if (rt == 1) ALISE_PREFILL_LAUNCH(prefill_attn_kernel_i4_g1);
        else ALISE_PREFILL_LAUNCH(prefill_attn_kernel_i4_g1_r2);
    } else if (rt == 1) {
        if (one_group) ALISE_PREFILL_LAUNCH(prefill_attn_kernel_g1);
        else ALISE_PREFILL_LAUNCH(prefill_attn_kernel_g2);
    } else {
        if (one_group) ALISE_PREFILL_LAUNCH(prefill_attn_kernel_g1_r2);
        else ALISE_PREFILL_LAUNCH(prefill_attn_kernel_g2_r2);
    }
#undef ALISE_PREFILL_LAUNCH
    return hipGetLastError();
}

}  // namespace alise
