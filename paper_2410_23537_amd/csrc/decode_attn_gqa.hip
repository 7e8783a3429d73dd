// Paged single-query attention for grouped-query layouts on the gfx950 matrix cores.
//
// With H / Hkv = qper query heads per KV head, every KV byte is used by qper queries, so
// q K^T and P V are real (small) matrix products (ALISE Sec. 2, Eq. 1-2, over the quantized
// cache of Sec. 3.2: INT8 with groups of 64 or 128 channels, INT4 with groups of 32, 64 or 128 -- see the note at the kernel).  One wave serves all query heads of one KV head for one tile of
// tokens; the work items of a tile are its KV heads.  Per step of 32 tokens:
//
//   S^T = K Q^T   v_mfma_f32_16x16x32_f16, A = K codes as fp16 (16 tokens x 32 channels),
//                 B = Q^T (32 channels x 16 query heads, the heads past qper are zero).
//                 The result has a query head per lane column and 4 tokens per lane, which
//                 is exactly the A-operand layout the second product needs for P.
//   O  += P V     A = p * lambda_v as fp16 (split into high and low parts so that no
//                 weight loses precision), B = V codes (32 tokens x 16 channels).
//
// The cache reaches the wave through LDS, by direct global -> LDS loads of 1 KiB (8 token
// rows) per instruction: fully coalesced, no vector registers in between, so the depth of
// the prefetch costs LDS space only.  (Fetching the operands in their matrix layouts
// straight from memory -- a 16-byte piece of 16 different rows per quarter wave -- kept the
// address unit busy over 70 % of the time and capped the kernel near 4.2 TB/s.)  The 16-byte
// pieces of a row are stored XOR-swizzled by the row number, which is free on the way in
// (a lane chooses which piece it fetches) and makes the operand reads conflict-free:
//   K: a lane reads 2 x 16 bytes of one token's row; a byte permute widens each code to the
//      fp16 subnormal code * 2^-24, which the matrix cores multiply exactly.  (The 1024 + code
//      form of the vector kernel would put a 1024 * sum(q) offset into the accumulator, and
//      its rounding -- harmless for small scales -- shows in the scores when outlier channels
//      make lambda_k large.)
//   V: the product contracts over tokens, but a row holds channels.  A lane reads one dword
//      (4 channels) from each of its 8 tokens and a byte permute picks the same channel out
//      of two dwords, leaving the fp16 subnormals code * 2^-24 of two tokens side by side --
//      which is the operand layout.  The matrix cores multiply subnormals exactly.
//
// A wave owns a fixed list of items (dealt out by rank in the longest-first order, odd
// rounds in reverse wave order) and treats it as one stream of steps: the producer side of
// the loop runs S - 1 steps ahead of the consumer side, across item boundaries.  What an
// item needs besides the cache (descriptor, block-table entries, query rows) also arrives
// by direct loads, ahead of time, into small rings beside the stages.  No load in the loop
// returns into a register, so the compiler places no wait of its own; every wait is placed
// here from a running count of issued loads.
//
// Softmax state (running maximum, denominator, weighted zero-points) lives in the lanes of
// the S^T layout and is brought to the rows of O only at the end of a tile.
#include "mfma_stream.h"
#include <atomic>
#include <type_traits>

namespace alise {
namespace {

// BITS = code width (8, or 4 with two channels per byte); NGRP = groups per token row (1, 2 or 4);
// QROWS = query rows kept per item (8 or 16, >= qper); S = stages of one step each.
//
// INT4 (groups of 32, 64 or 128 channels: four, two or one accumulator per tile).  A token's row is 64 bytes, so one 1 KiB load brings a whole
// 16-token tile; row r keeps its 16-byte piece c at position c ^ (r / 4 % 4).  K: chunk j of the
// first product is the 32 channels of piece j (one scale group); a lane's dword of it holds 8
// nibbles, which two masks on the dword and two on the dword shifted by a byte turn into fp16
// pairs code * 2^-24 (even channels) and 16 code * 2^-24 (odd channels) -- k-slots in the order
// 0 4 1 5 2 6 3 7, Q permuted likewise with its odd channels divided by 16.  V: the columns of a
// product are 16 channels of one 32-channel block b: lane n takes byte n % 4 of dword n / 4 of the
// block, i.e. channels 32 b + 2 n and 32 b + 2 n + 1 -- the low nibbles go to one product, the high
// nibbles (times 16, undone at the output) to another.
template <int BITS, int NGRP, int QROWS, int S>
__global__ __launch_bounds__(64) void decode_attn_gqa_kernel(AttnParams p)
{
    constexpr int D = 128, ROWB = D * BITS / 8;
    // one 16-token tile in LDS: K codes | V codes | K meta | V meta (INT8, two groups: 2 KiB | 2 KiB | 128 B | 128 B)
    constexpr int T_V = 16 * ROWB, T_KM = 32 * ROWB, T_VM = T_KM + 64 * NGRP;
    constexpr int TILEB = BITS == 8 ? 4352 : T_VM + 64 * NGRP;
    static_assert(TILEB % 128 == 0 && TILEB >= T_VM + 64 * NGRP, "tile layout");
    constexpr int STEPB = 2 * TILEB;
    constexpr int LOADS_PER_STEP = BITS == 8 ? 12 : 8;       // direct loads of one step
    constexpr int RD = 4, RG = 2, RQ = 1;       // rings: descriptors, page windows, query rows
    constexpr int QSLOT = QROWS * 256;
    // PACKED (INT4, at most 8 query heads per KV head).  A 16 x 16 tile of S^T has room for 16 query heads, and with 8
    // of them half of every step's score, exponential and weight arithmetic -- which is what this kernel's time goes
    // into: the vector-instruction issue is busy two thirds of the time, the matrix cores an eighth -- would be spent on
    // columns that hold no head.  So the first product is laid out block-diagonally: its 32 k-slots are 16 channels
    // of a token of the step's first tile (quarters 0 and 1 of the wave) and the same 16 channels of a token of the
    // second tile (quarters 2 and 3); column n < 8 of Q^T carries head n in the first half of the k-slots and zeros
    // in the second, column n >= 8 head n - 8 in the second half.  One product then gives 16 tokens x 8 heads of the
    // first tile in columns 0..7 and of the second tile in columns 8..15: eight products of 16 channels per step, as
    // before, but one accumulator tile per scale group instead of two half-empty ones, and four useful scores per
    // lane instead of eight half-useful ones.  The weights of column n + 8 travel to lane n (a rotation by 8 inside
    // the row of 16 lanes) to complete the A operand of the second product, whose k-slot order -- four tokens of the
    // first tile, then four of the second -- is the one it had.  Columns n and n + 8 are the same head: they share one
    // softmax reference, and their denominators and zero-point sums are added at the end.  The second product has the
    // same spare half: rows 8..15 of its A operand belong to no head, so they carry the low parts of the weights and
    // one product per V operand does what took two (the low sums land in rows 8..15 of O and join rows 0..7 at the
    // end of the item).  On this chip matrix and vector instructions of a SIMD's waves hardly overlap (a probe with
    // independent chains of both: 8.4 ms together against 5.5 and 4.8 ms alone), so every instruction saved counts.
    constexpr bool PACKED = BITS == 4 && QROWS == 8;
    constexpr int NQ = PACKED ? 8 : 4;          // products (k-chunks) per tile of S^T
    constexpr int OFF_DESC = S * STEPB, OFF_PG = OFF_DESC + RD * 16, OFF_Q = OFF_PG + RG * 256;
    static_assert(S >= 2 && S <= 4, "stage marks occupy four lanes");
    __shared__ __attribute__((aligned(128))) uint8_t lds[OFF_Q + RQ * QSLOT];

    const int lane = threadIdx.x;
    const int n = lane & 15;        // column of the matrix layouts: token (K), query head (S^T), channel (V, O)
    const int g = lane >> 4;        // quarter of the wave: 8 consecutive k-slots, 4 consecutive rows
    const int logP = p.c.logP, P = p.c.P, Hkv = p.c.Hkv, qper = p.qper, H = p.H;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)lds;
    lptr_t const ldsp = (lptr_t)lds;
    const int n_items = *p.ws.n_items;
    const uint32_t *order_words = reinterpret_cast<const uint32_t *>(p.ws.order);

    // ---- per-lane constants of the LDS layout.  A 1 KiB load covers 8 token rows; row r keeps
    // its 16-byte piece c at position c ^ r.  The array starts on a 128-byte boundary and every
    // stage, tile and row is a multiple of 128 bytes long, so the swizzle of an address is an
    // exclusive-or of its bits 4..6 with the row number.
    // what this lane fetches of a 1 KiB load
    const int src_lane = BITS == 8 ? (lane >> 3) * ROWB + (((lane & 7) ^ (lane >> 3)) * 16)
                                   : (lane >> 2) * ROWB + (((lane & 3) ^ ((lane >> 4) & 3)) * 16);
    // K operand, INT8: row n, pieces g and 4 + g (the second: the first with bit 6 flipped);
    // INT4: row n, dword g of piece j at (k_rd ^ 16 j)
    const uint32_t k_rd = BITS == 8 ? (n >> 3) * 1024 + ((n & 7) * 8 + (g ^ (n & 7))) * 16
                                    : n * 64 + ((n >> 2) & 3) * 16 + g * 4;
    // V operand, INT8: rows 4g + r, channels 64 * set + 4n .. (a dword): row r of set `set` sits at (v_rd ^ (16 r + 64 set)) + 128 r;
    // INT4: rows 4g + r, dword n / 4 of block b at (v_rd ^ 16 b) + 64 r
    const uint32_t v_rd = BITS == 8 ? T_V + (g >> 1) * 1024 + (g & 1) * 512 + (((n >> 2) ^ ((g & 1) * 4)) * 16) + (n & 3) * 4
                                    : T_V + g * 256 + g * 16 + (n >> 2) * 4;
    // PACKED: token n of tile g / 2; of piece j (at ^ 16 j) the dwords g % 2 and 2 + g % 2.  (Letting the quarters of the
    // second tile read the two dwords in the other order, so that the lanes of one read spread over 32 banks instead of 16,
    // took eight single reads instead of four double ones and measured the same.)
    const uint32_t k_rd_p = (g >> 1) * TILEB + n * 64 + ((n >> 2) & 3) * 16 + (g & 1) * 4;
    const uint32_t m_rd = g * 16 * NGRP + (PACKED ? (n >> 3) * TILEB : 0);        // meta of this lane's 4 tokens (PACKED: of the tile its column belongs to)
    const uint32_t v_sel = 0x0c000c00u | ((4u + (n & 3)) << 16) | (uint32_t)(n & 3);     // INT4: byte n % 4 of two dwords into the low bytes of two halves

    // ---- this wave's list of items (an item is a tile for one KV head)
    const int W = gridDim.x, w = blockIdx.x;
    auto item_at = [&](int r) {
        const int it = r * W + ((r & 1) ? W - 1 - w : w);
        return it < n_items ? it : -1;              // once -1, -1 for every later round
    };
    if (item_at(0) < 0) return;

    // ---- issue counts.  `marks` is a lane-indexed table of the value of `issued` when a
    // thing was issued: lanes 0..3 descriptors, 16..17 page windows, 20 query rows, 32.. stages.
    int issued = 0;
    int marks = 0;
    auto set_mark = [&](int idx) { marks = lane == idx ? issued : marks; };
    auto newer_than = [&](int idx) { return issued - __builtin_amdgcn_readlane(marks, idx); };

    auto issue_desc = [&](int r) {
        const int it = item_at(r);
        if (it < 0) return;
        if (lane < 4) dma4(order_words + (it / Hkv) * 4 + lane, ldsp + OFF_DESC + (r % RD) * 16);
        issued += 1;
        set_mark(r % RD);
    };
    auto read_desc = [&](int r) {
        const uint4 d = lds_read16(lds0 + OFF_DESC + (r % RD) * 16);
        // Clamped to what the plan kernel can write, so that every address derived from a
        // descriptor stays inside the caller's buffers whatever the bytes in LDS are.
        int4 c;
        c.x = min(max(__builtin_amdgcn_readfirstlane((int)d.x), 0), p.B - 1);
        c.y = min(max(__builtin_amdgcn_readfirstlane((int)d.y), 0), p.max_len - 1) & ~15;     // tiles start on a multiple of the split
        c.z = min(max(__builtin_amdgcn_readfirstlane((int)d.z), c.y + 1), min(c.y + p.ws.chunk_tokens, p.max_len));
        c.w = min(max(__builtin_amdgcn_readfirstlane((int)d.w), -1), p.ws.max_tiles - 1);
        return c;
    };
    // block-table entries of the item's tile (at most 64 pages)
    auto issue_pg = [&](int r) {
        if (item_at(r) < 0) return;
        const int4 d = read_desc(r);
        const int32_t *bt = p.block_tables + (int64_t)d.x * p.max_blocks;
        dma4(bt + min((d.y >> logP) + lane, (d.z - 1) >> logP), ldsp + OFF_PG + (r % RG) * 256);
        issued += 1;
        set_mark(16 + r % RG);
    };
    // the query rows of the item's KV head: row j = 256 bytes, QROWS of them (rows past qper repeat the first)
    auto issue_q = [&](int r, int i, int hk) {
#pragma unroll
        for (int c = 0; c < QROWS / 4; ++c) {
            const int row = c * 4 + g;
            const _Float16 *src = p.q + ((int64_t)i * H + hk * qper + (row < qper ? row : 0)) * D + n * 8;
            dma16(src, ldsp + OFF_Q + (r % RQ) * QSLOT + c * 1024);
        }
        issued += QROWS / 4;
        set_mark(20 + r % RQ);
    };

    // ---- producer state: the item being fetched
    int pr = -1, p_valid = 1, p_next = 0, p_hk = 0, p_t0 = 0, p_t1 = 0, p_ns = 1, p_s = 0, p_win = 0, p_pg = 0;
    int steps_issued = 0, steps_consumed = 0, c_entered = 0;
    // Entering item r overwrites the query rows of item r - RQ, which the consumer must have
    // taken into registers already.
    auto producer_may_enter = [&](int r) { return r - RQ < c_entered; };
    auto producer_enter = [&](int r) {
        pr = r;
        const int it = item_at(r);
        p_valid = it >= 0;
        p_next = 0;
        issue_desc(r + 2);
        if (item_at(r + 1) >= 0) {
            wait_newer(newer_than((r + 1) % RD));
            issue_pg(r + 1);
        }
        if (!p_valid) return;
        wait_newer(newer_than(16 + r % RG));        // covers the descriptor too: it was issued earlier
        const int4 d = read_desc(r);
        p_hk = it % Hkv;
        p_t0 = d.y;
        p_t1 = d.z;
        p_ns = (d.z - d.y + kStep - 1) / kStep;
        p_win = d.y >> logP;
        p_s = 0;
        p_pg = (int)lds_read4(lds0 + OFF_PG + (r % RG) * 256 + lane * 4);
        issue_q(r, d.x, p_hk);
    };
    // one step of the producer's item into the next stage
    auto produce = [&]() {
        const int st = steps_issued % S;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            int tx = p_t0 + p_s * kStep + x * 16;
            if (tx >= p_t1) tx -= 16;                       // second tile starts past the end: repeat the first
            const int page = min(max(__builtin_amdgcn_readlane(p_pg, (tx >> logP) - p_win), 0), p.c.num_pages - 1);
            const int blk = page * Hkv + p_hk;
            const int off = tx & (P - 1);
            const int64_t co = (int64_t)blk * p.c.cstride + (int64_t)off * ROWB;
            const int64_t mo = (int64_t)blk * p.c.mstride + (int64_t)off * NGRP * 4;
            lptr_t dst = ldsp + st * STEPB + x * TILEB;
            const uint8_t *kb = p.c.k_codes + co + src_lane;
            const uint8_t *vb = p.c.v_codes + co + src_lane;
            dma16_stream(kb, dst);
            if constexpr (BITS == 8) dma16_stream(kb + 1024, dst + 1024);
            dma16_stream(vb, dst + T_V);
            if constexpr (BITS == 8) dma16_stream(vb + 1024, dst + T_V + 1024);
            if (lane < 16 * NGRP) {
                dma4_stream(reinterpret_cast<const uint8_t *>(p.c.k_meta) + mo + lane * 4, dst + T_KM);
                dma4_stream(reinterpret_cast<const uint8_t *>(p.c.v_meta) + mo + lane * 4, dst + T_VM);
            }
        }
        issued += LOADS_PER_STEP;
        set_mark(32 + st);
        ++steps_issued;
        if (++p_s == p_ns) p_next = 1;                      // the item is fetched; the next one is entered when allowed
    };
    // keep the stages full
    auto fill = [&]() {
        for (;;) {
            if (p_next) {
                if (!producer_may_enter(pr + 1)) break;
                producer_enter(pr + 1);
            }
            if (!p_valid || steps_issued - steps_consumed >= S) break;
            produce();
        }
    };

    // ---- start: descriptors of the first items, the first page window
    issue_desc(0);
    issue_desc(1);
    ALISE_VMCNT(0);
    issue_pg(0);
    producer_enter(0);
    // the consumer of the step that is about to be eaten must not be overwritten: at most S - 1 ahead here
    for (;;) {
        if (p_next) {
            if (!producer_may_enter(pr + 1)) break;
            producer_enter(pr + 1);
        }
        if (!p_valid || steps_issued >= S - 1) break;
        produce();
    }

    // ---- consumer
    for (int cr = 0;; ++cr) {
        const int it = item_at(cr);
        if (it < 0) break;                          // wave-uniform
        const int4 cd = read_desc(cr);              // landed before the producer entered the item
        const int i = cd.x, t0 = cd.y, t1 = cd.z, part = cd.w;
        const int hk = it % Hkv;
        const int nsteps = (t1 - t0 + kStep - 1) / kStep;

        // ---- Q^T as the B operand of the four k-chunks: chunk j, slot g*8+e <-> channel (j/2)*64 + g*16 + (j%2)*8 + e
        h8_t qop[NQ];
        float qs[NGRP];             // sum of this query head's q over the channels of a group
        {
            wait_newer(newer_than(20 + cr % RQ));
            // query row n sits at (n / 4) * 1024 + (n % 4) * 256 of the slot: row c*4+g was written by quarter g of load c
            const uint32_t qa = lds0 + OFF_Q + (cr % RQ) * QSLOT + ((n % QROWS) >> 2) * 1024 + (n & 3) * 256;
            uint4 raw[NQ];
            // INT8: chunk j, slot g*8+e <-> channel (j/2)*64 + g*16 + (j%2)*8 + e;  INT4: channel 32 j + 8 g + {0 4 1 5 2 6 3 7}[e];
            // PACKED: product j, slot g*8+e <-> channel 16 j + 8 (g % 2) + {0 4 1 5 2 6 3 7}[e] of head n % 8, for the quarters of the column's tile
            if constexpr (PACKED) {
                const uint32_t qh = qa + (g & 1) * 16;
                lds_read16x4(qh, qh + 32, qh + 64, qh + 96, raw[0], raw[1], raw[2], raw[3]);
                lds_read16x4(qh + 128, qh + 160, qh + 192, qh + 224, raw[NQ - 4], raw[NQ - 3], raw[NQ - 2], raw[NQ - 1]);
            } else if constexpr (BITS == 8) lds_read16x4(qa + g * 32, qa + g * 32 + 16, qa + 128 + g * 32, qa + 128 + g * 32 + 16, raw[0], raw[1], raw[2], raw[3]);
            else lds_read16x4(qa + g * 16, qa + 64 + g * 16, qa + 128 + g * 16, qa + 192 + g * 16, raw[0], raw[1], raw[2], raw[3]);
            float part_sum[NGRP];
#pragma unroll
            for (int gr = 0; gr < NGRP; ++gr) part_sum[gr] = 0.0f;
            const bool q_here = PACKED ? ((n & 7) < qper && (g >> 1) == (n >> 3)) : n < qper;
#pragma unroll
            for (int j = 0; j < NQ; ++j) {
                h8_t v = pack8(raw[j].x, raw[j].y, raw[j].z, raw[j].w);
                if (!q_here) v = (h8_t)(_Float16)0.0f;
                float sacc = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) sacc += (float)v[e];
                part_sum[j * NGRP / NQ] += sacc;
                if constexpr (BITS == 4) {
                    const _Float16 sixteenth = (_Float16)0.0625f;       // the odd nibbles arrive 16 times too large
                    const h8_t w = {v[0], v[4], v[1] * sixteenth, v[5] * sixteenth, v[2], v[6], v[3] * sixteenth, v[7] * sixteenth};
                    v = w;
                }
                qop[j] = v;
            }
#pragma unroll
            for (int gr = 0; gr < NGRP; ++gr) {
                float v = part_sum[gr];
                v += __shfl_xor(v, 16);
                v += __shfl_xor(v, 32);
                qs[gr] = v;
            }
        }
        // Scores are kept in the units of the accumulator: t = sum_g lambda_k (acc_g - z_k sum(q_g) 2^-24), the true
        // score being t * scale24 (the softmax scale, log2 e and the 2^24 that the subnormal K codes lack).
        const float scale24 = p.scale_log2e * 16777216.0f;
        const float inv24 = 1.0f / scale24;
        const float lazy_t = kLazy * inv24;
        float nqs24[NGRP];                      // -sum(q) 2^-24
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) nqs24[gr] = -qs[gr] * (1.0f / 16777216.0f);
        ++c_entered;

        // m_ref: the running maximum in the units of t.  c_ref = bias - m_ref scale24: a weight is 2^(t scale24 + c_ref),
        // so -c_ref is the reference that the denominator and the sums are relative to.
        float m_ref = kFloor * inv24, l_part = 0.0f, z_part[NGRP];
        float bias = kWeightBias;           // see kWeightBias; wave-uniform
        float c_ref = __builtin_fmaf(-m_ref, scale24, bias);
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) z_part[gr] = 0.0f;
        f4_t o[8];                  // [set*4 + nu]: rows = query heads 4g..4g+3, column n <-> channel 64*set + 4n + nu
#pragma unroll
        for (int t = 0; t < 8; ++t) o[t] = (f4_t)0.0f;

        // One step of 32 tokens out of the LDS stage at `base`.  MASKED: the item's last step, which may hold
        // tokens past the item's end; the other steps spend no comparison and no select.
        auto step = [&](auto masked_c, int k, uint32_t base) {
            constexpr bool MASKED = decltype(masked_c)::value;
            // ---- S^T = K Q^T for the two 16-token tiles (PACKED: both tiles in one, see above)
            constexpr int NX = PACKED ? 1 : 2;      // tiles of S^T per step
            float s[NX][4];
            uint32_t vmraw[NX][4][NGRP];       // V (scale, zero) dwords of this lane's tokens; 0 where the token is masked
            float mx = kNegInf;
            uint4 kp[2][2];                // INT8: [tile][piece];  INT4: kp[tile][0] holds the dwords of the four chunks
            uint32_t kd[4][2];             // PACKED: [piece][which of this lane's two dwords of it]
            const uint32_t ka0 = base + k_rd, ma = base + m_rd;
            if constexpr (PACKED) {
                const uint32_t kb = base + k_rd_p;
                const uint32_t ka[4] = {kb, kb ^ 16u, kb ^ 32u, kb ^ 48u};
                lds_read2x4(ka, kd);
            } else if constexpr (BITS == 8) {
                const uint32_t ka1 = ka0 ^ 64u;
                lds_read16x4_at<0, 0, TILEB, TILEB>(ka0, ka1, ka0, ka1, kp[0][0], kp[0][1], kp[1][0], kp[1][1]);
            } else {
                const uint32_t ka[4] = {ka0, ka0 ^ 16u, ka0 ^ 32u, ka0 ^ 48u};
                uint32_t k0[4], k1[4];
                lds_read4x4x2<TILEB>(ka, k0, k1);
                kp[0][0] = make_uint4(k0[0], k0[1], k0[2], k0[3]);
                kp[1][0] = make_uint4(k1[0], k1[1], k1[2], k1[3]);
            }
            uint4 kmeta[NX][NGRP], vmeta[NX][NGRP];
            if constexpr (PACKED) {         // the four tokens of this lane's column: one tile's worth
                if constexpr (NGRP == 4) {
                    lds_read16x4_at<T_KM, T_KM + 16, T_KM + 32, T_KM + 48>(ma, ma, ma, ma, kmeta[0][0], kmeta[0][1], kmeta[0][2], kmeta[0][3]);
                    lds_read16x4_at<T_VM, T_VM + 16, T_VM + 32, T_VM + 48>(ma, ma, ma, ma, vmeta[0][0], vmeta[0][1], vmeta[0][2], vmeta[0][3]);
                } else if constexpr (NGRP == 2) {
                    lds_read16x4_at<T_KM, T_KM + 16, T_VM, T_VM + 16>(ma, ma, ma, ma, kmeta[0][0], kmeta[0][1], vmeta[0][0], vmeta[0][1]);
                } else {
                    lds_read16x2_at<T_KM, T_VM>(ma, ma, kmeta[0][0], vmeta[0][0]);
                }
            } else if constexpr (NGRP == 4) {
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
            for (int x = 0; x < NX; ++x) {
                f4_t acc[NGRP];
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) acc[gr] = (f4_t)0.0f;
#pragma unroll
                for (int j = 0; j < NQ; ++j) {
                    h8_t a;
                    if constexpr (PACKED) {
                        const uint32_t w0 = kd[j >> 1][j & 1], w1 = w0 >> 8;
                        a = pack8(w0 & 0x000F000Fu, w0 & 0x00F000F0u, w1 & 0x000F000Fu, w1 & 0x00F000F0u);
                    } else if constexpr (BITS == 8) {
                        const uint4 piece = kp[x][j / 2];
                        const uint32_t w0 = (j % 2) ? piece.z : piece.x, w1 = (j % 2) ? piece.w : piece.y;
                        a = pack8(__builtin_amdgcn_perm(0u, w0, 0x0c010c00u), __builtin_amdgcn_perm(0u, w0, 0x0c030c02u),
                                  __builtin_amdgcn_perm(0u, w1, 0x0c010c00u), __builtin_amdgcn_perm(0u, w1, 0x0c030c02u));
                    } else {
                        const uint4 d4 = kp[x][0];
                        const uint32_t w0 = j == 0 ? d4.x : j == 1 ? d4.y : j == 2 ? d4.z : d4.w, w1 = w0 >> 8;
                        a = pack8(w0 & 0x000F000Fu, w0 & 0x00F000F0u, w1 & 0x000F000Fu, w1 & 0x00F000F0u);
                    }
                    f4_t &dst = acc[j * NGRP / NQ];
                    dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, qop[j], dst, 0, 0, 0);
                }
                const int room = t1 - (t0 + k * kStep + (PACKED ? (n >> 3) : x) * 16 + g * 4);        // row r of this lane's S^T block is a token of the item iff r < room
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const bool valid = !MASKED || r < room;
                    float sv = 0.0f;
#pragma unroll
                    for (int gr = 0; gr < NGRP; ++gr) {
                        const h2_t kmh = as_h2(meta_of<NGRP>(kmeta[x], r, gr));     // the fp16 halves of the meta dword, read in place
                        const float u = __builtin_fmaf((float)kmh.y, nqs24[gr], acc[gr][r]);
                        sv = __builtin_fmaf((float)kmh.x, u, sv);
                        const uint32_t vm = meta_of<NGRP>(vmeta[x], r, gr);
                        vmraw[x][r][gr] = valid ? vm : 0u;
                    }
                    s[x][r] = valid ? sv : kNegInf;
                    mx = fmaxf(mx, s[x][r]);
                }
            }

            // ---- running maximum per query head, raised lazily; all four quarters hold the same value
            if (__builtin_amdgcn_ballot_w64(mx > m_ref + lazy_t) != 0) {
                float mq = fmaxf(mx, __shfl_xor(mx, 16));
                mq = fmaxf(mq, __shfl_xor(mq, 32));
                if constexpr (PACKED) mq = fmaxf(mq, __shfl_xor(mq, 8));        // columns n and n + 8 are the same head: one reference
                m_ref = (mq > m_ref + lazy_t) ? mq : m_ref;
                const float c_new = __builtin_fmaf(-m_ref, scale24, bias);
                const float f = __builtin_amdgcn_exp2f(c_new - c_ref);
                c_ref = c_new;
                l_part *= f;
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) z_part[gr] *= f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float fr = __shfl(f, 4 * g + r);          // factor of the query head in row 4g+r
#pragma unroll
                    for (int t = 0; t < 8; ++t) o[t][r] *= fr;
                }
            }

            // ---- a V scale of 2 or more in this step: the biased weights could leave the fp16 range (rare, wave-uniform)
            if (bias != 0.0f && __builtin_amdgcn_ballot_w64(max_low_half<NX * 4 * NGRP>(&vmraw[0][0][0]) >= 0x4000u) != 0) {
                bias = 0.0f;
                const float c_new = __builtin_fmaf(-m_ref, scale24, 0.0f);
                const float fb = __builtin_amdgcn_exp2f(c_new - c_ref);
                c_ref = c_new;
                l_part *= fb;
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) z_part[gr] *= fb;
#pragma unroll
                for (int t = 0; t < 8; ++t) o[t] *= fb;
            }

            // ---- weights p * lambda_v as fp16 high + low parts, in the A-operand order (tile, row).  The high
            // part is the product truncated to fp16, the low part what is left of the exact product.
            h8_t a_hi[NGRP], a_lo[NGRP];
            if constexpr (PACKED) {
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) a_hi[gr] = a_lo[gr] = (h8_t)(_Float16)0.0f;     // slots 4..7 are filled below
            }
#pragma unroll
            for (int x = 0; x < NX; ++x)
#pragma unroll
                for (int rr = 0; rr < 4; rr += 2) {
                    float pj[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        pj[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[x][rr + e], scale24, c_ref));
                        l_part += pj[e];
                    }
#pragma unroll
                    for (int gr = 0; gr < NGRP; ++gr) {
                        float wv[2];
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            const h2_t vmh = as_h2(vmraw[x][rr + e][gr]);
                            wv[e] = __builtin_fmaf((float)vmh.x, pj[e], 0.0f);
                            z_part[gr] = __builtin_fmaf((float)vmh.y, wv[e], z_part[gr]);
                        }
                        const h2_t hi = __builtin_bit_cast(h2_t, __builtin_amdgcn_cvt_pkrtz(wv[0], wv[1]));
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            a_hi[gr][x * 4 + rr + e] = hi[e];
                            a_lo[gr][x * 4 + rr + e] = (_Float16)__builtin_fmaf((float)as_h2(vmraw[x][rr + e][gr]).x, pj[e], -(float)hi[e]);
                        }
                    }
                }

            if constexpr (PACKED) {
                // One A operand instead of two.  Its rows 0..7 are the heads' high parts -- k-slots 0..3 the lane's own
                // (first tile), k-slots 4..7 the ones that column n + 8 holds for the same head (second tile) -- and its rows
                // 8..15, which no head uses, are the heads' LOW parts, so that one product per V operand accumulates the high
                // sums in rows 0..7 and the low sums in rows 8..15 of O; they are added at the end of the item.  Each dword is
                // one rotation by 8 inside the row of 16 lanes that only half of the lanes take (bank mask), the others keeping
                // their own part.
#pragma unroll
                for (int gr = 0; gr < NGRP; ++gr) {
                    typedef int32_t i4_t __attribute__((ext_vector_type(4)));
                    const i4_t hi = __builtin_bit_cast(i4_t, a_hi[gr]), lo = __builtin_bit_cast(i4_t, a_lo[gr]);
                    i4_t c;
                    c.x = __builtin_amdgcn_update_dpp(hi.x, lo.x, 0x128, 0xf, 0xc, false);      // lanes 8..15: the low part of lane n - 8
                    c.y = __builtin_amdgcn_update_dpp(hi.y, lo.y, 0x128, 0xf, 0xc, false);
                    c.z = __builtin_amdgcn_update_dpp(lo.x, hi.x, 0x128, 0xf, 0x3, false);      // lanes 0..7: the high part of lane n + 8
                    c.w = __builtin_amdgcn_update_dpp(lo.y, hi.y, 0x128, 0xf, 0x3, false);
                    a_hi[gr] = __builtin_bit_cast(h8_t, c);
                }
            }

            // ---- O += P V
            if constexpr (BITS == 8) {
                // byte nu of the dwords of two tokens -> two fp16 subnormals
                uint32_t va[8], vd[2][8];          // vd[tile][set * 4 + r]
                va[0] = v_rd + base;
#pragma unroll
                for (int t = 1; t < 8; ++t) va[t] = va[0] ^ (uint32_t)((t & 3) * 16 + (t >> 2) * 64);
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
                        f4_t &dst = o[set * 4 + nu];
                        dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_hi[gr], bv, dst, 0, 0, 0);
                        dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_lo[gr], bv, dst, 0, 0, 0);
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
                            f4_t &dst = o[b * 2 + m];
                            dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_hi[gr], bv, dst, 0, 0, 0);
                            if constexpr (!PACKED) dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_lo[gr], bv, dst, 0, 0, 0);
                        }
                    }
                }
            }
        };
        auto next_stage = [&]() -> uint32_t {
            fill();
            const int sg = steps_consumed % S;
            wait_newer(newer_than(32 + sg));
            return lds0 + sg * STEPB;
        };

        for (int k = 0; k < nsteps - 1; ++k) {
            const uint32_t base = next_stage();
            step(std::false_type{}, k, base);
            ++steps_consumed;
            // A wave lowers its own priority by a step with every 256 tokens it has done, wrapping after four: of the
            // waves of a SIMD the one that is behind goes first, so they finish together instead of the oldest long
            // before the youngest (see the vector kernel).
            if ((steps_consumed & 7) == 0) {        // wave-uniform; no memory operation inside
                switch ((steps_consumed >> 3) & 3) {
                case 0: __builtin_amdgcn_s_setprio(3); break;
                case 1: __builtin_amdgcn_s_setprio(2); break;
                case 2: __builtin_amdgcn_s_setprio(1); break;
                default: __builtin_amdgcn_s_setprio(0); break;
                }
            }
        }
        {
            const uint32_t base = next_stage();
            step(std::true_type{}, nsteps - 1, base);
            ++steps_consumed;
        }

        // ---- per query head: add the four quarters; then fetch the values of this lane's rows
        fill();                     // the stage just freed: keep loads in flight through the item's end and the next one's start
        if constexpr (PACKED) {        // rows 8..15 of O hold the sums of the low parts: quarter g + 2 has them for the rows of quarter g
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) o[t][r] += __shfl_xor(o[t][r], 32);
        }
        float l = l_part + __shfl_xor(l_part, 16);
        l += __shfl_xor(l, 32);
        if constexpr (PACKED) l += __shfl_xor(l, 8);       // the head's other column (the tokens of the second tiles)
        float zsum[NGRP];
#pragma unroll
        for (int gr = 0; gr < NGRP; ++gr) {
            float v = z_part[gr] + __shfl_xor(z_part[gr], 16);
            v += __shfl_xor(v, 32);
            if constexpr (PACKED) v += __shfl_xor(v, 8);
            zsum[gr] = v;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * g + r;                      // query head of the group
            const float l_row = __shfl(l, row);
            const float m_row = __shfl(-c_ref, row);             // the reference the denominator and the sums are relative to
            float z_row[NGRP];
#pragma unroll
            for (int gr = 0; gr < NGRP; ++gr) z_row[gr] = __shfl(zsum[gr], row);
            if (row < qper) {
                const int qh = hk * qper + row;
                if (part < 0) {
                    const float inv_l = 1.0f / l_row;
                    _Float16 *orow = p.out + ((int64_t)i * H + qh) * D;
                    if constexpr (BITS == 8) {
                        _Float16 *dst = orow + 4 * n;
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
#pragma unroll
                        for (int b = 0; b < 4; ++b) {           // column n of block b: channels 32 b + 2 n and 32 b + 2 n + 1
                            const float zr = z_row[b * NGRP / 4];
                            h2_t v;
                            v.x = (_Float16)(__builtin_fmaf(o[b * 2 + 0][r], 16777216.0f, -zr) * inv_l);
                            v.y = (_Float16)(__builtin_fmaf(o[b * 2 + 1][r], 1048576.0f, -zr) * inv_l);      // 2^24 / 16
                            *reinterpret_cast<h2_t *>(orow + 32 * b + 2 * n) = v;
                        }
                    }
                } else {
                    float *dst = p.ws.part + ((int64_t)part * H + qh) * (D + 2);
                    if (n == 0) { dst[0] = m_row; dst[1] = l_row; }
                    if constexpr (BITS == 4) {
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const float zr = z_row[b * NGRP / 4];
                            float2 v2;
                            v2.x = __builtin_fmaf(o[b * 2 + 0][r], 16777216.0f, -zr);
                            v2.y = __builtin_fmaf(o[b * 2 + 1][r], 1048576.0f, -zr);
                            *reinterpret_cast<float2 *>(dst + 2 + 32 * b + 2 * n) = v2;
                        }
                    } else
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
    }
    ALISE_VMCNT(0);     // nothing may still be on its way into LDS when the wave ends
}

template <int BITS, int NGRP, int QROWS, int S>
hipError_t launch_gqa_t(const AttnParams &p, int32_t num_cus, int32_t waves_per_cu, hipStream_t s)
{
    // one wave per workgroup; as many as the LDS lets a compute unit hold, unless the caller fixes the number
    // (asked once per kernel variant; two threads that ask at the same time store the same number)
    static std::atomic<int> resident{0};
    int occ = resident.load(std::memory_order_relaxed);
    if (occ == 0) {
        int n = 0;
        hipError_t oe = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, decode_attn_gqa_kernel<BITS, NGRP, QROWS, S>, 64, 0);
        occ = (oe == hipSuccess && n > 0) ? n : 4;
        resident.store(occ, std::memory_order_relaxed);
    }
    int waves = num_cus * (waves_per_cu > 0 ? waves_per_cu : occ);
    const int64_t max_items = (int64_t)p.ws.max_tiles * p.c.Hkv;
    if (waves > max_items) waves = (int)max_items;
    if (waves < 1) waves = 1;
    hipLaunchKernelGGL((decode_attn_gqa_kernel<BITS, NGRP, QROWS, S>), dim3(waves), dim3(64), 0, s, p);
    return hipGetLastError();
}

}  // namespace

bool gqa_mfma_applies(const CacheView &c, int32_t H)
{
    const int qper = H / c.Hkv;
    if (c.D != 128 || c.P < 16 || qper < 2 || qper > 16) return false;
    return (c.bits == 8 && (c.G == 128 || c.G == 64)) || (c.bits == 4 && (c.G == 128 || c.G == 64 || c.G == 32));
}

hipError_t launch_gqa_mfma(const AttnParams &p, int32_t num_cus, int32_t waves_per_cu, int32_t stages, hipStream_t s)
{
    const int ngrp = p.c.D / p.c.G;
    const bool small = p.qper <= 8;
#define ALISE_GQA_DISPATCH(SV)                                                                                        \
    do {                                                                                                              \
        if (p.c.bits == 4 && ngrp == 4)                                                                               \
            return small ? launch_gqa_t<4, 4, 8, SV>(p, num_cus, waves_per_cu, s) : launch_gqa_t<4, 4, 16, SV>(p, num_cus, waves_per_cu, s); \
        if (p.c.bits == 4 && ngrp == 2)                                                                               \
            return small ? launch_gqa_t<4, 2, 8, SV>(p, num_cus, waves_per_cu, s) : launch_gqa_t<4, 2, 16, SV>(p, num_cus, waves_per_cu, s); \
        if (p.c.bits == 4)                                                                                            \
            return small ? launch_gqa_t<4, 1, 8, SV>(p, num_cus, waves_per_cu, s) : launch_gqa_t<4, 1, 16, SV>(p, num_cus, waves_per_cu, s); \
        if (ngrp == 1)                                                                                                \
            return small ? launch_gqa_t<8, 1, 8, SV>(p, num_cus, waves_per_cu, s) : launch_gqa_t<8, 1, 16, SV>(p, num_cus, waves_per_cu, s); \
        return small ? launch_gqa_t<8, 2, 8, SV>(p, num_cus, waves_per_cu, s) : launch_gqa_t<8, 2, 16, SV>(p, num_cus, waves_per_cu, s);     \
    } while (0)
    // Two stages and more resident waves beat deeper prefetch with fewer waves (measured on the
    // 8-heads-per-KV-head workload: 209 us against 217-222 us for three and four stages).
    // INT4 stages are half the size and its steps are longer (four scale groups): three stages measured best there.
    if (stages == 0 && p.c.bits == 4) stages = 3;
    if (stages == 3) ALISE_GQA_DISPATCH(3);
    if (stages == 4) ALISE_GQA_DISPATCH(4);
    ALISE_GQA_DISPATCH(2);
#undef ALISE_GQA_DISPATCH
}

}  // namespace alise
