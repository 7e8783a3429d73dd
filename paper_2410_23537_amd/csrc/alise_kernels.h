// Internal launch interface between the C-ABI layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace alise {

// Geometry of the compressed cache, validated by the ABI layer.
struct CacheView {
    uint8_t *k_codes, *v_codes;
    uint32_t *k_meta, *v_meta;      // one dword per group: fp16 scale (low half), fp16 zero (high half)
    int32_t num_pages, P, logP, Hkv, D, bits, G, NG;
    int32_t row_code_bytes;         // D * bits / 8
    int32_t cstride, mstride;       // bytes between consecutive (page, head) blocks of the codes / meta arrays
};

// Workspace carved up by the ABI layer for one attention call.
struct AttnWorkspace {
    int32_t *n_items;       // [1]  tiles * H, written by the plan kernel
    int32_t *tile_base;     // [B+1] first tile of each request (exclusive scan of tile counts)
    int32_t *req_full_base; // [B] scratch of the plan kernel: first full tile of each request in the work order
    int32_t *n_merge;       // [1] requests with more than one split (0: the merge has nothing to do)
    int32_t *n_shared;      // [1] items before this one are dealt out among all waves, the rest among the favoured half
    int4 *order;            // [max_tiles] work order: (request, first token, end token, split buffer index or -1)
    float *part;            // [max_tiles * H][D + 2] = (m, l, o[D]) of every split
    int32_t max_tiles;
    int32_t chunk_tokens;   // largest tokens per split; the plan kernel halves it (down to min_chunk_tokens)
    int32_t min_chunk_tokens;   // while the batch would give fewer than min_items work items
    int32_t min_items;
    int32_t skew_permille;  // share of the work (its shortest items) that goes to the favoured waves only
};

// The tuning environment (ALISE_* variables), read once per process by the C-ABI layer.
struct Tuning {
    int32_t split_tokens = 0, split_tokens_gqa = 0;     // 0: chosen from the batch
    int32_t waves_per_cu = 0, loads_per_block = 0, min_items_per_wave = 0;
    int32_t xcd_skew_permille = 50;
    int32_t prefill_row_tiles = 2;
    bool prefill_split_weights = true;
    bool debug_validate = false;
};
const Tuning &tuning();

// Work items below which the plan kernel shortens the splits: every wave of a full grid (about eight waves per
// compute unit) should get ALISE_MIN_ITEMS_PER_WAVE items, by default four, or one on the matrix-core path, whose
// items are heavier to start.
inline int32_t plan_min_items(int32_t num_cus, bool gqa)
{
    const int32_t per_wave = tuning().min_items_per_wave;
    return num_cus * 8 * (per_wave > 0 ? per_wave : (gqa ? 1 : 4));
}

// True when the attention call takes the matrix-core path for grouped-query layouts
// (its tiles are shorter, so the workspace is carved differently).
bool gqa_mfma_applies(const CacheView &c, int32_t H);

hipError_t launch_quant_write(const CacheView &c, const void *k, const void *v,
                              const int64_t *slot_mapping, int32_t T, hipStream_t s);

// Workspace of one chunked-prefill call.
struct PrefillWorkspace {
    int32_t *n_tiles;       // [1] workgroup tiles in the table, written by the plan kernel
    int2 *table;            // [max_tiles] (request, row tile of the request's chunk)
    int32_t max_tiles;
};

// Shapes the matrix-core prefill kernels take (D = 128, P >= 16, 1..16 query heads per KV head; INT8 with G in {64, 128},
// INT4 with G in {32, 64, 128}).
bool prefill_mfma_applies(const CacheView &c, int32_t H);
int32_t prefill_tokens_per_workgroup(int32_t qper, int32_t row_tiles);

hipError_t launch_prefill_attn(const CacheView &c, const void *q, void *out, const int32_t *q_start,
                               const int32_t *block_tables, int32_t max_blocks, const int32_t *context_lens,
                               int32_t B, int32_t H, int32_t max_context_len, float softmax_scale,
                               const PrefillWorkspace &ws, hipStream_t s);

// Bytes of one (page, head) block in the offloaded form of a request.
int64_t swap_block_bytes(const CacheView &c);

// Gather (upload = false) or scatter (upload = true) the pages of one request; `packed` is
// device-accessible memory.
hipError_t launch_swap(const CacheView &c, const int32_t *block_table, int32_t num_tokens, void *packed,
                       bool upload, int32_t num_cus, hipStream_t s);

hipError_t launch_dequant_page(const CacheView &c, int32_t page, void *k_out, void *v_out,
                               hipStream_t s);

hipError_t launch_decode_attn(const CacheView &c, const void *q, void *out,
                              const int32_t *block_tables, int32_t max_blocks,
                              const int32_t *context_lens, int32_t B, int32_t H,
                              int32_t max_context_len, float softmax_scale,
                              const AttnWorkspace &ws, int32_t num_cus, int32_t waves_per_cu,
                              int32_t loads_per_block, int32_t phases, hipStream_t s);
// phases of launch_decode_attn: the plan (needs only the lengths; q, out and block_tables may be null) and the run;
// kPhaseKeepNegative: a request with a negative length is no request at all and its output row is left alone (by default it
// is an empty request and gets a zero row)
constexpr int32_t kPhasePlan = 1, kPhaseRun = 2, kPhaseKeepNegative = 4;

// Chunked prefill on the single-query kernel: writes, for every query token t of every chunk (rows q_start[i] .. q_start[i+1]-1
// belong to request i, whose chunk ends at its last cached token), lens[t] = its position + 1 and copies the entries of its
// request's block-table row that this length reaches into tables[t][...]; rows that no chunk owns get lens[t] = -1.
hipError_t launch_prefill_expand(const CacheView &c, const int32_t *q_start, const int32_t *block_tables, int32_t max_blocks,
                                 const int32_t *context_lens, int32_t B, int32_t total_q, int32_t max_context_len,
                                 int32_t *lens, int32_t *tables, int32_t blocks_per_row, hipStream_t s);

}  // namespace alise
