/*
 * alise_kv.h -- C ABI of the MI355X (gfx950) quantized, paged KV-cache decode path.
 *
 * The operations are the decode step of an LLM server that keeps its KV cache
 * compressed, and the movement of a preempted request's cache (ALISE, arXiv 2410.23537):
 *   - the cache stores b-bit integer codes with one (scale, zero-point) pair per
 *     group: x_q = round(x / lambda + z), x = lambda (x_q - z),
 *     lambda = (max - min) / (2^b - 1)                       [Sec. 3.2, "KV Compression"]
 *   - each decode iteration appends the new token's K/V to the cache and attends
 *     over all cached tokens                                  [Sec. 2, "LLM Inference"]
 *   - per head, Attn = softmax(q K^T / sqrt(d/h)) V; heads are concatenated
 *                                                             [Sec. 2, Eq. 1 and Eq. 2]
 *   - the cache is block-level (paged), as in PagedAttention  [Sec. 3.3]
 *
 * General rules
 *   - Every pointer named "device" is a HIP device pointer valid on the current
 *     device; every other pointer is a host pointer.  Nothing is retained after a
 *     call returns; the caller owns all buffers, including the workspace.
 *   - All calls enqueue work on `hip_stream` (a hipStream_t cast to void*, NULL =
 *     the default stream) and return without synchronising.
 *   - Return value: ALISE_OK or an error code below.  Arguments that can be
 *     checked on the host are checked before any HIP call, so the error paths
 *     need no GPU.  Contents of device arrays (slot or page indices out of range,
 *     duplicate slots in one call, context_lens[i] > max_context_len) are not
 *     checked: out-of-range indices are undefined behaviour; lengths above
 *     max_context_len are clamped to it.
 *   - With ALISE_DEBUG_VALIDATE=1 in the environment the calls check those contents
 *     too and return ALISE_INVALID_ARGUMENT without launching anything: slots outside
 *     the cache or used twice in one write, lengths outside [0, max_context_len],
 *     block-table entries that a length reaches outside [0, num_pages), a request
 *     longer than its block-table row, chunk boundaries that decrease or a chunk
 *     longer than its request, pages named twice in a swap, and -- for calls that run on
 *     the matrix cores -- a V scale of 256 or more among the tokens a length reaches (see
 *     "Value range" at alise_paged_decode_attn).  This copies the arrays
 *     to the host and waits for the stream: a debugging aid, not for serving.
 *
 * Exact arithmetic of the quantizer (so that codes and meta are reproducible bit
 * for bit).  With x_0..x_{G-1} one group widened to fp32, qmax = 2^bits - 1 and
 * every operation a single correctly rounded binary32 operation:
 *     mn = min(min_i x_i, 0)   mx = max(max_i x_i, 0)
 *     l32 = (mx - mn) / qmax
 *     scale = smallest fp16 >= l32, but at least 2^-14          (stored)
 *     inv = 1 / (float)scale
 *     zero = clamp(rint((-mn) * inv), 0, qmax)                   (stored as fp16, +0 if 0)
 *     code_i = clamp(rint(fma(x_i, inv, zero)), 0, qmax)         (rint: ties to even)
 * Dequantized value: (float)scale * (code - zero), exact in fp32.
 */
#ifndef ALISE_KV_H
#define ALISE_KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ALISE_OK = 0,
    ALISE_INVALID_ARGUMENT = 1,     /* null pointer, negative or inconsistent size            */
    ALISE_UNSUPPORTED = 2,          /* a shape outside the supported set listed below          */
    ALISE_WORKSPACE_TOO_SMALL = 3,
    ALISE_MISALIGNED = 4,           /* a pointer that must be 16-byte aligned is not           */
    ALISE_HIP_ERROR = 5             /* a HIP call or kernel launch failed                      */
};

/*
 * The compressed cache.  Caller-filled, passed by pointer, never retained.
 *
 * Layout (all device memory, row-major, 16-byte aligned bases):
 *   k_codes, v_codes : uint8 [num_pages][num_kv_heads][page_size][head_dim*bits/8]
 *                      bits = 4 packs channel 2i in the low nibble and channel
 *                      2i+1 in the high nibble of byte i.
 *   k_meta,  v_meta  : fp16  [num_pages][num_kv_heads][page_size][head_dim/group_size][2]
 *                      = (scale, zero-point) of each group of `group_size`
 *                      contiguous channels of one token's one head vector.
 * Slot s of the cache is page s / page_size, offset s % page_size.
 *
 * A (page, head) block is the [page_size][...] slab of one array.  The distance in bytes
 * between consecutive blocks is codes_block_stride for k_codes and v_codes and
 * meta_block_stride for k_meta and v_meta; 0 means dense (the shapes above, four separate
 * arrays).  Larger strides describe one allocation in which the four slabs of a (page, head)
 * pair sit next to each other -- block b at base + b * stride holds
 * [K codes | V codes | K meta | V meta], the four pointers name the four slabs of block 0 and
 * both strides equal the block size -- which is what the attention kernel streams best,
 * since a wave then reads one contiguous region per page.  Strides are multiples of 16 and at
 * least the dense slab size.
 *
 * Supported: bits in {4, 8}; head_dim in {64, 128}; group_size a divisor of
 * head_dim and a multiple of 128/bits (16 for INT8, 32 for INT4);
 * page_size a power of two in [8, 256]; num_pages * page_size < 2^31;
 * num_pages * num_kv_heads < 2^31; strides below 2^31.
 */
typedef struct alise_kv_cache {
    void *k_codes;
    void *v_codes;
    void *k_meta;
    void *v_meta;
    int32_t num_pages;
    int32_t page_size;
    int32_t num_kv_heads;
    int32_t head_dim;
    int32_t bits;
    int32_t group_size;
    int64_t codes_block_stride;     /* bytes; 0 = dense = page_size * head_dim * bits / 8      */
    int64_t meta_block_stride;      /* bytes; 0 = dense = page_size * (head_dim/group_size) * 4 */
} alise_kv_cache;

/* Bytes spanned by one codes array / one meta array of `c`, from its base pointer to the end
 * of its last block (0 if `c` is unsupported). */
size_t alise_kv_codes_bytes(const alise_kv_cache *c);
size_t alise_kv_meta_bytes(const alise_kv_cache *c);

/*
 * Quantize T new tokens and store them in the cache              [Sec. 3.2; Sec. 2]
 *   k, v          device, fp16 [T][num_kv_heads][head_dim], 16-byte aligned.
 *   slot_mapping  device, int64 [T]; token t goes to slot slot_mapping[t];
 *                 a negative slot skips the token.  Slots must be distinct.
 * Writes codes and meta of the addressed slots only.  T = 0 is a no-op.
 * K and V are finite numbers: a group that holds an infinity or a NaN gets unspecified codes, scale and
 * zero-point (nothing faults, the other groups are not affected).
 */
int alise_kv_quant_write(const alise_kv_cache *c, const void *k, const void *v,
                         const int64_t *slot_mapping, int32_t T, void *hip_stream);

/*
 * Workspace the attention call needs for these sizes (0 on invalid arguments).
 *
 * The size is bounded by what the cache can hold, not by B * max_context_len: long requests are cut
 * into splits of at most 2048 tokens whose partial results ((head_dim + 2) floats per query head)
 * wait in the workspace for the merge, and a batch has at most
 *     min(B * ceil(max_context_len / split), B + num_pages * page_size / split)
 * of them (for batches too small to fill the chip the split is shortened, down to 256 tokens, as far
 * as a fixed allowance of about 512 + B splits goes).  The second term assumes that the lengths of
 * one call add up to no more than num_pages * page_size tokens, i.e. that no page is counted for two
 * requests.  A call whose lengths exceed that (block tables that share pages between requests) and
 * whose splits do not fit writes nothing at all -- `out` is left untouched, no memory is overrun --
 * and ALISE_DEBUG_VALIDATE=1 reports lengths beyond the capacity as ALISE_INVALID_ARGUMENT.
 */
size_t alise_paged_decode_attn_workspace_bytes(const alise_kv_cache *c, int32_t B,
                                               int32_t num_q_heads, int32_t max_context_len);

/*
 * Single-query attention of B requests over their cached tokens   [Eq. 1, Eq. 2; Sec. 3.2]
 *   q, out        device, fp16 [B][num_q_heads][head_dim], 16-byte aligned.
 *   block_tables  device, int32 [B][max_blocks_per_seq]; entry j of request i is the
 *                 page holding its tokens j*page_size .. ; entries at index
 *                 >= ceil(L_i / page_size) are never read.
 *   context_lens  device, int32 [B]; L_i counts the token written in this step.
 *                 L_i <= 0 gives a zero output row.  Slots at positions >= L_i of
 *                 the last page are never interpreted.
 *   num_q_heads   a multiple of num_kv_heads; query head h reads KV head
 *                 h / (num_q_heads / num_kv_heads).
 *   softmax_scale 1/sqrt(head_dim) for Eq. 1.
 *   workspace     device, 256-byte aligned, at least
 *                 alise_paged_decode_attn_workspace_bytes(...) bytes; contents on
 *                 entry are irrelevant, contents on exit are unspecified.  Calls
 *                 that may overlap in time must use distinct workspaces.
 * out[i][h] = sum_t softmax_t(softmax_scale * q[i][h] . k^_t) v^_t over t < L_i, with
 * k^, v^ the dequantized rows; accumulated in fp32, rounded once to fp16.
 *
 * Value range.  Layouts with 2 to 16 query heads per KV head (head_dim 128, page_size >= 16, bits = 8
 * with group_size 64 or 128, or bits = 4 with group_size 32, 64 or 128) run on the matrix cores, where a
 * softmax weight times the V scale travels as a pair of fp16 numbers: V scales must stay below 256,
 * i.e. the range max - min of a V group below 65 280 (bits = 8) or 3 840 (bits = 4) -- always true for
 * fp16 activations of ordinary magnitude; beyond it the output saturates.  All other layouts have no
 * such limit.  alise_paged_prefill_attn has the same limit for every layout it takes.
 */
int alise_paged_decode_attn(const alise_kv_cache *c, const void *q, void *out,
                            const int32_t *block_tables, int32_t max_blocks_per_seq,
                            const int32_t *context_lens, int32_t B, int32_t num_q_heads,
                            int32_t max_context_len, float softmax_scale,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * alise_paged_decode_attn without a workspace argument, for callers that cannot allocate
 * device memory: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The workspace is a static device array inside the library, of
 * ALISE_STATIC_SCRATCH_BYTES bytes, which every GPU the library runs on holds until the
 * process ends.  The call allocates nothing on the host side of HIP or on the device (no
 * hipMalloc, hipFree or library routine that allocates); its first use on a device asks HIP for
 * the array's address there (hipGetSymbolAddress) and keeps it.
 *   - Arguments, results and status codes as for alise_paged_decode_attn (the output is bit for
 *     bit the same).  If alise_paged_decode_attn_workspace_bytes(c, B, num_q_heads,
 *     max_context_len) exceeds ALISE_STATIC_SCRATCH_BYTES the call returns
 *     ALISE_WORKSPACE_TOO_SMALL and launches nothing.
 *   - All calls on one GPU share that GPU's array: two such calls that may overlap in time (on
 *     two streams, or from two threads) race.  Nothing in the array has to be cleared between
 *     calls; what a call leaves there is unspecified.
 *   - ALISE_DEBUG_VALIDATE is not honoured (its checks copy device arrays to the host).
 */
#define ALISE_STATIC_SCRATCH_BYTES ((size_t)32 << 20)

int alise_paged_decode_attn_static(const alise_kv_cache *c, const void *q, void *out,
                                   const int32_t *block_tables, int32_t max_blocks_per_seq,
                                   const int32_t *context_lens, int32_t B, int32_t num_q_heads,
                                   int32_t max_context_len, float softmax_scale, void *hip_stream);

/*
 * The same attention in two calls, for a model of many layers              [Sec. 2, Eq. 1-2]
 *
 * How a batch is cut into work items depends on the lengths alone, and the lengths are the same for
 * every layer of one decode iteration.  alise_paged_decode_attn_plan does that part once (it reads
 * context_lens and writes the workspace); alise_paged_decode_attn_planned is
 * alise_paged_decode_attn without it, for each layer's cache, q and out in turn, on the same
 * workspace.  The cache geometry, B, num_q_heads, max_context_len and the contents of context_lens
 * must be those the plan was made with, and the tuning environment unchanged; the workspace must
 * not be touched in between except by these calls.  Results are bit for bit those of the single
 * call.  Arguments, checks and status codes as for alise_paged_decode_attn (the plan looks at no
 * cache pointer, so c->k_codes etc. may be NULL for it).
 */
int alise_paged_decode_attn_plan(const alise_kv_cache *c, const int32_t *context_lens, int32_t B,
                                 int32_t num_q_heads, int32_t max_context_len,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

int alise_paged_decode_attn_planned(const alise_kv_cache *c, const void *q, void *out,
                                    const int32_t *block_tables, int32_t max_blocks_per_seq,
                                    const int32_t *context_lens, int32_t B, int32_t num_q_heads,
                                    int32_t max_context_len, float softmax_scale,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Dequantize one page back to fp16                                 [Sec. 3.2]
 *   k_out, v_out  device, fp16 [page_size][num_kv_heads][head_dim], 16-byte aligned.
 * Every slot of the page is converted, written or not:
 * out = fp16_round_nearest_even(scale * (code - zero)).
 */
int alise_kv_dequant_page(const alise_kv_cache *c, int32_t page, void *k_out, void *v_out,
                          void *hip_stream);

/*
 * Chunked-prefill attention over the compressed cache        [Sec. 2 "LLM Inference", Eq. 1-2]
 *
 * The prefilling stage processes the prompt's tokens in one pass.  Here a request brings a
 * chunk of n_i query tokens; their K/V have already been quantized and written
 * (alise_kv_quant_write), so the cache holds L_i tokens including the chunk, the chunk at
 * positions L_i - n_i .. L_i - 1.  Query token j of the chunk attends, per head, to the cached
 * tokens 0 .. L_i - n_i + j (causal order), read from their quantized form like every other
 * token.  A chunk of one token is the decode step.
 *
 *   q, out        device, fp16 [total_q_tokens][num_q_heads][head_dim], 16-byte aligned: the
 *                 chunks of the B requests back to back.
 *   q_start       device, int32 [B + 1]: request i owns rows q_start[i] .. q_start[i+1] - 1;
 *                 q_start[0] = 0, nondecreasing, q_start[B] <= total_q_tokens (rows past q_start[B] are
 *                 not touched: a caller that captures the call in a graph sizes q, out and the workspace
 *                 for the largest chunk mix and changes q_start from replay to replay).  n_i = 0 is legal.
 *                 n_i > L_i is a caller error (the chunk is then cut to L_i rows).
 *   block_tables, max_blocks_per_seq, context_lens, max_context_len, softmax_scale, workspace:
 *                 as for alise_paged_decode_attn; the workspace size comes from
 *                 alise_paged_prefill_attn_workspace_bytes with the same B, total_q_tokens,
 *                 num_q_heads and max_context_len (0 on invalid arguments).
 * Every layout of the cache is taken.  Those with head_dim = 128, page_size >= 16, num_q_heads /
 * num_kv_heads between 1 and 16, and either bits = 8 with group_size 64 or 128, or bits = 4 with
 * group_size 32, 64 or 128, run on the matrix cores and need a workspace of a few bytes per query
 * token.  The others (head_dim 64, pages of 8 tokens, bits = 8 with groups of 16 or 32 channels, more
 * than 16 query heads per KV head) run on the single-query kernels, one request per query token whose
 * context ends at the token's position: correct and far slower (every query token reads its context
 * by itself), with a workspace of total_q_tokens * ceil(max_context_len / page_size) block-table
 * entries plus the split buffers of a single-query call over total_q_tokens requests.
 * out[t][h] = sum_u softmax_u(softmax_scale * q[t][h] . k^_u) v^_u over u <= position of t,
 * accumulated in fp32, rounded once to fp16.
 */
size_t alise_paged_prefill_attn_workspace_bytes(const alise_kv_cache *c, int32_t B, int32_t total_q_tokens,
                                                int32_t num_q_heads, int32_t max_context_len);

int alise_paged_prefill_attn(const alise_kv_cache *c, const void *q, void *out, const int32_t *q_start,
                             const int32_t *block_tables, int32_t max_blocks_per_seq,
                             const int32_t *context_lens, int32_t B, int32_t total_q_tokens,
                             int32_t num_q_heads, int32_t max_context_len, float softmax_scale,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Offload and upload of one request's cache            [Sec. 3.2 "Dynamic Swapping", Alg. 2]
 *
 * The paper's cache manager moves the whole KV cache of a preempted job between GPU memory
 * and CPU memory (request level), overlapped with computation; which job moves when (the
 * estimated wait time, the job limit M) is host-side scheduling and not part of this
 * library.  These two calls are the data movement: they gather the request's compressed
 * pages, found through its block table, into one contiguous buffer, and scatter such a
 * buffer into whatever pages the block table names at upload time.  Compressed bytes move
 * as they are; nothing is requantized.
 *
 *   block_table   device, int32 [ceil(num_tokens / page_size)]: the request's pages in
 *                 logical order (one row of the attention call's block_tables).
 *   packed        device-ACCESSIBLE memory, 16-byte aligned, at least
 *                 alise_kv_swap_bytes(c, num_tokens) bytes: either device memory (a staging
 *                 buffer that a copy engine then moves, hipMemcpyAsync) or pinned host
 *                 memory from hipHostMalloc, which the kernels read and write directly
 *                 over the host link.
 *   layout of packed: logical block j, KV head h at offset (j * num_kv_heads + h) * BB,
 *                 BB = 2 * page_size * head_dim*bits/8 + 2 * page_size * (head_dim/group_size) * 4,
 *                 holding [K codes | V codes | K meta | V meta] of that (page, head), each
 *                 in the canonical order.  Whole pages travel, the unused slots of the last
 *                 page included, so an upload reproduces every page bit for bit.
 * Run them on a stream of their own to overlap them with attention; a request must not be
 * attended to or written while it is in transit.  Beside an attention call prefer the device
 * buffer and let hipMemcpyAsync move it: both ways reach the rate of the host link, but a kernel
 * that reads or writes host memory itself slows an attention call running at the same time by
 * about a third on an MI355X, and the copy engine does not (measured; bench.py, `swap`).  num_tokens = 0 is legal and does nothing.
 */
size_t alise_kv_swap_bytes(const alise_kv_cache *c, int32_t num_tokens);

int alise_kv_swap_out(const alise_kv_cache *c, const int32_t *block_table, int32_t num_tokens,
                      void *packed, size_t packed_bytes, void *hip_stream);

int alise_kv_swap_in(const alise_kv_cache *c, const int32_t *block_table, int32_t num_tokens,
                     const void *packed, size_t packed_bytes, void *hip_stream);

/*
 * The tuning variables (ALISE_SPLIT_TOKENS, ALISE_SPLIT_TOKENS_GQA, ALISE_WAVES_PER_CU,
 * ALISE_LOADS_PER_BLOCK, ALISE_MIN_ITEMS_PER_WAVE, ALISE_XCD_SKEW, ALISE_PREFILL_ROW_TILES,
 * ALISE_PREFILL_WEIGHTS) and ALISE_DEBUG_VALIDATE are read from the environment once per process,
 * by the first call that needs them.  This call reads them again: for tests and tuning sweeps
 * that change them inside one process.  It must not run while another thread is inside the
 * library.  Workspace sizes depend on the split variables: ask for them again afterwards.
 */
void alise_reload_environment(void);

/* Static, human-readable name of a status code. */
const char *alise_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* ALISE_KV_H */
