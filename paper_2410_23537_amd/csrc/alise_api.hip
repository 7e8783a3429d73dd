// C-ABI layer: argument validation (host only, before any HIP call), workspace
// carving and kernel launches; with ALISE_DEBUG_VALIDATE=1 also checks of the device arrays.
// See include/alise_kv.h for the contract.
#include "../../include/alise_kv.h"
#include "alise_kernels.h"

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <mutex>
#include <vector>

// Workspace of alise_paged_decode_attn_static: a file-scope device array, so that the call needs no allocation
// by anybody.  Each GPU the library runs on holds its own copy until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress: the address that kernels, copies and fills may use is the one that
// call returns for the device that is current, asked once per device and kept in static_scratch_ptr.
constexpr size_t kStaticScratchBytes = ALISE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using alise::AttnWorkspace;
using alise::CacheView;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int ilog2_exact(int32_t v)
{
    if (v <= 0 || (v & (v - 1))) return -1;
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

// Shape checks shared by every entry point.
int check_cache(const alise_kv_cache *c, CacheView *out)
{
    if (!c) return ALISE_INVALID_ARGUMENT;
    if (c->num_pages <= 0 || c->page_size <= 0 || c->num_kv_heads <= 0 || c->head_dim <= 0 ||
        c->group_size <= 0)
        return ALISE_INVALID_ARGUMENT;
    if (c->bits != 4 && c->bits != 8) return ALISE_UNSUPPORTED;
    if (c->head_dim != 64 && c->head_dim != 128) return ALISE_UNSUPPORTED;
    if (c->head_dim % c->group_size != 0) return ALISE_UNSUPPORTED;
    if (c->group_size % (128 / c->bits) != 0) return ALISE_UNSUPPORTED;
    const int logP = ilog2_exact(c->page_size);
    if (logP < 3 || logP > 8) return ALISE_UNSUPPORTED;
    if ((int64_t)c->num_pages * c->page_size >= (int64_t)1 << 31) return ALISE_UNSUPPORTED;
    if ((int64_t)c->num_pages * c->num_kv_heads >= (int64_t)1 << 31) return ALISE_UNSUPPORTED;
    const int64_t dense_c = (int64_t)c->page_size * (c->head_dim * c->bits / 8);
    const int64_t dense_m = (int64_t)c->page_size * (c->head_dim / c->group_size) * 4;
    const int64_t cs = c->codes_block_stride ? c->codes_block_stride : dense_c;
    const int64_t ms = c->meta_block_stride ? c->meta_block_stride : dense_m;
    if (cs < dense_c || ms < dense_m || (cs & 15) || (ms & 15)) return ALISE_INVALID_ARGUMENT;
    if (cs >= (int64_t)1 << 31 || ms >= (int64_t)1 << 31) return ALISE_UNSUPPORTED;
    if (out) {
        out->k_codes = static_cast<uint8_t *>(c->k_codes);
        out->v_codes = static_cast<uint8_t *>(c->v_codes);
        out->k_meta = static_cast<uint32_t *>(c->k_meta);
        out->v_meta = static_cast<uint32_t *>(c->v_meta);
        out->num_pages = c->num_pages;
        out->P = c->page_size;
        out->logP = logP;
        out->Hkv = c->num_kv_heads;
        out->D = c->head_dim;
        out->bits = c->bits;
        out->G = c->group_size;
        out->NG = c->head_dim / c->group_size;
        out->row_code_bytes = c->head_dim * c->bits / 8;
        out->cstride = (int32_t)cs;
        out->mstride = (int32_t)ms;
    }
    return ALISE_OK;
}

int check_cache_pointers(const alise_kv_cache *c)
{
    if (!c->k_codes || !c->v_codes || !c->k_meta || !c->v_meta) return ALISE_INVALID_ARGUMENT;
    if (!aligned16(c->k_codes) || !aligned16(c->v_codes) || !aligned16(c->k_meta) || !aligned16(c->v_meta))
        return ALISE_MISALIGNED;
    return ALISE_OK;
}

// The tuning environment, read once per process (alise_reload_environment reads it again).
std::once_flag tuning_once;
alise::Tuning tuning_values;

long env_long(const char *name, long fallback)
{
    const char *e = std::getenv(name);
    return (e && *e) ? std::strtol(e, nullptr, 10) : fallback;
}

void read_tuning()
{
    alise::Tuning t;
    long v = env_long("ALISE_SPLIT_TOKENS", 0);
    t.split_tokens = (v < 64 || v > (1 << 20) || (v % 64) != 0) ? 0 : (int32_t)v;
    v = env_long("ALISE_SPLIT_TOKENS_GQA", 0);
    t.split_tokens_gqa = (v < 64 || v > (1 << 20) || (v % 64) != 0) ? 0 : (int32_t)v;
    v = env_long("ALISE_WAVES_PER_CU", 0);                      // a multiple of 4, at most 32; 0 = as many as fit
    t.waves_per_cu = (v < 4 || v > 32 || (v % 4) != 0) ? 0 : (int32_t)v;
    v = env_long("ALISE_LOADS_PER_BLOCK", 0);                   // 2, 3 or 4; 0 = the kernel's default for the bit width
    t.loads_per_block = (v < 2 || v > 4) ? 0 : (int32_t)v;
    v = env_long("ALISE_MIN_ITEMS_PER_WAVE", 0);                // 0 = the kernels' own defaults
    t.min_items_per_wave = (v < 0 || v > 1024) ? 0 : (int32_t)v;
    // Thousandths of an attention call's work that go to the waves of even workgroups only: 50 measured best on the
    // large INT4 batch (1145 us without, 1119 us with 34, 1110 us with 50, 1112 us with 70); 0 to 200, 0 = none.
    v = env_long("ALISE_XCD_SKEW", 50);
    t.xcd_skew_permille = (v < 0 || v > 200) ? 50 : (int32_t)v;
    const char *e = std::getenv("ALISE_PREFILL_ROW_TILES");     // row tiles per wave of the prefill kernels: two unless "1"
    t.prefill_row_tiles = (e && e[0] == '1' && e[1] == 0) ? 1 : 2;
    e = std::getenv("ALISE_PREFILL_WEIGHTS");                   // "single": one rounded fp16 number per softmax weight
    t.prefill_split_weights = !(e && e[0] == 's' && e[1] == 'i');
    // ALISE_DEBUG_VALIDATE=1: the calls also check what they are given in device memory (slots, lengths, block
    // tables, chunk boundaries).  That takes a copy to the host and a wait for the stream, so it is for debugging
    // only: without it the contents of device arrays are the caller's responsibility.
    e = std::getenv("ALISE_DEBUG_VALIDATE");
    t.debug_validate = e && e[0] == '1' && e[1] == 0;
    tuning_values = t;
}

// Tokens per split.  Long requests are cut into splits of this many tokens so that
// one long and many short requests fill the chip alike; ALISE_SPLIT_TOKENS overrides
// the default (a multiple of 64) for tuning.
// A split never spans more than 128 pages (64 on the matrix-core path): the attention
// kernel keeps a split's block-table entries in two registers (one), one entry per lane.
// A split longer than a page is therefore also a whole number of pages: the splits of a request
// start at multiples of the split length, and one that began inside a page would touch one page
// more than the window holds.
// Every item costs a wave a few microseconds at its end (the reduction over its token slots,
// the partial result), so splits are as long as that allows, up to 2048 tokens.
// The matrix-core path hands a whole group of query heads to one wave; starting and ending
// an item costs it several microseconds (query rows, partial results of up to 16 heads), so
// it takes the longest splits the 64-page window allows, up to 2048 tokens
// (ALISE_SPLIT_TOKENS_GQA overrides).
// Returns the largest split; *min_split is the smallest the plan kernel may fall back to
// when a batch is too small to give every wave several items (equal to the largest when
// the environment fixes the split).
int32_t split_tokens(int32_t page_size, bool gqa, int32_t *min_split)
{
    const alise::Tuning &t = alise::tuning();
    long v = gqa ? t.split_tokens_gqa : t.split_tokens;
    const bool fixed = v != 0;
    if (!fixed) v = 2048;
    const long window = gqa ? 64 : 128;         // pages whose block-table entries a wave keeps at hand
    if (v > window * page_size) v = window * page_size;
    if (v > page_size) v -= v % page_size;      // page sizes are powers of two up to 256, v a multiple of 64: v stays a multiple of 64
    long lo = fixed ? v : 256;
    if (lo > v) lo = v;
    if (min_split) *min_split = (int32_t)lo;
    return (int32_t)v;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool debug_validate() { return alise::tuning().debug_validate; }

template <class T>
int fetch_to_host(std::vector<T> &host, const T *dev, size_t n, hipStream_t s)
{
    host.resize(n);
    if (n == 0) return ALISE_OK;
    if (hipMemcpyAsync(host.data(), dev, n * sizeof(T), hipMemcpyDeviceToHost, s) != hipSuccess) return ALISE_HIP_ERROR;
    return hipStreamSynchronize(s) == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

// Lengths within [0, max_len], and the block-table entries that those lengths reach within [0, num_pages).
// `v_scale_limit`: the call runs on the matrix cores, where a V scale of 256 or more saturates the fp16 pair that carries
// weight times scale; every V scale that a length reaches is then read back and checked as well.
int validate_lens_and_tables(const CacheView &cv, const int32_t *block_tables, int32_t max_blocks, const int32_t *context_lens,
                             int32_t B, int32_t max_len, std::vector<int32_t> *lens_out, hipStream_t s, bool v_scale_limit = false)
{
    std::vector<int32_t> lens, bt;
    int st = fetch_to_host(lens, context_lens, (size_t)B, s);
    if (st != ALISE_OK) return st;
    st = fetch_to_host(bt, block_tables, (size_t)B * max_blocks, s);
    if (st != ALISE_OK) return st;
    int64_t sum = 0;
    for (int32_t i = 0; i < B; ++i) {
        if (lens[i] < 0 || lens[i] > max_len) return ALISE_INVALID_ARGUMENT;
        sum += lens[i];
        if (sum > (int64_t)cv.num_pages * cv.P) return ALISE_INVALID_ARGUMENT;     // more tokens than the cache holds: the workspace is not sized for that
        const int64_t nblk = ((int64_t)lens[i] + cv.P - 1) / cv.P;
        if (nblk > max_blocks) return ALISE_INVALID_ARGUMENT;
        for (int64_t b = 0; b < nblk; ++b) {
            const int32_t page = bt[(size_t)i * max_blocks + b];
            if (page < 0 || page >= cv.num_pages) return ALISE_INVALID_ARGUMENT;
        }
    }
    if (v_scale_limit) {
        std::vector<uint32_t> meta;
        const size_t span = ((size_t)cv.num_pages * cv.Hkv - 1) * (size_t)cv.mstride + (size_t)cv.P * cv.NG * 4;
        st = fetch_to_host(meta, cv.v_meta, span / 4, s);
        if (st != ALISE_OK) return st;
        for (int32_t i = 0; i < B; ++i)
            for (int32_t t = 0; t < lens[i]; ++t) {
                const int64_t page = bt[(size_t)i * max_blocks + t / cv.P];
                for (int32_t h = 0; h < cv.Hkv; ++h) {
                    const uint32_t *row = meta.data() + ((size_t)(page * cv.Hkv + h) * cv.mstride) / 4 + (size_t)(t % cv.P) * cv.NG;
                    for (int32_t g = 0; g < cv.NG; ++g)
                        if ((row[g] & 0x7fffu) >= 0x5c00u) return ALISE_INVALID_ARGUMENT;       // fp16 256.0, infinities and NaN above it
                }
            }
    }
    if (lens_out) lens_out->swap(lens);
    return ALISE_OK;
}

// How many tiles (request, token range of one split) a call can produce, which sizes the work order and the
// split buffers.  With splits of C tokens a batch has at most B * ceil(max_len / C) tiles, and no more than
// B + capacity / C, capacity = num_pages * page_size being all the tokens the cache can hold (every request adds
// at most one partial tile to the full ones).  The plan kernel starts from the largest split and halves it only
// for small batches -- while the tiles of the batch would give a full grid fewer than `min_items` work items --
// and never beyond what this bound holds (it checks), so the bound is taken at the largest split and widened to
// the most tiles such a small batch can end with, twice min_items' worth plus one per request; it never exceeds
// the bound at the smallest split.
int64_t max_tiles_of(const CacheView &c, int32_t B, int32_t H, int32_t max_len, bool bounded_by_capacity = true)
{
    const bool gqa = alise::gqa_mfma_applies(c, H);
    int32_t C_min = 0;
    const int32_t C = split_tokens(c.P, gqa, &C_min);
    const int64_t capacity = (int64_t)c.num_pages * c.P;
    auto bound = [&](int64_t split) {
        const int64_t per_req = ((int64_t)max_len + split - 1) / split;
        const int64_t by_length = (int64_t)B * std::max<int64_t>(per_req, 1);
        return bounded_by_capacity ? std::min(by_length, (int64_t)B + capacity / split) : by_length;
    };
    const int64_t items_per_tile = gqa ? c.Hkv : H;
    const int64_t small = (int64_t)B + (2 * alise::plan_min_items(256, gqa) + items_per_tile - 1) / items_per_tile;
    return std::max<int64_t>(1, std::min(bound(C_min), std::max(bound(C), small)));
}

// Workspace layout: [n_items, n_merge | tile_base[B+1] | req_full_base[B] |
// order[max_tiles] | part].
size_t carve_workspace(const CacheView &c, int32_t B, int32_t H, int32_t max_len, void *base,
                       AttnWorkspace *ws, bool bounded_by_capacity = true)
{
    int32_t C_min = 0;
    const int32_t C = split_tokens(c.P, alise::gqa_mfma_applies(c, H), &C_min);
    const int64_t max_tiles = max_tiles_of(c, B, H, max_len, bounded_by_capacity);
    size_t off = 256;       // header: n_items, n_merge
    const size_t off_base = off;
    off = align_up(off + sizeof(int32_t) * ((size_t)B + 1), 256);
    const size_t off_fb = off;
    off = align_up(off + sizeof(int32_t) * (size_t)B, 256);
    const size_t off_order = off;
    off = align_up(off + 16 * (size_t)max_tiles, 256);
    const size_t off_part = off;
    off = align_up(off + sizeof(float) * (size_t)max_tiles * H * (c.D + 2), 256);
    if (ws) {
        char *b = static_cast<char *>(base);
        ws->n_items = reinterpret_cast<int32_t *>(b);
        ws->tile_base = reinterpret_cast<int32_t *>(b + off_base);
        ws->req_full_base = reinterpret_cast<int32_t *>(b + off_fb);
        ws->n_merge = reinterpret_cast<int32_t *>(b + 4);
        ws->n_shared = reinterpret_cast<int32_t *>(b + 8);
        ws->skew_permille = alise::tuning().xcd_skew_permille;
        ws->order = reinterpret_cast<int4 *>(b + off_order);
        ws->part = reinterpret_cast<float *>(b + off_part);
        ws->max_tiles = (int32_t)max_tiles;
        ws->chunk_tokens = C;
        ws->min_chunk_tokens = C_min;
        ws->min_items = 0;      // set by the caller once the grid is known
    }
    return off;
}

int check_attn_sizes(const CacheView &c, int32_t B, int32_t H, int32_t max_len, bool bounded_by_capacity = true)
{
    if (B < 0 || H <= 0 || max_len < 0) return ALISE_INVALID_ARGUMENT;
    if (H % c.Hkv != 0) return ALISE_UNSUPPORTED;
    if (max_tiles_of(c, B, H, max_len, bounded_by_capacity) * H >= (int64_t)1 << 31) return ALISE_UNSUPPORTED;
    return ALISE_OK;
}

// Compute units of the current device, asked once per device (a race between two first calls writes the same value twice).
int num_compute_units()
{
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

constexpr int kMaxDevices = 64;
std::mutex static_scratch_mutex;
void *static_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (ALISE_HIP_ERROR if HIP cannot give it).
int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ALISE_HIP_ERROR;
    std::lock_guard<std::mutex> hold(static_scratch_mutex);
    if (!static_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return ALISE_HIP_ERROR;
        static_scratch_ptr[dev] = ptr;
    }
    *out = static_scratch_ptr[dev];
    return ALISE_OK;
}

}  // namespace

namespace alise {

const Tuning &tuning()
{
    std::call_once(tuning_once, read_tuning);
    return tuning_values;
}

}  // namespace alise

extern "C" {

void alise_reload_environment(void)
{
    std::call_once(tuning_once, read_tuning);       // so that a later first use does not overwrite what is read now
    read_tuning();
}

size_t alise_kv_codes_bytes(const alise_kv_cache *c)
{
    CacheView cv;
    if (check_cache(c, &cv) != ALISE_OK) return 0;
    const size_t blocks = (size_t)c->num_pages * c->num_kv_heads;
    return (blocks - 1) * (size_t)cv.cstride + (size_t)c->page_size * cv.row_code_bytes;
}

size_t alise_kv_meta_bytes(const alise_kv_cache *c)
{
    CacheView cv;
    if (check_cache(c, &cv) != ALISE_OK) return 0;
    const size_t blocks = (size_t)c->num_pages * c->num_kv_heads;
    return (blocks - 1) * (size_t)cv.mstride + (size_t)c->page_size * cv.NG * 4;
}

int alise_kv_quant_write(const alise_kv_cache *c, const void *k, const void *v,
                         const int64_t *slot_mapping, int32_t T, void *hip_stream)
{
    CacheView cv;
    int st = check_cache(c, &cv);
    if (st != ALISE_OK) return st;
    if (T < 0) return ALISE_INVALID_ARGUMENT;
    if (T == 0) return ALISE_OK;
    if (!k || !v || !slot_mapping) return ALISE_INVALID_ARGUMENT;
    st = check_cache_pointers(c);
    if (st != ALISE_OK) return st;
    if (!aligned16(k) || !aligned16(v)) return ALISE_MISALIGNED;
    if ((reinterpret_cast<uintptr_t>(slot_mapping) & 7u) != 0) return ALISE_MISALIGNED;
    if (debug_validate()) {
        std::vector<int64_t> slots;
        st = fetch_to_host(slots, slot_mapping, (size_t)T, static_cast<hipStream_t>(hip_stream));
        if (st != ALISE_OK) return st;
        const int64_t n_slots = (int64_t)cv.num_pages * cv.P;
        slots.erase(std::remove_if(slots.begin(), slots.end(), [](int64_t v) { return v < 0; }), slots.end());   // skipped tokens
        for (int64_t v : slots)
            if (v >= n_slots) return ALISE_INVALID_ARGUMENT;
        std::sort(slots.begin(), slots.end());
        if (std::adjacent_find(slots.begin(), slots.end()) != slots.end()) return ALISE_INVALID_ARGUMENT;    // two tokens, one slot
    }
    hipError_t e = alise::launch_quant_write(cv, k, v, slot_mapping, T, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

size_t alise_paged_decode_attn_workspace_bytes(const alise_kv_cache *c, int32_t B, int32_t num_q_heads,
                                               int32_t max_context_len)
{
    CacheView cv;
    if (check_cache(c, &cv) != ALISE_OK) return 0;
    if (check_attn_sizes(cv, B, num_q_heads, max_context_len) != ALISE_OK) return 0;
    return carve_workspace(cv, B, num_q_heads, max_context_len, nullptr, nullptr);
}

// The three forms of the attention call: plan + run in one (the lengths are new every time), the plan alone
// (once per decode step), the run alone (once per layer of that step, on the plan in the workspace).
static int decode_attn_call(const alise_kv_cache *c, const void *q, void *out,
                            const int32_t *block_tables, int32_t max_blocks_per_seq,
                            const int32_t *context_lens, int32_t B, int32_t num_q_heads,
                            int32_t max_context_len, float softmax_scale,
                            void *workspace, size_t workspace_bytes, int32_t phases, void *hip_stream,
                            bool use_static_scratch = false)
{
    const bool run = (phases & alise::kPhaseRun) != 0;
    CacheView cv;
    int st = check_cache(c, &cv);
    if (st != ALISE_OK) return st;
    st = check_attn_sizes(cv, B, num_q_heads, max_context_len);
    if (st != ALISE_OK) return st;
    if (B == 0) return ALISE_OK;
    if (run) {
        if (max_blocks_per_seq <= 0) return ALISE_INVALID_ARGUMENT;
        if ((int64_t)max_blocks_per_seq * cv.P < max_context_len) return ALISE_INVALID_ARGUMENT;
        if (!(softmax_scale == softmax_scale) || softmax_scale <= 0.0f) return ALISE_INVALID_ARGUMENT;
        if (!q || !out || !block_tables) return ALISE_INVALID_ARGUMENT;
    }
    if (!context_lens || (!workspace && !use_static_scratch)) return ALISE_INVALID_ARGUMENT;
    if (run) {
        st = check_cache_pointers(c);
        if (st != ALISE_OK) return st;
        if (!aligned16(q) || !aligned16(out)) return ALISE_MISALIGNED;
        if (reinterpret_cast<uintptr_t>(block_tables) & 3u) return ALISE_MISALIGNED;
    }
    if (reinterpret_cast<uintptr_t>(context_lens) & 3u) return ALISE_MISALIGNED;
    if (use_static_scratch) {
        // every host check has passed; the size is compared before the first HIP call
        if (carve_workspace(cv, B, num_q_heads, max_context_len, nullptr, nullptr) > kStaticScratchBytes)
            return ALISE_WORKSPACE_TOO_SMALL;
        st = static_scratch(&workspace);
        if (st != ALISE_OK) return st;
        workspace_bytes = kStaticScratchBytes;
    }
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ALISE_MISALIGNED;
    AttnWorkspace ws;
    const size_t need = carve_workspace(cv, B, num_q_heads, max_context_len, workspace, &ws);
    if (workspace_bytes < need) return ALISE_WORKSPACE_TOO_SMALL;
    if (debug_validate() && !use_static_scratch) {      // the checks copy to the host: not for a caller that must not allocate
        hipStream_t hs = static_cast<hipStream_t>(hip_stream);
        if (run) {
            st = validate_lens_and_tables(cv, block_tables, max_blocks_per_seq, context_lens, B, max_context_len, nullptr, hs,
                                          alise::gqa_mfma_applies(cv, num_q_heads));
            if (st != ALISE_OK) return st;
        } else {
            std::vector<int32_t> lens;
            st = fetch_to_host(lens, context_lens, (size_t)B, hs);
            if (st != ALISE_OK) return st;
            int64_t sum = 0;
            for (int32_t L : lens) {
                if (L < 0 || L > max_context_len) return ALISE_INVALID_ARGUMENT;
                sum += L;
            }
            if (sum > (int64_t)cv.num_pages * cv.P) return ALISE_INVALID_ARGUMENT;
        }
    }
    hipError_t e = alise::launch_decode_attn(cv, q, out, block_tables, max_blocks_per_seq, context_lens, B,
                                             num_q_heads, max_context_len, softmax_scale, ws,
                                             num_compute_units(), alise::tuning().waves_per_cu, alise::tuning().loads_per_block,
                                             phases, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

int alise_paged_decode_attn(const alise_kv_cache *c, const void *q, void *out,
                            const int32_t *block_tables, int32_t max_blocks_per_seq,
                            const int32_t *context_lens, int32_t B, int32_t num_q_heads,
                            int32_t max_context_len, float softmax_scale,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return decode_attn_call(c, q, out, block_tables, max_blocks_per_seq, context_lens, B, num_q_heads, max_context_len,
                            softmax_scale, workspace, workspace_bytes, alise::kPhasePlan | alise::kPhaseRun, hip_stream);
}

int alise_paged_decode_attn_static(const alise_kv_cache *c, const void *q, void *out,
                                   const int32_t *block_tables, int32_t max_blocks_per_seq,
                                   const int32_t *context_lens, int32_t B, int32_t num_q_heads,
                                   int32_t max_context_len, float softmax_scale, void *hip_stream)
{
    return decode_attn_call(c, q, out, block_tables, max_blocks_per_seq, context_lens, B, num_q_heads, max_context_len,
                            softmax_scale, nullptr, 0, alise::kPhasePlan | alise::kPhaseRun, hip_stream, true);
}

int alise_paged_decode_attn_plan(const alise_kv_cache *c, const int32_t *context_lens, int32_t B, int32_t num_q_heads,
                                 int32_t max_context_len, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return decode_attn_call(c, nullptr, nullptr, nullptr, 0, context_lens, B, num_q_heads, max_context_len, 1.0f, workspace,
                            workspace_bytes, alise::kPhasePlan, hip_stream);
}

int alise_paged_decode_attn_planned(const alise_kv_cache *c, const void *q, void *out,
                                    const int32_t *block_tables, int32_t max_blocks_per_seq,
                                    const int32_t *context_lens, int32_t B, int32_t num_q_heads,
                                    int32_t max_context_len, float softmax_scale,
                                    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return decode_attn_call(c, q, out, block_tables, max_blocks_per_seq, context_lens, B, num_q_heads, max_context_len,
                            softmax_scale, workspace, workspace_bytes, alise::kPhaseRun, hip_stream);
}

int alise_kv_dequant_page(const alise_kv_cache *c, int32_t page, void *k_out, void *v_out, void *hip_stream)
{
    CacheView cv;
    int st = check_cache(c, &cv);
    if (st != ALISE_OK) return st;
    if (page < 0 || page >= c->num_pages) return ALISE_INVALID_ARGUMENT;
    if (!k_out || !v_out) return ALISE_INVALID_ARGUMENT;
    st = check_cache_pointers(c);
    if (st != ALISE_OK) return st;
    if (!aligned16(k_out) || !aligned16(v_out)) return ALISE_MISALIGNED;
    hipError_t e = alise::launch_dequant_page(cv, page, k_out, v_out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

static size_t carve_prefill(const CacheView &cv, int32_t B, int32_t total_q, int32_t H, void *base,
                            alise::PrefillWorkspace *ws)
{
    const int tpw = alise::prefill_tokens_per_workgroup(H / cv.Hkv, 1);      // the smaller tile: an upper bound on the tile count
    const int64_t max_tiles = ((int64_t)total_q + tpw - 1) / tpw + B;
    const size_t bytes = align_up(256 + sizeof(int32_t) * 2 * (size_t)max_tiles, 256);
    if (ws) {
        char *b = static_cast<char *>(base);
        ws->n_tiles = reinterpret_cast<int32_t *>(b);
        ws->table = reinterpret_cast<int2 *>(b + 256);
        ws->max_tiles = (int32_t)max_tiles;
    }
    return bytes;
}

// Layouts without a matrix-core prefill kernel (head_dim 64, pages of 8 tokens, INT8 groups of 16 or 32 channels,
// more than 16 query heads per KV head) run on the single-query kernel: every query token of a chunk becomes a request
// of its own whose context ends at its position -- which is what the causal order means.  The workspace then holds
// the lengths and the block-table rows of these requests (one row of ceil(max_context_len / page_size) entries per
// query token, copied from its request's row) in front of the single-query call's own workspace.  That call's split
// buffers cannot be bounded by the cache's capacity here: the requests of one chunk share their pages.
struct PrefillFallback {
    int32_t *lens;          // [total_q] context length of every query token, -1 for rows that no chunk owns
    int32_t *tables;        // [total_q][blocks_per_row]
    int32_t blocks_per_row;
    void *attn_workspace;
    size_t attn_workspace_bytes;
};

static size_t carve_prefill_fallback(const CacheView &cv, int32_t total_q, int32_t H, int32_t max_len, void *base,
                                     PrefillFallback *fb)
{
    const int64_t blocks_per_row = std::max<int64_t>(1, ((int64_t)max_len + cv.P - 1) / cv.P);
    const size_t off_tables = align_up(sizeof(int32_t) * (size_t)total_q, 256);
    const size_t off_attn = align_up(off_tables + sizeof(int32_t) * (size_t)total_q * (size_t)blocks_per_row, 256);
    const size_t attn_bytes = carve_workspace(cv, total_q, H, max_len, nullptr, nullptr, false);
    if (fb) {
        char *b = static_cast<char *>(base);
        fb->lens = reinterpret_cast<int32_t *>(b);
        fb->tables = reinterpret_cast<int32_t *>(b + off_tables);
        fb->blocks_per_row = (int32_t)blocks_per_row;
        fb->attn_workspace = b + off_attn;
        fb->attn_workspace_bytes = attn_bytes;
    }
    return off_attn + attn_bytes;
}

static int check_prefill_sizes(const CacheView &cv, int32_t B, int32_t total_q, int32_t H, int32_t max_len)
{
    if (B < 0 || total_q < 0 || H <= 0 || max_len < 0) return ALISE_INVALID_ARGUMENT;
    if (H % cv.Hkv != 0) return ALISE_UNSUPPORTED;
    if ((int64_t)total_q * H >= (int64_t)1 << 31) return ALISE_UNSUPPORTED;
    if (((int64_t)total_q + B + 8) * cv.Hkv >= (int64_t)1 << 31) return ALISE_UNSUPPORTED;       // workgroups of the matrix-core kernels: (row tile, KV head) pairs
    if (!alise::prefill_mfma_applies(cv, H)) {
        const int64_t blocks_per_row = std::max<int64_t>(1, ((int64_t)max_len + cv.P - 1) / cv.P);
        if ((int64_t)total_q * blocks_per_row >= (int64_t)1 << 31) return ALISE_UNSUPPORTED;
        return check_attn_sizes(cv, total_q, H, max_len, false);
    }
    return ALISE_OK;
}

size_t alise_paged_prefill_attn_workspace_bytes(const alise_kv_cache *c, int32_t B, int32_t total_q_tokens,
                                                int32_t num_q_heads, int32_t max_context_len)
{
    CacheView cv;
    if (check_cache(c, &cv) != ALISE_OK) return 0;
    if (check_prefill_sizes(cv, B, total_q_tokens, num_q_heads, max_context_len) != ALISE_OK) return 0;
    if (!alise::prefill_mfma_applies(cv, num_q_heads))
        return carve_prefill_fallback(cv, std::max(total_q_tokens, 1), num_q_heads, max_context_len, nullptr, nullptr);
    return carve_prefill(cv, B, total_q_tokens, num_q_heads, nullptr, nullptr);
}

int alise_paged_prefill_attn(const alise_kv_cache *c, const void *q, void *out, const int32_t *q_start,
                             const int32_t *block_tables, int32_t max_blocks_per_seq,
                             const int32_t *context_lens, int32_t B, int32_t total_q_tokens,
                             int32_t num_q_heads, int32_t max_context_len, float softmax_scale,
                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    CacheView cv;
    int st = check_cache(c, &cv);
    if (st != ALISE_OK) return st;
    st = check_prefill_sizes(cv, B, total_q_tokens, num_q_heads, max_context_len);
    if (st != ALISE_OK) return st;
    if (B == 0 || total_q_tokens == 0) return ALISE_OK;
    if (max_blocks_per_seq <= 0) return ALISE_INVALID_ARGUMENT;
    if ((int64_t)max_blocks_per_seq * cv.P < max_context_len) return ALISE_INVALID_ARGUMENT;
    if (!(softmax_scale == softmax_scale) || softmax_scale <= 0.0f) return ALISE_INVALID_ARGUMENT;
    if (!q || !out || !q_start || !block_tables || !context_lens || !workspace) return ALISE_INVALID_ARGUMENT;
    st = check_cache_pointers(c);
    if (st != ALISE_OK) return st;
    if (!aligned16(q) || !aligned16(out)) return ALISE_MISALIGNED;
    if ((reinterpret_cast<uintptr_t>(block_tables) & 3u) || (reinterpret_cast<uintptr_t>(context_lens) & 3u) ||
        (reinterpret_cast<uintptr_t>(q_start) & 3u))
        return ALISE_MISALIGNED;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ALISE_MISALIGNED;
    const bool matrix_cores = alise::prefill_mfma_applies(cv, num_q_heads);
    alise::PrefillWorkspace ws;
    PrefillFallback fb;
    const size_t need = matrix_cores ? carve_prefill(cv, B, total_q_tokens, num_q_heads, workspace, &ws)
                                     : carve_prefill_fallback(cv, total_q_tokens, num_q_heads, max_context_len, workspace, &fb);
    if (workspace_bytes < need) return ALISE_WORKSPACE_TOO_SMALL;
    if (debug_validate()) {
        hipStream_t hs = static_cast<hipStream_t>(hip_stream);
        std::vector<int32_t> lens, qs;
        st = validate_lens_and_tables(cv, block_tables, max_blocks_per_seq, context_lens, B, max_context_len, &lens, hs, matrix_cores);
        if (st != ALISE_OK) return st;
        st = fetch_to_host(qs, q_start, (size_t)B + 1, hs);
        if (st != ALISE_OK) return st;
        if (qs[0] < 0 || qs[B] > total_q_tokens) return ALISE_INVALID_ARGUMENT;
        for (int32_t i = 0; i < B; ++i)
            if (qs[i + 1] < qs[i] || qs[i + 1] - qs[i] > lens[i]) return ALISE_INVALID_ARGUMENT;     // a chunk is part of its request
    }
    hipStream_t hs = static_cast<hipStream_t>(hip_stream);
    if (!matrix_cores) {
        hipError_t e = alise::launch_prefill_expand(cv, q_start, block_tables, max_blocks_per_seq, context_lens, B, total_q_tokens,
                                                    max_context_len, fb.lens, fb.tables, fb.blocks_per_row, hs);
        if (e != hipSuccess) return ALISE_HIP_ERROR;
        AttnWorkspace aws;
        carve_workspace(cv, total_q_tokens, num_q_heads, max_context_len, fb.attn_workspace, &aws, false);
        e = alise::launch_decode_attn(cv, q, out, fb.tables, fb.blocks_per_row, fb.lens, total_q_tokens, num_q_heads, max_context_len,
                                      softmax_scale, aws, num_compute_units(), alise::tuning().waves_per_cu,
                                      alise::tuning().loads_per_block,
                                      alise::kPhasePlan | alise::kPhaseRun | alise::kPhaseKeepNegative, hs);
        return e == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
    }
    hipError_t e = alise::launch_prefill_attn(cv, q, out, q_start, block_tables, max_blocks_per_seq, context_lens, B,
                                              num_q_heads, max_context_len, softmax_scale, ws, hs);
    return e == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

size_t alise_kv_swap_bytes(const alise_kv_cache *c, int32_t num_tokens)
{
    CacheView cv;
    if (check_cache(c, &cv) != ALISE_OK || num_tokens <= 0) return 0;
    const int64_t nblk = ((int64_t)num_tokens + cv.P - 1) / cv.P;
    return (size_t)(nblk * cv.Hkv * alise::swap_block_bytes(cv));
}

static int swap_call(const alise_kv_cache *c, const int32_t *block_table, int32_t num_tokens, void *packed,
                     size_t packed_bytes, bool upload, void *hip_stream)
{
    CacheView cv;
    int st = check_cache(c, &cv);
    if (st != ALISE_OK) return st;
    if (num_tokens < 0) return ALISE_INVALID_ARGUMENT;
    if ((int64_t)num_tokens > (int64_t)cv.num_pages * cv.P) return ALISE_INVALID_ARGUMENT;
    if (num_tokens == 0) return ALISE_OK;
    if (!block_table || !packed) return ALISE_INVALID_ARGUMENT;
    if (packed_bytes < alise_kv_swap_bytes(c, num_tokens)) return ALISE_INVALID_ARGUMENT;
    st = check_cache_pointers(c);
    if (st != ALISE_OK) return st;
    if (!aligned16(packed) || (reinterpret_cast<uintptr_t>(block_table) & 3u)) return ALISE_MISALIGNED;
    if (debug_validate()) {
        std::vector<int32_t> bt;
        st = fetch_to_host(bt, block_table, (size_t)(((int64_t)num_tokens + cv.P - 1) / cv.P), static_cast<hipStream_t>(hip_stream));
        if (st != ALISE_OK) return st;
        for (int32_t page : bt)
            if (page < 0 || page >= cv.num_pages) return ALISE_INVALID_ARGUMENT;
        std::sort(bt.begin(), bt.end());
        if (std::adjacent_find(bt.begin(), bt.end()) != bt.end()) return ALISE_INVALID_ARGUMENT;      // one page, two places in the request
    }
    hipError_t e = alise::launch_swap(cv, block_table, num_tokens, packed, upload, num_compute_units(),
                                      static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? ALISE_OK : ALISE_HIP_ERROR;
}

int alise_kv_swap_out(const alise_kv_cache *c, const int32_t *block_table, int32_t num_tokens,
                      void *packed, size_t packed_bytes, void *hip_stream)
{
    return swap_call(c, block_table, num_tokens, packed, packed_bytes, false, hip_stream);
}

int alise_kv_swap_in(const alise_kv_cache *c, const int32_t *block_table, int32_t num_tokens,
                     const void *packed, size_t packed_bytes, void *hip_stream)
{
    return swap_call(c, block_table, num_tokens, const_cast<void *>(packed), packed_bytes, true, hip_stream);
}

const char *alise_status_string(int status)
{
    switch (status) {
    case ALISE_OK: return "ALISE_OK";
    case ALISE_INVALID_ARGUMENT: return "ALISE_INVALID_ARGUMENT";
    case ALISE_UNSUPPORTED: return "ALISE_UNSUPPORTED";
    case ALISE_WORKSPACE_TOO_SMALL: return "ALISE_WORKSPACE_TOO_SMALL";
    case ALISE_MISALIGNED: return "ALISE_MISALIGNED";
    case ALISE_HIP_ERROR: return "ALISE_HIP_ERROR";
    default: return "ALISE_UNKNOWN_STATUS";
    }
}

}  // extern "C"
