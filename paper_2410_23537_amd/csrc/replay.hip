// The native serving loop around the library's own entry points (alise_replay.h).
//
// ALISE Sec. 3.1 "Preemptive Scheduling" decides the batch of every iteration, Sec. 3.2 "Dynamic
// Swapping" with Alg. 2 decides which preempted job's KV cache stays on the GPU; this file is the
// plumbing that turns those decisions into calls without ever waiting for the GPU in the steady
// state: a page free list, block tables, pinned host buffers recycled by size class, a device
// staging buffer between the swap kernels and the copy engine, a second stream for the swaps with two events that order it against the compute stream, and a ring of
// pinned staging buffers through which the metadata of an iteration (source rows, slots, chunk
// boundaries, lengths, block tables, page lists of the swaps) reaches the device in one copy per
// stream.  The only kernel here gathers the iteration's new token rows into contiguous K, V and Q
// buffers; everything else is alise_kv.h.
#include <algorithm>
#include <cstring>
#include <map>
#include <new>
#include <unordered_map>
#include <utility>
#include <vector>

#include <hip/hip_runtime.h>

#include "../../include/alise_replay.h"

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Row i of each destination is row rows[i] of its source.  One workgroup per token; rows are whole
// numbers of 16-byte units; a thread has four loads in flight before it stores.
__global__ __launch_bounds__(256) void gather_tokens_kernel(const int64_t *__restrict__ rows, const u32x4_t *__restrict__ k,
                                                            const u32x4_t *__restrict__ v, const u32x4_t *__restrict__ q,
                                                            u32x4_t *__restrict__ kd, u32x4_t *__restrict__ vd,
                                                            u32x4_t *__restrict__ qd, int32_t kv_units, int32_t q_units)
{
    const int64_t t = blockIdx.x, r = rows[t];
    const int n = 2 * kv_units + q_units;
    auto src_of = [&](int u) {
        return u < kv_units ? k + r * kv_units + u : u < 2 * kv_units ? v + r * kv_units + (u - kv_units) : q + r * q_units + (u - 2 * kv_units);
    };
    auto dst_of = [&](int u) {
        return u < kv_units ? kd + t * kv_units + u : u < 2 * kv_units ? vd + t * kv_units + (u - kv_units) : qd + t * q_units + (u - 2 * kv_units);
    };
    for (int base = threadIdx.x; base < n; base += 1024) {
        u32x4_t x[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (base + 256 * j < n) x[j] = __builtin_nontemporal_load(src_of(base + 256 * j));
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (base + 256 * j < n) *dst_of(base + 256 * j) = x[j];
    }
}

struct Job {
    int32_t s = 0;                  // prompt length
    int32_t L = 0;                  // tokens in the cache
    int64_t row = 0;                // the job's first row in the token arrays
    std::vector<int32_t> pages;
    void *host = nullptr;           // the offloaded form, pinned
    size_t host_bytes = 0, host_class = 0;
};

constexpr int kStages = 4;

struct Stage {
    uint8_t *main = nullptr, *side = nullptr;       // pinned
    hipEvent_t main_done = nullptr, side_done = nullptr;
    bool main_used = false, side_used = false;
};

struct Release {                    // host buffers that uploads still read until `ev` has passed
    hipEvent_t ev;
    std::vector<std::pair<void *, size_t>> bufs;
};

size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

}  // namespace

struct alise_replay {
    alise_kv_cache cache{};
    alise_sched_config scfg{};
    alise_replay_config cfg{};
    alise_sched *sched = nullptr;
    int32_t max_blocks = 0, kv_units = 0, q_units = 0;
    std::unordered_map<int64_t, Job> jobs;
    std::vector<int32_t> free_pages, pending_free;
    hipStream_t main = nullptr, side = nullptr;
    bool own_side = false;
    hipEvent_t iter_done = nullptr, swap_done = nullptr;
    Stage stage[kStages];
    int64_t iteration = 0;
    size_t main_cap = 0, side_cap = 0;
    uint8_t *dev_main = nullptr, *dev_side = nullptr;
    void *kbuf = nullptr, *vbuf = nullptr, *qbuf = nullptr;
    void *ws_dec = nullptr, *ws_pre = nullptr;
    void *swap_stage = nullptr;     // device staging of one request's offloaded form: the copy engine moves it over the host link
    size_t ws_dec_bytes = 0, ws_pre_bytes = 0;
    std::map<size_t, std::vector<void *>> host_pool;
    std::vector<Release> releases;
    std::vector<hipEvent_t> event_pool;
    // decision buffers of the scheduler
    std::vector<int64_t> d_batch, d_upload, d_offload;
    std::vector<int32_t> d_phase;
    alise_replay_stats stats{};
    bool broken = false;
    bool swaps_unseen = false;      // swap_done has been recorded since the compute stream last waited for it
};

namespace {

void *host_buffer(alise_replay *r, size_t nbytes, size_t *cls_out)
{
    size_t cls = 4096;
    while (cls < nbytes) cls <<= 1;
    *cls_out = cls;
    auto &pool = r->host_pool[cls];
    if (!pool.empty()) {
        void *p = pool.back();
        pool.pop_back();
        return p;
    }
    void *p = nullptr;
    if (hipHostMalloc(&p, cls, hipHostMallocDefault) != hipSuccess) return nullptr;
    return p;
}

// Host buffers whose upload copies have completed go back to the pool; nothing waits.
void recycle_released(alise_replay *r, bool wait)
{
    size_t keep = 0;
    for (size_t i = 0; i < r->releases.size(); ++i) {
        Release &rel = r->releases[i];
        const bool done = wait ? hipEventSynchronize(rel.ev) == hipSuccess : hipEventQuery(rel.ev) == hipSuccess;
        if (done) {
            for (auto &b : rel.bufs) r->host_pool[b.second].push_back(b.first);
            r->event_pool.push_back(rel.ev);
        } else {
            if (keep != i) r->releases[keep] = std::move(rel);
            ++keep;
        }
    }
    r->releases.resize(keep);
}

hipEvent_t take_event(alise_replay *r)
{
    if (!r->event_pool.empty()) {
        hipEvent_t e = r->event_pool.back();
        r->event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
    return e;
}

bool take_pages(alise_replay *r, std::vector<int32_t> &dst, int32_t n)
{
    if ((size_t)n > r->free_pages.size()) return false;
    for (int32_t i = 0; i < n; ++i) {
        dst.push_back(r->free_pages.back());
        r->free_pages.pop_back();
    }
    return true;
}

}  // namespace

extern "C" {

int alise_replay_create(const alise_kv_cache *cache, const alise_sched_config *sched_cfg,
                        const alise_replay_config *cfg, void *hip_stream, alise_replay **out)
{
    if (!cache || !sched_cfg || !cfg || !out) return ALISE_INVALID_ARGUMENT;
    *out = nullptr;
    if (cfg->num_q_heads < 1 || cfg->max_context < 2 || cfg->max_iter_tokens < 1 || cfg->reserved != 0 ||
        !(cfg->softmax_scale > 0.0f))
        return ALISE_INVALID_ARGUMENT;
    if (alise_kv_codes_bytes(cache) == 0) return ALISE_UNSUPPORTED;
    if (cfg->num_q_heads % cache->num_kv_heads != 0) return ALISE_INVALID_ARGUMENT;
    if (sched_cfg->max_batch < 1 || sched_cfg->gpu_job_limit < 1) return ALISE_INVALID_ARGUMENT;
    const int64_t mb = sched_cfg->max_batch, M = sched_cfg->gpu_job_limit;
    const int64_t max_blocks = (cfg->max_context + cache->page_size - 1) / cache->page_size;
    if ((int64_t)cfg->max_iter_tokens + mb >= ((int64_t)1 << 31) || mb * max_blocks >= ((int64_t)1 << 28))
        return ALISE_INVALID_ARGUMENT;

    alise_replay *r = new (std::nothrow) alise_replay();
    if (!r) return ALISE_HIP_ERROR;
    r->cache = *cache;
    r->scfg = *sched_cfg;
    r->cfg = *cfg;
    r->max_blocks = (int32_t)max_blocks;
    r->kv_units = cache->num_kv_heads * cache->head_dim * 2 / 16;
    r->q_units = cfg->num_q_heads * cache->head_dim * 2 / 16;
    r->main = static_cast<hipStream_t>(hip_stream);
    int st = alise_sched_create(sched_cfg, &r->sched);
    if (st != ALISE_OK) {
        delete r;
        return st;
    }
    const int32_t T = cfg->max_iter_tokens;
    r->ws_dec_bytes = alise_paged_decode_attn_workspace_bytes(cache, (int32_t)mb, cfg->num_q_heads, cfg->max_context);
    r->ws_pre_bytes = alise_paged_prefill_attn_workspace_bytes(cache, (int32_t)mb, T, cfg->num_q_heads, cfg->max_context);
    if (r->ws_dec_bytes == 0 || r->ws_pre_bytes == 0) {
        alise_replay_destroy(r);
        return ALISE_UNSUPPORTED;
    }
    // rows + slots, chunk boundaries, two length arrays, two block tables; each piece 16-byte aligned
    r->main_cap = 2 * align16((size_t)T * 8) + 3 * align16((size_t)(mb + 1) * 4) + 2 * align16((size_t)(mb * max_blocks) * 4);
    r->side_cap = align16((size_t)(2 * M * max_blocks) * 4);
    bool ok = true;
    if (cfg->overlap_swaps) {
        ok = ok && hipStreamCreateWithFlags(&r->side, hipStreamNonBlocking) == hipSuccess;
        r->own_side = ok;
    } else {
        r->side = r->main;
    }
    ok = ok && hipEventCreateWithFlags(&r->iter_done, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&r->swap_done, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventRecord(r->iter_done, r->main) == hipSuccess && hipEventRecord(r->swap_done, r->side) == hipSuccess;
    for (int i = 0; ok && i < kStages; ++i) {
        Stage &s = r->stage[i];
        ok = ok && hipHostMalloc((void **)&s.main, r->main_cap, hipHostMallocDefault) == hipSuccess;
        ok = ok && hipHostMalloc((void **)&s.side, r->side_cap, hipHostMallocDefault) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&s.main_done, hipEventDisableTiming) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&s.side_done, hipEventDisableTiming) == hipSuccess;
    }
    ok = ok && hipMalloc((void **)&r->dev_main, r->main_cap) == hipSuccess;
    ok = ok && hipMalloc((void **)&r->dev_side, r->side_cap) == hipSuccess;
    ok = ok && hipMalloc(&r->kbuf, (size_t)T * r->kv_units * 16) == hipSuccess;
    ok = ok && hipMalloc(&r->vbuf, (size_t)T * r->kv_units * 16) == hipSuccess;
    ok = ok && hipMalloc(&r->qbuf, (size_t)T * r->q_units * 16) == hipSuccess;
    ok = ok && hipMalloc(&r->ws_dec, r->ws_dec_bytes) == hipSuccess;
    ok = ok && hipMalloc(&r->ws_pre, r->ws_pre_bytes) == hipSuccess;
    ok = ok && hipMalloc(&r->swap_stage, alise_kv_swap_bytes(cache, cfg->max_context)) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        alise_replay_destroy(r);
        return ALISE_HIP_ERROR;
    }
    r->free_pages.reserve(cache->num_pages);
    for (int32_t p = cache->num_pages - 1; p >= 0; --p) r->free_pages.push_back(p);
    r->d_batch.resize(mb);
    r->d_phase.resize(mb);
    *out = r;
    return ALISE_OK;
}

int alise_replay_synchronize(alise_replay *r)
{
    if (!r) return ALISE_INVALID_ARGUMENT;
    if (hipStreamSynchronize(r->main) != hipSuccess) return ALISE_HIP_ERROR;
    if (r->own_side && hipStreamSynchronize(r->side) != hipSuccess) return ALISE_HIP_ERROR;
    return ALISE_OK;
}

void alise_replay_destroy(alise_replay *r)
{
    if (!r) return;
    (void)alise_replay_synchronize(r);
    recycle_released(r, true);
    for (auto &kv : r->jobs)
        if (kv.second.host) (void)hipHostFree(kv.second.host);
    for (auto &kv : r->host_pool)
        for (void *p : kv.second) (void)hipHostFree(p);
    for (hipEvent_t e : r->event_pool) (void)hipEventDestroy(e);
    for (Stage &s : r->stage) {
        if (s.main) (void)hipHostFree(s.main);
        if (s.side) (void)hipHostFree(s.side);
        if (s.main_done) (void)hipEventDestroy(s.main_done);
        if (s.side_done) (void)hipEventDestroy(s.side_done);
    }
    for (void *p : {(void *)r->dev_main, (void *)r->dev_side, r->kbuf, r->vbuf, r->qbuf, r->ws_dec, r->ws_pre, r->swap_stage})
        if (p) (void)hipFree(p);
    if (r->iter_done) (void)hipEventDestroy(r->iter_done);
    if (r->swap_done) (void)hipEventDestroy(r->swap_done);
    if (r->own_side) (void)hipStreamDestroy(r->side);
    alise_sched_destroy(r->sched);
    delete r;
}

int alise_replay_add_job(alise_replay *r, int64_t id, int64_t arrival, int32_t prompt_len, int32_t predicted_len,
                         int64_t token_row)
{
    if (!r || token_row < 0 || prompt_len < 1 || (int64_t)prompt_len + 1 > r->cfg.max_context ||
        prompt_len > r->cfg.max_iter_tokens)
        return ALISE_INVALID_ARGUMENT;
    const int st = alise_sched_add_job(r->sched, id, arrival, prompt_len, predicted_len);
    if (st != ALISE_OK) return st;
    Job &j = r->jobs[id];
    j.s = prompt_len;
    j.row = token_row;
    return ALISE_OK;
}

int32_t alise_replay_num_jobs(const alise_replay *r) { return r ? alise_sched_num_jobs(r->sched) : 0; }

int alise_replay_get_stats(const alise_replay *r, alise_replay_stats *s)
{
    if (!r || !s) return ALISE_INVALID_ARGUMENT;
    *s = r->stats;
    s->free_pages = (int32_t)(r->free_pages.size() + r->pending_free.size());
    s->live_jobs = alise_sched_num_jobs(r->sched);
    return ALISE_OK;
}

int alise_replay_iterate(alise_replay *r, const void *k_tokens, const void *v_tokens, const void *q_tokens, void *out,
                         alise_replay_iteration *it)
{
    if (!r || !it || !k_tokens || !v_tokens || !q_tokens || !out || r->broken) return ALISE_INVALID_ARGUMENT;
    if (!it->batch_ids || !it->batch_phase || !it->batch_out_row || !it->upload_ids || !it->offload_ids ||
        !it->offload_host || !it->offload_bytes || it->batch_cap < 0 || it->upload_cap < 0 || it->offload_cap < 0)
        return ALISE_INVALID_ARGUMENT;
    const alise_kv_cache *c = &r->cache;
    const int32_t P = c->page_size, n_jobs = alise_sched_num_jobs(r->sched);
    // the caller's lists must hold what the scheduler may decide, checked before it decides
    if (it->batch_cap < std::min(n_jobs, r->scfg.max_batch) || it->upload_cap < std::min(n_jobs, r->scfg.gpu_job_limit) ||
        it->offload_cap < std::min(n_jobs, r->scfg.gpu_job_limit))
        return ALISE_WORKSPACE_TOO_SMALL;
    if ((int32_t)r->d_upload.size() < n_jobs) {
        r->d_upload.resize(n_jobs);
        r->d_offload.resize(n_jobs);
    }
    alise_sched_decision d{};
    d.batch_ids = r->d_batch.data();
    d.batch_phase = r->d_phase.data();
    d.batch_cap = (int32_t)r->d_batch.size();
    d.upload_ids = r->d_upload.data();
    d.upload_cap = (int32_t)r->d_upload.size();
    d.offload_ids = r->d_offload.data();
    d.offload_cap = (int32_t)r->d_offload.size();
    int st = alise_sched_step(r->sched, &d);
    if (st != ALISE_OK) return st;
    it->n_batch = it->n_upload = it->n_offload = 0;
    it->model_time = d.model_time;
    it->n_prefill_tokens = it->n_decode_tokens = 0;
    if (d.n_batch == 0 && d.n_upload == 0 && d.n_offload == 0) return ALISE_OK;
    r->broken = true;               // cleared once the whole iteration is enqueued
    if (d.n_upload > it->upload_cap || d.n_offload > it->offload_cap || d.n_batch > it->batch_cap ||
        (int64_t)(d.n_upload + d.n_offload) * r->max_blocks * 4 > (int64_t)r->side_cap)
        return ALISE_WORKSPACE_TOO_SMALL;

    // ---- what the iteration needs, before anything is enqueued
    int64_t T = 0, n_pre_tokens = 0, pages_wanted = 0;
    int32_t n_pre = 0, n_dec = 0;
    for (int32_t i = 0; i < d.n_upload; ++i) {
        auto f = r->jobs.find(d.upload_ids[i]);
        if (f == r->jobs.end() || !f->second.host) return ALISE_INVALID_ARGUMENT;
        pages_wanted += (f->second.L + P - 1) / P;
    }
    for (int32_t i = 0; i < d.n_offload; ++i) {
        auto f = r->jobs.find(d.offload_ids[i]);
        if (f == r->jobs.end() || f->second.host) return ALISE_INVALID_ARGUMENT;
    }
    for (int32_t i = 0; i < d.n_batch; ++i) {
        auto f = r->jobs.find(d.batch_ids[i]);
        if (f == r->jobs.end()) return ALISE_INVALID_ARGUMENT;
        const Job &j = f->second;
        const int32_t t1 = j.L == 0 ? j.s : j.L + 1;
        if (t1 > r->cfg.max_context) return ALISE_INVALID_ARGUMENT;
        const bool is_upload = j.host != nullptr;
        pages_wanted += (t1 + P - 1) / P - (is_upload ? (j.L + P - 1) / P : (int64_t)j.pages.size());
        T += t1 - (j.L == 0 ? 0 : j.L);
        if (d.batch_phase[i] == 0) {
            ++n_pre;
            n_pre_tokens += j.s;
        } else {
            ++n_dec;
        }
    }
    if (T > r->cfg.max_iter_tokens || pages_wanted > (int64_t)(r->free_pages.size() + r->pending_free.size()))
        return ALISE_WORKSPACE_TOO_SMALL;

    recycle_released(r, false);
    Stage &sg = r->stage[r->iteration % kStages];
    if (sg.main_used && hipEventSynchronize(sg.main_done) != hipSuccess) return ALISE_HIP_ERROR;
    if (sg.side_used && hipEventSynchronize(sg.side_done) != hipSuccess) return ALISE_HIP_ERROR;
    sg.main_used = sg.side_used = false;

    // pages given up by the offloads and the finished jobs of the last iteration: every later writer is ordered
    // behind those copies and that iteration
    if (r->swaps_unseen) {          // nothing to wait for when no swap has been enqueued since the last wait
        if (hipStreamWaitEvent(r->main, r->swap_done, 0) != hipSuccess) return ALISE_HIP_ERROR;
        r->swaps_unseen = false;
    }
    r->free_pages.insert(r->free_pages.end(), r->pending_free.begin(), r->pending_free.end());
    r->pending_free.clear();

    // ---- the swaps
    if (d.n_offload + d.n_upload > 0) {
        if (hipStreamWaitEvent(r->side, r->iter_done, 0) != hipSuccess) return ALISE_HIP_ERROR;     // they see what the last iteration wrote
        int32_t *lists = reinterpret_cast<int32_t *>(sg.side);
        size_t n_ints = 0;
        std::vector<size_t> at(d.n_offload + d.n_upload);
        for (int32_t i = 0; i < d.n_offload; ++i) {
            Job &j = r->jobs[d.offload_ids[i]];
            at[i] = n_ints;
            std::memcpy(lists + n_ints, j.pages.data(), j.pages.size() * 4);
            n_ints += j.pages.size();
        }
        for (int32_t i = 0; i < d.n_upload; ++i) {
            Job &j = r->jobs[d.upload_ids[i]];
            if (!take_pages(r, j.pages, (j.L + P - 1) / P)) return ALISE_WORKSPACE_TOO_SMALL;
            at[d.n_offload + i] = n_ints;
            std::memcpy(lists + n_ints, j.pages.data(), j.pages.size() * 4);
            n_ints += j.pages.size();
        }
        if (hipMemcpyAsync(r->dev_side, sg.side, n_ints * 4, hipMemcpyHostToDevice, r->side) != hipSuccess ||
            hipEventRecord(sg.side_done, r->side) != hipSuccess)
            return ALISE_HIP_ERROR;
        sg.side_used = true;
        const int32_t *dev_lists = reinterpret_cast<const int32_t *>(r->dev_side);
        for (int32_t i = 0; i < d.n_offload; ++i) {
            Job &j = r->jobs[d.offload_ids[i]];
            const size_t n = alise_kv_swap_bytes(c, j.L);
            size_t cls = 0;
            void *buf = host_buffer(r, n, &cls);
            if (!buf) return ALISE_HIP_ERROR;
            // gathered into device memory by the kernel, moved to the host by the copy engine: a kernel that writes host
            // memory itself slows an attention call running beside it by a third, the copy engine does not
            st = alise_kv_swap_out(c, dev_lists + at[i], j.L, r->swap_stage, n, r->side);
            if (st != ALISE_OK) return st;
            if (hipMemcpyAsync(buf, r->swap_stage, n, hipMemcpyDeviceToHost, r->side) != hipSuccess) return ALISE_HIP_ERROR;
            r->pending_free.insert(r->pending_free.end(), j.pages.begin(), j.pages.end());
            j.pages.clear();
            j.host = buf;
            j.host_bytes = n;
            j.host_class = cls;
            it->offload_ids[i] = d.offload_ids[i];
            it->offload_host[i] = buf;
            it->offload_bytes[i] = n;
            r->stats.offloads += 1;
            r->stats.offload_bytes += (int64_t)n;
        }
        Release rel;
        rel.ev = nullptr;
        for (int32_t i = 0; i < d.n_upload; ++i) {
            Job &j = r->jobs[d.upload_ids[i]];
            if (hipMemcpyAsync(r->swap_stage, j.host, j.host_bytes, hipMemcpyHostToDevice, r->side) != hipSuccess)
                return ALISE_HIP_ERROR;
            st = alise_kv_swap_in(c, dev_lists + at[d.n_offload + i], j.L, r->swap_stage, j.host_bytes, r->side);
            if (st != ALISE_OK) return st;
            rel.bufs.emplace_back(j.host, j.host_class);
            r->stats.uploads += 1;
            r->stats.upload_bytes += (int64_t)j.host_bytes;
            j.host = nullptr;
            j.host_bytes = j.host_class = 0;
            it->upload_ids[i] = d.upload_ids[i];
        }
        if (hipEventRecord(r->swap_done, r->side) != hipSuccess) return ALISE_HIP_ERROR;
        r->swaps_unseen = true;
        if (!rel.bufs.empty()) {
            // the uploads read their host buffers until the swap stream has passed this point
            rel.ev = take_event(r);
            if (!rel.ev || hipEventRecord(rel.ev, r->side) != hipSuccess) return ALISE_HIP_ERROR;
            r->releases.push_back(std::move(rel));
            // a job that runs now needs its cache back first (the batch is short: a linear search)
            bool in_batch = false;
            for (int32_t i = 0; i < d.n_upload && !in_batch; ++i)
                in_batch = std::find(d.batch_ids, d.batch_ids + d.n_batch, d.upload_ids[i]) != d.batch_ids + d.n_batch;
            if (in_batch) {
                if (hipStreamWaitEvent(r->main, r->swap_done, 0) != hipSuccess) return ALISE_HIP_ERROR;
                r->swaps_unseen = false;
            }
        }
    }
    it->n_offload = d.n_offload;
    it->n_upload = d.n_upload;

    // ---- the batch: phase-0 jobs first, then phase-1 jobs, each group in batch order
    if (d.n_batch > 0) {
        uint8_t *blob = sg.main;
        size_t off = 0;
        auto carve = [&](size_t bytes) {
            const size_t at = off;
            off += align16(bytes);
            return at;
        };
        const size_t o_rows = carve((size_t)T * 8), o_slots = carve((size_t)T * 8), o_qstart = carve((size_t)(n_pre + 1) * 4),
                     o_lpre = carve((size_t)n_pre * 4), o_ldec = carve((size_t)n_dec * 4),
                     o_bpre = carve((size_t)n_pre * r->max_blocks * 4), o_bdec = carve((size_t)n_dec * r->max_blocks * 4);
        if (off > r->main_cap) return ALISE_WORKSPACE_TOO_SMALL;
        int64_t *rows = reinterpret_cast<int64_t *>(blob + o_rows), *slots = reinterpret_cast<int64_t *>(blob + o_slots);
        int32_t *q_start = reinterpret_cast<int32_t *>(blob + o_qstart), *l_pre = reinterpret_cast<int32_t *>(blob + o_lpre),
                *l_dec = reinterpret_cast<int32_t *>(blob + o_ldec), *b_pre = reinterpret_cast<int32_t *>(blob + o_bpre),
                *b_dec = reinterpret_cast<int32_t *>(blob + o_bdec);
        int64_t row_pre = 0, row_dec = n_pre_tokens;
        int32_t i_pre = 0, i_dec = 0, max_pre = 0, max_dec = 0;
        q_start[0] = 0;
        for (int32_t i = 0; i < d.n_batch; ++i) {
            Job &j = r->jobs[d.batch_ids[i]];
            const bool pre = d.batch_phase[i] == 0;
            const int32_t t0 = j.L == 0 ? 0 : j.L, t1 = j.L == 0 ? j.s : j.L + 1;
            const int32_t need = (t1 + P - 1) / P - (int32_t)j.pages.size();
            if (need > 0 && !take_pages(r, j.pages, need)) return ALISE_WORKSPACE_TOO_SMALL;
            int64_t &row = pre ? row_pre : row_dec;
            it->batch_ids[i] = d.batch_ids[i];
            it->batch_phase[i] = d.batch_phase[i];
            it->batch_out_row[i] = row;
            for (int32_t t = t0; t < t1; ++t, ++row) {
                rows[row] = j.row + t;
                slots[row] = (int64_t)j.pages[t / P] * P + t % P;
            }
            j.L = t1;
            int32_t *bt = pre ? b_pre + (size_t)i_pre * r->max_blocks : b_dec + (size_t)i_dec * r->max_blocks;
            std::memcpy(bt, j.pages.data(), j.pages.size() * 4);
            std::memset(bt + j.pages.size(), 0, (r->max_blocks - j.pages.size()) * 4);
            if (pre) {
                l_pre[i_pre] = t1;
                q_start[i_pre + 1] = (int32_t)row;
                max_pre = std::max(max_pre, t1);
                ++i_pre;
            } else {
                l_dec[i_dec] = t1;
                max_dec = std::max(max_dec, t1);
                ++i_dec;
            }
        }
        it->n_batch = d.n_batch;
        it->n_prefill_tokens = (int32_t)n_pre_tokens;
        it->n_decode_tokens = n_dec;
        if (hipMemcpyAsync(r->dev_main, blob, off, hipMemcpyHostToDevice, r->main) != hipSuccess ||
            hipEventRecord(sg.main_done, r->main) != hipSuccess)
            return ALISE_HIP_ERROR;
        sg.main_used = true;
        const uint8_t *dm = r->dev_main;
        hipLaunchKernelGGL(gather_tokens_kernel, dim3((uint32_t)T), dim3(256), 0, r->main,
                           reinterpret_cast<const int64_t *>(dm + o_rows), static_cast<const u32x4_t *>(k_tokens),
                           static_cast<const u32x4_t *>(v_tokens), static_cast<const u32x4_t *>(q_tokens),
                           static_cast<u32x4_t *>(r->kbuf), static_cast<u32x4_t *>(r->vbuf), static_cast<u32x4_t *>(r->qbuf),
                           r->kv_units, r->q_units);
        if (hipGetLastError() != hipSuccess) return ALISE_HIP_ERROR;
        st = alise_kv_quant_write(c, r->kbuf, r->vbuf, reinterpret_cast<const int64_t *>(dm + o_slots), (int32_t)T, r->main);
        if (st != ALISE_OK) return st;
        const size_t q_row_bytes = (size_t)r->q_units * 16;
        if (n_pre > 0) {
            st = alise_paged_prefill_attn(c, r->qbuf, out, reinterpret_cast<const int32_t *>(dm + o_qstart),
                                          reinterpret_cast<const int32_t *>(dm + o_bpre), r->max_blocks,
                                          reinterpret_cast<const int32_t *>(dm + o_lpre), n_pre, (int32_t)n_pre_tokens,
                                          r->cfg.num_q_heads, max_pre, r->cfg.softmax_scale, r->ws_pre, r->ws_pre_bytes, r->main);
            if (st != ALISE_OK) return st;
        }
        if (n_dec > 0) {
            st = alise_paged_decode_attn(c, static_cast<const uint8_t *>(r->qbuf) + n_pre_tokens * q_row_bytes,
                                         static_cast<uint8_t *>(out) + n_pre_tokens * q_row_bytes,
                                         reinterpret_cast<const int32_t *>(dm + o_bdec), r->max_blocks,
                                         reinterpret_cast<const int32_t *>(dm + o_ldec), n_dec, r->cfg.num_q_heads, max_dec,
                                         r->cfg.softmax_scale, r->ws_dec, r->ws_dec_bytes, r->main);
            if (st != ALISE_OK) return st;
        }
        r->stats.prefill_tokens += n_pre_tokens;
        r->stats.decode_tokens += n_dec;
    }
    if (hipEventRecord(r->iter_done, r->main) != hipSuccess) return ALISE_HIP_ERROR;
    r->stats.iterations += 1;
    r->iteration += 1;
    r->broken = false;
    return ALISE_OK;
}

int alise_replay_commit(alise_replay *r, int64_t elapsed, const int64_t *finished_ids, int32_t n_finished)
{
    if (!r || r->broken || n_finished < 0 || (n_finished > 0 && !finished_ids)) return ALISE_INVALID_ARGUMENT;
    const int st = alise_sched_commit(r->sched, elapsed, finished_ids, n_finished);
    if (st != ALISE_OK) return st;
    for (int32_t i = 0; i < n_finished; ++i) {
        auto f = r->jobs.find(finished_ids[i]);
        if (f == r->jobs.end()) continue;
        // the iteration that read these pages is ordered before any reuse
        r->pending_free.insert(r->pending_free.end(), f->second.pages.begin(), f->second.pages.end());
        r->jobs.erase(f);
    }
    return ALISE_OK;
}

}  // extern "C"
