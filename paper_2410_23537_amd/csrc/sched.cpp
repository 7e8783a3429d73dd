// Host-side speculative scheduler and swapping policy behind the C ABI of alise_sched.h.
//
// ALISE Sec. 3.1 (Eq. 3-5, "Preemptive Scheduling") and Sec. 3.2 ("Dynamic Swapping", the EWT
// equations, Alg. 2).  One pass per iteration over the live jobs: key every job (queue,
// estimated wait time, tie-breakers), sort once, then walk the sorted list queue by queue with
// the GPU job budget of Alg. 2.  The per-queue sums of the EWT equation come from one prefix
// pass over the queue totals, so the whole step is O(n log n) in the live jobs.
#include "../../include/alise_sched.h"

#include <algorithm>
#include <cstdint>
#include <limits>
#include <new>
#include <unordered_map>
#include <vector>

namespace {

enum Where : int32_t { kNoCache = 0, kOnGpu = 1, kOnHost = 2 };

struct Job {
    int64_t id, arrival;
    int64_t s;              // prompt length
    int64_t predicted;      // predicted output length; doubles on a misprediction
    int64_t generated;
    int64_t waited;         // ticks since the job last ran (or arrived)
    int32_t demotions;
    int32_t where;
    bool prefilled;
};

struct Keyed {
    int32_t queue;
    int64_t ewt;
    int32_t fresh;          // 0 for a job promoted by aging, 1 otherwise
    int64_t neg_wait;       // -waited for a promoted job, 0 otherwise
    int64_t remaining, arrival, id;
    size_t slot;            // index into the job table
};

}  // namespace

struct alise_sched {
    alise_sched_config cfg;
    std::vector<Job> jobs;
    std::unordered_map<int64_t, size_t> slot_of;
    std::vector<int64_t> last_batch;
    bool stepped = false;
    // scratch of step(), kept to avoid reallocating every iteration
    std::vector<Keyed> keyed;
    std::vector<int64_t> queue_total;
    std::vector<int32_t> queue_count;

    int64_t remaining(const Job &j) const
    {
        const int64_t per_token = cfg.alpha * j.s + cfg.beta;
        return (j.prefilled ? 0 : j.s * cfg.t0) + (j.predicted - j.generated) * per_token;
    }
    int32_t queue_of(const Job &j, int64_t rem) const
    {
        if (j.waited >= cfg.age_threshold) return 0;
        int32_t i = 0;
        while (i < cfg.num_queues - 1) {
            // limit0 * 2^i, read as "no bound" once it leaves the 64-bit range
            if (cfg.limit0 > (std::numeric_limits<int64_t>::max() >> i)) break;
            if (rem <= cfg.limit0 * ((int64_t)1 << i)) break;
            ++i;
        }
        const int64_t q = (int64_t)i + j.demotions;
        return (int32_t)std::min<int64_t>(q, cfg.num_queues - 1);
    }
};

extern "C" {

int alise_sched_create(const alise_sched_config *cfg, alise_sched **out)
{
    if (!cfg || !out) return ALISE_INVALID_ARGUMENT;
    if (cfg->num_queues < 1 || cfg->num_queues > 62 || cfg->max_batch < 1 || cfg->gpu_job_limit < 1 || cfg->reserved != 0)
        return ALISE_INVALID_ARGUMENT;
    if (cfg->limit0 < 1 || cfg->age_threshold < 1 || cfg->t0 < 0 || cfg->alpha < 0 || cfg->beta < 0) return ALISE_INVALID_ARGUMENT;
    alise_sched *s = new (std::nothrow) alise_sched;
    if (!s) return ALISE_HIP_ERROR;
    s->cfg = *cfg;
    *out = s;
    return ALISE_OK;
}

void alise_sched_destroy(alise_sched *s) { delete s; }

int alise_sched_add_job(alise_sched *s, int64_t id, int64_t arrival, int32_t prompt_len, int32_t predicted_len)
{
    if (!s || prompt_len < 1 || predicted_len < 1) return ALISE_INVALID_ARGUMENT;
    if (s->slot_of.count(id)) return ALISE_INVALID_ARGUMENT;
    Job j{};
    j.id = id;
    j.arrival = arrival;
    j.s = prompt_len;
    j.predicted = predicted_len;
    j.where = kNoCache;
    s->slot_of[id] = s->jobs.size();
    s->jobs.push_back(j);
    return ALISE_OK;
}

int32_t alise_sched_num_jobs(const alise_sched *s) { return s ? (int32_t)s->jobs.size() : 0; }

int alise_sched_step(alise_sched *s, alise_sched_decision *d)
{
    if (!s || !d) return ALISE_INVALID_ARGUMENT;
    if (d->batch_cap < 0 || d->upload_cap < 0 || d->offload_cap < 0 || d->order_cap < 0) return ALISE_INVALID_ARGUMENT;
    if ((d->batch_cap > 0 && (!d->batch_ids || !d->batch_phase)) || (d->upload_cap > 0 && !d->upload_ids) ||
        (d->offload_cap > 0 && !d->offload_ids) || (d->order_cap > 0 && (!d->order_ids || !d->order_queue || !d->order_ewt)))
        return ALISE_INVALID_ARGUMENT;
    const alise_sched_config &c = s->cfg;
    const size_t n = s->jobs.size();
    const bool want_order = d->order_cap > 0;
    if (want_order && (size_t)d->order_cap < n) return ALISE_WORKSPACE_TOO_SMALL;
    if ((size_t)d->batch_cap < std::min<size_t>(n, (size_t)c.max_batch)) return ALISE_WORKSPACE_TOO_SMALL;

    // ---- queue and remaining time of every job; the total of every queue
    s->keyed.resize(n);
    s->queue_total.assign(c.num_queues, 0);
    s->queue_count.assign(c.num_queues, 0);
    for (size_t k = 0; k < n; ++k) {
        const Job &j = s->jobs[k];
        Keyed &e = s->keyed[k];
        e.remaining = s->remaining(j);
        e.queue = s->queue_of(j, e.remaining);
        const bool aged = j.waited >= c.age_threshold;
        e.fresh = aged ? 0 : 1;
        e.neg_wait = aged ? -j.waited : 0;
        e.arrival = j.arrival;
        e.id = j.id;
        e.slot = k;
        s->queue_total[e.queue] += e.remaining;
        s->queue_count[e.queue] += 1;
    }
    // ---- EWT: the work in the queues before the job's own, or the time to promotion if that is sooner
    {
        int64_t ahead = 0;
        std::vector<int64_t> &tot = s->queue_total;         // becomes the exclusive prefix sum
        for (int32_t q = 0; q < c.num_queues; ++q) {
            const int64_t mine = tot[q];
            tot[q] = ahead;
            ahead += mine;
        }
        for (size_t k = 0; k < n; ++k) {
            Keyed &e = s->keyed[k];
            const int64_t promote = std::max<int64_t>(c.age_threshold - s->jobs[e.slot].waited, 0);
            e.ewt = std::min(tot[e.queue], promote);
        }
    }
    std::sort(s->keyed.begin(), s->keyed.end(), [](const Keyed &a, const Keyed &b) {
        if (a.queue != b.queue) return a.queue < b.queue;
        if (a.ewt != b.ewt) return a.ewt < b.ewt;
        if (a.fresh != b.fresh) return a.fresh < b.fresh;
        if (a.neg_wait != b.neg_wait) return a.neg_wait < b.neg_wait;
        if (a.remaining != b.remaining) return a.remaining < b.remaining;
        if (a.arrival != b.arrival) return a.arrival < b.arrival;
        return a.id < b.id;
    });

    // ---- Alg. 2 with the budget of M jobs; a first pass counts, so that nothing changes if a list does not fit
    for (int pass = 0; pass < 2; ++pass) {
        int64_t budget = c.gpu_job_limit;
        int32_t n_batch = 0, n_up = 0, n_off = 0;
        int64_t pre_time = 0, dec_time = 0;
        size_t k = 0;
        for (int32_t q = 0; q < c.num_queues; ++q) {
            const int32_t len = s->queue_count[q];
            for (int32_t i = 0; i < len; ++i, ++k) {
                const Keyed &e = s->keyed[k];
                Job &j = s->jobs[e.slot];
                if (i < budget) {
                    if (j.where == kOnHost) {
                        if (pass) { d->upload_ids[n_up] = j.id; }
                        ++n_up;
                    }
                    if (n_batch < c.max_batch) {
                        if (pass) {
                            d->batch_ids[n_batch] = j.id;
                            d->batch_phase[n_batch] = j.prefilled ? 1 : 0;
                            if (j.prefilled) dec_time = std::max(dec_time, c.alpha * j.s + c.beta);
                            else pre_time += j.s * c.t0;
                        }
                        ++n_batch;
                    }
                } else if (j.where == kOnGpu) {
                    if (pass) { d->offload_ids[n_off] = j.id; }
                    ++n_off;
                }
                if (pass && want_order) {
                    d->order_ids[k] = e.id;
                    d->order_queue[k] = e.queue;
                    d->order_ewt[k] = e.ewt;
                }
            }
            budget = std::max<int64_t>(budget - len, 0);
        }
        if (!pass) {
            if (n_up > d->upload_cap || n_off > d->offload_cap) return ALISE_WORKSPACE_TOO_SMALL;
        } else {
            d->n_batch = n_batch;
            d->n_upload = n_up;
            d->n_offload = n_off;
            d->n_order = want_order ? (int32_t)n : 0;
            d->model_time = pre_time + dec_time;
        }
    }
    for (int32_t i = 0; i < d->n_upload; ++i) s->jobs[s->slot_of[d->upload_ids[i]]].where = kOnGpu;
    for (int32_t i = 0; i < d->n_offload; ++i) s->jobs[s->slot_of[d->offload_ids[i]]].where = kOnHost;
    s->last_batch.assign(d->batch_ids, d->batch_ids + d->n_batch);
    s->stepped = true;
    return ALISE_OK;
}

int alise_sched_commit(alise_sched *s, int64_t elapsed, const int64_t *finished_ids, int32_t n_finished)
{
    if (!s || elapsed < 0 || n_finished < 0 || (n_finished > 0 && !finished_ids) || !s->stepped) return ALISE_INVALID_ARGUMENT;
    for (int32_t i = 0; i < n_finished; ++i)
        if (std::find(s->last_batch.begin(), s->last_batch.end(), finished_ids[i]) == s->last_batch.end()) return ALISE_INVALID_ARGUMENT;
    for (Job &j : s->jobs) j.waited += elapsed;
    for (int64_t id : s->last_batch) {
        Job &j = s->jobs[s->slot_of[id]];
        j.generated += 1;                   // the prompt's iteration yields the first token
        j.prefilled = true;
        j.where = kOnGpu;
        j.waited = 0;
        if (j.generated >= j.predicted) {   // a misprediction, unless the job ends right now (then it is removed below)
            j.predicted *= 2;
            j.demotions += 1;
        }
    }
    for (int32_t i = 0; i < n_finished; ++i) {
        auto it = s->slot_of.find(finished_ids[i]);
        if (it == s->slot_of.end()) continue;       // named twice
        const size_t k = it->second, last = s->jobs.size() - 1;
        s->slot_of.erase(it);
        if (k != last) {
            s->jobs[k] = s->jobs[last];
            s->slot_of[s->jobs[k].id] = k;
        }
        s->jobs.pop_back();
    }
    s->stepped = false;
    s->last_batch.clear();
    return ALISE_OK;
}

}  // extern "C"
