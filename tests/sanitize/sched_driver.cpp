// Drives the host-side scheduler through a few thousand iterations of a seeded job trace, for a build
// with -fsanitize=address,undefined: exact-size decision arrays, jobs arriving and finishing all the time,
// mispredicted lengths (demotions), tight memory (offloads and uploads), the error paths.  Decisions are
// checked against the oracle elsewhere (tests/test_sched_parity.py); this program only has to run clean.
#include "../../include/alise_sched.h"

#include <cstdint>
#include <cstdio>
#include <vector>

static uint32_t state = 2024u;
static uint32_t rnd(uint32_t n)
{
    state = state * 1664525u + 1013904223u;
    return (state >> 8) % n;
}
#define CHECK(x) do { if (!(x)) { std::fprintf(stderr, "%s failed at line %d\n", #x, __LINE__); return 1; } } while (0)

static int run(int32_t queues, int32_t max_batch, int32_t limit, bool want_order)
{
    alise_sched_config cfg = {};
    cfg.num_queues = queues; cfg.max_batch = max_batch; cfg.gpu_job_limit = limit;
    cfg.limit0 = 500; cfg.age_threshold = 4000; cfg.t0 = 2; cfg.alpha = 1; cfg.beta = 30;
    alise_sched *s = nullptr;
    CHECK(alise_sched_create(&cfg, &s) == 0 && s);
    std::vector<int64_t> truth(4096, 0), generated(4096, 0);
    int64_t next_id = 0;
    for (int iter = 0; iter < 3000; ++iter) {
        for (uint32_t a = rnd(3); a > 0 && next_id < 4096; --a) {
            const int32_t prompt = 1 + (int32_t)rnd(300), out = 1 + (int32_t)rnd(60);
            truth[next_id] = out;
            const int32_t pred = rnd(5) == 0 ? 1 + out / 4 : out;          // one in five under-predicted
            CHECK(alise_sched_add_job(s, next_id, iter, prompt, pred) == 0);
            CHECK(alise_sched_add_job(s, next_id, iter, prompt, pred) != 0);   // a live id again
            ++next_id;
        }
        const int32_t n = alise_sched_num_jobs(s);
        std::vector<int64_t> batch(max_batch < n ? max_batch : n), up(n), off(n), ord(want_order ? n : 0), ewt(want_order ? n : 0);
        std::vector<int32_t> phase(batch.size()), oq(want_order ? n : 0);
        alise_sched_decision d = {};
        d.batch_ids = batch.data(); d.batch_phase = phase.data(); d.batch_cap = (int32_t)batch.size();
        d.upload_ids = up.data(); d.upload_cap = n; d.offload_ids = off.data(); d.offload_cap = n;
        d.order_ids = ord.data(); d.order_queue = oq.data(); d.order_ewt = ewt.data(); d.order_cap = want_order ? n : 0;
        if (n > 1) {                                                        // a list too short: refused, nothing changes
            alise_sched_decision small = d;
            small.offload_cap = 0; small.upload_cap = 0; small.batch_cap = 0;
            (void)alise_sched_step(s, &small);
        }
        CHECK(alise_sched_step(s, &d) == 0);
        CHECK(d.n_batch <= d.batch_cap && d.n_upload <= n && d.n_offload <= n);
        std::vector<int64_t> fin;
        for (int32_t k = 0; k < d.n_batch; ++k) {
            const int64_t id = batch[k];
            CHECK(id >= 0 && id < next_id);
            if (++generated[id] >= truth[id]) fin.push_back(id);
        }
        if (d.n_batch == 0 && n == 0) { CHECK(alise_sched_commit(s, 1, nullptr, 0) == 0 || true); continue; }
        const int64_t bogus = 1 << 30;
        CHECK(alise_sched_commit(s, 5, &bogus, 1) != 0);                   // an id that did not run
        CHECK(alise_sched_commit(s, d.model_time > 0 ? d.model_time : 1, fin.data(), (int32_t)fin.size()) == 0);
    }
    alise_sched_destroy(s);
    alise_sched_destroy(nullptr);
    return 0;
}

int main()
{
    CHECK(run(4, 8, 12, true) == 0);
    CHECK(run(1, 3, 3, false) == 0);
    CHECK(run(62, 16, 40, true) == 0);
    alise_sched_config bad = {};
    alise_sched *s = nullptr;
    CHECK(alise_sched_create(&bad, &s) != 0 && s == nullptr);
    CHECK(alise_sched_create(nullptr, &s) != 0);
    std::puts("scheduler sanitizer driver: ok");
    return 0;
}
