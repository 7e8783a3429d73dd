"""Pins for the oracle of the speculative scheduler and the swapping decisions (ALISE Sec. 3.1,
Eq. 3-5 and "Preemptive Scheduling"; Sec. 3.2 "Dynamic Swapping", the EWT equations, Alg. 2).
CPU only.

Pins: hand-worked values of Eq. 3-5, of the queue bounds, of EWT and of one pass of Alg. 2;
the textbook policies the scheduler must reduce to (shortest remaining time first with one
queue, perfect predictions and one job per iteration, against a brute-force SRTF written here;
first come first served when all predictions are equal); the demote-and-double sequence of a
mispredicted job; the starvation bound that aging gives; invariants on seeded traces."""
import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2410_23537_amd import workloads as wl

BIG = 10 ** 12


def cfg(**kw):
    base = dict(num_queues=1, limit0=BIG, age_threshold=BIG, max_batch=1, gpu_job_limit=10 ** 6, t0=0, alpha=0, beta=1)
    base.update(kw)
    return so.Config(**base)


def test_remaining_time_is_eq_3_to_5_on_the_rest_of_the_job():
    s = so.Scheduler(cfg(t0=2, alpha=1, beta=10))
    s.add_job(0, 0, 100, 5)
    j = s.jobs[0]
    assert s.remaining(j) == 100 * 2 + 5 * (1 * 100 + 10) == 750          # T_pre(s) + T_dec(s, n)
    j.prefilled, j.generated = True, 1
    assert s.remaining(j) == 4 * 110 == 440                              # the prompt is done, four tokens to go


@pytest.mark.parametrize("r, want", [(1, 0), (100, 0), (101, 1), (200, 1), (201, 2), (400, 2), (401, 3), (10 ** 9, 3)])
def test_queue_bounds_double(r, want):
    s = so.Scheduler(cfg(num_queues=4, limit0=100))
    s.add_job(0, 0, 1, r)                # beta = 1, nothing else: remaining time = predicted length
    assert s.level(s.jobs[0]) == want


def test_ewt_is_the_smaller_of_the_work_ahead_and_the_time_to_promotion():
    K = 1000
    s = so.Scheduler(cfg(num_queues=2, limit0=60, age_threshold=K, max_batch=4))
    for id, n in enumerate((30, 50, 200, 300)):
        s.add_job(id, 0, 1, n)
    s.jobs[2].waited = K - 20
    d = s.step()
    assert d.order == [0, 1, 2, 3] and d.level == [0, 0, 1, 1]
    # nothing is ahead of the highest queue; 30 + 50 ticks of work are ahead of the second one;
    # job 2 is promoted in 20 ticks, sooner than that work is done
    assert d.ewt == [0, 0, 20, 80]


def test_one_pass_of_alg_2_by_hand():
    # M = 3.  Q0 = {a, b} in the GPU; Q1 = {c offloaded, d in the GPU}; Q2 = {e in the GPU}.
    # Q0 takes two places, one is left: c (first of Q1) is uploaded, d is offloaded, the budget is spent, e is offloaded.
    s = so.Scheduler(cfg(num_queues=3, limit0=10, gpu_job_limit=3, max_batch=2))
    for id, n in enumerate((5, 8, 15, 18, 100)):
        s.add_job(id, 0, 1, n)
    for id, st in enumerate((so.RESIDENT, so.RESIDENT, so.OFFLOADED, so.RESIDENT, so.RESIDENT)):
        s.jobs[id].state, s.jobs[id].prefilled, s.jobs[id].generated = st, True, 1
    d = s.step()
    assert d.level == [0, 0, 1, 1, 2]
    assert d.upload == [2] and d.offload == [3, 4]
    assert d.batch == [0, 1] and d.phase == [1, 1]
    assert [s.jobs[i].state for i in range(5)] == [so.RESIDENT, so.RESIDENT, so.RESIDENT, so.OFFLOADED, so.OFFLOADED]
    # a job without a cache is neither uploaded nor offloaded, but takes a place
    s2 = so.Scheduler(cfg(num_queues=1, gpu_job_limit=1))
    s2.add_job(0, 0, 1, 3)
    s2.add_job(1, 0, 1, 9)
    s2.jobs[1].state, s2.jobs[1].prefilled, s2.jobs[1].generated = so.RESIDENT, True, 1
    d = s2.step()
    assert d.batch == [0] and d.phase == [0] and d.upload == [] and d.offload == [1]


def _srtf_brute_force(arrival, n):
    """Textbook preemptive shortest-remaining-time-first, one unit of work per tick, ties by arrival then index."""
    left = list(n)
    done = {}
    now = 0
    while len(done) < len(n):
        live = [i for i in range(len(n)) if arrival[i] <= now and left[i] > 0]
        if not live:
            now = min(arrival[i] for i in range(len(n)) if left[i] > 0)
            continue
        i = min(live, key=lambda i: (left[i], arrival[i], i))
        left[i] -= 1
        now += 1
        if left[i] == 0:
            done[i] = now
    return done


def _run_unit_ticks(c, arrival, n, pred):
    """Drive the scheduler with a clock of one tick per iteration (every iteration yields one token per job of
    the batch, the prompt's iteration included).  Returns (first job of every batch, completion time per job)."""
    s = so.Scheduler(c)
    left, done, heads = list(n), {}, []
    now = 0
    while len(done) < len(n):
        for i in range(len(n)):
            if arrival[i] == now:
                s.add_job(i, now, 1, pred[i])
        if s.jobs:
            d = s.step()
            heads.append(d.batch[0])
            fin = []
            for id in d.batch:
                left[id] -= 1
                if left[id] == 0:
                    fin.append(id)
                    done[id] = now + 1
            s.commit(d, 1, fin)
        now += 1
    return heads, done


def test_one_queue_and_perfect_predictions_is_shortest_remaining_time_first():
    assert _run_unit_ticks(cfg(), [0, 0, 0, 0], [5, 2, 9, 1], [5, 2, 9, 1])[1] == {3: 1, 1: 3, 0: 8, 2: 17}
    # a short job that arrives later preempts the long one
    assert _run_unit_ticks(cfg(), [0, 3], [10, 2], [10, 2])[1] == {1: 5, 0: 12}
    rng = np.random.default_rng(12)
    for _ in range(5):
        m = 12
        arrival = np.sort(rng.integers(0, 40, m)).tolist()
        n = rng.integers(1, 15, m).tolist()
        _, done = _run_unit_ticks(cfg(), arrival, n, n)
        assert done == _srtf_brute_force(arrival, n)


def test_equal_predictions_are_first_come_first_served():
    arrival, n = [0, 1, 2, 3], [4, 4, 4, 4]
    heads, done = _run_unit_ticks(cfg(), arrival, n, n)
    assert heads == [0] * 4 + [1] * 4 + [2] * 4 + [3] * 4
    assert done == {0: 4, 1: 8, 2: 12, 3: 16}


def test_a_mispredicted_job_is_demoted_and_its_prediction_doubled():
    s = so.Scheduler(cfg(num_queues=4))
    s.add_job(0, 0, 1, 2)                 # predicted 2, truly 5
    levels, preds = [], []
    for it in range(5):
        d = s.step()
        levels.append(d.level[0])
        preds.append(s.jobs[0].predicted)
        s.commit(d, 1, [0] if it == 4 else [])
    assert preds == [2, 2, 4, 4, 8]       # doubled when the 2nd and the 4th token came out without an end
    assert levels == [0, 0, 1, 1, 2]
    assert not s.jobs


def test_aging_bounds_the_wait():
    K = 25
    c = cfg(num_queues=2, limit0=5, age_threshold=K, max_batch=2)
    s = so.Scheduler(c)
    s.add_job(0, 0, 1, 500)               # the long job; two fresh one-token jobs arrive every tick
    nxt = 1
    ran_at = None
    for now in range(200):
        for _ in range(2):
            s.add_job(nxt, now, 1, 1)
            nxt += 1
        d = s.step()
        if 0 in d.batch:
            ran_at = now
            assert d.order[0] == 0 and d.level[0] == 0          # promoted to the head of the highest queue
            break
        s.commit(d, 1, d.batch)
    assert ran_at == K                    # waited exactly K ticks, not one more


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_invariants_on_seeded_traces(seed):
    arrival, s, n, pred = (a.tolist() for a in wl.job_trace(60, seed, mean_gap=30.0))
    c = so.Config(num_queues=4, limit0=2000, age_threshold=20000, max_batch=8, gpu_job_limit=12, t0=2, alpha=1, beta=20)
    trace, done = so.simulate(c, arrival, s, n, pred)
    assert sorted(done) == list(range(60))                        # every job ends
    tokens = np.zeros(60, np.int64)
    state = {}
    for now, d, elapsed in trace:
        assert 1 <= len(d.batch) <= c.max_batch and len(set(d.batch)) == len(d.batch)
        assert sorted(d.order) == sorted(set(d.order)) and set(d.batch) <= set(d.order)
        assert d.batch == d.order[:len(d.batch)]                  # the batch is the head of the priority order
        assert d.level == sorted(d.level)
        for id in d.upload:
            assert state.get(id) == "off"
            state[id] = "gpu"
        for id in d.offload:
            assert state.get(id) == "gpu"
            state[id] = "off"
        for id, ph in zip(d.batch, d.phase):
            assert (ph == 0) == (tokens[id] == 0)
            assert state.get(id, "new") in ("gpu", "new")         # never runs from the host
            state[id] = "gpu"
            tokens[id] += 1
            if tokens[id] == n[id]:
                del state[id]
        assert sum(1 for v in state.values() if v == "gpu") <= c.gpu_job_limit
        assert elapsed > 0
    assert tokens.tolist() == n
    assert any(d.offload for _, d, _ in trace) and any(d.upload for _, d, _ in trace)        # the trace does exercise Alg. 2


def test_model_time_of_an_iteration():
    s = so.Scheduler(cfg(max_batch=4, t0=3, alpha=2, beta=7))
    for id, (sl, st) in enumerate(((10, 0), (20, 0), (5, 1), (40, 1))):
        s.add_job(id, 0, sl, 100)
        if st:
            s.jobs[id].prefilled, s.jobs[id].generated, s.jobs[id].state = True, 1, so.RESIDENT
    d = s.step()
    assert sorted(d.batch) == [0, 1, 2, 3]
    # two prompts of 10 and 20 tokens one after the other (Eq. 4), the decode jobs together, as slow as the one with the longest input (Eq. 5)
    assert s.model_time(d) == 3 * 10 + 3 * 20 + (2 * 40 + 7)
