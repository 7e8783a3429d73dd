"""Parity of the C++ scheduler (alise_sched.h) with the oracle (ALISE Sec. 3.1 Eq. 3-5 and
"Preemptive Scheduling"; Sec. 3.2 EWT and Alg. 2): the same seeded job traces through both,
every iteration's batch, phases, uploads, offloads, full priority order, queues, EWT values
and model time compared bit for bit.  Host code only: runs without a GPU."""
import ctypes

import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2410_23537_amd import workloads as wl


@pytest.fixture(scope="module")
def B():
    from paper_2410_23537_amd import binding
    return binding


CONFIGS = {
    "four_queues": dict(num_queues=4, limit0=2000, age_threshold=20000, max_batch=8, gpu_job_limit=12, t0=2, alpha=1, beta=20),
    "one_queue_fcfs_like": dict(num_queues=1, limit0=10 ** 9, age_threshold=10 ** 12, max_batch=4, gpu_job_limit=1000, t0=1, alpha=0, beta=5),
    "tight_memory": dict(num_queues=3, limit0=500, age_threshold=3000, max_batch=4, gpu_job_limit=4, t0=3, alpha=2, beta=10),
    "aging_dominates": dict(num_queues=6, limit0=100, age_threshold=400, max_batch=2, gpu_job_limit=6, t0=1, alpha=1, beta=1),
    "many_queues": dict(num_queues=62, limit0=1, age_threshold=10 ** 6, max_batch=16, gpu_job_limit=20, t0=5, alpha=3, beta=50),
}


def _run_both(B, cfg, jobs, max_iters=200000):
    arrival, s, n_true, n_pred = (a.tolist() for a in jobs)
    n = len(arrival)
    o = so.Scheduler(so.Config(**cfg))
    p = B.Scheduler(**cfg)
    nxt = sorted(range(n), key=lambda i: (arrival[i], i))
    k, now, iters, swaps = 0, 0, 0, 0
    gen = [0] * n
    while True:
        while k < n and arrival[nxt[k]] <= now:
            i = nxt[k]
            o.add_job(i, arrival[i], s[i], n_pred[i])
            p.add_job(i, arrival[i], s[i], n_pred[i])
            k += 1
        assert p.num_jobs() == len(o.jobs)
        if not o.jobs:
            if k == n:
                break
            now = arrival[nxt[k]]
            continue
        want = o.step()
        got = p.step()
        assert got["batch"] == want.batch and got["phase"] == want.phase, f"iteration {iters}"
        assert got["upload"] == want.upload and got["offload"] == want.offload, f"iteration {iters}"
        assert got["order"] == want.order and got["queue"] == want.level and got["ewt"] == want.ewt, f"iteration {iters}"
        elapsed = o.model_time(want)
        assert got["model_time"] == elapsed
        fin = []
        for id in want.batch:
            gen[id] += 1
            if gen[id] >= n_true[id]:
                fin.append(id)
        o.commit(want, elapsed, fin)
        p.commit(elapsed, fin)
        now += elapsed
        iters += 1
        swaps += len(want.upload) + len(want.offload)
        assert iters < max_iters
    return iters, swaps


@pytest.mark.parametrize("name", list(CONFIGS))
@pytest.mark.parametrize("seed", [1, 7])
def test_every_decision_matches_the_oracle(B, name, seed):
    iters, swaps = _run_both(B, CONFIGS[name], wl.job_trace(80, seed, mean_gap=25.0))
    assert iters > 100
    if name in ("tight_memory", "four_queues", "aging_dominates"):
        assert swaps > 0                      # the trace does exercise Alg. 2


def test_heavy_misprediction_and_bursts(B):
    jobs = wl.job_trace(120, 5, mean_gap=3.0, pred_error=0.5, underestimates=0.5)
    _run_both(B, CONFIGS["tight_memory"], jobs)


def test_overflow_guard_of_the_queue_bounds(B):
    cfg = dict(num_queues=62, limit0=2 ** 40, age_threshold=10 ** 15, max_batch=2, gpu_job_limit=3, t0=10 ** 6, alpha=10 ** 4, beta=10 ** 6)
    _run_both(B, cfg, wl.job_trace(20, 3, mean_gap=10.0))


def test_arguments(B):
    lib = B.raw()
    h = ctypes.c_void_p()
    good = dict(num_queues=2, max_batch=2, gpu_job_limit=2, reserved=0, limit0=10, age_threshold=10, t0=0, alpha=0, beta=1)
    for bad in (dict(num_queues=0), dict(num_queues=63), dict(max_batch=0), dict(gpu_job_limit=0), dict(reserved=1),
                dict(limit0=0), dict(age_threshold=0), dict(t0=-1), dict(alpha=-1), dict(beta=-1)):
        c = B.alise_sched_config(**{**good, **bad})
        assert lib.alise_sched_create(ctypes.byref(c), ctypes.byref(h)) == B.ALISE_INVALID_ARGUMENT
    c = B.alise_sched_config(**good)
    assert lib.alise_sched_create(None, ctypes.byref(h)) == B.ALISE_INVALID_ARGUMENT
    assert lib.alise_sched_create(ctypes.byref(c), None) == B.ALISE_INVALID_ARGUMENT
    assert lib.alise_sched_create(ctypes.byref(c), ctypes.byref(h)) == B.ALISE_OK
    assert lib.alise_sched_add_job(h, 1, 0, 0, 5) == B.ALISE_INVALID_ARGUMENT
    assert lib.alise_sched_add_job(h, 1, 0, 5, 0) == B.ALISE_INVALID_ARGUMENT
    assert lib.alise_sched_add_job(h, 1, 0, 5, 5) == B.ALISE_OK
    assert lib.alise_sched_add_job(h, 1, 0, 5, 5) == B.ALISE_INVALID_ARGUMENT           # already live
    for id in (2, 3, 4):
        assert lib.alise_sched_add_job(h, id, 0, 5, 5 + id) == B.ALISE_OK
    assert lib.alise_sched_num_jobs(h) == 4
    assert lib.alise_sched_commit(h, 1, None, 0) == B.ALISE_INVALID_ARGUMENT            # nothing stepped yet
    ids, ph = (ctypes.c_int64 * 8)(), (ctypes.c_int32 * 8)()
    d = B.alise_sched_decision(ids, ph, 1, 0, ids, 8, 0, ids, 8, 0, None, None, None, 0, 0, 0)
    assert lib.alise_sched_step(h, ctypes.byref(d)) == B.ALISE_WORKSPACE_TOO_SMALL      # two jobs per batch, room for one
    d.batch_cap = 8
    d.order_ids, d.order_cap = ids, 8                                                   # order wanted, but two of its arrays missing
    assert lib.alise_sched_step(h, ctypes.byref(d)) == B.ALISE_INVALID_ARGUMENT
    d.order_ids, d.order_cap = None, 0
    assert lib.alise_sched_step(h, ctypes.byref(d)) == B.ALISE_OK
    assert d.n_batch == 2 and list(ids[:2]) == [1, 2] and d.n_order == 0
    bad = (ctypes.c_int64 * 1)(4)
    assert lib.alise_sched_commit(h, 1, bad, 1) == B.ALISE_INVALID_ARGUMENT             # job 4 was not in the batch
    assert lib.alise_sched_commit(h, -1, None, 0) == B.ALISE_INVALID_ARGUMENT
    fin = (ctypes.c_int64 * 1)(1)
    assert lib.alise_sched_commit(h, 1, fin, 1) == B.ALISE_OK
    assert lib.alise_sched_num_jobs(h) == 3
    assert lib.alise_sched_commit(h, 1, None, 0) == B.ALISE_INVALID_ARGUMENT            # committed already
    lib.alise_sched_destroy(h)
    lib.alise_sched_destroy(None)
    assert lib.alise_sched_num_jobs(None) == 0
