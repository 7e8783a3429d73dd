"""CPU oracle of the speculative scheduler and of the swapping decisions (ALISE Sec. 3.1
"Predicting Execution Runtime", Eq. 3-5; "Preemptive Scheduling"; Sec. 3.2 "Dynamic Swapping",
the EWT equations and Alg. 2).

TEST INFRASTRUCTURE ONLY: plain, slow Python that takes the paper's steps in the paper's order.
Nothing in the product path may import it; it shares no code with the C++ scheduler.

All times are integer ticks, all state is integer: two implementations of the same readings
must produce the same decisions bit for bit.

Readings where the paper is silent or at odds with itself (all listed in the design notes):
  S1  the remaining time of a job is Eq. 3-5 on what is left of it: the prefill term s*T0 while
      the prompt has not been processed, plus (predicted - generated) decode iterations of
      alpha*s + beta each, s the INPUT length as in Eq. 5.
  S2  h priority queues; queue i (0 = highest) takes jobs whose remaining time is at most
      limit0 * 2^i, the last queue everything else; recomputed every iteration.
  S3  a job that exceeds its predicted length has the prediction doubled and is demoted by one
      queue for good (demotions add to the queue index of S2, capped at the last queue).
  S4  virtual aging: a job that has waited K ticks since it last ran (or arrived) sits at the
      head of the highest queue until it runs (several such jobs: the longest wait first), which
      is what keeps it from starving; T_promote(J, K) = max(K - waited, 0).
  S5  EWT(J) = min(sum of the remaining times of the jobs in queues of higher priority than
      J's, T_promote(J, K)); inside a queue jobs are sorted by EWT, ties: promoted jobs (S4)
      first, then by remaining time, then arrival, then id.
  S6  Alg. 2: walking the queues in priority order with a budget of M jobs, the first jobs of
      each queue (in its EWT order) stay in or are uploaded to the GPU while the budget lasts,
      the rest are offloaded if they are there; the budget shrinks by the queue's length, not
      below zero.  (The printed listing offloads in its else-branch also jobs that are in the GPU
      and within the limit; the text says they are kept, and the text is followed.)  A job
      whose prompt has not been processed holds no cache: it is neither uploaded nor offloaded,
      but it counts against the budget once it is within it.
  S7  the batch of an iteration is the first max_batch jobs of that order that are within the
      budget; a job runs its whole prompt in one iteration (its first token comes out of it),
      then one token per iteration.
  S8  the model time of an iteration: the prefill terms of its prefill jobs add up, its decode
      jobs run together and take the longest alpha*s + beta among them.
"""
from __future__ import annotations

from dataclasses import dataclass, field

NEW, RESIDENT, OFFLOADED = 0, 1, 2


@dataclass
class Config:
    num_queues: int          # h
    limit0: int              # remaining-time bound of the highest queue, ticks
    age_threshold: int       # K, ticks
    max_batch: int
    gpu_job_limit: int       # M
    t0: int                  # Eq. 4
    alpha: int               # Eq. 5
    beta: int


@dataclass
class Job:
    id: int
    arrival: int
    s: int                   # input length
    predicted: int           # predicted output length (doubles on misprediction)
    generated: int = 0
    prefilled: bool = False
    demotions: int = 0
    waited: int = 0
    state: int = NEW


@dataclass
class Decision:
    batch: list = field(default_factory=list)        # job ids, in priority order
    phase: list = field(default_factory=list)        # 0 = prefill, 1 = decode, per batch entry
    upload: list = field(default_factory=list)       # job ids whose cache comes back to the GPU
    offload: list = field(default_factory=list)      # job ids whose cache leaves the GPU
    order: list = field(default_factory=list)        # every live job id in priority order
    level: list = field(default_factory=list)        # its queue
    ewt: list = field(default_factory=list)          # its estimated wait time


class Scheduler:
    def __init__(self, cfg: Config):
        assert cfg.num_queues >= 1 and cfg.max_batch >= 1 and cfg.gpu_job_limit >= 1
        self.cfg = cfg
        self.jobs: dict[int, Job] = {}

    # ---- Eq. 3-5 on the rest of a job (S1)
    def remaining(self, j: Job) -> int:
        c = self.cfg
        t = 0 if j.prefilled else j.s * c.t0
        return t + (j.predicted - j.generated) * (c.alpha * j.s + c.beta)

    def t_promote(self, j: Job) -> int:
        return max(self.cfg.age_threshold - j.waited, 0)

    def level(self, j: Job) -> int:
        c = self.cfg
        if j.waited >= c.age_threshold:                  # S4
            return 0
        r = self.remaining(j)
        i = 0
        while i < c.num_queues - 1 and r > c.limit0 * (1 << i):     # S2
            i += 1
        return min(i + j.demotions, c.num_queues - 1)    # S3

    def add_job(self, id: int, arrival: int, s: int, predicted: int) -> None:
        assert id not in self.jobs and s >= 1 and predicted >= 1
        self.jobs[id] = Job(id, arrival, s, predicted)

    def step(self) -> Decision:
        c = self.cfg
        queues = [[] for _ in range(c.num_queues)]
        for j in self.jobs.values():
            queues[self.level(j)].append(j)
        d = Decision()
        ahead = 0                                        # remaining time of all jobs in higher queues (Eq. EWT)
        budget = c.gpu_job_limit
        for lvl, q in enumerate(queues):
            ewt = {j.id: min(ahead, self.t_promote(j)) for j in q}                      # S5
            aged = lambda j: j.waited >= c.age_threshold
            q.sort(key=lambda j: (ewt[j.id], 0 if aged(j) else 1, -j.waited if aged(j) else 0,
                                  self.remaining(j), j.arrival, j.id))
            for i, j in enumerate(q):                    # Alg. 2 (S6)
                d.order.append(j.id)
                d.level.append(lvl)
                d.ewt.append(ewt[j.id])
                if i < budget:
                    if j.state == OFFLOADED:
                        d.upload.append(j.id)
                    if len(d.batch) < c.max_batch:       # S7
                        d.batch.append(j.id)
                        d.phase.append(1 if j.prefilled else 0)
                elif j.state == RESIDENT:
                    d.offload.append(j.id)
            budget = max(budget - len(q), 0)
            ahead += sum(self.remaining(j) for j in q)
        for id in d.upload:
            self.jobs[id].state = RESIDENT
        for id in d.offload:
            self.jobs[id].state = OFFLOADED
        return d

    def model_time(self, d: Decision) -> int:
        """S8."""
        c = self.cfg
        pre = sum(self.jobs[id].s * c.t0 for id, ph in zip(d.batch, d.phase) if ph == 0)
        dec = max([c.alpha * self.jobs[id].s + c.beta for id, ph in zip(d.batch, d.phase) if ph == 1], default=0)
        return pre + dec

    def commit(self, d: Decision, elapsed: int, finished) -> None:
        """The batch of `d` ran and took `elapsed` ticks; `finished`: ids of its jobs that ended."""
        ran = set(d.batch)
        finished = set(finished)
        assert finished <= ran
        for j in list(self.jobs.values()):
            if j.id in ran:
                j.generated += 1                         # a prefill yields the first token
                j.prefilled = True
                j.state = RESIDENT
                j.waited = 0
                if j.id in finished:
                    del self.jobs[j.id]
                elif j.generated >= j.predicted:         # S3
                    j.predicted *= 2
                    j.demotions += 1
            else:
                j.waited += elapsed


def simulate(cfg: Config, arrival, s, n_true, n_pred, max_iters=1_000_000):
    """Run a job set to completion with the model time of S8 as the clock.  Returns the list of
    (now, Decision, elapsed) and the completion time per job."""
    sched = Scheduler(cfg)
    n = len(arrival)
    nxt = sorted(range(n), key=lambda i: (arrival[i], i))
    k = 0
    now = 0
    trace, done_at = [], {}
    gen = [0] * n
    for _ in range(max_iters):
        while k < n and arrival[nxt[k]] <= now:
            i = nxt[k]
            sched.add_job(i, arrival[i], s[i], n_pred[i])
            k += 1
        if not sched.jobs:
            if k == n:
                break
            now = arrival[nxt[k]]                        # idle until the next arrival
            continue
        d = sched.step()
        elapsed = sched.model_time(d)
        fin = []
        for id in d.batch:
            gen[id] += 1
            if gen[id] >= n_true[id]:
                fin.append(id)
        sched.commit(d, elapsed, fin)
        now += elapsed
        for id in fin:
            done_at[id] = now
        trace.append((now - elapsed, d, elapsed))
    else:
        raise RuntimeError("simulate: iteration limit reached")
    return trace, done_at
