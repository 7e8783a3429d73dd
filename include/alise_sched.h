/*
 * alise_sched.h -- C ABI of the host-side speculative scheduler and KV-cache swapping policy.
 *
 * ALISE (arXiv 2410.23537): jobs are ordered at every iteration by their estimated remaining
 * execution time in a set of priority queues, with virtual aging against starvation and
 * demote-and-double on a misprediction [Sec. 3.1 "Predicting Execution Runtime", Eq. 3-5, and
 * "Preemptive Scheduling"]; the KV caches of preempted jobs are kept in, uploaded to or
 * offloaded from GPU memory by their estimated wait time under a job limit M [Sec. 3.2
 * "Dynamic Swapping", the EWT equations and Alg. 2].  This object takes the decisions; moving
 * the bytes is alise_kv_swap_out / alise_kv_swap_in of alise_kv.h, running the batch is the
 * attention calls there.  The output-length predictor (Sec. 3.1, Alg. 1) is not here: a
 * predicted length comes in with every job.
 *
 * Everything is host memory and host arithmetic, in integer ticks of the caller's choice; no
 * HIP call is made.  The scheduler object owns its job table (the one place in this library
 * that allocates: host memory, at create and add_job); every array in a decision belongs to
 * the caller.  Calls on one object must not overlap.  Status codes are those of alise_kv.h.
 *
 * The rules, where the paper leaves them open:
 *   remaining(J) = (prompt not yet processed ? s * t0 : 0) + (predicted - generated) * (alpha * s + beta),
 *       s the prompt length                                                      [Eq. 3-5]
 *   queue(J) = 0 if J has waited age_threshold ticks since it last ran or arrived (aging), else
 *       min(num_queues - 1, i + demotions), i the smallest index with remaining <= limit0 * 2^i
 *       (the last queue takes the rest)
 *   EWT(J) = min(sum of remaining(.) over the jobs in queues before J's,
 *                max(age_threshold - waited, 0))                                 [the EWT equations]
 *   order: by queue; inside a queue by EWT, then aged jobs first (longest wait first), then
 *       remaining time, arrival, id
 *   residency [Alg. 2]: walking the queues with a budget of gpu_job_limit jobs, the first jobs of
 *       each queue are within the budget while it lasts; the budget shrinks by the queue's
 *       length (not below zero).  Within the budget: a job whose cache is on the host is uploaded.
 *       Outside: a job whose cache is on the GPU is offloaded.  A job that has not run yet
 *       holds no cache and is neither, but takes a place.
 *   batch: the first max_batch jobs of the order that are within the budget; a job's first
 *       iteration processes its whole prompt (phase 0) and yields its first token, every
 *       later one (phase 1) yields one token
 *   commit: jobs of the batch: generated += 1, waited = 0, cache on the GPU; finished ones
 *       leave; one that reaches its predicted length without finishing has the prediction
 *       doubled and is demoted by one queue for good.  Every other job: waited += elapsed.
 *   model time of a batch: sum of s * t0 over its phase-0 jobs + the largest alpha * s + beta
 *       among its phase-1 jobs.
 */
#ifndef ALISE_SCHED_H
#define ALISE_SCHED_H

#include "alise_kv.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct alise_sched alise_sched;

typedef struct {
    int32_t num_queues;         /* h >= 1, at most 62                                         */
    int32_t max_batch;          /* jobs per iteration, >= 1                                   */
    int32_t gpu_job_limit;      /* M >= 1: jobs whose cache may sit in GPU memory             */
    int32_t reserved;           /* 0                                                          */
    int64_t limit0;             /* remaining-time bound of queue 0, ticks, >= 1               */
    int64_t age_threshold;      /* K, ticks, >= 1                                             */
    int64_t t0, alpha, beta;    /* Eq. 4-5, ticks, >= 0                                       */
} alise_sched_config;

/*
 * One iteration's decision.  The caller sets the pointers and capacities; step() fills the
 * arrays and the counts.  order_* may all be NULL (order_cap 0) when the full order is not
 * wanted.  Ids are in priority order in every list.
 */
typedef struct {
    int64_t *batch_ids;   int32_t *batch_phase;  int32_t batch_cap;   int32_t n_batch;
    int64_t *upload_ids;  int32_t upload_cap;    int32_t n_upload;
    int64_t *offload_ids; int32_t offload_cap;   int32_t n_offload;
    int64_t *order_ids;   int32_t *order_queue;  int64_t *order_ewt;  int32_t order_cap;  int32_t n_order;
    int64_t model_time;   /* out: the model time of the batch, ticks */
} alise_sched_decision;

/* ALISE_INVALID_ARGUMENT for a NULL pointer or a field outside the ranges above. */
int alise_sched_create(const alise_sched_config *cfg, alise_sched **out);
void alise_sched_destroy(alise_sched *s);          /* NULL is allowed */

/*
 * A new job [Sec. 3.1: its profile enters the priority queues].  prompt_len >= 1,
 * predicted_len >= 1; an id already live is ALISE_INVALID_ARGUMENT.
 */
int alise_sched_add_job(alise_sched *s, int64_t id, int64_t arrival, int32_t prompt_len, int32_t predicted_len);

int32_t alise_sched_num_jobs(const alise_sched *s);

/*
 * Order the live jobs, decide residency and pick the batch (the rules above).  Applies the
 * uploads and offloads to the scheduler's own record of where each cache is.  A list that
 * does not fit its capacity gives ALISE_WORKSPACE_TOO_SMALL and changes nothing (batch:
 * min(max_batch, jobs); upload, offload, order: at most the number of live jobs).
 * With no live job all counts are 0.
 */
int alise_sched_step(alise_sched *s, alise_sched_decision *d);

/*
 * The batch of the last step() has run and took `elapsed` >= 0 ticks; finished_ids names
 * those of its jobs that ended (an id that was not in the batch: ALISE_INVALID_ARGUMENT,
 * nothing changes).  Without a step() since the last commit: ALISE_INVALID_ARGUMENT.
 */
int alise_sched_commit(alise_sched *s, int64_t elapsed, const int64_t *finished_ids, int32_t n_finished);

#ifdef __cplusplus
}
#endif
#endif /* ALISE_SCHED_H */
