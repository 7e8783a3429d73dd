/*
 * alise_replay.h -- C ABI of the native serving loop: the scheduler's decisions turned into calls.
 *
 * ALISE (arXiv 2410.23537) plans every iteration with its speculative scheduler [Sec. 3.1
 * "Preemptive Scheduling"], keeps, uploads or offloads the KV caches of preempted jobs by their
 * estimated wait time [Sec. 3.2 "Dynamic Swapping", Alg. 2] overlapped with the iteration's
 * compute, and runs the batch over the compressed paged cache [Sec. 3.2 "KV Compression",
 * Sec. 3.3].  This object is the loop around one attention layer's worth of that: it owns a
 * scheduler (alise_sched.h), the page free list and block tables of a cache (alise_kv.h), pinned
 * host buffers for offloaded requests (filled and read by the copy engine through a device staging
 * buffer: alise_kv_swap_out / _in gather and scatter in device memory), a second stream and the
 * events that order it against the caller's, and at every iteration it
 *     offloads the jobs that lost their place (their pages are free one iteration later),
 *     uploads the ones that got one,
 *     quantizes and writes the new K/V of the batch (whole prompts for jobs in their first
 *         iteration, one token for the others),
 *     runs chunked-prefill attention for the former and single-query attention for the latter,
 * all through the entry points of alise_kv.h, with no host synchronisation in the steady state:
 * per-iteration metadata travels through a ring of pinned staging buffers.
 *
 * Where the tokens come from: three device arrays of fp16 rows, k_tokens and v_tokens
 * [rows][num_kv_heads][head_dim] and q_tokens [rows][num_q_heads][head_dim]; a job whose
 * token_row is r finds its token t (prompt tokens first, then generated ones) in row r + t of
 * each.  In a model these would be the projections of the layer's input; here the caller
 * supplies them, so that a run can be reproduced and checked.
 *
 * Where the results go: `out`, device fp16 [max_iter_tokens][num_q_heads][head_dim].  The
 * phase-0 jobs of the batch come first, in batch order, each with one row per prompt token; the
 * phase-1 jobs follow with one row each.  batch_out_row[i] is the first row of batch job i.
 *
 * Streams: everything is enqueued on the stream given at create and, with overlap_swaps, on a
 * stream of the object's own (default priority); iterate() and commit() return without waiting
 * for the GPU.  The token arrays and `out` of an iteration must stay untouched until that
 * stream has passed the iteration.  Calls on one object must not overlap.  All pages of the
 * cache belong to the object from create to destroy.  Status codes are those of alise_kv.h.
 */
#ifndef ALISE_REPLAY_H
#define ALISE_REPLAY_H

#include "alise_kv.h"
#include "alise_sched.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct alise_replay alise_replay;

typedef struct {
    int32_t num_q_heads;        /* a multiple of the cache's num_kv_heads                              */
    int32_t max_context;        /* most tokens a job's cache may reach: prompt + generated, >= 2       */
    int32_t max_iter_tokens;    /* most new tokens of one iteration: the prompts of its phase-0 jobs
                                   plus one per phase-1 job, >= 1                                      */
    int32_t overlap_swaps;      /* nonzero: offloads and uploads run on a stream of the object's own   */
    float softmax_scale;        /* 1/sqrt(head_dim) for Eq. 1                                          */
    int32_t reserved;           /* 0                                                                   */
} alise_replay_config;

/*
 * What one iteration did.  The caller sets the pointers and capacities (batch: max_batch of the
 * scheduler is enough; upload and offload: gpu_job_limit is enough); iterate() fills the arrays
 * and counts.  Ids are in the scheduler's priority order in every list.
 */
typedef struct {
    int64_t *batch_ids;   int32_t *batch_phase;  int64_t *batch_out_row;  int32_t batch_cap;  int32_t n_batch;
    int64_t *upload_ids;  int32_t upload_cap;    int32_t n_upload;
    int64_t *offload_ids; const void **offload_host;  size_t *offload_bytes;  int32_t offload_cap;  int32_t n_offload;
    int64_t model_time;           /* the model time of the batch, ticks (alise_sched.h)                */
    int32_t n_prefill_tokens;     /* rows of `out` that phase-0 jobs own                               */
    int32_t n_decode_tokens;      /* rows after them, one per phase-1 job                              */
} alise_replay_iteration;

typedef struct {
    int64_t iterations, prefill_tokens, decode_tokens, offloads, uploads, offload_bytes, upload_bytes;
    int32_t free_pages;           /* pages on the free list or on their way back to it                 */
    int32_t live_jobs;
} alise_replay_stats;

/*
 * Allocates the object: host tables, the scheduler, pinned staging, device staging for the
 * gathered tokens and the metadata, the workspaces of both attention calls for the largest
 * iteration the configuration allows, one stream and a few events.  `hip_stream` is the stream
 * every iteration runs on (NULL = the default stream).  ALISE_INVALID_ARGUMENT for a NULL
 * pointer or a field outside its range, ALISE_UNSUPPORTED for a cache layout alise_kv.h does
 * not take, ALISE_HIP_ERROR if an allocation fails.
 */
int alise_replay_create(const alise_kv_cache *cache, const alise_sched_config *sched_cfg,
                        const alise_replay_config *cfg, void *hip_stream, alise_replay **out);

/* Waits for the GPU work of the object, then frees everything it owns.  NULL is allowed. */
void alise_replay_destroy(alise_replay *r);

/*
 * A new job [Sec. 3.1].  prompt_len >= 1, prompt_len + 1 <= max_context, prompt_len <=
 * max_iter_tokens, token_row >= 0; otherwise as alise_sched_add_job.
 */
int alise_replay_add_job(alise_replay *r, int64_t id, int64_t arrival, int32_t prompt_len,
                         int32_t predicted_len, int64_t token_row);

int32_t alise_replay_num_jobs(const alise_replay *r);

/*
 * Plans one iteration (alise_sched_step) and enqueues all of its work.  offload_host[i] is the
 * pinned host buffer (hipHostMalloc) that holds the offloaded form of offload_ids[i] in the
 * layout of alise_kv_swap_out, offload_bytes[i] bytes of it: complete once the GPU has passed the
 * iteration (alise_replay_synchronize), valid until the job is uploaded again.  Host buffers come in
 * power-of-two sizes and are recycled once their upload has passed; an offload that finds none of its
 * size free allocates one (hipHostMalloc), which is the only allocation after create.
 * Errors: ALISE_WORKSPACE_TOO_SMALL if a list does not fit its capacity (nothing has changed), if
 * the iteration's new tokens exceed max_iter_tokens, or if the cache has too few free pages for
 * the uploads and the batch (size the pool for gpu_job_limit + max_batch jobs of max_context
 * tokens); in the last two cases the scheduler has already taken its decision and the object can
 * only be destroyed.  With no live job all counts are 0 and nothing is enqueued.
 */
int alise_replay_iterate(alise_replay *r, const void *k_tokens, const void *v_tokens, const void *q_tokens,
                         void *out, alise_replay_iteration *it);

/*
 * The batch of the last iterate() took `elapsed` ticks; finished_ids names those of its jobs
 * that ended (alise_sched_commit).  Their pages return to the free list behind the iteration
 * that read them.  A job may still generate after reaching max_context - 1 tokens only if it
 * finishes now: the next iteration would not fit (ALISE_INVALID_ARGUMENT from that iterate()).
 */
int alise_replay_commit(alise_replay *r, int64_t elapsed, const int64_t *finished_ids, int32_t n_finished);

/* Waits until the GPU has finished everything the object has enqueued, on both streams. */
int alise_replay_synchronize(alise_replay *r);

int alise_replay_get_stats(const alise_replay *r, alise_replay_stats *s);

#ifdef __cplusplus
}
#endif
#endif /* ALISE_REPLAY_H */
