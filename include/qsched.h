/* qsched.h -- C ABI of the host-side scheduler that sits above the MoE-layer calls of qmoe.h.
 *
 * Paper: section "System Architecture".  A scheduler receives prompts (jobs) over time; its
 * dispatcher puts each new job into the prefill queue of its priority class and, for every output
 * token the model produces, puts the job into the decode queue of its class; its batch engine builds
 * the next batch from the four FCFS queues {LS, BE} x {prefill, decode} with the "Batch Selection
 * Logic" (Algorithm 1).  The inference engine reports back after each stage and the scheduler tells
 * it whether to stop the running batch (closed loop, same section): sched_preempt_wanted.
 *
 * Everything here is host code: all pointers are host pointers, nothing touches the GPU.  A sched
 * object is not thread-safe; calls on one object must be serialised by the caller.
 *
 * Every function that returns int32_t returns SCHED_OK (0) or SCHED_NONE (1) on success and a
 * negative SCHED_E_* code on error; sched_last_error() then describes the failure (thread-local
 * string, valid until the next failing call on the thread).
 */
#ifndef QSCHED_H
#define QSCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sched sched;

enum {
    SCHED_OK = 0,
    SCHED_NONE = 1,      /* sched_next_batch: all four queues are empty */
    SCHED_E_ARG = -1,    /* null pointer, unknown class or queue, capacity too small */
    SCHED_E_JOB = -2     /* job id already known (submit), unknown, or not in a running batch (token) */
};

/* Priority class of a job. */
enum { SCHED_BE = 0, SCHED_LS = 1 };
/* Stage of a batch. */
enum { SCHED_PREFILL = 0, SCHED_DECODE = 1 };
/* Queue numbers for sched_queue_len. */
enum { SCHED_Q_LS_PREFILL = 0, SCHED_Q_BE_PREFILL = 1, SCHED_Q_LS_DECODE = 2, SCHED_Q_BE_DECODE = 3 };

/* What sched_next_batch hands out besides the job ids. */
typedef struct sched_batch {
    uint32_t n;       /* jobs in the batch, 1 .. batch_size */
    uint32_t n_ls;    /* the first n_ls of them are LS jobs, the rest BE jobs */
    int32_t stage;    /* SCHED_PREFILL or SCHED_DECODE: a batch never mixes the two */
} sched_batch;

/* Creates a scheduler whose batches hold at most batch_size jobs (BatchSize of Algorithm 1,
 * counted in jobs; >= 1).  Returns NULL on a bad argument. */
sched *sched_create(uint32_t batch_size);
void sched_destroy(sched *s);

/* Dispatcher, new prompt: job (any id not currently known to s) joins the tail of the prefill queue
 * of class cls (SCHED_LS or SCHED_BE). */
int32_t sched_submit(sched *s, uint64_t job, int32_t cls);

/* Dispatcher, output token: job must be in a batch handed out by sched_next_batch and not yet
 * reported.  finished != 0: that was its last token, the job leaves the system (its id may be
 * submitted again).  Otherwise it joins the tail of the decode queue of its class. */
int32_t sched_token(sched *s, uint64_t job, int32_t finished);

/* Batch engine, Algorithm 1 (GetNextBatch).  In this order: a full batch of LS decode jobs if there
 * are at least batch_size of them; else LS prefill jobs, filled up with BE prefill jobs; else LS
 * decode jobs, filled up with BE decode jobs; else BE decode jobs; else BE prefill jobs.  Jobs are
 * taken from the head of their queue, in queue order; LS jobs come first in jobs[].
 * jobs: host array of capacity cap >= batch_size, receives out->n ids.  The jobs are then "running":
 * in no queue until sched_token is called for them.  Returns SCHED_NONE (out->n = 0) if all queues
 * are empty. */
int32_t sched_next_batch(sched *s, uint64_t *jobs, uint32_t cap, sched_batch *out);

/* Closed-loop signal for the engine, asked at a preemption point (after an expert chunk) of the batch
 * it is executing: 1 if that batch holds BE jobs only (running->n_ls == 0) and an LS prompt waits in
 * the LS prefill queue, i.e. the engine should park the batch and ask for the next one; else 0.
 * Negative on a null argument. */
int32_t sched_preempt_wanted(const sched *s, const sched_batch *running);

/* Jobs waiting in queue q (SCHED_Q_*); 0 for an unknown queue or null s. */
uint32_t sched_queue_len(const sched *s, int32_t q);
/* Jobs currently handed out in batches and not yet reported by sched_token. */
uint32_t sched_running(const sched *s);

const char *sched_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* QSCHED_H */
