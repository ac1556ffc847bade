// Host-side scheduler: dispatcher, four FCFS queues, batch selection (no device code in this file).
//
// Paper: section "System Architecture" and its Algorithm 1.  Queues are std::deque<uint64_t>;
// a hash map holds, for every live job, its class and where it is (queued for prefill, queued for
// decode, running), which is what makes the dispatcher's error checks O(1).
#include "qsched.h"

#include <cstdarg>
#include <cstdio>
#include <deque>
#include <new>
#include <unordered_map>

namespace {

thread_local char g_err[256] = "";

int32_t fail(int32_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

enum Where : uint8_t { W_PREFILL_QUEUE, W_DECODE_QUEUE, W_RUNNING };

struct Job {
    uint8_t cls;
    Where where;
};

}  // namespace

struct sched {
    uint32_t batch_size;
    std::deque<uint64_t> q[4];   // indexed by SCHED_Q_*
    std::unordered_map<uint64_t, Job> jobs;
    uint32_t running = 0;

    // Moves up to `room` jobs from the head of queue qi to out[n...]; returns how many.
    uint32_t take(int qi, uint32_t room, uint64_t *out, uint32_t n) {
        uint32_t got = 0;
        std::deque<uint64_t> &dq = q[qi];
        while (got < room && !dq.empty()) {
            const uint64_t id = dq.front();
            dq.pop_front();
            jobs[id].where = W_RUNNING;
            out[n + got] = id;
            ++got;
        }
        running += got;
        return got;
    }
};

extern "C" {

const char *sched_last_error(void) { return g_err; }

sched *sched_create(uint32_t batch_size) {
    if (batch_size == 0) {
        fail(SCHED_E_ARG, "sched_create: batch_size must be at least 1");
        return nullptr;
    }
    sched *s = new (std::nothrow) sched();
    if (!s) {
        fail(SCHED_E_ARG, "sched_create: out of host memory");
        return nullptr;
    }
    s->batch_size = batch_size;
    return s;
}

void sched_destroy(sched *s) { delete s; }

int32_t sched_submit(sched *s, uint64_t job, int32_t cls) {
    if (!s) return fail(SCHED_E_ARG, "sched_submit: null scheduler");
    if (cls != SCHED_LS && cls != SCHED_BE) return fail(SCHED_E_ARG, "sched_submit: class %d is neither LS nor BE", cls);
    if (s->jobs.count(job)) return fail(SCHED_E_JOB, "sched_submit: job %llu is already in the system", (unsigned long long)job);
    s->jobs[job] = Job{(uint8_t)cls, W_PREFILL_QUEUE};
    s->q[cls == SCHED_LS ? SCHED_Q_LS_PREFILL : SCHED_Q_BE_PREFILL].push_back(job);
    return SCHED_OK;
}

int32_t sched_token(sched *s, uint64_t job, int32_t finished) {
    if (!s) return fail(SCHED_E_ARG, "sched_token: null scheduler");
    auto it = s->jobs.find(job);
    if (it == s->jobs.end()) return fail(SCHED_E_JOB, "sched_token: unknown job %llu", (unsigned long long)job);
    if (it->second.where != W_RUNNING)
        return fail(SCHED_E_JOB, "sched_token: job %llu is queued, not in a running batch", (unsigned long long)job);
    --s->running;
    if (finished) {
        s->jobs.erase(it);
        return SCHED_OK;
    }
    it->second.where = W_DECODE_QUEUE;
    s->q[it->second.cls == SCHED_LS ? SCHED_Q_LS_DECODE : SCHED_Q_BE_DECODE].push_back(job);
    return SCHED_OK;
}

int32_t sched_next_batch(sched *s, uint64_t *jobs, uint32_t cap, sched_batch *out) {
    if (!s || !jobs || !out) return fail(SCHED_E_ARG, "sched_next_batch: null argument");
    if (cap < s->batch_size) return fail(SCHED_E_ARG, "sched_next_batch: capacity %u is below the batch size %u", cap, s->batch_size);
    const uint32_t B = s->batch_size;
    out->n = 0;
    out->n_ls = 0;
    out->stage = SCHED_PREFILL;
    // primary queue of the batch and the BE queue it may be filled from (-1: none)
    int first, fill;
    if (s->q[SCHED_Q_LS_DECODE].size() >= B) { first = SCHED_Q_LS_DECODE; fill = -1; }
    else if (!s->q[SCHED_Q_LS_PREFILL].empty()) { first = SCHED_Q_LS_PREFILL; fill = SCHED_Q_BE_PREFILL; }
    else if (!s->q[SCHED_Q_LS_DECODE].empty()) { first = SCHED_Q_LS_DECODE; fill = SCHED_Q_BE_DECODE; }
    else if (!s->q[SCHED_Q_BE_DECODE].empty()) { first = SCHED_Q_BE_DECODE; fill = -1; }
    else if (!s->q[SCHED_Q_BE_PREFILL].empty()) { first = SCHED_Q_BE_PREFILL; fill = -1; }
    else return SCHED_NONE;

    uint32_t n = s->take(first, B, jobs, 0);
    if (first == SCHED_Q_LS_DECODE || first == SCHED_Q_LS_PREFILL) out->n_ls = n;
    if (fill >= 0 && n < B) n += s->take(fill, B - n, jobs, n);
    out->n = n;
    out->stage = (first == SCHED_Q_LS_DECODE || first == SCHED_Q_BE_DECODE) ? SCHED_DECODE : SCHED_PREFILL;
    return SCHED_OK;
}

int32_t sched_preempt_wanted(const sched *s, const sched_batch *running) {
    if (!s || !running) return fail(SCHED_E_ARG, "sched_preempt_wanted: null argument");
    return (running->n_ls == 0 && !s->q[SCHED_Q_LS_PREFILL].empty()) ? 1 : 0;
}

uint32_t sched_queue_len(const sched *s, int32_t q) {
    if (!s || q < 0 || q > 3) return 0;
    return (uint32_t)s->q[q].size();
}

uint32_t sched_running(const sched *s) { return s ? s->running : 0; }

}  // extern "C"
