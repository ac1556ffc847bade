/*
 * qmoe — one priority-ordered, preemptible Mixture-of-Experts layer on AMD MI355X (gfx950).
 *
 * C ABI of the hot path of QLLM (arXiv 2503.09304): the MoE block re-organised into per-expert
 * FIFO queues (Sec. 3.3, "queues per expert") whose latency-sensitive (LS) entries run before
 * best-effort (BE) ones (Abstract; Sec. 3.2, Algorithm 1) and which can be stopped at expert
 * granularity and resumed without repeating finished work (Introduction, "Fine-Grained
 * Expert-Level Preemption"; Sec. 3.1, "Top-k expert selection").
 *
 * One layer-batch goes through
 *
 *     moe_route -> moe_permute -> moe_expert_run / moe_expert_run_units (any number of calls),
 *               or moe_expert_enqueue .. moe_expert_collect -> moe_combine / moe_combine_complete
 *
 * Every return of moe_expert_run is a preemption point: the caller may run other contexts (for
 * instance a newly arrived LS batch) before calling it again with the saved cursor.
 *
 * Conventions that hold for every call
 *  - Pointers marked [device] are GPU global memory owned by the caller; [host] are ordinary host
 *    pointers.  The library allocates no device memory and creates no stream.  (It allocates one
 *    small pinned host buffer per context at the first moe_route, freed by moe_destroy.)
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *    work and return, except moe_permute, which waits until the per-expert counts are on the host,
 *    moe_expert_collect, which waits for the stream, and moe_profile_read, which waits for its events.
 *    All calls on one context must be issued on one stream, or be ordered by the caller.
 *  - Return value: moe_status.  Negative = error; in that case nothing was enqueued and the
 *    context is unchanged (MOE_E_HIP excepted, where the HIP runtime failed half-way).
 *    moe_last_error() gives a thread-local description of the last error.
 *  - Tensors are dense row-major.  dtype MOE_F32: x, weights, y are float.  MOE_BF16: they are
 *    bfloat16 (16-bit patterns), all products are accumulated in fp32, the SwiGLU activation is
 *    rounded to bf16 once, y is rounded to bf16 once.  Router logits, gate weights and the
 *    per-assignment expert outputs are fp32 in both modes.
 *  - Inputs are assumed finite; behaviour with NaN/Inf is unspecified.
 *  - For MOE_BF16, H and F must be multiples of 64.
 */
#ifndef QMOE_H
#define QMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx; /* opaque host object: one per in-flight layer-batch */

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

typedef enum {
    MOE_OK = 0,            /* success; for moe_expert_run: units remain                        */
    MOE_DONE = 1,          /* moe_expert_run: every unit has been executed                     */
    MOE_E_ARG = -1,        /* bad argument (null pointer, size out of range, stale cursor)      */
    MOE_E_STATE = -2,      /* call out of order for this context                                */
    MOE_E_INCOMPLETE = -3, /* moe_combine asked for a class whose expert work is not finished   */
    MOE_E_WORKSPACE = -4,  /* workspace too small or misaligned                                 */
    MOE_E_HIP = -5         /* a HIP runtime call failed                                          */
} moe_status;

typedef struct {
    int32_t E;          /* experts, 1..256                                                      */
    int32_t k;          /* experts per token, 1..min(E,32)                                      */
    int32_t H;          /* hidden size                                                          */
    int32_t F;          /* SwiGLU intermediate size                                             */
    int32_t dtype;      /* moe_dtype                                                            */
    int32_t chunk_rows; /* C: most rows of one work unit, 1..256                                */
    int32_t max_tokens; /* capacity of the context, N <= max_tokens, max_tokens*k < 2^31        */
    int32_t down_ksplit; /* K-split of the down projection: 0 = choose from the configuration, 1 = none,
                            2 or 4 = that many contiguous K ranges, each summed on its own, added in
                            ascending order ((p0+p1)+p2)+p3 (bf16, F % (64*down_ksplit) == 0 only).
                            0 picks 1 unless max_tokens*k <= 256*E (weight-streaming shapes, where
                            the split supplies the parallelism): there it picks the fewest ranges
                            (1, 2, 4) for which E * ceil(H/256) * ranges reaches the 256 compute
                            units, as far as F allows (with 4-bit weights and decode-sized batches 4
                            ranges are faster than that choice: set it).  Choose 4 for a
                            context whose batches are fed a few units per call so that they can be
                            stopped quickly: a launch of few units has only H/256 workgroups per unit in
                            the down projection without the split.  Part of the
                            configuration, never of a launch: results of one context do not depend on it
                            changing, because it cannot change.                                          */
} moe_config;

typedef struct {
    const void *Wg; /* [device] router weight  [H,E]   row-major (E contiguous)                 */
    const void *W1; /* [device] gate_proj      [E,F,H] (H contiguous)                           */
    const void *W3; /* [device] up_proj        [E,F,H] (H contiguous)                           */
    const void *W2; /* [device] down_proj      [E,H,F] (F contiguous)                           */
    int32_t layout; /* MOE_W_ROWMAJOR: the shapes above.  MOE_W_PACKED: written by moe_pack_weights */
    const void *S1; /* [device] 4-bit layouts only: block scales of W1, W3, W2 (else NULL)          */
    const void *S3;
    const void *S2;
} moe_weights;

/* Weight layouts.  MOE_W_PACKED (bf16 only) stores every expert matrix M [R,K] (R % 32 == 0,
 * K % 16 == 0) as 1 KiB blocks in the order a wave's MFMA B operand consumes them, so that a wave
 * streams its weight rows with fully contiguous loads:
 *     element (r, k)  ->  (((r/32) * (K/16) + k/16) * 64 + (r%32) + 32*((k%16)/8)) * 8 + k%8
 * per expert, experts back to back (same total size as row-major); Wg is stored transposed and
 * padded: [ceil16(E), H], rows >= E zero. */
enum { MOE_W_ROWMAJOR = 0, MOE_W_PACKED = 1, MOE_W_MXFP4_ROWMAJOR = 2, MOE_W_MXFP4 = 3 };

/* 4-bit expert weights (the paper evaluates its model with 4-bit quantised weights and 16-bit
 * activations, Sec. 4 "Models and Dataset", without naming a format; this library takes the open
 * microscaling FP4 format): an element is a 4-bit float e2m1 (sign, 2 exponent bits, 1 mantissa bit:
 * +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}), every 32 consecutive elements along K share one scale byte e8m0
 * (2^(byte-127)); value = element * scale, always exactly a bf16.  cfg.dtype stays MOE_BF16 (x, y and
 * the activation are bf16, Wg is bf16 [H,E]); only W1, W3, W2 are 4-bit.
 * MOE_W_MXFP4_ROWMAJOR (input of moe_pack_weights only): W1/W3 [E,F,H/2] and W2 [E,H,F/2] bytes, the
 * element with even k in the low nibble; S1/S3 [E,F,H/32], S2 [E,H,F/32] scale bytes.
 * MOE_W_MXFP4 (what moe_route / moe_expert_run accept): per expert and matrix M [R,K] (R % 32 == 0,
 * K % 64 == 0) the codes as 1 KiB blocks, block (r/32, k/64) at ((r/32)*(K/64) + k/64) * 1024 bytes,
 * inside it lane l = r%32 + 32*((k%16)/8) owns 16 bytes: 4 little-endian words, word (k%64)/16 holds
 * the 8 elements k%8 = 0..7 (element j in bits 4j..4j+3); the scales as 64-byte blocks in the same
 * block order, row r%32 owning 2 bytes: the scales of k%64 < 32 and of k%64 >= 32.  Same sizes as
 * the row-major form.  Wg as in MOE_W_PACKED. */

/* Where a layer-batch stands in its work-unit list.  A plain value: keeping a copy of it (and the
 * context's workspace) is all a preempted batch needs in order to resume. */
typedef struct {
    uint32_t next_unit; /* first unit not yet executed                                          */
    uint32_t n_units;   /* length of the list                                                   */
} moe_cursor;

/* One preemptible piece of expert work: `rows` consecutive entries of one expert's queue, all of
 * one priority class, starting at sorted position `row0`. */
typedef struct {
    int32_t expert;
    int32_t cls; /* 0 = LS, 1 = BE */
    int32_t row0;
    int32_t rows; /* 1..chunk_rows */
} moe_unit;

enum { MOE_CLASS_LS = 1, MOE_CLASS_BE = 2, MOE_CLASS_ALL = 3,
       MOE_Y_F32 = 4 /* moe_combine: or-ed into class_mask, y is float [n_tokens,H] whatever the context's dtype */ };

typedef enum {
    MOE_GET_LOGITS = 0,     /* float   [N,E]    router logits (bias included)                   */
    MOE_GET_TOPK_IDX = 1,   /* int32   [N,k]    chosen experts, slot 0 = largest logit          */
    MOE_GET_TOPK_W = 2,     /* float   [N,k]    renormalised gate weights                       */
    MOE_GET_COUNTS = 3,     /* int32   [E,2]    queue lengths, column 0 = LS, 1 = BE            */
    MOE_GET_OFFSETS = 4,    /* int32   [2E+1]   running total in order e0-LS, e0-BE, e1-LS, ... */
    MOE_GET_PERM = 5,       /* int32   [N*k]    sorted position -> assignment id n*k+slot       */
    MOE_GET_INV = 6,        /* int32   [N*k]    assignment id -> sorted position                */
    MOE_GET_EXPERT_OUT = 7, /* float   [N*k,H]  expert output of each sorted position           */
    MOE_GET_ACT = 8,        /* dtype   [N*k,F]  SwiGLU activation of each sorted position       */
    MOE_GET_UNITS = 9       /* moe_unit[n_units] the device copy of the work-unit list          */
} moe_what;

/* Bytes of device workspace a context of this configuration needs; 0 if the configuration is
 * invalid.  The workspace holds the state a preempted batch must keep (routing metadata, queue
 * order, finished expert rows: Introduction, paragraph on granular state management; Discussion,
 * "Limitations") plus scratch. */
size_t moe_workspace_bytes(const moe_config *cfg);

/* Creates a context over `workspace` ([device], 256-byte aligned, >= moe_workspace_bytes(cfg)).
 * Touches no GPU state.  The workspace must outlive the context.  Two environment variables are read
 * here, both for tests: QMOE_REPORT_SPIN_MS (see moe_permute) and QMOE_GATE_UP_WAVE_COLUMNS (16, 20,
 * 24, 28 or 32: every bf16 gate-up launch of the context gives each wave that many output columns
 * instead of the width the launch would pick; results do not depend on it). */
int32_t moe_create(const moe_config *cfg, void *workspace, size_t workspace_bytes, moe_ctx **out);

/* Frees the host object (and its pinned buffer).  Does not wait for enqueued work: the caller makes
 * sure that nothing of this context is still on a stream.  Between moe_expert_enqueue and
 * moe_expert_collect the kernels of the sequence read and write the pinned buffer, so the call is
 * refused with MOE_E_STATE (nothing is freed): collect first. */
int32_t moe_destroy(moe_ctx *ctx);

/* One-time re-layout of the weights at model load (outside any timed region).  src: row-major
 * weights, layout MOE_W_ROWMAJOR (bf16) or MOE_W_MXFP4_ROWMAJOR (4-bit codes and scales).  dst:
 * caller-allocated [device] buffers, W1/W3/W2 (and S1/S3/S2 for the 4-bit form) of the same sizes as
 * the sources, Wg of ceil16(E)*H bf16 elements; on success dst->layout is set to MOE_W_PACKED or
 * MOE_W_MXFP4.  The expert kernels produce bit-identical results for the row-major and the packed
 * bf16 layout.  cfg->dtype must be MOE_BF16 (MOE_E_ARG otherwise).  Enqueues on `stream` and returns. */
int32_t moe_pack_weights(const moe_config *cfg, const moe_weights *src, moe_weights *dst, void *stream);

/* Router (Sec. 2.1 and 2.2).
 *   logits[n,e] = sum_h x[n,h]*Wg[h,e] + logit_bias[e]      (fp32 accumulation)
 *   slot j of token n = j-th expert in the order (logit descending, expert index ascending)
 *   w[n,j] = exp(l_j - l_0) / sum_{i<k} exp(l_i - l_0)      (softmax renormalised over the k)
 * x [device] [n_tokens,H]; logit_bias [device] float[E] or NULL; 0 <= n_tokens <= max_tokens.
 * Starts a new layer-batch on the context: earlier results in the workspace are discarded. */
int32_t moe_route(moe_ctx *ctx, const void *x, int32_t n_tokens, const moe_weights *w,
                  const float *logit_bias, void *stream);

/* The router for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same kernels and same results as moe_route with row-major
 * weights, bit for bit, but no context, no workspace and no allocation of any kind (device, pinned or
 * host): the one scratch buffer the bf16 router needs (Wg transposed and padded, ceil16(E)*H bf16)
 * lives in a 2 MiB array in the library's device image, one copy per GPU, held until the process ends.
 *   cfg: E, k, H and dtype are used.  x [device] [n_tokens,H]; Wg [device] [H,E] row-major;
 *   logit_bias [device] float[E] or NULL; outputs [device]: logits float[n_tokens,E], topk_idx
 *   int32[n_tokens,k], topk_w float[n_tokens,k].
 * MOE_E_ARG if ceil16(E)*H*2 exceeds 2 MiB (bf16) or an argument is bad; nothing is enqueued then.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (different streams,
 * different threads) race; calls on one stream are ordered and each rewrites what it reads. */
int32_t moe_route_noalloc(const moe_config *cfg, const void *x, int32_t n_tokens, const void *Wg,
                          const float *logit_bias, float *logits, int32_t *topk_idx, float *topk_w, void *stream);

/* Per-expert priority queues (Sec. 3.3 per-expert FIFO; Sec. 3.2 LS before BE): a stable counting
 * sort of the n_tokens*k assignments by (expert ascending, LS before BE, token ascending).
 * prio [device] uint8[n_tokens], non-zero = LS.  Produces counts, offsets, perm, inv and the
 * work-unit list: phase LS then phase BE; inside a phase experts ascending; inside one expert's
 * sub-queue consecutive chunks of chunk_rows rows, the last one short; empty sub-queues give no
 * unit.  Waits for the counts (the engine's report to the scheduler after the router stage,
 * Sec. 3.2): the kernel stores them into pinned host memory as soon as it knows them and the call
 * polls for that, so it returns while the rest of the permutation may still be running; whatever is
 * enqueued on the stream afterwards is ordered behind it.  If the report does not arrive within
 * 200 ms (environment variable QMOE_REPORT_SPIN_MS at moe_create, 0 = never poll) the call waits for
 * the stream instead.  Returns the cursor {0, n_units} in *cursor ([host]). */
int32_t moe_permute(moe_ctx *ctx, const uint8_t *prio, moe_cursor *cursor, void *stream);

/* Expert work, resumable (Sec. 3.1 "Top-k expert selection"; Introduction, contribution 3).
 * Executes the next max_units units that have not run yet, in list order, starting at
 * cursor->next_unit (the first unit that has not run): for each row r of a unit of expert e, with
 * token n = perm[r] / k,
 *     act[r,:] = silu(W1[e] x[n,:]) (.) (W3[e] x[n,:]),   out[r,:] = W2[e] act[r,:]
 * and advances *cursor ([host], in/out).  max_units = UINT32_MAX runs to the end.  x and w must be
 * the tensors given to moe_route, unchanged.  *cursor must be the value last returned for this
 * context (MOE_E_ARG otherwise): no unit is ever executed twice.  Results do not depend on how
 * the unit list is split into calls, bit for bit.
 * Order on the device: list order holds from call to call (everything one call enqueues runs before
 * what the next call enqueues).  Inside one call the bf16 kernels take the call's units expert by
 * expert, so that an expert's LS and BE rows share one pass over its weights: a call that spans both
 * phases finishes its LS rows with the rest.  A caller that wants the LS rows out first cuts the
 * call at the end of the LS phase (the units with cls == 0 come first in the list: moe_units), runs
 * moe_combine(MOE_CLASS_LS), then carries on; that costs a second pass over the weights of every
 * expert that holds rows of both classes.
 * Returns MOE_OK while units remain, MOE_DONE when every unit has run. */
int32_t moe_expert_run(moe_ctx *ctx, const void *x, const moe_weights *w, uint32_t max_units,
                       moe_cursor *cursor, void *stream);

/* Expert work in an order the caller chooses (Sec. 3.1 "User-defined scheduling policies", Sec. 3.2:
 * policies at the granularity of experts, e.g. selective expert execution).  unit_ids [host]
 * uint32[n]: indices into the context's unit list (moe_units), distinct, each not yet executed; any
 * order (honoured from call to call; inside one call the device takes the units expert by expert, see
 * moe_expert_run).  The arithmetic per row is that of moe_expert_run, bit for bit.  On a bad id (out of range,
 * repeated, already executed) nothing runs and MOE_E_ARG is returned.  *cursor ([host], may be
 * NULL) receives the context's cursor afterwards: next_unit = first unit that has not run, so
 * moe_expert_run can carry on from it.  Returns MOE_OK while units remain, MOE_DONE when all ran. */
int32_t moe_expert_run_units(moe_ctx *ctx, const void *x, const moe_weights *w, const uint32_t *unit_ids,
                             uint32_t n, moe_cursor *cursor, void *stream);

/* Expert work enqueued ahead and stopped from the device side, at the granularity of a work unit
 * (Discussion, Sec. 6, paragraph on overlapping preemption with execution: named there as future work).
 * moe_expert_enqueue puts ALL units that have not run yet on the stream, as launches of
 * units_per_launch units each, and returns without waiting.  moe_expert_stop sets the context's stop
 * word (a plain store to host memory that is mapped into the device; it may come from another thread
 * than the one that enqueued).  Every workgroup of the sequence looks at that word when it starts:
 * once it is set, workgroups that have not started yet do nothing, so the sequence ends as soon as
 * the workgroups in flight have finished their tiles (a fraction of one unit's duration), whatever
 * units_per_launch is; the launches behind the stop are closed as a whole by a one-thread gate kernel
 * in front of each.  No kernel waits or spins.  The workgroups count themselves per row range; a
 * down-projection workgroup runs only if all gate-up workgroups of its rows ran, and a small kernel
 * behind the last launch reports, per row range, whether all its down-projection workgroups ran.
 * Work of other contexts may be enqueued on the stream at any time; it runs behind whatever the
 * sequence still executes.
 * moe_expert_collect waits for the stream, reads the report, books the units whose rows are all
 * complete as executed (a unit whose rows were only partly computed when the stop took effect is
 * not booked: it runs again, in full and to the same bits, when the batch resumes), clears the stop
 * word and returns the cursor in *cursor ([host]); MOE_DONE if every unit has run, MOE_OK otherwise
 * (then carry on with moe_expert_enqueue or moe_expert_run; units booked out of list order are
 * skipped).  The arithmetic is that of moe_expert_run, bit for bit.
 * Between enqueue and collect every other call on the context fails with MOE_E_STATE. */
int32_t moe_expert_enqueue(moe_ctx *ctx, const void *x, const moe_weights *w, uint32_t units_per_launch,
                           void *stream);
int32_t moe_expert_stop(moe_ctx *ctx);
int32_t moe_expert_collect(moe_ctx *ctx, moe_cursor *cursor, void *stream);

/* Gate-weighted combine of complete tokens (Sec. 3.1: only fully processed tokens contribute to
 * the next layer's hidden state):
 *     y[n,:] = sum_{j=0..k-1, in slot order} w[n,j] * out[inv[n*k+j], :]
 * accumulated in fp32 from zero in that fixed order, rounded once to the output type.
 * class_mask selects which tokens' rows of y ([device] [n_tokens,H]) are written: MOE_CLASS_LS,
 * MOE_CLASS_BE or MOE_CLASS_ALL; rows of other tokens are left untouched.  If a selected class
 * still has unexecuted units the call fails with MOE_E_INCOMPLETE.  With MOE_Y_F32 or-ed in, y is
 * float and receives the fp32 sums unrounded: for a bf16 context the bf16 y is exactly that value
 * rounded once to nearest-even, so the flag shows a caller (and the tests) the result before the
 * one rounding the output type costs. */
int32_t moe_combine(moe_ctx *ctx, void *y, int32_t class_mask, void *stream);

/* Combine of whatever is complete (Sec. 3.1 "Top-k expert selection": fully and partially processed
 * tokens are told apart, only complete ones contribute).  A token is complete when the units holding
 * all k of its assignments have been executed, in whatever order and by whichever call.  Rows of y
 * ([device] [n_tokens,H]) of complete tokens are written exactly as moe_combine writes them; rows of
 * the other tokens are left untouched.  complete ([device] uint8[n_tokens], may be NULL) receives 1
 * for complete tokens, 0 for the others.  Never fails with MOE_E_INCOMPLETE. */
int32_t moe_combine_complete(moe_ctx *ctx, void *y, uint8_t *complete, void *stream);

/* Read-back for tests and schedulers: a [device] pointer into the workspace and its size in bytes
 * for the current layer-batch.  Valid until the next moe_route on this context.
 * MOE_GET_EXPERT_OUT on a context whose down projection is K-split (down_ksplit, chosen or implied):
 * the kernels keep the K ranges' partial sums apart and moe_combine adds them as it reads them, so
 * this request first enqueues, on the stream of the context's last expert launch, a kernel that adds
 * them ((p0+p1)+p2)+p3 into the returned array for the rows executed so far: read it in stream order
 * or after synchronising. */
int32_t moe_get(moe_ctx *ctx, int32_t what, const void **dev_ptr, size_t *bytes);

/* Host copy of the context's work-unit list (after moe_permute).  Writes at most `cap` entries to
 * out ([host], may be NULL when cap is 0) and the full count to *n_units. */
int32_t moe_units(moe_ctx *ctx, moe_unit *out, uint32_t cap, uint32_t *n_units);

/* The work-unit list as a pure host function of the queue lengths: cnt [host] int32[E][2]
 * (column 0 = LS).  Same list moe_permute builds.  Needs no GPU. */
int32_t moe_plan_units(const int32_t *cnt, int32_t E, int32_t chunk_rows, moe_unit *out,
                       uint32_t cap, uint32_t *n_units);

/* Per-kernel timing for benchmarks.  moe_profile(ctx, kinds) makes moe_expert_run bracket the kernel
 * launches of the selected kinds with a pair of HIP events on the caller's stream (events are
 * created on demand and kept by the context); kinds is a bit mask, bit MOE_PROF_x per kind,
 * MOE_PROF_ALL for every kind, 0 turns the bracketing off.  Each bracketed launch costs a few
 * microseconds of stream time.  moe_profile_read waits for the recorded events, adds up elapsed
 * milliseconds and launch counts per kernel kind since the last read into ms / launches ([host],
 * MOE_PROF_KINDS entries each) and forgets them. */
enum { MOE_PROF_GATE_UP = 0, MOE_PROF_DOWN = 1, MOE_PROF_DOWN_REDUCE = 2 /* unused: no such launch any more */,
       MOE_PROF_KINDS = 3, MOE_PROF_ALL = 7 };
int32_t moe_profile(moe_ctx *ctx, int32_t kinds);
int32_t moe_profile_read(moe_ctx *ctx, float *ms, uint32_t *launches);

/* Yardstick for profiles of the MFMA-bound kernels (no part of the method): one launch of `workgroups`
 * workgroups of 4 waves, each wave running iters * 8 bf16 MFMAs (32x32x16, 32768 flop each) on
 * register operands taken once from a_bf16 and b_bf16 ([device], at least 4096 bf16 each, e.g. the
 * first rows of x and of W1, so that the operands carry the workload's bit patterns); no memory
 * traffic inside the loop.  sink: [device] one float (never written in practice).
 * flop = workgroups * 4 * iters * 8 * 32768. */
int32_t moe_probe_mfma(const void *a_bf16, const void *b_bf16, int32_t iters, int32_t workgroups, float *sink, void *stream);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char *moe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* QMOE_H */
