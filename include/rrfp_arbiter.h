/* Ready-set arbiter of one pipeline stage and a discrete-event simulator of a whole pipeline.
 *
 * Host code only (no GPU calls).  The arbiter is the event-driven execution loop of App. A,
 * Algorithm 1, turned inside out: message arrivals are posted into the ready buffers
 * (arbiter_post_ready), the compute thread asks for the next task when it is free (arbiter_next)
 * and reports completions (arbiter_complete).  The selected task is the one the hint order ranks
 * first AMONG READY TASKS; unready work is skipped, never waited for (Sec. 5).
 *
 * Hint orders: BF (App. A: each round a ready backward first, then a ready forward), FB, B-priority,
 * F-priority (Sec. 7.7), BFW (Sec. 7.1: a weight task W per (microbatch, chunk), ready once the local
 * B has completed, dispatched only when neither B nor F is ready), and FIXED_1F1B (the fixed-order
 * baseline of Sec. 7.1: the planned sequence is binding, the stage waits for its head).
 * Within a direction: forward takes the smallest chunk, backward and W the largest; ties go to the
 * smallest microbatch (App. A).
 * Backpressure (App. C.2): with buffer_limit > 0, D = n_f - n_b is taken before every arbitration;
 * at D >= limit a one-chunk stage dispatches no forward and waits for backward work (a ready W may
 * still run); a multi-chunk stage completes microbatches one by one in index order
 * (F_0..F_{C-1}, B_{C-1}..B_0), waiting for the next required task.
 *
 * All functions return ARB_OK / ARB_TASK / ARB_WAIT / ARB_DONE or a negative error; nothing is
 * thrown across the boundary.  An arbiter is used from one thread at a time.
 */
#ifndef RRFP_ARBITER_H
#define RRFP_ARBITER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ARB_F = 0, ARB_B = 1, ARB_W = 2 };
enum { ARB_HINT_BF = 0, ARB_HINT_FB = 1, ARB_HINT_B_PRIO = 2, ARB_HINT_F_PRIO = 3, ARB_HINT_BFW = 4,
       ARB_HINT_FIXED_1F1B = 5 };
enum { ARB_OK = 0, ARB_WAIT = 0, ARB_TASK = 1, ARB_DONE = 2, ARB_EINVAL = -1, ARB_ESTATE = -2 };

typedef struct {
  int32_t n_microbatches;   /* M */
  int32_t n_chunks;         /* C model chunks on this stage (1 = non-interleaved) */
  int32_t hint;             /* ARB_HINT_* */
  int32_t buffer_limit;     /* 0 = no backpressure */
  int32_t stage;            /* index of this stage in the pipeline */
  int32_t n_stages;         /* N; stage 0 admits the first chunk's forwards itself, stage N-1 turns
                               the last chunk's forward output into its own backward input */
} arbiter_config;

typedef struct { int32_t dir, microbatch, chunk; } arbiter_task;

typedef struct arbiter arbiter_t;

/* Host memory owned by the library until arbiter_destroy.  NULL + arbiter_last_error(NULL) on error. */
arbiter_t* arbiter_create(const arbiter_config* cfg);
void arbiter_destroy(arbiter_t* a);
/* Start of an iteration: clears buffers and counters; at stage 0 every (microbatch, chunk 0) forward is ready. */
int arbiter_reset(arbiter_t* a);
/* A message arrived: the forward input (dir ARB_F) or the backward input (ARB_B) of (microbatch, chunk).
 * ARB_ESTATE if it is already present or done, or if a backward input arrives before the local forward ran. */
int arbiter_post_ready(arbiter_t* a, int32_t dir, int32_t microbatch, int32_t chunk);
/* One arbitration.  ARB_TASK: *out is removed from its ready buffer and is now in flight (at most one
 * task in flight); ARB_WAIT: nothing may run now, call again after the next arbiter_post_ready;
 * ARB_DONE: every task of the iteration has completed. */
int arbiter_next(arbiter_t* a, arbiter_task* out);
/* The task returned by the last arbiter_next has finished executing. */
int arbiter_complete(arbiter_t* a, const arbiter_task* t);
/* out[0..4] = n_f, n_b, n_w, 1 if D >= limit right now, number of completed tasks. */
int arbiter_counters(const arbiter_t* a, int64_t out[5]);
const char* arbiter_last_error(const arbiter_t* a);

/* ---- pipeline simulator (simplified setting of Sec. 6 plus a constant message latency) ------------
 * N stages, one task at a time per stage, M microbatches, C chunks; durations in seconds, row-major
 * [stage][chunk][microbatch]; a stage arbitrates whenever it is idle and something changed.
 * Jitter (Sec. 7.6): per stage e <- 0.9 e + 0.1 c over the tasks it runs (e starts at the first c); with
 * probability jitter_p the task is lengthened by alpha * max(base, e) * (0.5 + r), r uniform in [0,1);
 * the two uniforms come from a counter-based generator keyed by (seed, stage, dir, microbatch, chunk), so
 * two runs with different hint orders see the same pattern per task. */
typedef struct {
  int32_t n_stages, n_microbatches, n_chunks, hint, buffer_limit;
  int32_t mode;             /* 0 full iteration, 1 forward-only reference, 2 backward-only reference */
  double latency;           /* seconds added to every inter-stage message */
  double jitter_p, jitter_base, jitter_alpha;
  uint64_t jitter_seed;
} rrfp_sim_config;

typedef struct { int32_t stage, dir, microbatch, chunk; double start, end; } rrfp_sim_event;

typedef struct {
  double makespan;
  int64_t n_events;         /* tasks executed (trace entries written = min(n_events, trace_cap)) */
  int32_t deadlock;         /* 1 if the run stopped with unfinished work and nothing in flight */
} rrfp_sim_result;

/* dur_w may be NULL unless hint is BFW.  per_stage (may be NULL) receives 4 doubles per stage:
 * busy seconds, peak retained forward inputs, peak backward inputs, peak D seen at an arbitration.
 * trace (may be NULL) receives the executed tasks in dispatch order (global time order, stage order
 * within one time). */
int rrfp_sim_run(const rrfp_sim_config* cfg, const double* dur_f, const double* dur_b, const double* dur_w,
                 rrfp_sim_result* result, double* per_stage, rrfp_sim_event* trace, int64_t trace_cap);

/* ---- the same event loop, one dispatch at a time (for a runtime that enqueues real stage tasks) -------
 * rrfp_sim_run is a loop over these calls with durations from its tables.  A runtime on one GPU drives them
 * itself: rrfp_pipe_next advances the virtual clock to the next dispatch (completions, message arrivals after
 * the latency, and one arbitration per idle stage, in stage order: Sec. 4.1, Sec. 5, App. A) and names the task
 * and the producer of its input tensor; the caller enqueues stage_F / stage_B / stage_W for it, measures or
 * chooses its duration and reports it with rrfp_pipe_set_duration before the next rrfp_pipe_next.  With
 * jitter_p > 0 in the configuration the delay of Sec. 7.6 for this task (F and B only) is drawn by the
 * library, added to the task's duration and returned, so that the caller can put rrfp_delay(delay) behind the
 * task on its stream.  mode must be 0 for real runs; modes 1 and 2 are the reference executions of Sec. 6. */
typedef struct rrfp_pipe rrfp_pipe_t;
typedef struct {
  int32_t stage, dir, microbatch, chunk;
  int32_t src_stage, src_chunk;   /* (stage, chunk) whose task of the same direction and microbatch produced this
                                     task's input; -1, -1 = the caller's tensor (the pipeline input for F at the
                                     first virtual stage, the output gradient for B at the last).  For W: -1, -1. */
  double start;                   /* virtual time of the dispatch */
} rrfp_pipe_dispatch;
/* NULL + arbiter_last_error(NULL) on an invalid configuration.  Host memory, freed by rrfp_pipe_destroy. */
rrfp_pipe_t* rrfp_pipe_create(const rrfp_sim_config* cfg);
void rrfp_pipe_destroy(rrfp_pipe_t* p);
/* ARB_TASK: *out is the next dispatched task; ARB_DONE: every task of the iteration has completed;
 * ARB_ESTATE: the previous task still waits for its duration, or the pipeline stalled (unfinished work and
 * nothing in flight); ARB_EINVAL: NULL argument. */
int rrfp_pipe_next(rrfp_pipe_t* p, rrfp_pipe_dispatch* out);
/* Duration in seconds (>= 0) of the task rrfp_pipe_next returned last.  *delay_seconds (may be NULL) receives
 * the injected jitter delay (0 if none), *end (may be NULL) the task's virtual completion time
 * start + (seconds + delay). */
int rrfp_pipe_set_duration(rrfp_pipe_t* p, double seconds, double* delay_seconds, double* end);

/* ---- jitter injector for real task streams (Sec. 7.6) ----------------------------------------------
 * The per-stage state of the jitter model above, for a runtime that measures its own tasks: feed the
 * measured compute time of each F/B task of the stage in execution order; the return value is the
 * delay in seconds to add behind that task (0 when none is injected).  Same moving average, same
 * counter-based uniforms as the simulator. */
typedef struct jitter jitter_t;
jitter_t* jitter_create(double p, double base_seconds, double alpha, uint64_t seed, int32_t stage,
                        int32_t n_microbatches, int32_t n_chunks);
void jitter_destroy(jitter_t* j);
double jitter_next_delay(jitter_t* j, int32_t dir, int32_t microbatch, int32_t chunk, double compute_seconds);

/* Enqueues on `stream` (a hipStream_t of the current device, NULL = the null stream) a one-wavefront
 * kernel that returns once `seconds` of the device's constant-rate wall clock have passed: the
 * device-side sleep the paper adds to a task's stream.  0 <= seconds <= 1; the kernel also stops after a
 * bounded number of polls, so it ends even if the clock did not advance.  Returns ARB_OK, ARB_EINVAL,
 * or ARB_ESTATE (a HIP call failed); rrfp_delay_last_error() has the text (thread-local). */
int rrfp_delay(double seconds, void* stream);
const char* rrfp_delay_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
