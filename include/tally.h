/*
 * tally.h -- C ABI of the block-level kernel scheduling library for one MI355X (gfx950).
 *
 * Problem statement (Section 4, "Tally: system design"): one high-priority job and
 * best-effort job(s) share a single GPU.  High-priority kernels are dispatched at once
 * in their original form; best-effort kernels are run at thread-block granularity,
 * either as sliced launches or as preemptible persistent-worker kernels, so that they
 * release the compute units within microseconds (Section 4.1, Section 4.2).
 *
 * Conventions
 *   - Every function returns TALLY_OK (0) or a negative tally_status.  No exception
 *     crosses the boundary.  Out-parameters are written only on success.
 *   - "device pointer" = address in the GPU's HBM valid on the current device;
 *     "host pointer" = ordinary process memory.  Pointers inside tally_*_args are
 *     DEVICE pointers owned by the caller, who keeps them alive until the job that
 *     uses them is COMPLETE or freed.  The args struct itself is HOST memory and is
 *     copied at launch.
 *   - Streams are HIP streams (hipStream_t passed as void*), borrowed, never destroyed
 *     here, and must have the default priority.
 *   - The logical grid of a kernel is a function of its arguments (see the args
 *     structs); tally_logical_grid() computes it and the launch calls reject any other.
 *   - Threading: tally_preempt() and tally_progress() may be called from any thread
 *     while a job runs.  All other calls on one context are serialised by the caller.
 */
#ifndef TALLY_H
#define TALLY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TALLY_OK = 0,
  TALLY_ERR_INVALID_ARG = -1, /* null pointer, zero size, unknown kernel, wrong grid/args size */
  TALLY_ERR_BAD_STATE = -2,   /* e.g. resume of a job that is still running                   */
  TALLY_ERR_HIP = -3,         /* a HIP call failed; tally_last_hip_error() has the code        */
  TALLY_ERR_NOMEM = -4,
  TALLY_ERR_UNSUPPORTED = -5  /* kernel needs all blocks co-resident (Section 6: kernels with
                                 inter-block synchronisation are never sliced or preempted)    */
} tally_status;

/* Job states, after the running()/stopped() predicates of the scheduling algorithm
 * (Section 4.2, Figure 4). */
typedef enum {
  TALLY_JOB_QUEUED = 0,
  TALLY_JOB_RUNNING = 1,
  TALLY_JOB_STOPPED = 2,  /* drained after a preemption, progress < total */
  TALLY_JOB_COMPLETE = 3
} tally_job_state;

typedef enum {
  TALLY_K_SAXPY = 0,          /* y <- a*x + y, fp32                                         */
  TALLY_K_REDUCE_SUM = 1,     /* partial[b] = sum of 4096 consecutive fp32                  */
  TALLY_K_REDUCE_FINAL = 2,   /* total (fp64) = sum of the partials; one block              */
  TALLY_K_GEMM_BF16 = 3,      /* C = A * B, bf16 in/out, fp32 accumulate, 256x256 tiles     */
  TALLY_K_GEMV_BF16 = 4,      /* y = W * x, bf16 in/out, fp32 accumulate                    */
  TALLY_K_SOFTMAX_F32 = 5,    /* row softmax, fp32                                          */
  TALLY_K_LAYERNORM_F32 = 6,  /* row LayerNorm with gain and bias, fp32                     */
  TALLY_K_ATTN_DECODE_BF16 = 7, /* one query per head over a bf16 K/V cache (native only)   */
  TALLY_K_GEMM_BF16_SMALL = 8,  /* same operator as GEMM_BF16 with 32x32 tiles, ragged edges */
  TALLY_K_GEMM_BF16_N128 = 9,   /* same operator with tiles of 256 rows x 128 columns         */
  TALLY_K_COUNT = 10
} tally_kernel_id;

typedef struct { uint32_t x, y, z; } tally_dim3;

/* ---- kernel arguments (host structs holding device pointers) --------------------- */

/* Block b covers elements [256 b, 256 b + 256); thread t handles 256 b + t if < n. */
typedef struct { const float *x; float *y; float a; uint32_t n; } tally_saxpy_args;

/* Block b sums x[4096 b .. 4096 b + 4096) (256 threads x 16 elements, ragged tail
 * allowed) into partial[b].  grid.x = ceil(n / 4096). */
typedef struct { const float *x; float *partial; uint64_t n; } tally_reduce_sum_args;

/* One block: *total = sum(partial[0..count)), carried in fp64. */
typedef struct { const float *partial; double *total; uint32_t count; } tally_reduce_final_args;

/* C[z] (m x n, row-major, ld = n) = A[z] (m x k, row-major) * B[z] (k x n) where B is
 * stored K-contiguous: Bt[z] is n x k row-major.  All bf16 bit patterns; products are
 * accumulated in fp32 and rounded to nearest-even bf16 once.  Batch z uses element
 * strides stride_a/b/c.  Block (bx, by, bz) owns the output tile rows [Tm by, Tm by + Tm),
 * columns [Tn bx, Tn bx + Tn) of batch bz.  GEMM_BF16: Tm = Tn = 256, m and n multiples of
 * 256; GEMM_BF16_N128: Tm = 256, Tn = 128, m a multiple of 256 and n of 128;
 * GEMM_BF16_SMALL: Tm = Tn = 32, any m, n.  k a multiple of 32 in all three.  A, Bt (and
 * C, except for GEMM_BF16_SMALL) 16-byte aligned, strides multiples of 8 elements. */
typedef struct {
  const uint16_t *A; const uint16_t *Bt; uint16_t *C;
  uint32_t m, n, k, batch;
  uint64_t stride_a, stride_b, stride_c;
  uint32_t lda, ldb;  /* elements between consecutive rows of A / of Bt; 0 means k.  Rows
                         that are a large power of two apart (k = 16384: 32 KB) crowd into a
                         few cache sets and the tiled kernels lose 40 % of their rate; a
                         padded leading dimension (k + 256) restores it.  Multiples of 8. */
} tally_gemm_bf16_args;

/* y[r] = sum_k W[r][k] x[k]; W is n x k row-major.  Block b owns rows [4b, 4b+4), one
 * 64-lane wave per row.  k must be a multiple of 8. */
typedef struct { const uint16_t *x; const uint16_t *W; uint16_t *y; uint32_t n, k; } tally_gemv_bf16_args;

/* Row-wise kernels: block b owns rows [4b, 4b+4), one wave per row; rows are cols
 * fp32 apart.  cols <= 8192. */
typedef struct { const float *x; float *y; uint32_t rows, cols; } tally_softmax_f32_args;
typedef struct {
  const float *x; const float *gamma; const float *beta; float *y;
  uint32_t rows, cols; float eps;
} tally_layernorm_f32_args;

/* out[h] = softmax(q[h] . K[:,h,:]^T / sqrt(dim)) . V[:,h,:]; q, out: heads x dim;
 * K, V: tokens x heads x dim; dim must be 128.  `scratch` is caller-owned device memory
 * of tally_attn_decode_scratch_bytes(heads) bytes (split partial results). */
typedef struct {
  const uint16_t *q; const uint16_t *K; const uint16_t *V; uint16_t *out; void *scratch;
  uint32_t tokens, heads, dim;
} tally_attn_decode_args;

typedef struct {
  uint32_t kernel_id;        /* tally_kernel_id                                           */
  tally_dim3 grid, block;    /* LOGICAL grid and block, as the original kernel is launched */
  const void *args;          /* host pointer to the matching tally_*_args                  */
  size_t args_size;          /* sizeof of that struct                                      */
} tally_kernel_desc;

/* Per-logical-block coverage record, written by the transformed kernels when a job is
 * created with coverage enabled (test/diagnostic).  `count` is incremented atomically;
 * b[] is the block index the kernel rebuilt from the offset or task index. */
typedef struct { uint32_t count, bx, by, bz, segment, worker; } tally_cover_rec;

typedef struct tally_ctx tally_ctx; /* owns flags, counters, status words, marker words */
typedef struct tally_job tally_job; /* one best-effort kernel instance and its progress  */

/* ---- context ---------------------------------------------------------------------- */

/* Create a context on the current device for one high-priority and one best-effort
 * stream (Section 4: one high-priority task next to best-effort tasks).  The two
 * hipStream_t stay the caller's (never destroyed here; default priority expected).  The
 * call allocates the context's device and pinned host words, creates the stream the relay
 * kernels use, and times a few microsecond-long kernels on the streams to choose it
 * (see tally_stream_report): it synchronises both streams and takes some milliseconds, so
 * call it while they are idle.  TALLY_ERR_NOMEM / TALLY_ERR_HIP (tally_last_hip_error())
 * on failure, with nothing left allocated. */
int tally_create(tally_ctx **out, void *hip_stream_hi, void *hip_stream_be);
int tally_destroy(tally_ctx *ctx); /* all jobs must have been freed */

/* Logical grid/block of a kernel for given arguments (host struct). */
int tally_logical_grid(uint32_t kernel_id, const void *args, size_t args_size,
                       tally_dim3 *grid, tally_dim3 *block);
size_t tally_attn_decode_scratch_bytes(uint32_t heads);

/* ---- the three launch forms ------------------------------------------------------- */

/* Original form: one launch of the whole logical grid on the high-priority stream
 * (on_hi_stream != 0) or on the best-effort stream (Section 4.2: high-priority
 * kernels are launched with the default configuration).  Asynchronous. */
int tally_launch_native(tally_ctx *ctx, const tally_kernel_desc *desc, int on_hi_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the decode-attention launch of
 * tally_launch_native with its split records kept in a device array that is part of the
 * library instead of caller-provided scratch.  args->scratch is ignored (may be NULL);
 * everything else is as for TALLY_K_ATTN_DECODE_BF16.  The call allocates nothing and calls
 * no allocating routine.  Limit: heads <= TALLY_ATTN_STATIC_MAX_HEADS (the array takes
 * about 1 MiB on every GPU the library runs on, until the process ends);
 * TALLY_ERR_INVALID_ARG beyond it, TALLY_ERR_BAD_STATE if the current device is not the
 * context's.  Nothing in the array has to start at zero (every record is written before it
 * is read).  All calls on one GPU share the array: two calls whose kernels overlap in time
 * (e.g. one per stream) race; calls on one stream are ordered by the stream. */
#define TALLY_ATTN_STATIC_MAX_HEADS 128
int tally_launch_attn_decode_static(tally_ctx *ctx, const tally_attn_decode_args *args,
                                    int on_hi_stream);

/* Sliced form (Section 4.1, slicing transformation): the grid is cut into sub-kernels
 * of slice_blocks consecutive logical blocks (last one: the remainder); each sub-kernel
 * receives a block offset and rebuilds its logical block index as offset + blockIdx.
 * At most max_in_flight (>= 1; 1 = "one at a time", Section 4.2) sub-kernels are
 * enqueued; this call issues the first ones, tally_pump() the following.
 * coverage != 0 allocates per-block coverage records. */
int tally_launch_sliced(tally_ctx *ctx, const tally_kernel_desc *desc, uint32_t slice_blocks,
                        uint32_t max_in_flight, int coverage, tally_job **out);

/* Preemptible persistent-worker form (Section 4.1, preemption transformation):
 * num_workers worker blocks loop { check flag; fetch-and-add the global task counter;
 * map the task index to the logical block index; run the block; barrier }.
 * `chunk` (>= 1) is the number of consecutive task indices taken per fetch; 1 is the
 * paper's form.  A fetched index is always executed before the worker exits.
 * num_workers must not exceed tally_max_workers(): every worker has to be resident at
 * once (Section 4.2 draws its candidates from the multiples of the compute-unit count
 * that fit).  Workgroups that wait for room keep their hardware queue's dispatcher busy,
 * and then neither the relay of the preemption flag nor a high-priority kernel is sure
 * to start before the kernel ends.  TALLY_ERR_INVALID_ARG otherwise. */
int tally_launch_ptb(tally_ctx *ctx, const tally_kernel_desc *desc, uint32_t num_workers,
                     uint32_t chunk, int coverage, tally_job **out);

/* Measured ceiling of the bf16 matrix pipe on this device, for the roofline: a register-only
 * loop of independent 32x32x16 MFMAs (random operand bits), one wave per SIMD on every
 * compute unit, 4096 MFMAs per wave as in one 256x256x4096 tile; best of `reps` launches on
 * the best-effort stream, timed with HIP events.  Allocates and frees a few KB. */
int tally_mfma_ceiling_tflops(tally_ctx *ctx, uint32_t reps, double *tflops);

/* What one workgroup of a kernel occupies on a compute unit: LDS bytes, 64-lane waves,
 * registers per lane (vector and accumulation registers together, as allocated).
 * form 0: persistent-worker kernel, 1: original form.  The scheduler uses these figures
 * for admission among best-effort clients and to decide whether paused best-effort
 * workers leave room for the high-priority kernels. */
int tally_kernel_footprint(tally_ctx *ctx, uint32_t kernel_id, int form, uint32_t *lds_bytes,
                           uint32_t *waves, uint32_t *regs_per_lane);

/* Largest worker count of the persistent-worker form of this kernel whose workgroups are
 * all resident at once on an otherwise idle GPU: compute units x workgroups per unit. */
int tally_max_workers(tally_ctx *ctx, const tally_kernel_desc *desc, uint32_t *max_workers);

/* preempt_best_effort_kernel() of the scheduling algorithm (Section 4.2, Figure 4), acting
 * as Section 4.1 describes: non-blocking.  Persistent-worker job: raise its preemption
 * signal (one host store; the device folds it into the global task counter, so that every
 * later fetch of a task index fails); workers finish the block(s) they hold and exit,
 * leaving the progress in the task index.  Sliced job: stop issuing sub-kernels (those
 * already enqueued finish).  No-op on STOPPED / COMPLETE jobs.  Callable from any thread. */
int tally_preempt(tally_job *job);

/* Extension for blocks that last far longer than the turnaround threshold (a 256x256 GEMM
 * tile over a long K lasts 120 us and more): tally_preempt() plus a request that workers of
 * kernels which support it pause INSIDE their block, keeping registers and LDS, so that the
 * high-priority kernel runs beside them undisturbed.  The pause ends when tally_end_pause()
 * withdraws it or when a block's pause budget (tally_set_yield_bound_us) is spent.  Only
 * use it when the high-priority kernels fit beside the paused workgroups
 * (tally_kernel_footprint); otherwise they wait for the pause to end.  Other kernels and
 * sliced jobs: same as tally_preempt(). */
int tally_preempt_pausing(tally_job *job);

/* kernel.resume() of Figure 4: continue a STOPPED job from its saved task counter / block
 * offset (Section 4.1: the progress of the execution is held in the global task index; a
 * kernel that terminated early is resumed from the point at which it ended).  The task
 * counter is not reset.  BAD_STATE while RUNNING; no-op when COMPLETE. */
int tally_resume(tally_job *job);

/* Budget of tally_preempt_pausing(): the longest time one block may spend paused, all its
 * pauses together, in microseconds (default 1000; 0 disables pausing).  It keeps a
 * high-priority kernel that does not fit beside the paused workers from waiting for ever.
 * Applies to jobs launched after the call. */
int tally_set_yield_bound_us(tally_ctx *ctx, uint32_t us);

/* How often a pausing body looks at the pause word: every `steps` of its inner loop (a power
 * of two up to 1024; default 4, about 2 us of a GEMM tile).  Each look stalls the workgroup
 * for a memory round trip, so fewer steps buy a faster pause with best-effort throughput
 * (measured on a 4096^3 GEMM: 16 -> 4 steps costs 1.6 % alone and takes 3 us off the median
 * and 1.5 us off the 99th percentile of a co-located 4096 x 4096 GEMV).
 * Applies to jobs launched after the call. */
int tally_set_yield_every(tally_ctx *ctx, uint32_t steps);

/* End the pause of tally_preempt_pausing(): paused workers go on and finish their block.
 * The preemption itself stands (its signal is in the task counter): workers still leave at
 * their next block boundary and the job becomes STOPPED.  No-op otherwise.  Any thread. */
int tally_end_pause(tally_job *job);

/* running() / stopped() of Figure 4, and the progress Section 4.1 keeps in the task index:
 * non-blocking snapshot.  done_blocks = task indices handed out so far, at most total, as
 * last published by the device; exact once the job is STOPPED or COMPLETE, when every block
 * below it has run and none above it (the prefix property).  Any out pointer may be null.
 * Callable from any thread. */
int tally_progress(tally_job *job, uint64_t *done_blocks, uint64_t *total_blocks, int *state);

/* One visit of a best-effort client in the loop of Figure 4 (Section 4.2: sub-kernels are
 * launched one at a time).  Sliced jobs: retire finished sub-kernels and, unless preempted,
 * enqueue the next ones.  Persistent-worker jobs: refresh the state.  Non-blocking. */
int tally_pump(tally_job *job);

/* Wait for the drain Section 4.1 describes (after a preemption signal every worker finishes
 * its current block and exits) or for completion: blocks (host spin, pumping a sliced job)
 * until the job is STOPPED or COMPLETE, then synchronises the best-effort stream so that
 * outputs are visible.  TALLY_ERR_BAD_STATE if the device could not report the progress of
 * a preempted segment (never seen; the job then cannot be resumed). */
int tally_wait(tally_job *job, int *state);
int tally_job_free(tally_job *job); /* waits for in-flight launches of the job first */

/* ---- test / diagnostic ------------------------------------------------------------- */

/* Deterministic preemption "at counter value stop_at": the workers treat stop_at as
 * the end of the grid, which is what a preemption observed exactly when the counter
 * reached stop_at produces; the job ends STOPPED with progress == stop_at (or COMPLETE
 * if stop_at >= total). */
int tally_launch_ptb_until(tally_ctx *ctx, const tally_kernel_desc *desc, uint32_t num_workers,
                           uint32_t chunk, uint64_t stop_at, int coverage, tally_job **out);
int tally_resume_until(tally_job *job, uint64_t stop_at);

/* Copy the coverage records (one tally_cover_rec per logical block, x-fastest linear
 * order) to host memory.  Job must be STOPPED or COMPLETE. */
int tally_coverage(tally_job *job, void *host_records, size_t bytes);

/* Enqueue, on the high-priority (or best-effort) stream, a marker that stores `value`
 * into the context's host-visible word for that stream once all earlier work on the
 * stream has finished; tally_marker_read() returns the last stored value. */
int tally_marker(tally_ctx *ctx, int on_hi_stream, uint32_t value);
int tally_marker_read(tally_ctx *ctx, int on_hi_stream, uint32_t *value);

/* Time from tally_preempt() to the device reporting the job drained, in microseconds
 * (host clock); negative if the last segment was not preempted. */
int tally_last_preempt_latency_us(tally_job *job, double *us);

int tally_last_hip_error(void);
const char *tally_strerror(int status);
int tally_device_info(uint32_t *num_cus, uint32_t *lds_bytes_per_cu, uint32_t *wave_size);

/* Hardware queues (Section 4.2: a high-priority kernel is dispatched the moment it arrives).
 * The command processors (one per die) serve the queues through four pipes each.  A kernel
 * resident on a queue that shares the high-priority queue's pipe, on any die, delays the
 * start of every high-priority kernel with workgroups there by about 10 us.  The library measures
 * this when it creates a stream for resident best-effort work (relays; the further clients'
 * stream pairs) and sets aside streams that, busy beside the ones already in use, delay the
 * high-priority one.  *be_delays_hi: bit 0, the caller's own best-effort stream does
 * (create the two streams one right after the other to avoid it); bit 1, more streams were
 * needed than there are free pipes (from the second best-effort client on) and one was
 * taken although it delays.  *set_aside: streams created and left unused so far.  Either
 * pointer may be null. */
int tally_stream_report(tally_ctx *ctx, int *be_delays_hi, uint32_t *set_aside);

/* ---- profile-guided configuration (Section 4.2) ------------------------------------ */

typedef struct {
  uint32_t kind;          /* 0 = persistent workers, 1 = sliced                          */
  uint32_t param;         /* worker count, or blocks per slice                            */
  uint32_t chunk;         /* persistent workers: task indices per fetch; sliced: slices
                             enqueued at a time (0 and 1 both mean one, as in the paper)   */
  float latency_ms;       /* mean whole-kernel latency over the profiling runs            */
  float turnaround_ms;    /* Eq. 1 for persistent workers; sliced: one slice's time times
                             the slices enqueued at a time                                 */
} tally_config;

/* Eq. 1: kernel_latency * worker_blocks / total_blocks (times `chunk`). */
double tally_ptb_turnaround_ms(double kernel_latency_ms, uint32_t worker_blocks, uint32_t chunk,
                               uint64_t total_blocks);

/* Best-performing candidate whose turnaround estimate is <= threshold_ms; if none
 * complies, the one with the smallest estimate.  Returns its index or a negative status. */
int tally_select_config(const tally_config *cands, uint32_t n, double threshold_ms);

/* Measure every candidate configuration of a kernel on the best-effort stream (`runs`
 * timed executions each, after one warm-up; the kernel really runs, so its outputs are
 * written `runs`+1 times per candidate), fill latency and turnaround, choose under
 * threshold_ms and cache the choice per (kernel, grid, block).  cands: in/out array.
 * Turnaround of a persistent-worker candidate is Eq. 1; for a kernel whose workers pause
 * inside their blocks while preempted (and with the pause enabled, see
 * tally_set_yield_bound_us) it is the time of ONE block times the share of a block
 * between two pause points, since that is when the execution units are handed over. */
int tally_profile(tally_ctx *ctx, const tally_kernel_desc *desc, tally_config *cands, uint32_t n,
                  uint32_t runs, double threshold_ms, uint32_t *chosen);
/* lookup_launch_config() of Figure 4: the fixed choice for (kernel, grid, block);
 * TALLY_ERR_BAD_STATE while none is fixed. */
int tally_lookup_config(tally_ctx *ctx, const tally_kernel_desc *desc, tally_config *out);

/* get_candidate_configs() of Figure 4 (Section 4.2): persistent-worker counts that are
 * multiples of the compute-unit count up to tally_max_workers(), each with 1, 4 and 16 task
 * indices per fetch where every worker then still has a fetch to make, and slices of
 * 1/1 (the whole grid in one launch: what a kernel shorter than the threshold needs),
 * 1/2, 1/4, ... 1/256 of the grid.  Writes at most cap entries (latency and turnaround zero)
 * and their number. */
int tally_candidate_configs(tally_ctx *ctx, const tally_kernel_desc *desc, tally_config *out,
                            uint32_t cap, uint32_t *n);

/* The profiling record of (kernel, grid, block) as it stands: candidates (latency = mean of
 * the samples so far), samples per candidate, index of the fixed choice or -1.  *n = 0 if
 * the kernel has never been seen.  out / samples may be NULL. */
int tally_profile_table(tally_ctx *ctx, const tally_kernel_desc *desc, tally_config *out, uint32_t cap,
                        uint32_t *n, uint32_t *samples, int *chosen);
int tally_profile_reset(tally_ctx *ctx);   /* forget every measurement and choice */

/* ---- two-stream priority scheduler (Section 4.2, Figure 4) ------------------------- */

/* The priority-aware scheduler as a running service.  Clients hand it kernels: the
 * high-priority client's are dispatched at once in their original form after the running
 * best-effort kernels have been told to give way (Figure 4, the high-priority branch);
 * best-effort clients' kernels are queued per client and launched, resumed or continued
 * slice by slice only while no high-priority request is in flight (the best-effort branch).
 * A best-effort kernel submitted without a configuration gets one as Section 4.2 describes:
 * lookup_launch_config(), and while none is fixed launch_and_profile(): each real
 * invocation of the kernel runs under the next unmeasured candidate of its candidate set
 * and is that candidate's measurement; when every candidate has `profile_runs` samples the
 * best-performing one whose turnaround estimate is within the threshold is fixed and reused.
 * The scheduler is built on the calls above (launch, preempt, resume, pump, progress).
 *
 * Threads: the best-effort clients are served by a thread the scheduler owns (it sleeps
 * while no client has work).  tally_sched_submit_hi / tally_sched_poll must come from one
 * thread (the high-priority client's); tally_sched_submit_be / tally_sched_stats from any.
 * While a scheduler exists, do not call launch functions on its context yourself. */
typedef struct tally_sched tally_sched;

#define TALLY_SCHED_NO_PAUSE 1u      /* never ask workers to pause inside their blocks        */
typedef struct {
  uint32_t policy;          /* 0 = priority scheduling with preemption (the method)
                               1 = priority scheduling, best-effort kernels as submitted
                               2 = no scheduling: everything dispatched on arrival          */
  uint32_t n_be_clients;    /* 0 .. 8; client 0 uses the context's best-effort stream, the
                               others a stream pair of their own.  n clients need 2 + 2n
                               hardware queues: the process must have been started with
                               GPU_MAX_HW_QUEUES at least that (HIP's default is 4), else
                               TALLY_ERR_UNSUPPORTED                                        */
  double threshold_ms;      /* turnaround-latency threshold of the profile-guided choice;
                               0 = the paper's default, 0.0316 ms                           */
  uint32_t profile_runs;    /* invocations averaged per candidate; 0 = 10 (Section 4.2)     */
  uint32_t flags;           /* TALLY_SCHED_*                                                */
} tally_sched_opts;

int tally_sched_create(tally_ctx *ctx, const tally_sched_opts *opts, tally_sched **out);
/* Stops the best-effort thread (kernels in flight are preempted at block boundaries and
 * dropped where they stand, queued ones discarded), waits for the streams, frees. */
int tally_sched_destroy(tally_sched *s);

#define TALLY_SUBMIT_LOOP 1u         /* when the kernel completes it goes to the back of its
                                        client's queue again (a training loop's step)        */
#define TALLY_SUBMIT_END_OF_STEP 2u  /* completing it counts one step of the client           */
/* Queue one best-effort kernel for `client`.  The descriptor and its args struct are copied;
 * the device buffers they point to stay the caller's and must outlive the kernel.  config:
 * persistent workers / sliced / native (kind 0 / 1 / 2) as given, or NULL to have the
 * profiler choose. */
int tally_sched_submit_be(tally_sched *s, uint32_t client, const tally_kernel_desc *kernel,
                          const tally_config *config, uint32_t flags);

/* One high-priority request of n kernels: preempt_best_effort_kernel() for every
 * best-effort client (workers pause inside long blocks if all n kernels fit beside them,
 * else they only give way at block boundaries), then launch the kernels in their original
 * form on the high-priority stream.  One request at a time: TALLY_ERR_BAD_STATE while the
 * previous one is in flight. */
int tally_sched_submit_hi(tally_sched *s, const tally_kernel_desc *kernels, uint32_t n);

/* Non-blocking: has the request in flight completed?  When it has, the best-effort clients
 * are released (and paused workers go on) unless more_pending says that another request
 * follows at once.  Also reports an error of the best-effort thread. */
int tally_sched_poll(tally_sched *s, int more_pending, int *hi_in_flight);

/* Switch the best-effort side off (running kernels are preempted and stay stopped) or on. */
int tally_sched_enable_be(tally_sched *s, int enable);

typedef struct {
  uint64_t hi_requests_done;
  uint64_t be_kernels_done;            /* over all clients                                   */
  uint64_t be_steps_done;              /* client 0: kernels flagged END_OF_STEP completed    */
  uint64_t be_client_kernels_done[8];
  uint64_t n_preempts;                 /* drains that followed a preemption request          */
  uint64_t profile_samples;            /* invocations that served as a candidate's measurement */
  uint64_t configs_fixed;              /* kernels whose configuration the profiler has fixed  */
} tally_sched_stats_t;
int tally_sched_stats(tally_sched *s, tally_sched_stats_t *out);
/* Move up to cap recorded preemption latencies (request -> drained, microseconds, host
 * clock) into out; the scheduler keeps the 4096 oldest not yet taken. */
int tally_sched_take_preempt_latencies(tally_sched *s, double *out, uint32_t cap, uint32_t *n);

typedef struct {
  const tally_kernel_desc *kernel; /* one best-effort kernel of the step                   */
  tally_config config;             /* kind 0/1 as above; kind 2 = native (untransformed);
                                      kind 3 = chosen by the profiler                       */
} tally_be_item;

typedef struct {
  /* inputs */
  const tally_kernel_desc *hi_kernels; uint32_t n_hi_kernels; /* one high-priority request  */
  const double *arrivals_us; uint32_t n_arrivals; /* open-loop arrival times from t0        */
  const tally_be_item *be_items; uint32_t n_be_items; /* one best-effort step, repeated      */
  uint32_t policy;            /* as tally_sched_opts.policy                                  */
  double tail_us;             /* keep feeding best-effort work this long after last arrival  */
  /* outputs (host arrays owned by the caller) */
  double *latency_us;         /* n_arrivals: scheduled arrival -> completion observed        */
  double *preempt_latency_us; uint32_t preempt_cap; uint32_t n_preempts; /* per preemption   */
  uint64_t be_kernels_done;   /* best-effort kernels completed inside the window             */
  uint64_t be_steps_done;
  double window_us;           /* wall time of the run (start of the clock to the last request
                                 completed and the tail elapsed; teardown is not in it)      */
  double *issue_us;           /* optional (may be NULL), n_arrivals: scheduled arrival -> the
                                 request's launch calls have returned on the host            */
  /* several best-effort clients (Figure 4 loops over them): be_items is the concatenation
   * of the clients' steps, client c owning be_client_items[c] consecutive items.  NULL / 0 =
   * one client owning every item; at most 8 clients.  be_steps_done counts client 0's. */
  const uint32_t *be_client_items; uint32_t n_be_clients;
  uint64_t *be_client_kernels_done; /* optional output, n_be_clients entries                */
  /* profile-guided items (kind 3) */
  double threshold_ms; uint32_t profile_runs; uint32_t sched_flags;   /* as tally_sched_opts */
  uint64_t profile_samples, configs_fixed;                            /* outputs             */
  /* Alternating measurement: with be_toggle_every = T > 0 the best-effort side is switched
   * off (tally_sched_enable_be) for arrivals [0, T), on for [T, 2T), off for [2T, 3T) ...,
   * so that one run yields the high-priority job's latencies alone and co-located under the
   * same host and machine conditions.  be_enabled_us (output) is the time the best-effort
   * side was switched on; be_kernels_done counts what completed in the whole window. */
  uint32_t be_toggle_every;
  double be_enabled_us;
} tally_sched_run_t;

/* Replay driver over the scheduler: creates one, submits every best-effort item as a looping
 * step, then plays the arrival list on the calling thread (tally_sched_submit_hi at each
 * arrival time, tally_sched_poll until it completes) until every arrival has completed and
 * tail_us has elapsed, and destroys the scheduler.  n_arrivals == 0 runs the best-effort job
 * alone for tail_us; n_be_items == 0 runs the high-priority job alone. */
int tally_sched_run(tally_ctx *ctx, tally_sched_run_t *run);

#ifdef __cplusplus
}
#endif
#endif /* TALLY_H */
