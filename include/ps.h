/*
 * ps.h -- C ABI of a GPU-resident parameter service for gfx950 (MI355X).
 *
 * The service does what the paper's aggregation servers do (Section 2,
 * "Background and Motivation"; Section 3.1, "System Overview"): it hosts the
 * master copy of every registered job's parameters, collects the gradient
 * pushes of the job's W workers, aggregates them, updates the master copy with
 * the aggregated result, and answers pulls.  Aggregations are tensor-scale and
 * independent of each other (Section 2.2), so they are not grouped by job: one
 * call aggregates a list of blocks that may belong to many jobs, the way the
 * paper packs several jobs' aggregations onto one server (Section 3.1).  The
 * key of a piece of state is (job id, block id), as in Appendix A where the
 * agent rewrites a tensor's key to (job ID, tensor ID).
 *
 * A BLOCK is a contiguous slice of one layer (tensor) of at most
 * max_block_bytes/4 binary32 values: as many full blocks as fit, then one
 * remainder block.  Blocks are numbered per job in registration order.
 *
 * Arithmetic of one aggregation of a block (binary32, every operation rounded
 * separately, no fused multiply-add unless PS_FLAG_FP_CONTRACT is set):
 *     S  = ((g_0 + g_1) + g_2) + ... + g_{W-1}          fixed worker order
 *     d  = S + wd * p ;   v' = mu * v + d ;   p' = p - lr * v'
 * and the block's telemetry value sum_i S_i^2 accumulated in binary64.
 *
 * Conventions
 *   - Every function returns a status (PS_OK = 0, errors negative) unless
 *     stated otherwise.  Nothing throws across this boundary: a failed host
 *     allocation inside the library comes back as PS_ERR_NOMEM.
 *   - "device" pointers address GPU memory of the current HIP device; "host"
 *     pointers address ordinary memory.  The library never takes ownership of a
 *     pointer passed in.
 *   - stream arguments are hipStream_t values passed as void* (NULL = the
 *     default stream).  Device work is enqueued on that stream and not waited
 *     for; the caller synchronises.
 *   - One context is guarded by one mutex: calls on the same context may come
 *     from several threads.  Aggregation, pull and telemetry of a block are
 *     ordered by the streams the caller uses.
 */
#ifndef PS_H_
#define PS_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PS_MAX_W 32                 /* most workers per job (push mask is 32 bits) */
#define PS_DEFAULT_BLOCK_BYTES (4u << 20)
#define PS_DEFAULT_SMALL_ELEMS 4096u
#define PS_ALIGN_BYTES 256u          /* alignment of every block inside the arena */
#define PS_GRAD_ALIGN_BYTES 16u      /* alignment required of pushed gradients */

enum {
  PS_OK = 0,
  PS_ERR_ARG = -1,         /* null pointer, W outside [1, PS_MAX_W], numel <= 0, non-finite scalar */
  PS_ERR_BAD_JOB = -2,     /* unknown or unregistered job id */
  PS_ERR_BAD_BLOCK = -3,   /* block id outside the job */
  PS_ERR_BAD_WORKER = -4,  /* worker outside [0, W) */
  PS_ERR_DUP_PUSH = -5,    /* this worker already pushed this block in this round */
  PS_ERR_NOT_READY = -6,   /* a listed block has not received all W pushes */
  PS_ERR_DUP_BLOCK = -7,   /* the same block appears twice in one list */
  PS_ERR_ALIGN = -8,       /* pointer not aligned as required */
  PS_ERR_NOMEM = -9,       /* arena exhausted, or a host/device allocation failed */
  PS_ERR_NO_DEVICE = -10,  /* the context was created without an arena (planning only) */
  PS_ERR_HIP = -11,        /* a HIP runtime call failed; see ps_last_error */
  PS_ERR_CAPACITY = -12,   /* an output array is too small; the needed count is reported */
  PS_ERR_NOT_OWNER = -13,  /* the block's master copy is not (or no longer) held by this context */
  PS_ERR_BUSY = -14,       /* the block has pushes pending: it cannot start to migrate now */
  PS_ERR_NO_ROOM = -15     /* scheduling: no Aggregator cluster has room for the job (ps_sched.h) */
};

/* Where a block's master copy is, as seen by one context. */
enum {
  PS_OWNER_HERE = 0,       /* this context holds it and aggregates it */
  PS_OWNER_LEAVING = 1,    /* migration announced: still readable here, no pushes, no updates */
  PS_OWNER_ELSEWHERE = 2   /* another context holds it */
};

enum {
  PS_FLAG_FP_CONTRACT = 1u /* use fused multiply-add in the update (not bit-exact with
                              the separately rounded definition; error <= 1e-6 relative) */
};

typedef struct ps_ctx ps_ctx;
typedef int32_t ps_job_t;

typedef struct ps_config {
  uint64_t max_block_bytes;   /* 0 = PS_DEFAULT_BLOCK_BYTES; a multiple of 256, at most 1 GiB */
  uint32_t small_block_elems; /* blocks of at most this many values take the small-block
                                 path; 0 = PS_DEFAULT_SMALL_ELEMS; at most 4096 */
  uint32_t flags;             /* PS_FLAG_* */
  void* arena_dev;            /* device memory for the master copies, 256-byte aligned,
                                 owned by the caller, must outlive the context.
                                 NULL = planning context: layouts, push state and wave
                                 packing work, anything touching the device returns
                                 PS_ERR_NO_DEVICE */
  uint64_t arena_bytes;
  uint32_t launch_tiles;      /* tiles (4096 values each) per kernel launch of the large-block
                                 path; 0 = as many as the chip holds at once (2048 on MI355X);
                                 a larger value switches the store hold off for that launch */
  int32_t store_hold_permille; /* a launch's workgroups keep their results in registers and
                                 store them only once this fraction (in 1/1000) of the
                                 launch's predicted read time has passed since they
                                 started, so that reads and writes reach HBM in separate
                                 bursts; 0 = default (980), negative = no hold, at most 2000 */
  int32_t store_stagger_permille; /* the workgroups of a launch release their stores one after
                                 the other in address order, spread over this fraction (in
                                 1/1000) of the time the launch's stores take at the read
                                 rate, so that the writes reach HBM as a paced sweep;
                                 0 = default (835), negative = all at once, at most 4000;
                                 without a hold there is no spread either */
  int32_t reserved_;           /* 0 */
} ps_config;

typedef struct ps_block_ref {
  ps_job_t job;
  int32_t block;
} ps_block_ref;

typedef struct ps_block_info {
  int32_t layer;          /* index of the layer this block is a slice of */
  int32_t W;              /* workers of the job */
  int64_t layer_offset;   /* first element of the block inside its layer */
  int64_t numel;          /* elements in the block */
  int64_t flat_offset;    /* first element of the block inside the job's flat layout
                             (every layer starts on a 256-byte boundary; a layer's blocks
                             are contiguous).  Parameters, momentum and, by convention of
                             ps_push_flat, a worker's gradient buffer share this layout. */
  int64_t round;          /* aggregations applied to this block so far */
  uint32_t push_mask;     /* bit w set = worker w has pushed for the current round */
  uint32_t small_path;    /* 1 if the block takes the small-block path */
  uint32_t owner;         /* PS_OWNER_* */
  uint32_t reserved_;
} ps_block_info;

typedef struct ps_block_stats {
  double grad_norm2;      /* sum_i S_i^2 of the block's last completed aggregation */
  int64_t round;          /* the block's round counter after that aggregation, written by
                             the GPU together with the value (0 = never aggregated) */
} ps_block_stats;

typedef struct ps_wave_stats {
  int64_t n_blocks;        /* blocks in the list */
  int64_t n_params;        /* sum of their numel */
  int64_t n_large_tiles;   /* workgroups taking a tile of a large-path block */
  int64_t n_small_blocks;  /* blocks routed to the small-block path */
  int64_t n_small_bins;    /* workgroups taking a bin of small-path blocks */
  int64_t small_params;    /* parameters in small-path blocks */
  uint64_t algorithmic_bytes; /* sum over blocks of (4 W + 16) * numel */
  uint64_t small_algorithmic_bytes; /* the part of that in small-path blocks */
  int64_t n_launches;      /* aggregation kernel launches the list is cut into */
  double est_seconds;      /* predicted GPU time of the wave on MI355X: per launch, bytes read
                              at the read rate, then bytes written at the write rate (ps_rates:
                              7.0 TB/s each), plus 1.4 us; plus 5 us a wave.  Within a few per
                              cent of the measured time for waves of tens of megabytes and more
                              (a planning context assumes launches of 2048 tiles, what an
                              MI355X holds at once); an execution time e_t for
                              ps_sched_assign (the paper's profiler, Section 3.3.1) */
} ps_wave_stats;

typedef struct ps_rates_info {
  double read_bytes_per_sec;   /* HBM rate of a launch's read phase */
  double write_bytes_per_sec;  /* ... and of its write phase */
  int32_t reserved_[2];        /* 0 */
} ps_rates_info;

typedef struct ps_timing {
  int64_t n_waves;     /* waves measured since ps_timing_enable */
  int64_t n_launches;  /* aggregation kernel launches in those waves */
  double upload_ms;    /* host->device copy of the wave's tables */
  double agg_ms;       /* the aggregation launches, first start to last end */
  double norms_ms;     /* per-block telemetry reduction */
  double total_ms;     /* all of the above, GPU time (sums over waves) */
} ps_timing;

/* --- life cycle ---------------------------------------------------------- */

/* Create a context.  cfg is copied.  The library's own device tables are small
 * and grow on demand inside ps_aggregate; ps_create itself allocates 8 MiB of
 * pinned host memory (the staging buffer of ps_aggregate_noalloc).  The arena
 * is not touched.
 * Errors: PS_ERR_ARG (bad cfg, misaligned arena, small_block_elems > 4096). */
int32_t ps_create(const ps_config* cfg, ps_ctx** out_ctx);

/* Destroy a context and free the library's own tables.  The caller must have
 * synchronised every stream that was passed to this context.  NULL is allowed. */
void ps_destroy(ps_ctx* ctx);

/* Bytes of arena a job with these layers occupies (parameters + momentum, with
 * alignment padding), so the caller can size the arena before ps_create. */
int32_t ps_job_arena_bytes(const ps_config* cfg, const int64_t* layer_numel, int32_t n_layers,
                           uint64_t* out_bytes);

/* --- registration (the paper's job registration + per-tensor Init) -------- */

/* Register a job: split every layer into blocks, carve parameter and momentum
 * shards out of the arena, zero the momentum, and set the parameters from
 * init_params (host array of n_layers DEVICE pointers, layer l holding
 * layer_numel[l] floats; the array itself or single entries may be NULL = zeros).
 * The copies are enqueued on stream.  *out_job receives the id, *out_n_blocks
 * the number of blocks.  Errors: PS_ERR_ARG, PS_ERR_NOMEM, PS_ERR_HIP. */
int32_t ps_register_job(ps_ctx* ctx, const int64_t* layer_numel, int32_t n_layers, int32_t W,
                        float lr, float momentum, float wd, const float* const* init_params,
                        void* stream, ps_job_t* out_job, int32_t* out_n_blocks);

/* Register a job whose master copies live in another context for now: same
 * layout and arena use as ps_register_job, but every block starts as
 * PS_OWNER_ELSEWHERE and can only be filled by ps_migrate_copy.  This is the
 * receiving side of the paper's tensor migration (Section 3.2, Appendix B). */
int32_t ps_register_shadow_job(ps_ctx* ctx, const int64_t* layer_numel, int32_t n_layers, int32_t W,
                               float lr, float momentum, float wd, void* stream, ps_job_t* out_job,
                               int32_t* out_n_blocks);

/* Job exit (Section 3.3.2: when a job leaves, what it held is given back).
 * Forget a job.  Its arena space is reused only if it was the most recently
 * registered live job (the arena is a stack).  Pending pushes are dropped.
 * Waves that name the job must have completed (synchronise their streams first):
 * the job's telemetry memory is released here and its arena space may be handed
 * to the next registration. */
int32_t ps_unregister_job(ps_ctx* ctx, ps_job_t job);

/* Number of blocks / flat elements (with padding) of a job; negative = error. */
int32_t ps_job_n_blocks(ps_ctx* ctx, ps_job_t job);
int64_t ps_job_flat_numel(ps_ctx* ctx, ps_job_t job);

/* One row of the table that says where a piece of a job's state lives and in
 * what condition: the counterpart of the agent's mapping from (job ID, tensor
 * ID) to the Aggregator holding the tensor (Section 3.1; Appendix A), at block
 * granularity, with the owner field a pull response would carry during a
 * migration (Appendix B). */
int32_t ps_job_block_info(ps_ctx* ctx, ps_job_t job, int32_t block, ps_block_info* out);

/* --- push (worker -> service) -------------------------------------------- */

/* The paper's Push (Section 2: after the backward pass of a tensor each worker
 * pushes its gradient of that tensor to the server; Appendix A: the request
 * carries the key and the worker).  Records worker's gradient for (job, block)
 * for the block's current round.  grad_dev: DEVICE pointer to numel floats, 16-byte aligned, owned by the
 * caller; it is read, never written, by the aggregation that consumes it and
 * must stay valid and unchanged until that aggregation has completed on its
 * stream.  No data is copied.  Errors: BAD_JOB, BAD_BLOCK, BAD_WORKER,
 * DUP_PUSH, ALIGN, ARG (NULL). */
int32_t ps_push(ps_ctx* ctx, ps_job_t job, int32_t block, int32_t worker, const float* grad_dev);

/* Push every block of the job from one worker whose gradient buffer grad_flat_dev
 * (DEVICE, 256-byte aligned, ps_job_flat_numel floats) uses the job's flat
 * layout.  All-or-nothing: on error no block is marked. */
int32_t ps_push_flat(ps_ctx* ctx, ps_job_t job, int32_t worker, const float* grad_flat_dev);

/* --- wave packing ---------------------------------------------------------- */

/* Build the block list of one wave in which each listed job contributes one
 * round.  Within a job, blocks come in back-propagation arrival order (last
 * registered layer first, ascending offset inside a layer: Section 2.1).  Jobs
 * are interleaved by fractional position: the k-th of n blocks of a job sits at
 * (k + 1/2)/n; ascending position, ties to the job listed first.  Writes at most
 * cap entries to out (host) and the total to *out_n; PS_ERR_CAPACITY if
 * cap is too small (then *out_n is still the needed count).  A job listed twice
 * is PS_ERR_DUP_BLOCK. */
int32_t ps_pack_wave(ps_ctx* ctx, const ps_job_t* jobs, int32_t n_jobs, ps_block_ref* out,
                     int64_t cap, int64_t* out_n);

/* Split a block list by readiness (late requests, Section 3.3.1 "Handling
 * Outliers"): blocks that have all W pushes go to out_ready, the others to
 * out_late, both in list order and each with room for n entries.  The caller
 * aggregates out_ready now and decides with ps_sched_admit_late whether a late
 * block may still join this cycle or waits for the next.  Validates ids,
 * duplicates and ownership like ps_aggregate; changes no state. */
int32_t ps_split_ready(ps_ctx* ctx, const ps_block_ref* block_list, int64_t n,
                       ps_block_ref* out_ready, int64_t* out_n_ready, ps_block_ref* out_late,
                       int64_t* out_n_late);

/* Validate a block list exactly as ps_aggregate would, and report how it would
 * be laid out on the GPU.  Changes no state, touches no device. */
int32_t ps_plan_wave(ps_ctx* ctx, const ps_block_ref* block_list, int64_t n, ps_wave_stats* out);

/* The same report for a list whose pushes need not be in yet (ids, duplicates
 * and ownership are still checked): what a wave of these blocks would cost. */
int32_t ps_estimate_wave(ps_ctx* ctx, const ps_block_ref* block_list, int64_t n, ps_wave_stats* out);

/* --- aggregate (the hot path) --------------------------------------------- */

/* Model aggregation (Section 2: once a tensor's gradients are in from all
 * workers the server aggregates them and updates the master copy with the
 * result; Section 3.1: one Aggregator serves the aggregations of many jobs; the
 * list is one cycle's worth of them, Section 3.3.1).  Aggregates every block of
 * block_list (host array of n entries): sums the W pushed gradients in worker
 * order and applies the update to the block's parameter and momentum shards, on
 * stream.  All-or-nothing: the whole list is validated first (BAD_JOB,
 * BAD_BLOCK, DUP_BLOCK, NOT_OWNER, NOT_READY if a block lacks a push: the
 * paper's aggregation is synchronous) and nothing is launched or changed on
 * error; NO_DEVICE on a planning context; HIP if the runtime refuses a call.
 * On success every listed block's push mask is cleared and its round advances
 * by one.  n = 0 is a no-op.  The launch tables of the previous call are reused
 * when the list and the pushed pointers are the same as then.  Waves on
 * different streams that touch the same block must be ordered by the caller. */
int32_t ps_aggregate(ps_ctx* ctx, const ps_block_ref* block_list, int64_t n, void* stream);

/* ps_aggregate for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * validation, same kernels and same results as ps_aggregate, but the call
 * allocates nothing on the device or through HIP (no hipMalloc, hipFree,
 * hipHostMalloc, no event or stream creation): the wave's tables and the
 * per-tile telemetry partials go into a device array of fixed size that is
 * part of the library image (8 MiB per GPU, held until the process ends),
 * through a pinned staging buffer that ps_create allocated.  A wave whose tables
 * do not fit (16 bytes per tile of 4096 values plus 64 + 8 W bytes per block:
 * about 2 G parameters in one wave, or some 25 000 blocks of 32 workers) is
 * refused with PS_ERR_CAPACITY and nothing is launched or consumed;
 * ps_last_error says how many bytes it needed.  Every use of the array on one
 * GPU -- from any context, thread or stream -- is serialised: a call holds a
 * per-GPU lock while it runs on the host, and its device work is ordered after
 * the previous use of the array by an event.  Tables are re-used when the list
 * and the pushed pointers repeat and no other call has used the array since;
 * otherwise the call first waits on the host for the previous use to finish
 * (the staging buffer is about to be rewritten).  Event timing
 * (ps_timing_enable) does not cover these waves.  Other errors as ps_aggregate. */
int32_t ps_aggregate_noalloc(ps_ctx* ctx, const ps_block_ref* block_list, int64_t n, void* stream);

/* --- pull (service -> worker) and inspection ------------------------------- */

/* The paper's Pull (Section 2: workers fetch the updated parameters before the
 * next iteration).  Borrowed DEVICE pointers to the block's parameters /
 * momentum: no copy is made, the worker reads the master copy in place.  They stay
 * valid until the job is unregistered; their contents are those of the last
 * aggregation enqueued for the block, in stream order.  A block that has
 * migrated away (PS_OWNER_ELSEWHERE) is PS_ERR_NOT_OWNER: pull from its new
 * owner; one that is only leaving (PS_OWNER_LEAVING) still answers. */
int32_t ps_pull(ps_ctx* ctx, ps_job_t job, int32_t block, const float** out_param_dev,
                int64_t* out_numel);
int32_t ps_pull_momentum(ps_ctx* ctx, ps_job_t job, int32_t block, const float** out_mom_dev,
                         int64_t* out_numel);

/* Pull as a copy: enqueue on stream a device-to-device copy of the block's
 * parameters into dst_dev (DEVICE, numel floats, owned by the caller) -- the
 * stand-in for the paper's server-to-worker transfer when a worker wants its own
 * replica.  Ordered after updates enqueued on the same stream (and after the
 * arrival of a shard that has just migrated here); updates running on other
 * streams are the caller's to order.  Errors as ps_pull, PS_ERR_HIP. */
int32_t ps_pull_copy(ps_ctx* ctx, ps_job_t job, int32_t block, float* dst_dev, void* stream);

/* Base DEVICE pointers of the job's flat parameter and momentum arrays
 * (ps_job_flat_numel floats each; block b starts at flat_offset).  Regions of
 * blocks this context does not own hold stale or unset data. */
int32_t ps_pull_flat(ps_ctx* ctx, ps_job_t job, const float** out_param_dev,
                     const float** out_mom_dev, int64_t* out_flat_numel);

/* Telemetry of a block's last aggregation: what the service measures about the
 * aggregations it runs, for whoever schedules them (the paper's job and server
 * profilers, Section 3.1, whose figures feed the assignment scheme of Section
 * 3.3.1; the quantity itself, the squared norm of the aggregated gradient, is
 * this library's choice).  The GPU writes the value together with the round it
 * belongs to, in one 16-byte store into host-visible memory, at the end of the
 * wave; the call reads that pair.  To see the round just enqueued, synchronise
 * the wave's stream first; without that the pair is that of an earlier round,
 * with its own round number. */
int32_t ps_telemetry(ps_ctx* ctx, ps_job_t job, int32_t block, ps_block_stats* out);

/* --- migration of a block's master copy between contexts ------------------- */
/* The paper moves a tensor between Aggregators inside the window in which its
 * master copy is idle -- after the last pull of an iteration and before the next
 * update -- and keeps two rules: the old owner stops serving it once the move is
 * announced, and the new owner never updates it before the copy is complete
 * (Section 3.2 "Tensor Migration"; Appendix B).  Here an Aggregator is a
 * context; both contexts hold the job (ps_register_job in one,
 * ps_register_shadow_job in the other, same layers and W).
 *
 * ps_migrate_begin   announce (the paper's MIGRATE_INIT): the block must have no
 *                    pending pushes (PS_ERR_BUSY otherwise).  It becomes
 *                    PS_OWNER_LEAVING: pulls still work, pushes and aggregation
 *                    return PS_ERR_NOT_OWNER.
 * ps_migrate_cancel  undo an announcement.
 * ps_migrate_copy    the paper's TENSOR_COPY: enqueue on stream the copy of the
 *                    parameter and momentum shards and of the round counter from
 *                    src to dst, ordered after src's updates in flight.  dst owns
 *                    the block from this call on and may take pushes at once; its
 *                    first ps_aggregate naming the block is ordered after the
 *                    copy on whatever stream it runs (TENSOR_COPY_DONE).  src
 *                    becomes PS_OWNER_ELSEWHERE.  If the shard had itself
 *                    arrived at src by a copy not yet waited for, the new copy
 *                    is ordered after that one.
 * ps_migrate_many    announce and copy n blocks (ids in blocks, host array) of
 *                    one job in one call, e.g. a whole job when an Aggregator is
 *                    recycled (Section 3.3.2).  Blocks may be owned or already
 *                    announced; all are checked before any moves (same errors
 *                    as above, PS_ERR_DUP_BLOCK for a repeated id; both jobs
 *                    must have been registered with the same layers and block
 *                    size, else PS_ERR_ARG).  Runs of consecutive block ids
 *                    move in one kernel launch, and the new owner waits on
 *                    one event for all of them. */
int32_t ps_migrate_begin(ps_ctx* ctx, ps_job_t job, int32_t block);
int32_t ps_migrate_cancel(ps_ctx* ctx, ps_job_t job, int32_t block);
int32_t ps_migrate_copy(ps_ctx* src, ps_job_t src_job, int32_t block, ps_ctx* dst, ps_job_t dst_job,
                        void* stream);
int32_t ps_migrate_many(ps_ctx* src, ps_job_t src_job, const int32_t* blocks, int32_t n, ps_ctx* dst,
                        ps_job_t dst_job, void* stream);

/* --- measurement ------------------------------------------------------------ */

/* The HBM rates behind the launch timing and behind ps_wave_stats.est_seconds
 * (the service's server profiler, Section 3.1: how fast this Aggregator is):
 * 7.0 TB/s each, fitted to launch times on MI355X.  They are fixed: a read
 * probe at start-up and reports from the launches themselves were both tried
 * and both timed the launches worse than these figures on every MI355X
 * measured.  store_hold_permille and store_stagger_permille scale what is
 * derived from them.  The rates change timing only, never results. */
int32_t ps_rates(ps_ctx* ctx, ps_rates_info* out);

/* Event timing of the waves, for measurement.  on == 1: from now on every
 * ps_aggregate brackets its aggregation launches with two HIP events on the
 * wave's stream (agg_ms; upload_ms and norms_ms stay 0 and total_ms = agg_ms).
 * on == 2: four events, so that the table upload and the telemetry reduction
 * are timed too.  Each event costs the stream a few microseconds.  The elapsed
 * times are summed per kind.  Resets the sums.  on == 0 stops it. */
int32_t ps_timing_enable(ps_ctx* ctx, int32_t on);
/* Wait for every wave this context has enqueued, then report the sums. */
int32_t ps_timing_read(ps_ctx* ctx, ps_timing* out);

/* --- diagnostics ----------------------------------------------------------- */

/* Static, never NULL. */
const char* ps_strerror(int32_t status);
/* Detail of the last failure this context reported with PS_ERR_HIP, or with
 * PS_ERR_CAPACITY from ps_aggregate_noalloc ("" if none).  Valid until the next
 * call on the context. */
const char* ps_last_error(ps_ctx* ctx);
/* Library version as major*10000 + minor*100 + patch. */
int32_t ps_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PS_H_ */
