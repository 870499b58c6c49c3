/*
 * ps_sched.h -- C ABI of the assignment and scaling logic of the parameter
 * service (host only; no device is touched).
 *
 * This is the paper's Section 3.3, "Model Aggregation Management":
 *   - cyclic execution: an Aggregator's cycle C_n is the largest profiled
 *     iteration duration D_j among the jobs it serves; a job with a shorter
 *     iteration runs floor(C_n / D_j) times per cycle, which stretches its
 *     iteration to d_j = C_n / floor(C_n / D_j);
 *   - the assignment heuristic (Pseudocode 1): an Aggregator qualifies for a new
 *     task of job k if no job on it, nor k, would lose LossLimit or more of its
 *     speed ((d_j - D_j) / d_j >= LossLimit disqualifies); among the qualified,
 *     the one with the least free time per cycle that still holds the task's
 *     execution time e_t wins (ties: lowest id); otherwise a new Aggregator is
 *     allocated;
 *   - late requests ("Handling Outliers in Cyclic Execution");
 *   - scaling on job exit (Section 3.3.2): empty Aggregators are released, then
 *     the least-loaded ones are drained into the others without allocating;
 *   - best-fit choice of an Aggregator cluster (Section 3.3.3).
 * An "Aggregator" here is a logical destination of waves (a GPU, or a share of
 * one); a "task" is one model aggregation per iteration (a tensor or a block)
 * with execution time e_t, e.g. the measured kernel time of its block.
 *
 * All functions return PS_OK (0) or a negative PS_ERR_* of ps.h unless stated.
 * A scheduler object is not thread-safe; guard it externally.
 */
#ifndef PS_SCHED_H_
#define PS_SCHED_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PS_SCHED_DEFAULT_LOSS_LIMIT 0.1

typedef struct ps_sched ps_sched;

typedef struct ps_sched_agg_stats {
  double cycle;      /* C_n (0 if it holds no task) */
  double busy;       /* W_n: aggregation time within one cycle */
  double free_time;  /* C_n - W_n */
  int32_t n_jobs;
  int32_t n_tasks;
} ps_sched_agg_stats;

typedef struct ps_sched_job_stats {
  double D;          /* profiled iteration duration */
  double d;          /* current iteration duration: the slowest of its Aggregators */
  double loss;       /* (d - D) / d */
  int32_t n_tasks;
  int32_t n_aggregators;
} ps_sched_job_stats;

typedef struct ps_sched_wave {
  int64_t num, den;  /* the wave starts num/den of the way through the cycle (reduced) */
  int32_t first;     /* its jobs are out_jobs[first .. first+count) in ascending id */
  int32_t count;
} ps_sched_wave;

/* loss_limit <= 0 selects the default 0.1; values >= 1 are PS_ERR_ARG. */
int32_t ps_sched_create(double loss_limit, ps_sched** out);
void ps_sched_destroy(ps_sched* s);

/* Register a job with profiled iteration duration D > 0 (any time unit, the
 * same for every D and e). */
int32_t ps_sched_add_job(ps_sched* s, double D, int32_t* out_job);

/* Pseudocode 1 for one new task of `job` with execution time e > 0.  Writes the
 * task id and the Aggregator chosen (possibly newly allocated). */
int32_t ps_sched_assign(ps_sched* s, int32_t job, double e, int32_t* out_task,
                        int32_t* out_aggregator);

/* The first half of Pseudocode 1 for one Aggregator: returns 1 and writes the
 * estimated cycle and free time if a task of `job` may go there, 0 if the loss
 * limit rules it out, negative on error. */
int32_t ps_sched_estimate(ps_sched* s, int32_t aggregator, int32_t job, double* out_cycle,
                          double* out_free);

/* Job exit.  Removes the job's tasks, releases empty Aggregators, then drains
 * least-loaded Aggregators (load = busy / cycle, ties to the highest id) into the
 * others, largest task first, without allocating, until one cannot be drained.
 * Writes the released ids in order (at most cap; *out_n is the full count). */
int32_t ps_sched_remove_job(ps_sched* s, int32_t job, int32_t* out_released, int32_t cap,
                            int32_t* out_n);

/* Scaling up on arrival (Section 3.3.2): the caller has measured that `job` runs
 * slower than standalone.  Allocates one more Aggregator and assigns the whole
 * job again (its tasks in id order, Pseudocode 1 each) with the new one among
 * the destinations; Aggregators left empty are released.  Repeat while the
 * measured loss stays above the limit.  Writes the new Aggregator's id (which
 * is released again if no task landed there). */
int32_t ps_sched_scale_up_job(ps_sched* s, int32_t job, int32_t* out_new_aggregator);

int32_t ps_sched_aggregator_info(ps_sched* s, int32_t aggregator, ps_sched_agg_stats* out);
int32_t ps_sched_job_info(ps_sched* s, int32_t job, ps_sched_job_stats* out);
int32_t ps_sched_task_info(ps_sched* s, int32_t task, int32_t* out_aggregator, int32_t* out_job,
                           double* out_e);

/* Ids of the live Aggregators in ascending order (at most cap; *out_n = count). */
int32_t ps_sched_aggregators(ps_sched* s, int32_t* out_ids, int32_t cap, int32_t* out_n);

/* The waves of one cycle of an Aggregator, in order of start: a job that runs r
 * times per cycle appears in the waves starting at 0, 1/r, ..., (r-1)/r of the
 * cycle.  PS_ERR_CAPACITY if an output array is too small (counts still set). */
int32_t ps_sched_cycle_plan(ps_sched* s, int32_t aggregator, ps_sched_wave* out_waves,
                            int32_t cap_waves, int32_t* out_n_waves, int32_t* out_jobs,
                            int32_t cap_jobs, int32_t* out_n_jobs);

/* Late request: 1 if it may still run in the current cycle (cycle - elapsed -
 * remaining_scheduled >= e_late), 0 if it waits for the next cycle. */
int32_t ps_sched_admit_late(double cycle, double elapsed, double remaining_scheduled, double e_late);

/* Index of the cluster with sufficient but least free time, -1 if none fits. */
int32_t ps_sched_best_fit_cluster(const double* free_time, int32_t n, double demand);

#ifdef __cplusplus
}
#endif
#endif /* PS_SCHED_H_ */
