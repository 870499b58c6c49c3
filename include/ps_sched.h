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
 *   - scaling on job arrival (Section 3.3.2): a job measured slow gets one more
 *     Aggregator and is assigned again;
 *   - Aggregator clusters (Section 3.3.3): pMaster forwards a job to the best-fit
 *     cluster, whose controller assigns it (ps_pmaster_*, at the end).
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

/* Scaling up on arrival (Section 3.3.2: a new job that runs slower than alone
 * gets one more Aggregator and is assigned again as a whole, repeatedly, until
 * its loss is within the limit).  The caller has measured that `job` is slow.
 * Allocates one more Aggregator for the job and assigns all its tasks again in
 * id order.  The Aggregators added for this job -- by earlier calls and by this
 * one -- are offered first, oldest first: a task goes to the first of them that
 * passes the loss test and has free time >= e; a task none of them holds goes
 * through Pseudocode 1 over the other Aggregators.  (Plain best fit over all
 * Aggregators would put every task back where it was: it never prefers the
 * emptiest destination.)  Tasks of other jobs do not move; Aggregators left
 * empty are released.  Writes the new Aggregator's id (released again if no
 * task landed there) and the number of the job's tasks whose Aggregator
 * changed.  Repeat while the measured loss stays above the limit and that
 * number is not 0; at 0 the job sits on Aggregators of its own. */
int32_t ps_sched_scale_up_job(ps_sched* s, int32_t job, int32_t* out_new_aggregator, int32_t* out_moved);

int32_t ps_sched_aggregator_info(ps_sched* s, int32_t aggregator, ps_sched_agg_stats* out);
int32_t ps_sched_job_info(ps_sched* s, int32_t job, ps_sched_job_stats* out);
int32_t ps_sched_task_info(ps_sched* s, int32_t task, int32_t* out_aggregator, int32_t* out_job,
                           double* out_e);

/* Ids of the live Aggregators in ascending order (at most cap; *out_n = count). */
int32_t ps_sched_aggregators(ps_sched* s, int32_t* out_ids, int32_t cap, int32_t* out_n);

/* The waves of one cycle of an Aggregator, in order of start: a job that runs r
 * times per cycle appears in the waves starting at 0, 1/r, ..., (r-1)/r of the
 * cycle.  PS_ERR_CAPACITY if an output array is too small (counts still set);
 * PS_ERR_ARG if a job would run more than 65536 times per cycle. */
int32_t ps_sched_cycle_plan(ps_sched* s, int32_t aggregator, ps_sched_wave* out_waves,
                            int32_t cap_waves, int32_t* out_n_waves, int32_t* out_jobs,
                            int32_t cap_jobs, int32_t* out_n_jobs);

/* Late request: 1 if it may still run in the current cycle (cycle - elapsed -
 * remaining_scheduled >= e_late), 0 if it waits for the next cycle. */
int32_t ps_sched_admit_late(double cycle, double elapsed, double remaining_scheduled, double e_late);

/* Index of the cluster with sufficient but least free resource (ties: the
 * lowest index), -1 if none fits. */
int32_t ps_sched_best_fit_cluster(const double* free_resource, int32_t n, double demand);

/* --- Aggregator clusters (Section 3.3.3) ------------------------------------
 * The pool of Aggregators is split into independent clusters.  Each cluster has
 * a controller that assigns model aggregations among its own Aggregators only
 * (a ps_sched; Aggregator, job and task ids are local to the cluster).  pMaster
 * keeps each cluster's remaining free resource and places a new job in two
 * steps: it forwards the job to the best-fit cluster -- sufficient but least
 * free resource for the job's total demand -- and that cluster's controller
 * then runs Pseudocode 1 for every task of the job, so a job takes resource
 * from one cluster.  When a job exits, the controller removes it (releasing and
 * recycling Aggregators inside the cluster) and the exit is reported to
 * pMaster, whose book gets the job's demand back.
 *
 * The book is kept in units of Aggregators from profiled job information only:
 * a cluster of capacity M offers M; a job with iteration duration D and task
 * execution times e_t consumes sum(e_t) / D; free = M - sum of the demands of
 * the jobs forwarded there.  Not thread-safe; guard externally. */
typedef struct ps_pmaster ps_pmaster;

typedef struct ps_pmaster_cluster_stats {
  double capacity;       /* Aggregators the cluster offers */
  double used;           /* sum of the demands of its jobs */
  double free_resource;  /* capacity - used */
  int32_t n_jobs;
  int32_t n_aggregators; /* Aggregators its controller has allocated right now */
} ps_pmaster_cluster_stats;

/* loss_limit as for ps_sched_create; every controller uses it. */
int32_t ps_pmaster_create(double loss_limit, ps_pmaster** out);
/* Destroys the controllers too.  NULL is allowed. */
void ps_pmaster_destroy(ps_pmaster* m);

/* Add a cluster offering `capacity` (> 0) Aggregators' worth of resource. */
int32_t ps_pmaster_add_cluster(ps_pmaster* m, double capacity, int32_t* out_cluster);
int32_t ps_pmaster_n_clusters(ps_pmaster* m);

/* Job arrival.  D: profiled iteration duration; e: host array of the n_tasks
 * (>= 1) execution times, all > 0, in the order the tasks are to be assigned.
 * Chooses the cluster, registers the job with its controller and assigns every
 * task there.  Writes pMaster's job id, the cluster, and per task the
 * controller's task id and the Aggregator chosen (out_tasks / out_aggregators:
 * host arrays of n_tasks, either may be NULL).  PS_ERR_NO_ROOM if no cluster
 * has free resource >= sum(e)/D: nothing is registered (adding clusters or
 * capacity is the periodic scaling policy's business, not this call's). */
int32_t ps_pmaster_forward_job(ps_pmaster* m, double D, const double* e, int32_t n_tasks,
                               int32_t* out_job, int32_t* out_cluster, int32_t* out_tasks,
                               int32_t* out_aggregators);

/* Job exit: ps_sched_remove_job in the job's cluster (out_released, cap, out_n
 * as there, ids local to the cluster), then the report: pMaster forgets the job
 * and the cluster's free resource grows by its demand. */
int32_t ps_pmaster_job_exit(ps_pmaster* m, int32_t job, int32_t* out_cluster, int32_t* out_released,
                            int32_t cap, int32_t* out_n);

/* ps_sched_scale_up_job inside the job's cluster.  The job's demand, and with
 * it pMaster's book, does not change. */
int32_t ps_pmaster_scale_up_job(ps_pmaster* m, int32_t job, int32_t* out_new_aggregator,
                                int32_t* out_moved);

int32_t ps_pmaster_cluster_info(ps_pmaster* m, int32_t cluster, ps_pmaster_cluster_stats* out);
/* The job's cluster, its id inside that cluster's controller, and its demand. */
int32_t ps_pmaster_job_info(ps_pmaster* m, int32_t job, int32_t* out_cluster, int32_t* out_local_job,
                            double* out_demand);

/* The cluster's controller, borrowed (NULL if there is no such cluster): for
 * the inspection calls above (ps_sched_task_info, ps_sched_aggregators,
 * ps_sched_cycle_plan, ...).  Changing it directly (assign, remove, add_job)
 * leaves pMaster's book out of step. */
ps_sched* ps_pmaster_controller(ps_pmaster* m, int32_t cluster);

#ifdef __cplusplus
}
#endif
#endif /* PS_SCHED_H_ */
