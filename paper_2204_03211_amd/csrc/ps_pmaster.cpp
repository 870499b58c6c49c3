// Aggregator clusters (host only): the paper's Section 3.3.3.  pMaster keeps
// the remaining free resource of every cluster and forwards a new job to the
// best-fit one by the job's total demand; the cluster's controller -- one
// ps_sched per cluster, reached through its own C entry points -- assigns the
// job's tasks among the cluster's Aggregators; a job takes resource from one
// cluster; an exit is reported back and returns the job's demand to the
// cluster's book.
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "../../include/ps.h"
#include "../../include/ps_sched.h"

namespace {

struct PmJob {
  int32_t cluster = -1;
  int32_t local = -1;   // the job's id inside its cluster's controller
  double demand = 0.0;  // sum of its tasks' execution times per unit of time, in Aggregators
  bool live = false;
};

}  // namespace

struct ps_pmaster {
  double limit = PS_SCHED_DEFAULT_LOSS_LIMIT;
  std::vector<double> capacity;
  std::vector<ps_sched*> controller;
  std::vector<PmJob> jobs;

  bool cluster_ok(int32_t c) const { return c >= 0 && (size_t)c < capacity.size(); }
  bool job_ok(int32_t j) const { return j >= 0 && (size_t)j < jobs.size() && jobs[j].live; }
  // pMaster's own book: demands of the jobs forwarded to c, added in job order
  double used(int32_t c) const {
    double total = 0.0;
    for (const PmJob& j : jobs)
      if (j.live && j.cluster == c) total += j.demand;
    return total;
  }
};

#define PS_NO_THROW catch (...) { return PS_ERR_NOMEM; }

extern "C" {

int32_t ps_pmaster_create(double loss_limit, ps_pmaster** out) try {
  if (!out) return PS_ERR_ARG;
  *out = nullptr;
  if (!(loss_limit < 1.0)) return PS_ERR_ARG;
  ps_pmaster* m = new (std::nothrow) ps_pmaster();
  if (!m) return PS_ERR_NOMEM;
  if (loss_limit > 0) m->limit = loss_limit;
  *out = m;
  return PS_OK;
} PS_NO_THROW

void ps_pmaster_destroy(ps_pmaster* m) {
  if (!m) return;
  for (ps_sched* s : m->controller) ps_sched_destroy(s);
  delete m;
}

int32_t ps_pmaster_add_cluster(ps_pmaster* m, double capacity, int32_t* out_cluster) try {
  if (!m || !(capacity > 0) || !std::isfinite(capacity)) return PS_ERR_ARG;
  // room in both lists first, so that neither can be left one entry ahead of the other
  m->controller.reserve(m->controller.size() + 1);
  m->capacity.reserve(m->capacity.size() + 1);
  ps_sched* s = nullptr;
  const int32_t st = ps_sched_create(m->limit, &s);
  if (st != PS_OK) return st;
  m->controller.push_back(s);
  m->capacity.push_back(capacity);
  if (out_cluster) *out_cluster = (int32_t)m->capacity.size() - 1;
  return PS_OK;
} PS_NO_THROW

int32_t ps_pmaster_n_clusters(ps_pmaster* m) { return m ? (int32_t)m->capacity.size() : PS_ERR_ARG; }

int32_t ps_pmaster_forward_job(ps_pmaster* m, double D, const double* e, int32_t n_tasks, int32_t* out_job,
                               int32_t* out_cluster, int32_t* out_tasks, int32_t* out_aggregators) try {
  if (!m || !e || n_tasks < 1 || !(D > 0) || !std::isfinite(D)) return PS_ERR_ARG;
  double total = 0.0;
  for (int32_t i = 0; i < n_tasks; ++i) {
    if (!(e[i] > 0) || !std::isfinite(e[i])) return PS_ERR_ARG;
    total += e[i];
  }
  const double need = total / D;
  std::vector<double> free_now(m->capacity.size());
  for (size_t c = 0; c < free_now.size(); ++c) free_now[c] = m->capacity[c] - m->used((int32_t)c);
  const int32_t c = ps_sched_best_fit_cluster(free_now.data(), (int32_t)free_now.size(), need);
  if (c < 0) return PS_ERR_NO_ROOM;
  m->jobs.reserve(m->jobs.size() + 1);  // nothing below may fail half-way
  ps_sched* ctl = m->controller[c];
  int32_t local = -1;
  int32_t st = ps_sched_add_job(ctl, D, &local);
  if (st != PS_OK) return st;
  for (int32_t i = 0; i < n_tasks; ++i) {
    int32_t t = -1, n = -1;
    st = ps_sched_assign(ctl, local, e[i], &t, &n);
    if (st != PS_OK) {  // out of host memory inside the controller: take the job out again
      int32_t dummy = 0;
      (void)ps_sched_remove_job(ctl, local, nullptr, 0, &dummy);
      return st;
    }
    if (out_tasks) out_tasks[i] = t;
    if (out_aggregators) out_aggregators[i] = n;
  }
  PmJob j;
  j.cluster = c; j.local = local; j.demand = need; j.live = true;
  m->jobs.push_back(j);
  if (out_job) *out_job = (int32_t)m->jobs.size() - 1;
  if (out_cluster) *out_cluster = c;
  return PS_OK;
} PS_NO_THROW

int32_t ps_pmaster_job_exit(ps_pmaster* m, int32_t job, int32_t* out_cluster, int32_t* out_released,
                            int32_t cap, int32_t* out_n) try {
  if (!m || cap < 0 || (cap > 0 && !out_released)) return PS_ERR_ARG;
  if (!m->job_ok(job)) return PS_ERR_BAD_JOB;
  PmJob& j = m->jobs[job];
  const int32_t st = ps_sched_remove_job(m->controller[j.cluster], j.local, out_released, cap, out_n);
  if (st != PS_OK) return st;
  if (out_cluster) *out_cluster = j.cluster;
  j.live = false;  // the report: the cluster's book gets the demand back
  return PS_OK;
} PS_NO_THROW

int32_t ps_pmaster_scale_up_job(ps_pmaster* m, int32_t job, int32_t* out_new_aggregator, int32_t* out_moved) try {
  if (!m) return PS_ERR_ARG;
  if (!m->job_ok(job)) return PS_ERR_BAD_JOB;
  const PmJob& j = m->jobs[job];
  return ps_sched_scale_up_job(m->controller[j.cluster], j.local, out_new_aggregator, out_moved);
} PS_NO_THROW

int32_t ps_pmaster_cluster_info(ps_pmaster* m, int32_t cluster, ps_pmaster_cluster_stats* out) try {
  if (!m || !out) return PS_ERR_ARG;
  if (!m->cluster_ok(cluster)) return PS_ERR_BAD_BLOCK;
  out->capacity = m->capacity[cluster];
  out->used = m->used(cluster);
  out->free_resource = out->capacity - out->used;
  out->n_jobs = 0;
  for (const PmJob& j : m->jobs) out->n_jobs += (j.live && j.cluster == cluster) ? 1 : 0;
  out->n_aggregators = 0;
  (void)ps_sched_aggregators(m->controller[cluster], nullptr, 0, &out->n_aggregators);  // count only
  return PS_OK;
} PS_NO_THROW

int32_t ps_pmaster_job_info(ps_pmaster* m, int32_t job, int32_t* out_cluster, int32_t* out_local_job,
                            double* out_demand) try {
  if (!m) return PS_ERR_ARG;
  if (!m->job_ok(job)) return PS_ERR_BAD_JOB;
  if (out_cluster) *out_cluster = m->jobs[job].cluster;
  if (out_local_job) *out_local_job = m->jobs[job].local;
  if (out_demand) *out_demand = m->jobs[job].demand;
  return PS_OK;
} PS_NO_THROW

ps_sched* ps_pmaster_controller(ps_pmaster* m, int32_t cluster) {
  return (m && m->cluster_ok(cluster)) ? m->controller[cluster] : nullptr;
}

}  // extern "C"
