// Assignment and scaling of model aggregations (host only): cyclic execution,
// the assignment heuristic, late requests, recycling on job exit, cluster best
// fit -- the paper's Section 3.3.  Jobs and tasks are kept in flat vectors; an
// Aggregator holds, per job in ascending id, that job's tasks in arrival order.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <map>
#include <new>
#include <numeric>
#include <vector>

#include "../../include/ps.h"
#include "../../include/ps_sched.h"

namespace {

struct Task {
  int32_t agg = -1;
  int32_t job = -1;
  double e = 0;
  bool live = false;
};

struct Agg {
  bool live = false;
  std::map<int32_t, std::vector<int32_t>> by_job;  // job -> task ids, arrival order
};

double stretched(double C, double D) { return std::max(D, C / std::floor(C / D)); }
double lost(double d, double D) { return (d - D) / d; }

}  // namespace

struct ps_sched {
  double limit = PS_SCHED_DEFAULT_LOSS_LIMIT;
  std::vector<double> D;        // per job; <= 0 once the job has left
  std::vector<Task> tasks;
  std::vector<Agg> aggs;
  std::map<int32_t, std::vector<int32_t>> own;  // job -> Aggregators added for it by scale-up, oldest first

  bool job_ok(int32_t j) const { return j >= 0 && (size_t)j < D.size() && D[j] > 0; }
  bool agg_ok(int32_t n) const { return n >= 0 && (size_t)n < aggs.size() && aggs[n].live; }

  double cycle(int32_t n) const {
    double c = 0.0;
    for (const auto& kv : aggs[n].by_job) c = std::max(c, D[kv.first]);
    return c;
  }
  double busy(int32_t n, double C) const {
    double total = 0.0;
    for (const auto& kv : aggs[n].by_job) {
      const double d = stretched(C, D[kv.first]);
      double sum = 0.0;
      for (int32_t t : kv.second) sum += tasks[t].e;
      total += std::floor(C / d) * sum;
    }
    return total;
  }
  // Pseudocode 1, first loop body.  Returns false if the loss limit rejects n.
  bool estimate(int32_t n, int32_t k, double* C_est, double* F_est) const {
    const double C = std::max(cycle(n), D[k]);
    bool k_seen = false;
    for (const auto& kv : aggs[n].by_job) {
      if (kv.first == k) k_seen = true;
      if (lost(stretched(C, D[kv.first]), D[kv.first]) >= limit) return false;
    }
    if (!k_seen && lost(stretched(C, D[k]), D[k]) >= limit) return false;
    *C_est = C;
    *F_est = C - busy(n, C);
    return true;
  }
  int32_t allocate() {
    aggs.emplace_back();
    aggs.back().live = true;
    return (int32_t)aggs.size() - 1;
  }
  // Best-fit destination, or -1.
  int32_t choose(int32_t k, double e, int32_t exclude) const {
    int32_t best = -1;
    double best_f = 0.0;
    for (int32_t n = 0; n < (int32_t)aggs.size(); ++n) {
      if (!aggs[n].live || n == exclude) continue;
      double C, F;
      if (!estimate(n, k, &C, &F)) continue;
      if (F >= e && (best < 0 || F < best_f)) { best = n; best_f = F; }
    }
    return best;
  }
  // Hand an Aggregator back; no job keeps it as one of its own.
  void release(int32_t n) {
    aggs[n].live = false;
    for (auto it = own.begin(); it != own.end();) {
      auto& v = it->second;
      v.erase(std::remove(v.begin(), v.end(), n), v.end());
      it = v.empty() ? own.erase(it) : std::next(it);
    }
  }
  int32_t choose_excluding(int32_t k, double e, const std::vector<int32_t>& skip) const {
    int32_t best = -1;
    double best_f = 0.0;
    for (int32_t n = 0; n < (int32_t)aggs.size(); ++n) {
      if (!aggs[n].live || std::find(skip.begin(), skip.end(), n) != skip.end()) continue;
      double C, F;
      if (!estimate(n, k, &C, &F)) continue;
      if (F >= e && (best < 0 || F < best_f)) { best = n; best_f = F; }
    }
    return best;
  }
  void place(int32_t n, int32_t t) {
    tasks[t].agg = n;
    aggs[n].by_job[tasks[t].job].push_back(t);
  }
  void unplace(int32_t t) {
    auto& a = aggs[tasks[t].agg];
    auto it = a.by_job.find(tasks[t].job);
    auto& v = it->second;
    v.erase(std::find(v.begin(), v.end(), t));
    if (v.empty()) a.by_job.erase(it);
  }
  bool drain(int32_t victim) {
    std::vector<int32_t> todo;
    for (const auto& kv : aggs[victim].by_job) todo.insert(todo.end(), kv.second.begin(), kv.second.end());
    std::sort(todo.begin(), todo.end(), [&](int32_t a, int32_t b) {
      if (tasks[a].e != tasks[b].e) return tasks[a].e > tasks[b].e;
      return a < b;
    });
    // tasks stay listed on the victim while copies are tried elsewhere
    std::vector<int32_t> moved;
    for (int32_t t : todo) {
      const int32_t n = choose(tasks[t].job, tasks[t].e, victim);
      if (n < 0) {
        for (int32_t m : moved) {  // roll back
          auto& a = aggs[tasks[m].agg];
          auto it = a.by_job.find(tasks[m].job);
          it->second.erase(std::find(it->second.begin(), it->second.end(), m));
          if (it->second.empty()) a.by_job.erase(it);
          tasks[m].agg = victim;
        }
        return false;
      }
      aggs[n].by_job[tasks[t].job].push_back(t);
      tasks[t].agg = n;
      moved.push_back(t);
    }
    aggs[victim].by_job.clear();
    return true;
  }
};

// No C++ exception leaves the library; see the same macro in ps_service.cpp.
#define PS_NO_THROW catch (...) { return PS_ERR_NOMEM; }

extern "C" {

int32_t ps_sched_create(double loss_limit, ps_sched** out) try {
  if (!out) return PS_ERR_ARG;
  *out = nullptr;
  if (!(loss_limit < 1.0)) return PS_ERR_ARG;
  ps_sched* s = new (std::nothrow) ps_sched();
  if (!s) return PS_ERR_NOMEM;
  if (loss_limit > 0) s->limit = loss_limit;
  *out = s;
  return PS_OK;
} PS_NO_THROW

void ps_sched_destroy(ps_sched* s) { delete s; }

int32_t ps_sched_add_job(ps_sched* s, double D, int32_t* out_job) try {
  if (!s || !out_job || !(D > 0) || !std::isfinite(D)) return PS_ERR_ARG;
  s->D.push_back(D);
  *out_job = (int32_t)s->D.size() - 1;
  return PS_OK;
} PS_NO_THROW

int32_t ps_sched_assign(ps_sched* s, int32_t job, double e, int32_t* out_task, int32_t* out_aggregator) try {
  if (!s || !(e > 0) || !std::isfinite(e)) return PS_ERR_ARG;
  if (!s->job_ok(job)) return PS_ERR_BAD_JOB;
  int32_t n = s->choose(job, e, -1);
  if (n < 0) n = s->allocate();
  Task t;
  t.job = job; t.e = e; t.live = true;
  s->tasks.push_back(t);
  const int32_t id = (int32_t)s->tasks.size() - 1;
  s->place(n, id);
  if (out_task) *out_task = id;
  if (out_aggregator) *out_aggregator = n;
  return PS_OK;
} PS_NO_THROW

int32_t ps_sched_estimate(ps_sched* s, int32_t aggregator, int32_t job, double* out_cycle, double* out_free) try {
  if (!s) return PS_ERR_ARG;
  if (!s->job_ok(job)) return PS_ERR_BAD_JOB;
  if (!s->agg_ok(aggregator)) return PS_ERR_BAD_BLOCK;
  double C = 0, F = 0;
  if (!s->estimate(aggregator, job, &C, &F)) return 0;
  if (out_cycle) *out_cycle = C;
  if (out_free) *out_free = F;
  return 1;
} PS_NO_THROW

int32_t ps_sched_remove_job(ps_sched* s, int32_t job, int32_t* out_released, int32_t cap, int32_t* out_n) try {
  if (!s || cap < 0 || (cap > 0 && !out_released)) return PS_ERR_ARG;
  if (!s->job_ok(job)) return PS_ERR_BAD_JOB;
  std::vector<int32_t> released;
  for (auto& a : s->aggs) {
    if (!a.live) continue;
    auto it = a.by_job.find(job);
    if (it == a.by_job.end()) continue;
    for (int32_t t : it->second) s->tasks[t].live = false;
    a.by_job.erase(it);
  }
  s->D[job] = -1.0;
  s->own.erase(job);
  for (int32_t n = 0; n < (int32_t)s->aggs.size(); ++n)
    if (s->aggs[n].live && s->aggs[n].by_job.empty()) {
      s->release(n);
      released.push_back(n);
    }
  for (;;) {
    int32_t victim = -1, live = 0;
    double load = 0.0;
    for (int32_t n = 0; n < (int32_t)s->aggs.size(); ++n) {
      if (!s->aggs[n].live) continue;
      ++live;
      const double C = s->cycle(n);
      const double l = s->busy(n, C) / C;
      if (victim < 0 || l < load || (l == load && n > victim)) { victim = n; load = l; }
    }
    if (live <= 1 || !s->drain(victim)) break;
    s->release(victim);
    released.push_back(victim);
  }
  if (out_n) *out_n = (int32_t)released.size();
  for (int32_t i = 0; i < (int32_t)released.size() && i < cap; ++i) out_released[i] = released[i];
  return PS_OK;
} PS_NO_THROW

int32_t ps_sched_scale_up_job(ps_sched* s, int32_t job, int32_t* out_new_aggregator, int32_t* out_moved) try {
  if (!s) return PS_ERR_ARG;
  if (!s->job_ok(job)) return PS_ERR_BAD_JOB;
  std::vector<int32_t> mine, before;
  for (int32_t t = 0; t < (int32_t)s->tasks.size(); ++t)
    if (s->tasks[t].live && s->tasks[t].job == job) mine.push_back(t);
  for (int32_t t : mine) {
    before.push_back(s->tasks[t].agg);
    s->unplace(t);
  }
  const int32_t fresh = s->allocate();
  s->own[job].push_back(fresh);
  for (int32_t t : mine) {
    const double e = s->tasks[t].e;
    int32_t n = -1;
    // the Aggregators added for this job come first, oldest first
    for (int32_t cand : s->own[job]) {
      double C, F;
      if (s->estimate(cand, job, &C, &F) && F >= e) { n = cand; break; }
    }
    if (n < 0) n = s->choose_excluding(job, e, s->own[job]);
    if (n < 0) n = s->allocate();
    s->place(n, t);
  }
  for (int32_t n = 0; n < (int32_t)s->aggs.size(); ++n)
    if (s->aggs[n].live && s->aggs[n].by_job.empty()) s->release(n);
  int32_t moved = 0;
  for (size_t i = 0; i < mine.size(); ++i) moved += s->tasks[mine[i]].agg != before[i] ? 1 : 0;
  if (out_new_aggregator) *out_new_aggregator = fresh;
  if (out_moved) *out_moved = moved;
  return PS_OK;
} PS_NO_THROW

int32_t ps_sched_aggregator_info(ps_sched* s, int32_t aggregator, ps_sched_agg_stats* out) try {
  if (!s || !out) return PS_ERR_ARG;
  if (!s->agg_ok(aggregator)) return PS_ERR_BAD_BLOCK;
  const double C = s->cycle(aggregator);
  out->cycle = C;
  out->busy = C > 0 ? s->busy(aggregator, C) : 0.0;
  out->free_time = C - out->busy;
  out->n_jobs = (int32_t)s->aggs[aggregator].by_job.size();
  out->n_tasks = 0;
  for (const auto& kv : s->aggs[aggregator].by_job) out->n_tasks += (int32_t)kv.second.size();
  return PS_OK;
} PS_NO_THROW

int32_t ps_sched_job_info(ps_sched* s, int32_t job, ps_sched_job_stats* out) try {
  if (!s || !out) return PS_ERR_ARG;
  if (!s->job_ok(job)) return PS_ERR_BAD_JOB;
  const double D = s->D[job];
  double d = D;
  bool any = false;
  out->n_tasks = 0;
  out->n_aggregators = 0;
  for (int32_t n = 0; n < (int32_t)s->aggs.size(); ++n) {
    if (!s->aggs[n].live) continue;
    auto it = s->aggs[n].by_job.find(job);
    if (it == s->aggs[n].by_job.end()) continue;
    const double dn = stretched(s->cycle(n), D);
    d = any ? std::max(d, dn) : dn;
    any = true;
    out->n_tasks += (int32_t)it->second.size();
    out->n_aggregators += 1;
  }
  out->D = D;
  out->d = d;
  out->loss = lost(d, D);
  return PS_OK;
} PS_NO_THROW

int32_t ps_sched_task_info(ps_sched* s, int32_t task, int32_t* out_aggregator, int32_t* out_job, double* out_e) try {
  if (!s) return PS_ERR_ARG;
  if (task < 0 || (size_t)task >= s->tasks.size() || !s->tasks[task].live) return PS_ERR_BAD_BLOCK;
  if (out_aggregator) *out_aggregator = s->tasks[task].agg;
  if (out_job) *out_job = s->tasks[task].job;
  if (out_e) *out_e = s->tasks[task].e;
  return PS_OK;
} PS_NO_THROW

int32_t ps_sched_aggregators(ps_sched* s, int32_t* out_ids, int32_t cap, int32_t* out_n) try {
  if (!s || !out_n || cap < 0 || (cap > 0 && !out_ids)) return PS_ERR_ARG;
  int32_t k = 0;
  for (int32_t n = 0; n < (int32_t)s->aggs.size(); ++n)
    if (s->aggs[n].live) {
      if (k < cap) out_ids[k] = n;
      ++k;
    }
  *out_n = k;
  return k > cap ? PS_ERR_CAPACITY : PS_OK;
} PS_NO_THROW

int32_t ps_sched_cycle_plan(ps_sched* s, int32_t aggregator, ps_sched_wave* out_waves, int32_t cap_waves,
                            int32_t* out_n_waves, int32_t* out_jobs, int32_t cap_jobs, int32_t* out_n_jobs) try {
  if (!s || !out_n_waves || !out_n_jobs || cap_waves < 0 || cap_jobs < 0) return PS_ERR_ARG;
  if ((cap_waves > 0 && !out_waves) || (cap_jobs > 0 && !out_jobs)) return PS_ERR_ARG;
  if (!s->agg_ok(aggregator)) return PS_ERR_BAD_BLOCK;
  const double C = s->cycle(aggregator);
  // (num, den) reduced -> jobs; ordered by num/den through cross-multiplication
  struct Key {
    int64_t num, den;
    bool operator<(const Key& o) const { return (__int128)num * o.den < (__int128)o.num * den; }
  };
  std::map<Key, std::vector<int32_t>> at;
  for (const auto& kv : s->aggs[aggregator].by_job) {
    const int64_t r = (int64_t)std::floor(C / s->D[kv.first]);
    for (int64_t i = 0; i < r; ++i) {
      const int64_t g = std::gcd(i, r);
      at[Key{i / g, r / g}].push_back(kv.first);
    }
  }
  int32_t nw = 0, nj = 0;
  for (const auto& kv : at) {
    if (nw < cap_waves) {
      out_waves[nw].num = kv.first.num;
      out_waves[nw].den = kv.first.den;
      out_waves[nw].first = nj;
      out_waves[nw].count = (int32_t)kv.second.size();
    }
    for (int32_t j : kv.second) {
      if (nj < cap_jobs) out_jobs[nj] = j;
      ++nj;
    }
    ++nw;
  }
  *out_n_waves = nw;
  *out_n_jobs = nj;
  return (nw > cap_waves || nj > cap_jobs) ? PS_ERR_CAPACITY : PS_OK;
} PS_NO_THROW

int32_t ps_sched_admit_late(double cycle, double elapsed, double remaining_scheduled, double e_late) {
  return (cycle - elapsed) - remaining_scheduled >= e_late ? 1 : 0;
}

int32_t ps_sched_best_fit_cluster(const double* free_time, int32_t n, double demand) {
  if (!free_time || n <= 0) return -1;
  int32_t best = -1;
  for (int32_t i = 0; i < n; ++i)
    if (free_time[i] >= demand && (best < 0 || free_time[i] < free_time[best])) best = i;
  return best;
}

}  // extern "C"
