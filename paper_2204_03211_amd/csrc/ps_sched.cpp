// Assignment and scaling of model aggregations (host only): cyclic execution,
// the assignment heuristic, late requests, recycling on job exit, scaling up on
// arrival -- the paper's Section 3.3.
//
// Bookkeeping.  Every Aggregator keeps a ledger: per job it serves (ascending
// id), that job's tasks in arrival order and the running sum of their execution
// times, plus the Aggregator's cycle (the largest profiled iteration among its
// jobs).  An estimate for a new task then costs one pass over the jobs of an
// Aggregator, not over its tasks: a job brings thousands of tasks, an
// Aggregator serves a handful of jobs.  Sums are always formed left to right
// in arrival order (a removal recomputes the job's sum from its remaining
// tasks), so every figure is reproducible to the last bit.
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

// One job's share of one Aggregator.
struct Share {
  std::vector<int32_t> tasks;  // arrival order
  double e_sum = 0.0;          // their execution times added in that order
};

struct Ledger {
  bool live = false;
  std::map<int32_t, Share> share;  // job -> its share, ascending job id
  double cycle = 0.0;              // C_n: max profiled iteration of the jobs here, 0 if none
};

// d_j of a job with profiled iteration D under cycle C, and the loss that goes with it
inline double runs_per_cycle(double C, double D) { return std::floor(C / D); }
inline double iteration_under(double C, double D) { return std::max(D, C / runs_per_cycle(C, D)); }
inline double speed_loss(double d, double D) { return (d - D) / d; }

}  // namespace

struct ps_sched {
  double limit = PS_SCHED_DEFAULT_LOSS_LIMIT;
  std::vector<double> D;        // per job; <= 0 once the job has left
  std::vector<Task> tasks;
  std::vector<Ledger> aggs;
  std::map<int32_t, std::vector<int32_t>> own;  // job -> Aggregators added for it by scale-up, oldest first

  bool job_ok(int32_t j) const { return j >= 0 && (size_t)j < D.size() && D[j] > 0; }
  bool agg_ok(int32_t n) const { return n >= 0 && (size_t)n < aggs.size() && aggs[n].live; }
  bool empty(int32_t n) const { return aggs[n].share.empty(); }
  double cycle(int32_t n) const { return aggs[n].cycle; }

  // --- ledger operations ---------------------------------------------------
  void ledger_add(int32_t n, int32_t t) {
    Ledger& a = aggs[n];
    Share& sh = a.share[tasks[t].job];
    sh.tasks.push_back(t);
    sh.e_sum += tasks[t].e;
    a.cycle = std::max(a.cycle, D[tasks[t].job]);
  }
  void ledger_remove(int32_t n, int32_t t) {
    Ledger& a = aggs[n];
    auto it = a.share.find(tasks[t].job);
    Share& sh = it->second;
    sh.tasks.erase(std::find(sh.tasks.begin(), sh.tasks.end(), t));
    if (sh.tasks.empty()) {
      a.share.erase(it);
      a.cycle = 0.0;
      for (const auto& kv : a.share) a.cycle = std::max(a.cycle, D[kv.first]);
    } else {
      sh.e_sum = 0.0;
      for (int32_t q : sh.tasks) sh.e_sum += tasks[q].e;
    }
  }
  void ledger_drop_job(int32_t n, int32_t job) {
    Ledger& a = aggs[n];
    a.share.erase(job);
    a.cycle = 0.0;
    for (const auto& kv : a.share) a.cycle = std::max(a.cycle, D[kv.first]);
  }

  // W_n: aggregation time within one cycle of length C
  double busy(int32_t n, double C) const {
    double total = 0.0;
    for (const auto& kv : aggs[n].share)
      total += runs_per_cycle(C, iteration_under(C, D[kv.first])) * kv.second.e_sum;
    return total;
  }

  // The first half of the assignment scheme for one Aggregator and a task of
  // job k: the cycle if k joined, whether anybody (k included) would lose the
  // limit or more, and the free time left.
  bool estimate(int32_t n, int32_t k, double* C_est, double* F_est) const {
    const Ledger& a = aggs[n];
    const double C = std::max(a.cycle, D[k]);
    for (const auto& kv : a.share)
      if (speed_loss(iteration_under(C, D[kv.first]), D[kv.first]) >= limit) return false;
    if (!a.share.count(k) && speed_loss(iteration_under(C, D[k]), D[k]) >= limit) return false;
    *C_est = C;
    *F_est = C - busy(n, C);
    return true;
  }

  int32_t allocate() {
    aggs.emplace_back();
    aggs.back().live = true;
    return (int32_t)aggs.size() - 1;
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

  // The second half: among the live Aggregators not in `skip` that qualify and
  // have room for e, the one with the least free time (first such id on ties);
  // -1 if none.
  int32_t best_fit(int32_t k, double e, const int32_t* skip, size_t n_skip) const {
    int32_t best = -1;
    double best_f = 0.0;
    for (int32_t n = 0; n < (int32_t)aggs.size(); ++n) {
      if (!aggs[n].live || std::find(skip, skip + n_skip, n) != skip + n_skip) continue;
      double C, F;
      if (!estimate(n, k, &C, &F) || F < e) continue;
      if (best < 0 || F < best_f) { best = n; best_f = F; }
    }
    return best;
  }

  void place(int32_t n, int32_t t) {
    tasks[t].agg = n;
    ledger_add(n, t);
  }
  void unplace(int32_t t) { ledger_remove(tasks[t].agg, t); }

  // Recycling: every task of the victim must find room elsewhere, largest
  // first, with no allocation.  The victim's own ledger is left as it is while
  // destinations are tried (it is not a destination), so a failed attempt only
  // has to take the tentative entries out of the destinations again.
  bool drain(int32_t victim) {
    std::vector<int32_t> todo;
    for (const auto& kv : aggs[victim].share) todo.insert(todo.end(), kv.second.tasks.begin(), kv.second.tasks.end());
    std::sort(todo.begin(), todo.end(), [&](int32_t a, int32_t b) {
      if (tasks[a].e != tasks[b].e) return tasks[a].e > tasks[b].e;
      return a < b;
    });
    std::vector<int32_t> tentative;
    for (int32_t t : todo) {
      const int32_t n = best_fit(tasks[t].job, tasks[t].e, &victim, 1);
      if (n < 0) {
        for (int32_t m : tentative) {
          ledger_remove(tasks[m].agg, m);
          tasks[m].agg = victim;
        }
        return false;
      }
      ledger_add(n, t);
      tasks[t].agg = n;
      tentative.push_back(t);
    }
    aggs[victim].share.clear();
    aggs[victim].cycle = 0.0;
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
  int32_t n = s->best_fit(job, e, nullptr, 0);
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
  for (int32_t n = 0; n < (int32_t)s->aggs.size(); ++n) {
    if (!s->aggs[n].live) continue;
    auto it = s->aggs[n].share.find(job);
    if (it == s->aggs[n].share.end()) continue;
    for (int32_t t : it->second.tasks) s->tasks[t].live = false;
    s->ledger_drop_job(n, job);
  }
  s->D[job] = -1.0;
  s->own.erase(job);
  for (int32_t n = 0; n < (int32_t)s->aggs.size(); ++n)
    if (s->aggs[n].live && s->empty(n)) {
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
    if (n < 0) n = s->best_fit(job, e, s->own[job].data(), s->own[job].size());
    if (n < 0) n = s->allocate();
    s->place(n, t);
  }
  for (int32_t n = 0; n < (int32_t)s->aggs.size(); ++n)
    if (s->aggs[n].live && s->empty(n)) s->release(n);
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
  out->n_jobs = (int32_t)s->aggs[aggregator].share.size();
  out->n_tasks = 0;
  for (const auto& kv : s->aggs[aggregator].share) out->n_tasks += (int32_t)kv.second.tasks.size();
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
    auto it = s->aggs[n].share.find(job);
    if (it == s->aggs[n].share.end()) continue;
    const double dn = iteration_under(s->cycle(n), D);
    d = any ? std::max(d, dn) : dn;
    any = true;
    out->n_tasks += (int32_t)it->second.tasks.size();
    out->n_aggregators += 1;
  }
  out->D = D;
  out->d = d;
  out->loss = speed_loss(d, D);
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
  for (const auto& kv : s->aggs[aggregator].share) {
    const double runs = std::floor(C / s->D[kv.first]);
    if (runs > 65536.0) return PS_ERR_ARG;  // iterations that far apart do not share a cycle plan
    const int64_t r = (int64_t)runs;
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
