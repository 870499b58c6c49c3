// Host-only exercise of the service's planning paths and of the scheduler, built
// with AddressSanitizer and UBSan by tests/test_native_sanitizers.py.  No device
// is touched: contexts are planning contexts (no arena), and the two functions
// that live in the kernel file are stubbed here.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <random>
#include <thread>
#include <vector>

#include "../../include/ps.h"
#include "../../include/ps_sched.h"
#include "../../paper_2204_03211_amd/csrc/ps_internal.h"

int ps_launch_wave(const PsWaveTables&, void*, uint32_t* launched) { *launched = 0; return 0; }
int ps_static_scratch(PsStaticScratch** out) { *out = nullptr; return 1; }
void ps_static_scratch_lock(PsStaticScratch*) {}
void ps_static_scratch_unlock(PsStaticScratch*) {}
int ps_launch_zero(float*, uint64_t, void*) { return 0; }
int ps_launch_copy(const float*, float*, const float*, float*, uint64_t, void*, uint32_t, double, uint32_t) { return 0; }
uint32_t ps_resident_copy_workgroups() { return 2048; }
uint32_t ps_resident_workgroups(uint32_t) { return 2048; }

#define CHECK(x) do { if (!(x)) { std::printf("CHECK failed: %s (line %d)\n", #x, __LINE__); std::exit(1); } } while (0)

static void service_rounds(uint64_t seed) {
  std::mt19937_64 rng(seed);
  ps_config cfg{};
  cfg.max_block_bytes = (uint64_t)(1 + rng() % 64) * 256;
  cfg.small_block_elems = (uint32_t)(rng() % 4097);
  ps_ctx* ctx = nullptr;
  CHECK(ps_create(&cfg, &ctx) == PS_OK);
  std::vector<ps_job_t> jobs;
  std::vector<int32_t> Ws;
  const int n_jobs = 1 + (int)(rng() % 5);
  for (int j = 0; j < n_jobs; ++j) {
    std::vector<int64_t> layers(1 + rng() % 6);
    for (auto& n : layers) n = 1 + (int64_t)(rng() % 20000);
    const int32_t W = 1 + (int32_t)(rng() % 32);
    ps_job_t job = -1;
    int32_t nb = 0;
    CHECK(ps_register_job(ctx, layers.data(), (int32_t)layers.size(), W, 0.1f, 0.9f, 1e-4f, nullptr,
                          nullptr, &job, &nb) == PS_OK);
    CHECK(nb == ps_job_n_blocks(ctx, job));
    jobs.push_back(job);
    Ws.push_back(W);
  }
  int64_t need = 0;
  CHECK(ps_pack_wave(ctx, jobs.data(), n_jobs, nullptr, 0, &need) == (need ? PS_ERR_CAPACITY : PS_OK));
  std::vector<ps_block_ref> wave((size_t)need);
  CHECK(ps_pack_wave(ctx, jobs.data(), n_jobs, wave.data(), need, &need) == PS_OK);
  const float* fake = reinterpret_cast<const float*>(uintptr_t(1) << 20);
  for (int j = 0; j < n_jobs; ++j)
    for (int32_t w = 0; w < Ws[j]; ++w) {
      if (rng() % 7 == 0 && w == Ws[j] - 1) continue;  // leave a job incomplete now and then
      CHECK(ps_push_flat(ctx, jobs[j], w, fake) == PS_OK);
    }
  std::vector<ps_block_ref> ready((size_t)need), late((size_t)need);
  int64_t nr = 0, nl = 0;
  CHECK(ps_split_ready(ctx, wave.data(), need, ready.data(), &nr, late.data(), &nl) == PS_OK);
  CHECK(nr + nl == need);
  ps_wave_stats st{};
  CHECK(ps_plan_wave(ctx, ready.data(), nr, &st) == PS_OK);
  CHECK(st.n_blocks == nr);
  if (nl) CHECK(ps_plan_wave(ctx, wave.data(), need, &st) == PS_ERR_NOT_READY);
  CHECK(ps_aggregate(ctx, ready.data(), nr, nullptr) == (nr ? PS_ERR_NO_DEVICE : PS_OK));
  // shuffled and truncated lists, duplicates, bad ids
  for (int k = 0; k < 4 && nr > 1; ++k) {
    std::vector<ps_block_ref> l(ready.begin(), ready.begin() + nr);
    std::shuffle(l.begin(), l.end(), rng);
    l.resize(1 + rng() % l.size());
    CHECK(ps_plan_wave(ctx, l.data(), (int64_t)l.size(), &st) == PS_OK);
    l.push_back(l[0]);
    CHECK(ps_plan_wave(ctx, l.data(), (int64_t)l.size(), &st) == PS_ERR_DUP_BLOCK);
    l.back().block = 1 << 30;
    CHECK(ps_plan_wave(ctx, l.data(), (int64_t)l.size(), &st) == PS_ERR_BAD_BLOCK);
  }
  // migration bookkeeping against a second planning context (stops at the device)
  {
    ps_ctx* other = nullptr;
    CHECK(ps_create(&cfg, &other) == PS_OK);
    std::vector<int64_t> layers = {5000, 7, 300};
    ps_job_t a = -1, b = -1;
    int32_t nb = 0, nb2 = 0;
    CHECK(ps_register_job(ctx, layers.data(), 3, 2, 0.1f, 0.9f, 0.0f, nullptr, nullptr, &a, &nb) == PS_OK);
    CHECK(ps_register_shadow_job(other, layers.data(), 3, 2, 0.1f, 0.9f, 0.0f, nullptr, &b, &nb2) == PS_OK);
    CHECK(nb == nb2 && nb >= 3);
    std::vector<int32_t> ids((size_t)nb);
    for (int32_t i = 0; i < nb; ++i) ids[(size_t)i] = i;
    std::shuffle(ids.begin(), ids.end(), rng);
    CHECK(ps_migrate_begin(ctx, a, ids[0]) == PS_OK);
    CHECK(ps_migrate_begin(ctx, a, ids[0]) == PS_ERR_NOT_OWNER);
    CHECK(ps_migrate_many(ctx, a, ids.data(), nb, other, b, nullptr) == PS_ERR_NO_DEVICE);
    CHECK(ps_migrate_copy(ctx, a, ids[0], other, b, nullptr) == PS_ERR_NO_DEVICE);
    CHECK(ps_migrate_cancel(ctx, a, ids[0]) == PS_OK);
    ids.push_back(ids[1]);
    CHECK(ps_migrate_many(ctx, a, ids.data(), nb + 1, other, b, nullptr) == PS_ERR_DUP_BLOCK);
    CHECK(ps_push(ctx, a, ids[2], 1, reinterpret_cast<const float*>(uintptr_t(1) << 20)) == PS_OK);
    CHECK(ps_migrate_many(ctx, a, ids.data(), nb, other, b, nullptr) == PS_ERR_BUSY);
    CHECK(ps_migrate_many(other, b, ids.data(), 1, ctx, a, nullptr) == PS_ERR_NOT_OWNER);
    CHECK(ps_unregister_job(other, b) == PS_OK);
    ps_destroy(other);
  }
  if (n_jobs > 1) CHECK(ps_unregister_job(ctx, jobs[0]) == PS_OK);
  ps_destroy(ctx);
}

static void scheduler_rounds(uint64_t seed) {
  std::mt19937_64 rng(seed);
  ps_sched* s = nullptr;
  CHECK(ps_sched_create(0.0, &s) == PS_OK);
  std::vector<int32_t> live;
  const double Ds[] = {3, 4, 5, 6, 7.5, 9, 10, 12, 24};
  for (int step = 0; step < 300; ++step) {
    const unsigned r = (unsigned)(rng() % 100);
    if (r < 12 || live.empty()) {
      int32_t j = -1;
      CHECK(ps_sched_add_job(s, Ds[rng() % 9], &j) == PS_OK);
      live.push_back(j);
    } else if (r < 90) {
      int32_t t = -1, n = -1;
      CHECK(ps_sched_assign(s, live[rng() % live.size()], 0.05 + (double)(rng() % 40) / 64.0, &t, &n) == PS_OK);
      ps_sched_agg_stats a{};
      CHECK(ps_sched_aggregator_info(s, n, &a) == PS_OK);
      std::vector<ps_sched_wave> waves(64);
      std::vector<int32_t> js(512);
      int32_t nw = 0, nj = 0;
      const int32_t rc = ps_sched_cycle_plan(s, n, waves.data(), 64, &nw, js.data(), 512, &nj);
      CHECK(rc == PS_OK || rc == PS_ERR_CAPACITY);
    } else if (r < 94) {
      int32_t fresh = -1, moved = -1;
      CHECK(ps_sched_scale_up_job(s, live[rng() % live.size()], &fresh, &moved) == PS_OK);
      CHECK(moved >= 0);
    } else {
      const size_t i = rng() % live.size();
      int32_t rel[64], nrel = 0;
      CHECK(ps_sched_remove_job(s, live[i], rel, 64, &nrel) == PS_OK);
      live.erase(live.begin() + (long)i);
    }
  }
  ps_sched_destroy(s);
}

static void pmaster_rounds(uint64_t seed) {
  std::mt19937_64 rng(seed);
  ps_pmaster* m = nullptr;
  CHECK(ps_pmaster_create(0.0, &m) == PS_OK);
  for (int c = 0; c < 3; ++c) CHECK(ps_pmaster_add_cluster(m, 1.0 + (double)(rng() % 6) / 2.0, nullptr) == PS_OK);
  std::vector<int32_t> live;
  const double Ds[] = {3, 4, 5, 6, 7.5, 9, 10, 12, 24};
  for (int step = 0; step < 200; ++step) {
    const unsigned r = (unsigned)(rng() % 100);
    if (r < 55 || live.empty()) {
      const double D = Ds[rng() % 9];
      std::vector<double> e(1 + rng() % 8);
      for (double& x : e) x = (double)(1 + rng() % 23) * D / 64.0;
      std::vector<int32_t> t(e.size()), a(e.size());
      int32_t j = -1, c = -1;
      const int32_t rc = ps_pmaster_forward_job(m, D, e.data(), (int32_t)e.size(), &j, &c, t.data(), a.data());
      CHECK(rc == PS_OK || rc == PS_ERR_NO_ROOM);
      if (rc == PS_OK) {
        live.push_back(j);
        ps_sched* ctl = ps_pmaster_controller(m, c);
        CHECK(ctl != nullptr);
        int32_t where = -1;
        CHECK(ps_sched_task_info(ctl, t[0], &where, nullptr, nullptr) == PS_OK && where == a[0]);
      }
    } else if (r < 75) {
      int32_t fresh = -1, moved = -1;
      CHECK(ps_pmaster_scale_up_job(m, live[rng() % live.size()], &fresh, &moved) == PS_OK);
    } else {
      const size_t i = rng() % live.size();
      int32_t rel[64], nrel = 0, c = -1;
      CHECK(ps_pmaster_job_exit(m, live[i], &c, rel, 64, &nrel) == PS_OK);
      live.erase(live.begin() + (long)i);
    }
    ps_pmaster_cluster_stats cs{};
    CHECK(ps_pmaster_cluster_info(m, (int32_t)(rng() % 3), &cs) == PS_OK);
  }
  ps_pmaster_destroy(m);
}

// Several threads on the same two planning contexts (a context is guarded by
// one mutex; calls that take two contexts lock them in address order).  Each
// thread works on jobs of its own, so every status is known.
static void worker_thread(ps_ctx* a, ps_ctx* b, uint64_t seed, bool forward) {
  std::mt19937_64 rng(seed);
  const float* fake = reinterpret_cast<const float*>(uintptr_t(1) << 20);
  for (int it = 0; it < 60; ++it) {
    ps_ctx* src = forward ? a : b;
    ps_ctx* dst = forward ? b : a;
    std::vector<int64_t> layers(1 + rng() % 4);
    for (auto& n : layers) n = 1 + (int64_t)(rng() % 9000);
    const int32_t W = 1 + (int32_t)(rng() % 8);
    ps_job_t job = -1, shadow = -1;
    int32_t nb = 0, nb2 = 0;
    CHECK(ps_register_job(src, layers.data(), (int32_t)layers.size(), W, 0.1f, 0.9f, 1e-4f, nullptr, nullptr,
                          &job, &nb) == PS_OK);
    CHECK(ps_register_shadow_job(dst, layers.data(), (int32_t)layers.size(), W, 0.1f, 0.9f, 1e-4f, nullptr,
                                 &shadow, &nb2) == PS_OK);
    CHECK(nb == nb2 && nb > 0);
    std::vector<int32_t> ids((size_t)nb);
    for (int32_t i = 0; i < nb; ++i) ids[(size_t)i] = i;
    // both contexts are locked, in whatever order the two directions ask for them
    CHECK(ps_migrate_many(src, job, ids.data(), nb, dst, shadow, nullptr) == PS_ERR_NO_DEVICE);
    for (int32_t w = 0; w < W; ++w) CHECK(ps_push_flat(src, job, w, fake) == PS_OK);
    int64_t need = 0;
    CHECK(ps_pack_wave(src, &job, 1, nullptr, 0, &need) == PS_ERR_CAPACITY && need == nb);
    std::vector<ps_block_ref> wave((size_t)need);
    CHECK(ps_pack_wave(src, &job, 1, wave.data(), need, &need) == PS_OK);
    ps_wave_stats st{};
    CHECK(ps_plan_wave(src, wave.data(), need, &st) == PS_OK && st.n_blocks == nb);
    CHECK(ps_estimate_wave(src, wave.data(), need, &st) == PS_OK && st.est_seconds > 0.0);
    CHECK(ps_aggregate(src, wave.data(), need, nullptr) == PS_ERR_NO_DEVICE);
    ps_block_info bi{};
    CHECK(ps_job_block_info(src, job, nb - 1, &bi) == PS_OK && bi.W == W);
    ps_block_stats bs{};
    CHECK(ps_telemetry(src, job, 0, &bs) == PS_OK && bs.round == 0);
    CHECK(ps_migrate_many(src, job, ids.data(), nb, dst, shadow, nullptr) == PS_ERR_BUSY);
    CHECK(ps_unregister_job(dst, shadow) == PS_OK);
    CHECK(ps_unregister_job(src, job) == PS_OK);
  }
}

static void threaded_rounds() {
  ps_config cfg{};
  cfg.max_block_bytes = 4096;
  ps_ctx *a = nullptr, *b = nullptr;
  CHECK(ps_create(&cfg, &a) == PS_OK && ps_create(&cfg, &b) == PS_OK);
  std::vector<std::thread> th;
  for (int k = 0; k < 4; ++k) th.emplace_back(worker_thread, a, b, (uint64_t)(100 + k), k % 2 == 0);
  for (auto& t : th) t.join();
  ps_destroy(a);
  ps_destroy(b);
}

int main(int argc, char** argv) {
  if (argc > 1 && std::strcmp(argv[1], "threads") == 0) {
    threaded_rounds();
    std::printf("host thread driver: ok\n");
    return 0;
  }
  for (uint64_t seed = 1; seed <= 40; ++seed) service_rounds(seed);
  for (uint64_t seed = 1; seed <= 10; ++seed) scheduler_rounds(seed);
  for (uint64_t seed = 1; seed <= 10; ++seed) pmaster_rounds(seed);
  std::printf("host sanitize driver: ok\n");
  return 0;
}
