// Host side of the parameter service: job registry, block-descriptor table,
// push state, wave packer and wave planner, behind the C ABI of ps.h.
//
// The paper's agent keeps a table from (job, tensor) to the server that owns the
// tensor (Section 3.1; Appendix A); here every block lives on the one GPU and the
// table maps (job, block) to its parameter / momentum shards in the arena.  The
// paper's server runs the aggregations of several jobs in one cycle (Section
// 3.3); here that is one ps_aggregate call over a list of blocks.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/ps.h"
#include "ps_internal.h"

namespace {

constexpr uint64_t kAlignElems = PS_ALIGN_BYTES / 4;

inline uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// The event that marks the arrival of migrated shard content.  One copy call
// may bring many blocks; they share one event.
struct Arrival {
  hipEvent_t ev = nullptr;
  int32_t refs = 0;
};

struct Block {
  int32_t layer;
  int64_t layer_off;
  int64_t numel;
  int64_t flat_off;
  int64_t round = 0;
  uint32_t mask = 0;
  uint64_t wave_stamp = 0;  // id of the last list that named this block (duplicate check)
  uint8_t owner = PS_OWNER_HERE;   // PS_OWNER_*
  Arrival* ready = nullptr;        // shard content arrives by a copy: wait for this first (else null)
  const float* grad[PS_MAX_W];
};

struct Job {
  bool live = false;
  int32_t W = 0;
  float lr = 0, mu = 0, wd = 0;
  uint32_t full_mask = 0;
  std::vector<int64_t> layer_numel;
  std::vector<Block> blocks;
  std::vector<int32_t> arrival;  // block ids, last layer first
  int64_t flat_numel = 0;        // elements, padded
  uint64_t arena_off = 0;        // bytes from arena base: [p flat][v flat]
  uint64_t arena_bytes = 0;
  float* p = nullptr;
  float* v = nullptr;
  PsStat* stat = nullptr;        // host-visible, one {value, round} per block, written by the GPU
};

// HIP events bracketing the phases of one measured wave.
struct TimingSet {
  hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
  bool pending = false;
  bool all_phases = false;  // four events recorded (else only ev[1], ev[2] around the launches)
  int64_t launches = 0;
};
constexpr int kTimingSets = 8;

struct Plan {
  std::vector<uint64_t> sig;           // what the tables depend on: the list and its gradient pointers
  std::vector<ps_block_ref> list;      // the list itself, and the context's pointer generation when the
  uint64_t ptr_gen = 0;                //   tables were built: equal list + equal generation = equal sig
  std::vector<int64_t> round_at_build; // per list position: the block's round before the first wave
  int64_t uses = 0;                    // waves launched with these tables
  std::vector<unsigned char> recs;     // PsBlockRec + W pointers per listed block
  std::vector<uint32_t> rec_of;        // record offset (8-byte units) per list position
  std::vector<uint32_t> large_order;   // list positions of large-path blocks, launch order
  std::vector<PsTile> tiles;
  std::vector<PsChunk> chunks;
  std::vector<PsSmallEntry> small_entries;
  std::vector<PsBin> bins;
  std::vector<uint32_t> large_recs;
  ps_wave_stats stats{};
};

// Device + pinned-host buffers holding the tables of one wave, and the host
// side of that wave's plan.  A slot whose plan matches the next call is reused
// without rebuilding or uploading anything.
struct Slot {
  char* host = nullptr;
  char* dev = nullptr;
  size_t host_cap = 0, dev_cap = 0;
  hipEvent_t done = nullptr;
  bool in_flight = false;
  hipStream_t stream = nullptr;  // stream of the wave that last used the slot
  bool valid = false;            // plan and device tables are in step
  uint64_t generation = 0;       // static scratch only: its generation when these tables went in
  Plan plan;
  PsWaveTables tables{};
};
constexpr int kSlots = 4;

}  // namespace

struct ps_ctx {
  std::mutex mu;
  ps_config cfg{};
  int64_t cap_elems = 0;
  std::vector<Job> jobs;
  uint64_t arena_top = 0;
  uint64_t wave_counter = 0;
  uint64_t ptr_gen = 1;          // bumped whenever a push records a pointer other than the one before
  Slot slots[kSlots];
  int next_slot = 0;
  int last_slot = -1;            // slot of the most recent wave (candidate for reuse)
  Slot static_slot;              // ps_aggregate_noalloc: pinned staging from ps_create, device side = the static array
  PsStaticScratch* sscratch = nullptr;  // this GPU's static array (looked up in ps_create)
  TimingSet tsets[kTimingSets];
  int next_tset = 0;
  Plan plan;                     // scratch of ps_plan_wave
  std::vector<uint64_t> sig;     // scratch: signature of the list being validated
  std::string last_error;
  int32_t timing_level = 0;     // 0 off, 1 aggregation launches only, 2 every phase
  ps_timing timing{};
  double clock_hz = 1.0e8;      // rate of the device's wall clock
  int64_t n_ready_pending = 0;  // blocks whose migrated content has not been waited for yet
  std::vector<Arrival*> arrivals;       // every arrival event ever created (owned)
  std::vector<Arrival*> arrivals_free;  // those no block refers to
  uint32_t resident_tiles[PS_MAX_W + 1] = {};  // per W: workgroups the chip holds at once (0 = unknown)
  uint32_t copy_resident = 0;    // the same for the migration copy kernel
  double read_rate = PS_READ_BYTES_PER_SEC;    // bytes/s a launch's read phase sustains
  double write_rate = PS_WRITE_BYTES_PER_SEC;  // bytes/s of its write phase
};

namespace {

int32_t normalise_config(const ps_config* in, ps_config* out) {
  if (!in) return PS_ERR_ARG;
  *out = *in;
  if (out->max_block_bytes == 0) out->max_block_bytes = PS_DEFAULT_BLOCK_BYTES;
  if (out->small_block_elems == 0) out->small_block_elems = PS_DEFAULT_SMALL_ELEMS;
  if (out->max_block_bytes % PS_ALIGN_BYTES != 0) return PS_ERR_ARG;
  if (out->max_block_bytes > (1ull << 30)) return PS_ERR_ARG;  // byte offsets inside a block are 32-bit
  if (out->small_block_elems > PS_SMALL_MAX_ELEMS) return PS_ERR_ARG;
  if (out->flags & ~uint32_t(PS_FLAG_FP_CONTRACT)) return PS_ERR_ARG;
  if (out->store_hold_permille > 2000) return PS_ERR_ARG;
  if (out->store_stagger_permille > 4000 || out->reserved_ != 0) return PS_ERR_ARG;
  if (out->arena_dev && (reinterpret_cast<uintptr_t>(out->arena_dev) % PS_ALIGN_BYTES)) return PS_ERR_ARG;
  return PS_OK;
}

// Flat layout of a job: every layer starts at a multiple of 64 elements.
int32_t layout_layers(const int64_t* layer_numel, int32_t n_layers, int64_t cap_elems,
                      std::vector<Block>* blocks, int64_t* flat_numel) {
  if (!layer_numel || n_layers <= 0) return PS_ERR_ARG;
  int64_t flat = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    const int64_t n = layer_numel[l];
    if (n <= 0 || n > (int64_t(1) << 40)) return PS_ERR_ARG;
    for (int64_t off = 0; off < n; off += cap_elems) {
      if (blocks) {
        Block b{};
        b.layer = l;
        b.layer_off = off;
        b.numel = (n - off < cap_elems) ? n - off : cap_elems;
        b.flat_off = flat + off;
        blocks->push_back(b);
      }
    }
    flat = (int64_t)round_up((uint64_t)(flat + n), kAlignElems);
  }
  *flat_numel = flat;
  return PS_OK;
}

Job* find_job(ps_ctx* c, ps_job_t job) {
  if (job < 0 || (size_t)job >= c->jobs.size() || !c->jobs[job].live) return nullptr;
  return &c->jobs[job];
}

int32_t hip_fail(ps_ctx* c, hipError_t e, const char* what);

Arrival* arrival_get(ps_ctx* c) {
  if (!c->arrivals_free.empty()) {
    Arrival* a = c->arrivals_free.back();
    c->arrivals_free.pop_back();
    return a;
  }
  Arrival* a = new Arrival();
  if (hipEventCreateWithFlags(&a->ev, hipEventDisableTiming) != hipSuccess) {
    delete a;
    return nullptr;
  }
  c->arrivals.push_back(a);
  return a;
}

// The block no longer needs its arrival event (it was waited for, or the block goes away).
void arrival_drop(ps_ctx* c, Block& b) {
  if (!b.ready) return;
  if (--b.ready->refs == 0) c->arrivals_free.push_back(b.ready);
  b.ready = nullptr;
  c->n_ready_pending -= 1;
}

void arrival_attach(ps_ctx* c, Block& b, Arrival* a) {
  arrival_drop(c, b);
  b.ready = a;
  a->refs += 1;
  c->n_ready_pending += 1;
}

int32_t hip_fail(ps_ctx* c, hipError_t e, const char* what) {
  c->last_error = std::string(what) + ": " + hipGetErrorString(e);
  return PS_ERR_HIP;
}
#define PS_HIP(c, call)                                  \
  do {                                                   \
    hipError_t e_ = (call);                              \
    if (e_ != hipSuccess) return hip_fail(c, e_, #call); \
  } while (0)

// What a plan for a (validated) list depends on besides the context's fixed
// layout: the blocks named and the gradient pointers pushed for them.
void gather_signature(ps_ctx* c, const ps_block_ref* list, int64_t n) {
  c->sig.clear();
  for (int64_t i = 0; i < n; ++i) {
    const Job& j = c->jobs[list[i].job];
    const Block& b = j.blocks[list[i].block];
    c->sig.push_back(((uint64_t)(uint32_t)list[i].job << 32) | (uint32_t)list[i].block);
    for (int32_t w = 0; w < j.W; ++w)
      c->sig.push_back((b.mask >> w) & 1u ? (uint64_t)reinterpret_cast<uintptr_t>(b.grad[w]) : 0);
  }
}

// Validate a block list.  Changes nothing but c->wave_counter, the blocks'
// duplicate stamps and (if asked) c->sig.
int32_t validate_list(ps_ctx* c, const ps_block_ref* list, int64_t n, bool need_pushes,
                      bool gather_sig = true) {
  if (n < 0 || (n > 0 && !list)) return PS_ERR_ARG;
  if (n > 0x7FFFFFF0ll) return PS_ERR_ARG;
  const uint64_t stamp = ++c->wave_counter;
  for (int64_t i = 0; i < n; ++i) {
    Job* j = find_job(c, list[i].job);
    if (!j) return PS_ERR_BAD_JOB;
    if (list[i].block < 0 || (size_t)list[i].block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
    Block& b = j->blocks[list[i].block];
    if (b.wave_stamp == stamp) return PS_ERR_DUP_BLOCK;
    b.wave_stamp = stamp;
    if (b.owner != PS_OWNER_HERE) return PS_ERR_NOT_OWNER;
    if (need_pushes && b.mask != j->full_mask) return PS_ERR_NOT_READY;
  }
  if (gather_sig) gather_signature(c, list, n);
  return PS_OK;
}

// Timing of a plan's launches: when each launch's reads are expected to be
// over (hold), how its stores are spread after that (stagger), and how long the
// wave will take.
void retime_plan(const ps_ctx* c, Plan& P) {
  const int32_t pm = c->cfg.store_hold_permille;
  const double frac = pm < 0 ? 0.0 : (pm == 0 ? PS_DEFAULT_HOLD_PERMILLE : pm) / 1000.0;
  const int32_t sm = c->cfg.store_stagger_permille;
  const double sfrac = (pm < 0 || sm < 0) ? 0.0 : (sm == 0 ? PS_DEFAULT_STAGGER_PERMILLE : sm) / 1000.0;
  // predicted GPU time of the wave: each launch reads, then writes (the store
  // hold separates the two), plus a fixed cost per launch and per wave
  double est = PS_EST_WAVE_SECONDS;
  for (PsChunk& ch : P.chunks) {
    // holding only pays when the whole launch is resident; a larger launch (a
    // caller's launch_tiles) would make every later generation wait again
    const uint32_t resident = c->resident_tiles[ch.W <= PS_MAX_W ? ch.W : 0];
    const bool fits = resident == 0 || ch.end - ch.begin <= resident;
    const double read_ticks = (double)ch.read_bytes / c->read_rate * c->clock_hz;
    // never longer than half a millisecond, whatever the tables say: a resident
    // launch reads for far less, and every wave must leave its wait soon
    ch.hold_ticks = fits ? (uint32_t)std::min(frac * read_ticks, 5.0e-4 * c->clock_hz) : 0u;
    // per workgroup index: the time one tile's stores (parameters and momentum)
    // take at the read-phase rate, scaled; bounded so that index * value stays
    // inside 32 bits and the whole spread of a resident launch below 100 us
    const double tile_ticks = (double)PS_TILE_ELEMS * 8.0 / c->read_rate * c->clock_hz;
    ch.stagger_q16 = (uint32_t)std::min(sfrac * tile_ticks * 65536.0, 1.0e-4 * c->clock_hz / 2048.0 * 65536.0);
    const double params = (double)ch.read_bytes / (4.0 * ch.W + 8.0);
    est += (double)ch.read_bytes / c->read_rate + 8.0 * params / c->write_rate + PS_EST_LAUNCH_SECONDS;
  }
  if (P.chunks.empty() && !P.bins.empty()) est += PS_EST_LAUNCH_SECONDS;
  P.stats.est_seconds = est;
}

// Lay out the tables of a validated list's wave in P.
void layout_plan(ps_ctx* c, const ps_block_ref* list, int64_t n, Plan& P) {
  P.recs.clear(); P.rec_of.clear(); P.large_order.clear(); P.tiles.clear(); P.chunks.clear();
  P.small_entries.clear(); P.bins.clear(); P.large_recs.clear();
  P.stats = ps_wave_stats{};
  P.list.assign(list, list + n);
  P.ptr_gen = c->ptr_gen;
  P.round_at_build.resize((size_t)n);
  P.uses = 0;
  const uint32_t small_max = c->cfg.small_block_elems;

  // one record per listed block, in list order; small blocks go to bins
  P.rec_of.resize((size_t)n);
  PsBin bin{0, 0, 0, 0};
  auto close_bin = [&]() {
    if (bin.count) P.bins.push_back(bin);
    bin = PsBin{(uint32_t)P.small_entries.size(), 0, 0, 0};
  };
  for (int64_t i = 0; i < n; ++i) {
    Job& j = c->jobs[list[i].job];
    Block& b = j.blocks[list[i].block];
    P.round_at_build[(size_t)i] = b.round;
    PsBlockRec d{};
    d.p = j.p ? j.p + b.flat_off : nullptr;
    d.v = j.v ? j.v + b.flat_off : nullptr;
    d.stat = j.stat ? j.stat + list[i].block : nullptr;
    d.round0 = b.round + 1;
    d.n = (uint32_t)b.numel;
    d.W = (uint32_t)j.W;
    d.lr = j.lr; d.mu = j.mu; d.wd = j.wd;
    const size_t at = P.recs.size();
    P.rec_of[(size_t)i] = (uint32_t)(at / PS_REC_UNIT);
    P.recs.resize(at + sizeof(PsBlockRec) + sizeof(const float*) * (size_t)j.W);
    const float** gp = reinterpret_cast<const float**>(P.recs.data() + at + sizeof(PsBlockRec));
    for (int32_t w = 0; w < j.W; ++w) gp[w] = (b.mask >> w) & 1u ? b.grad[w] : nullptr;
    if (d.n <= small_max) {
      const uint32_t q = (d.n + 3) / 4;
      // a bin is closed once it gives every lane a quad, or when a table is full
      if (bin.count && (bin.quads >= PS_WG || bin.count == PS_BIN_MAX_BLOCKS ||
                        bin.quads + q > PS_BIN_MAX_QUADS || bin.nptrs + d.W > PS_BIN_MAX_PTRS))
        close_bin();
      P.small_entries.push_back(PsSmallEntry{P.rec_of[(size_t)i], bin.quads, bin.nptrs, 0});
      bin.count += 1;
      bin.quads += q;
      bin.nptrs += d.W;
      P.stats.n_small_blocks += 1;
      P.stats.small_params += d.n;
      P.stats.small_algorithmic_bytes += (uint64_t)(4 * j.W + 16) * d.n;
    } else {
      P.large_order.push_back((uint32_t)i);
    }
    std::memcpy(P.recs.data() + at, &d, sizeof(d));
    P.stats.n_params += d.n;
    P.stats.algorithmic_bytes += (uint64_t)(4 * j.W + 16) * d.n;
  }
  close_bin();

  // launch order of the large path.  Blocks are independent, so any
  // order gives the same result; tiles of one worker count are made adjacent
  // (most workers first); inside a class, one job's blocks stay together, which
  // keeps the number of HBM streams touched at any moment small; and a job's
  // blocks go in ascending address order, so that the workgroups of a launch,
  // which start in index order, sweep every array upwards through one
  // contiguous range (measured: the arrival order, last layer first, costs
  // 1.4 % at W = 2 when layers are not whole launches, a random order 5 %).
  std::stable_sort(P.large_order.begin(), P.large_order.end(), [&](uint32_t a, uint32_t b) {
    const Job& ja = c->jobs[list[a].job];
    const Job& jb = c->jobs[list[b].job];
    if (ja.W != jb.W) return ja.W > jb.W;
    if (list[a].job != list[b].job) return list[a].job < list[b].job;
    return ja.blocks[list[a].block].flat_off < jb.blocks[list[b].block].flat_off;
  });
  uint32_t cur_w = 0;
  PsChunk chunk{0, 0, 0, 0, 0};
  for (uint32_t i : P.large_order) {
    PsBlockRec* d = reinterpret_cast<PsBlockRec*>(P.recs.data() + (size_t)P.rec_of[i] * PS_REC_UNIT);
    d->tile0 = (uint32_t)P.tiles.size();
    d->ntiles = (d->n + PS_TILE_ELEMS - 1) / PS_TILE_ELEMS;
    if (d->W != cur_w && chunk.end > chunk.begin) {
      P.chunks.push_back(chunk);
      chunk.begin = chunk.end;
      chunk.read_bytes = 0;
    }
    cur_w = d->W;
    chunk.W = cur_w;
    uint32_t limit = c->cfg.launch_tiles ? c->cfg.launch_tiles : ps_chunk_tiles(cur_w);
    if (c->resident_tiles[cur_w] && limit > c->resident_tiles[cur_w]) limit = c->resident_tiles[cur_w];
    // the first launch also carries the small-path bins: leave them room
    if (P.chunks.empty() && limit > 2 * P.bins.size()) limit -= (uint32_t)P.bins.size();
    for (uint32_t t = 0; t < d->ntiles; ++t) {
      P.tiles.push_back(PsTile{P.rec_of[i], t * PS_TILE_ELEMS});
      const uint32_t len = std::min<uint32_t>(PS_TILE_ELEMS, d->n - t * PS_TILE_ELEMS);
      chunk.read_bytes += (uint64_t)(4 * cur_w + 8) * len;
      if (++chunk.end - chunk.begin >= limit) {
        P.chunks.push_back(chunk);
        chunk.begin = chunk.end;
        chunk.read_bytes = 0;
      }
    }
    P.large_recs.push_back(P.rec_of[i]);
  }
  if (chunk.end > chunk.begin) P.chunks.push_back(chunk);
  retime_plan(c, P);
  P.stats.est_seconds = n > 0 ? P.stats.est_seconds : 0.0;

  P.stats.n_blocks = n;
  P.stats.n_large_tiles = (int64_t)P.tiles.size();
  P.stats.n_small_bins = (int64_t)P.bins.size();
  P.stats.n_launches = (int64_t)std::max<size_t>(P.chunks.size(), P.bins.empty() ? 0 : 1);
}

// Wall-clock ticks a copy launch holds its data per tile it moves: the tile's
// bytes read (parameters and momentum) at the pure-read rate, scaled.
double copy_hold_ticks_per_tile(const ps_ctx* c) {
  const int32_t pm = c->cfg.store_hold_permille;
  if (pm < 0) return 0.0;
  // the caller's knob scales the copy's hold in the same proportion as the aggregation's
  const double frac = PS_COPY_HOLD_PERMILLE / 1000.0 * (pm == 0 ? 1.0 : (double)pm / PS_DEFAULT_HOLD_PERMILLE);
  return frac * (double)PS_TILE_ELEMS * 8.0 / c->read_rate * c->clock_hz;
}

// Extra hold per workgroup index of a launch, in 1/65536 ticks: the time the
// stores of one tile (parameters and momentum) take at the read-phase rate,
// scaled by the configured fraction.  Bounded so that index * value stays far
// inside 32 bits and the whole spread below 100 us for any resident launch.
uint32_t copy_stagger_q16(const ps_ctx* c) {
  const int32_t pm = c->cfg.store_stagger_permille;
  if (pm < 0 || c->cfg.store_hold_permille < 0) return 0;
  const double frac = (pm == 0 ? PS_COPY_STAGGER_PERMILLE : (uint32_t)pm) / 1000.0;
  const double ticks_per_tile = frac * (double)PS_TILE_ELEMS * 8.0 / c->read_rate * c->clock_hz;
  return (uint32_t)std::min(ticks_per_tile * 65536.0, 1.0e-4 * c->clock_hz / 2048.0 * 65536.0);
}

// Wait for the wave that last used the slot.
int32_t slot_retire(ps_ctx* c, Slot& s) {
  if (!s.in_flight) return PS_OK;
  PS_HIP(c, hipEventSynchronize(s.done));
  s.in_flight = false;
  return PS_OK;
}

// Wait for a measured wave and add its event times to the sums.
int32_t timing_harvest(ps_ctx* c, TimingSet& t) {
  if (!t.pending) return PS_OK;
  PS_HIP(c, hipEventSynchronize(t.ev[t.all_phases ? 3 : 2]));
  t.pending = false;
  float agg = 0;
  PS_HIP(c, hipEventElapsedTime(&agg, t.ev[1], t.ev[2]));
  float up = 0, norms = 0, tot = agg;
  if (t.all_phases) {
    PS_HIP(c, hipEventElapsedTime(&up, t.ev[0], t.ev[1]));
    PS_HIP(c, hipEventElapsedTime(&norms, t.ev[2], t.ev[3]));
    PS_HIP(c, hipEventElapsedTime(&tot, t.ev[0], t.ev[3]));
  }
  c->timing.n_waves += 1;
  c->timing.n_launches += t.launches;
  c->timing.upload_ms += up;
  c->timing.agg_ms += agg;
  c->timing.norms_ms += norms;
  c->timing.total_ms += tot;
  return PS_OK;
}

int32_t slot_reserve(ps_ctx* c, Slot& s, size_t host_bytes, size_t dev_bytes) {
  {
    const int32_t st = slot_retire(c, s);
    if (st != PS_OK) return st;
  }
  if (!s.done) PS_HIP(c, hipEventCreateWithFlags(&s.done, hipEventDisableTiming));
  if (host_bytes > s.host_cap) {
    if (s.host) PS_HIP(c, hipHostFree(s.host));
    s.host = nullptr; s.host_cap = 0;
    const size_t cap = round_up(host_bytes + host_bytes / 2, 4096);
    PS_HIP(c, hipHostMalloc((void**)&s.host, cap, hipHostMallocDefault));
    s.host_cap = cap;
  }
  if (dev_bytes > s.dev_cap) {
    if (s.dev) PS_HIP(c, hipFree(s.dev));
    s.dev = nullptr; s.dev_cap = 0;
    const size_t cap = round_up(dev_bytes + dev_bytes / 2, 4096);
    PS_HIP(c, hipMalloc((void**)&s.dev, cap));
    s.dev_cap = cap;
  }
  return PS_OK;
}

template <class T>
size_t place(size_t* cursor, size_t count) {
  const size_t at = round_up(*cursor, 256);
  *cursor = at + count * sizeof(T);
  return at;
}

// Where the tables of a plan sit inside a slot's buffer.
struct Offsets {
  size_t recs, tiles, small, bins, large, upload, part, total;
};

Offsets offsets_of(const Plan& P) {
  Offsets o{};
  size_t cur = 0;
  o.recs = place<unsigned char>(&cur, P.recs.size());
  o.tiles = place<PsTile>(&cur, P.tiles.size());
  o.small = place<PsSmallEntry>(&cur, P.small_entries.size());
  o.bins = place<PsBin>(&cur, P.bins.size());
  o.large = place<uint32_t>(&cur, P.large_recs.size());
  o.upload = cur;
  o.part = place<double>(&cur, P.tiles.size());
  o.total = cur;
  return o;
}

void stage_tables(const Plan& P, const Offsets& o, char* host) {
  auto put = [&](size_t at, const void* src, size_t bytes) { if (bytes) std::memcpy(host + at, src, bytes); };
  put(o.recs, P.recs.data(), P.recs.size());
  put(o.tiles, P.tiles.data(), P.tiles.size() * sizeof(PsTile));
  put(o.small, P.small_entries.data(), P.small_entries.size() * sizeof(PsSmallEntry));
  put(o.bins, P.bins.data(), P.bins.size() * sizeof(PsBin));
  put(o.large, P.large_recs.data(), P.large_recs.size() * sizeof(uint32_t));
}

void bind_tables(const ps_ctx* c, Slot& s, const Offsets& o, char* dev) {
  const Plan& P = s.plan;
  PsWaveTables& t = s.tables;
  t = PsWaveTables{};
  t.recs = reinterpret_cast<const unsigned char*>(dev + o.recs);
  t.tiles = reinterpret_cast<const PsTile*>(dev + o.tiles);
  t.n_tiles = (uint32_t)P.tiles.size();
  t.chunks = P.chunks.data();
  t.n_chunks = (uint32_t)P.chunks.size();
  t.tile_part = reinterpret_cast<double*>(dev + o.part);
  t.small_entries = reinterpret_cast<const PsSmallEntry*>(dev + o.small);
  t.bins = reinterpret_cast<const PsBin*>(dev + o.bins);
  t.n_bins = (uint32_t)P.bins.size();
  t.large_recs = reinterpret_cast<const uint32_t*>(dev + o.large);
  t.n_large_blocks = (uint32_t)P.large_recs.size();
  t.fp_contract = (c->cfg.flags & PS_FLAG_FP_CONTRACT) != 0;
}

struct ScratchGuard {
  PsStaticScratch* s;
  explicit ScratchGuard(PsStaticScratch* x) : s(x) { if (s) ps_static_scratch_lock(s); }
  ~ScratchGuard() { if (s) ps_static_scratch_unlock(s); }
};

}  // namespace

// No C++ exception leaves the library.  What this code can raise are failed
// host allocations (containers growing), so that is what the caller is told.
#define PS_NO_THROW catch (...) { return PS_ERR_NOMEM; }

extern "C" {

int32_t ps_version(void) { return 100; }

const char* ps_strerror(int32_t s) {
  switch (s) {
    case PS_OK: return "ok";
    case PS_ERR_ARG: return "invalid argument";
    case PS_ERR_BAD_JOB: return "unknown job";
    case PS_ERR_BAD_BLOCK: return "block id outside the job";
    case PS_ERR_BAD_WORKER: return "worker outside [0, W)";
    case PS_ERR_DUP_PUSH: return "worker already pushed this block in this round";
    case PS_ERR_NOT_READY: return "block has not received all W pushes";
    case PS_ERR_DUP_BLOCK: return "block listed twice";
    case PS_ERR_ALIGN: return "pointer not aligned as required";
    case PS_ERR_NOMEM: return "out of arena or memory";
    case PS_ERR_NO_DEVICE: return "planning context: no device arena";
    case PS_ERR_HIP: return "HIP runtime call failed";
    case PS_ERR_CAPACITY: return "output array too small";
    case PS_ERR_NOT_OWNER: return "block's master copy is not held by this context";
    case PS_ERR_BUSY: return "block has pushes pending";
    case PS_ERR_NO_ROOM: return "no Aggregator cluster has room for the job";
    default: return "unknown status";
  }
}

const char* ps_last_error(ps_ctx* ctx) { return ctx ? ctx->last_error.c_str() : ""; }

int32_t ps_create(const ps_config* cfg, ps_ctx** out_ctx) try {
  if (!out_ctx) return PS_ERR_ARG;
  *out_ctx = nullptr;
  ps_config n{};
  const int32_t st = normalise_config(cfg, &n);
  if (st != PS_OK) return st;
  ps_ctx* c = new (std::nothrow) ps_ctx();
  if (!c) return PS_ERR_NOMEM;
  c->cfg = n;
  c->cap_elems = (int64_t)(n.max_block_bytes / 4);
  // a planning context plans for the GPU the figures were fitted on: MI355X holds 2048 workgroups at once
  for (uint32_t w = 0; w <= PS_MAX_W; ++w) c->resident_tiles[w] = 2048;
  if (n.arena_dev) {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0)
      c->clock_hz = 1000.0 * khz;
    for (uint32_t w = 0; w <= PS_MAX_W; ++w) c->resident_tiles[w] = ps_resident_workgroups(w);
    c->copy_resident = ps_resident_copy_workgroups();
    // everything ps_aggregate_noalloc will need, so that it never allocates:
    // this GPU's static array and a pinned staging buffer of the same size
    if (ps_static_scratch(&c->sscratch) != 0 ||
        hipHostMalloc((void**)&c->static_slot.host, PS_STATIC_SCRATCH_BYTES, hipHostMallocDefault) != hipSuccess) {
      delete c;
      return PS_ERR_HIP;
    }
    c->static_slot.host_cap = PS_STATIC_SCRATCH_BYTES;
  }
  *out_ctx = c;
  return PS_OK;
} PS_NO_THROW

void ps_destroy(ps_ctx* c) {
  if (!c) return;
  for (Slot& s : c->slots) {
    if (s.in_flight) (void)hipEventSynchronize(s.done);
    if (s.done) (void)hipEventDestroy(s.done);

    if (s.host) (void)hipHostFree(s.host);
    if (s.dev) (void)hipFree(s.dev);
  }
  if (c->static_slot.host) (void)hipHostFree(c->static_slot.host);
  for (TimingSet& t : c->tsets)
    for (hipEvent_t e : t.ev)
      if (e) (void)hipEventDestroy(e);
  for (Job& j : c->jobs) {
    if (j.stat && c->cfg.arena_dev) (void)hipHostFree(j.stat);
    else delete[] j.stat;
  }
  for (Arrival* a : c->arrivals) {
    (void)hipEventDestroy(a->ev);
    delete a;
  }
  delete c;
}

int32_t ps_job_arena_bytes(const ps_config* cfg, const int64_t* layer_numel, int32_t n_layers,
                           uint64_t* out_bytes) try {
  if (!out_bytes) return PS_ERR_ARG;
  ps_config n{};
  int32_t st = normalise_config(cfg, &n);
  if (st != PS_OK) return st;
  int64_t flat = 0;
  st = layout_layers(layer_numel, n_layers, (int64_t)(n.max_block_bytes / 4), nullptr, &flat);
  if (st != PS_OK) return st;
  *out_bytes = (uint64_t)flat * 4 * 2;
  return PS_OK;
} PS_NO_THROW

static int32_t register_job(ps_ctx* c, const int64_t* layer_numel, int32_t n_layers, int32_t W, float lr,
                            float momentum, float wd, const float* const* init_params, void* stream,
                            ps_job_t* out_job, int32_t* out_n_blocks, bool shadow) {
  if (!c || !out_job) return PS_ERR_ARG;
  if (W < 1 || W > PS_MAX_W) return PS_ERR_ARG;
  if (!std::isfinite(lr) || !std::isfinite(momentum) || !std::isfinite(wd)) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job j;
  int32_t st = layout_layers(layer_numel, n_layers, c->cap_elems, &j.blocks, &j.flat_numel);
  if (st != PS_OK) return st;
  if (j.blocks.size() > 0x7FFFFFF0u) return PS_ERR_ARG;
  j.W = W; j.lr = lr; j.mu = momentum; j.wd = wd;
  j.full_mask = (W == 32) ? 0xFFFFFFFFu : ((1u << W) - 1u);
  j.layer_numel.assign(layer_numel, layer_numel + n_layers);
  // arrival order: last registered layer first, ascending offset inside a layer
  {
    const int32_t nb = (int32_t)j.blocks.size();
    j.arrival.reserve(nb);
    int32_t end = nb;
    while (end > 0) {
      int32_t begin = end;
      const int32_t layer = j.blocks[end - 1].layer;
      while (begin > 0 && j.blocks[begin - 1].layer == layer) --begin;
      for (int32_t b = begin; b < end; ++b) j.arrival.push_back(b);
      end = begin;
    }
  }
  j.arena_bytes = (uint64_t)j.flat_numel * 4 * 2;
  j.arena_off = c->arena_top;
  const size_t nb = j.blocks.size();
  const bool device = c->cfg.arena_dev != nullptr;
  if (device) {
    if (j.arena_off + j.arena_bytes > c->cfg.arena_bytes) return PS_ERR_NOMEM;
    char* base = static_cast<char*>(c->cfg.arena_dev) + j.arena_off;
    j.p = reinterpret_cast<float*>(base);
    j.v = j.p + j.flat_numel;
    PS_HIP(c, hipHostMalloc((void**)&j.stat, nb * sizeof(PsStat), hipHostMallocDefault));
    hipStream_t s = static_cast<hipStream_t>(stream);
    // parameters' padding and all momentum start at zero
    hipError_t e = (hipError_t)ps_launch_zero(j.p, j.arena_bytes / 4, stream);
    if (e == hipSuccess && init_params) {
      int64_t flat = 0;
      for (int32_t l = 0; l < n_layers && e == hipSuccess; ++l) {
        if (init_params[l])
          e = hipMemcpyAsync(j.p + flat, init_params[l], (size_t)layer_numel[l] * 4,
                             hipMemcpyDeviceToDevice, s);
        flat = (int64_t)round_up((uint64_t)(flat + layer_numel[l]), kAlignElems);
      }
    }
    if (e != hipSuccess) {
      (void)hipHostFree(j.stat);
      return hip_fail(c, e, "initialising the job's shards");
    }
  } else {
    j.stat = new (std::nothrow) PsStat[nb];
    if (!j.stat) return PS_ERR_NOMEM;
  }
  for (size_t b = 0; b < nb; ++b) j.stat[b] = PsStat{0.0, 0};
  if (shadow)
    for (Block& b : j.blocks) b.owner = PS_OWNER_ELSEWHERE;
  j.live = true;
  c->arena_top = round_up(j.arena_off + j.arena_bytes, PS_ALIGN_BYTES);
  c->jobs.push_back(std::move(j));
  *out_job = (ps_job_t)(c->jobs.size() - 1);
  if (out_n_blocks) *out_n_blocks = (int32_t)nb;
  return PS_OK;
}

int32_t ps_register_job(ps_ctx* c, const int64_t* layer_numel, int32_t n_layers, int32_t W, float lr,
                        float momentum, float wd, const float* const* init_params, void* stream,
                        ps_job_t* out_job, int32_t* out_n_blocks) try {
  return register_job(c, layer_numel, n_layers, W, lr, momentum, wd, init_params, stream, out_job,
                      out_n_blocks, /*shadow=*/false);
} PS_NO_THROW

int32_t ps_register_shadow_job(ps_ctx* c, const int64_t* layer_numel, int32_t n_layers, int32_t W,
                               float lr, float momentum, float wd, void* stream, ps_job_t* out_job,
                               int32_t* out_n_blocks) try {
  return register_job(c, layer_numel, n_layers, W, lr, momentum, wd, nullptr, stream, out_job,
                      out_n_blocks, /*shadow=*/true);
} PS_NO_THROW

int32_t ps_unregister_job(ps_ctx* c, ps_job_t job) try {
  if (!c) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  j->live = false;
  for (Block& b : j->blocks) arrival_drop(c, b);
  if (j->stat && c->cfg.arena_dev) (void)hipHostFree(j->stat);
  else delete[] j->stat;
  j->stat = nullptr;
  j->blocks.clear(); j->blocks.shrink_to_fit();
  // pop the arena stack past every dead job on top
  uint64_t top = 0;
  for (const Job& o : c->jobs)
    if (o.live) top = std::max<uint64_t>(top, round_up(o.arena_off + o.arena_bytes, PS_ALIGN_BYTES));
  c->arena_top = top;
  return PS_OK;
} PS_NO_THROW

int32_t ps_job_n_blocks(ps_ctx* c, ps_job_t job) try {
  if (!c) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  return j ? (int32_t)j->blocks.size() : PS_ERR_BAD_JOB;
} PS_NO_THROW

int64_t ps_job_flat_numel(ps_ctx* c, ps_job_t job) try {
  if (!c) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  return j ? j->flat_numel : (int64_t)PS_ERR_BAD_JOB;
} PS_NO_THROW

int32_t ps_job_block_info(ps_ctx* c, ps_job_t job, int32_t block, ps_block_info* out) try {
  if (!c || !out) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
  const Block& b = j->blocks[block];
  out->layer = b.layer;
  out->W = j->W;
  out->layer_offset = b.layer_off;
  out->numel = b.numel;
  out->flat_offset = b.flat_off;
  out->round = b.round;
  out->push_mask = b.mask;
  out->small_path = b.numel <= (int64_t)c->cfg.small_block_elems ? 1u : 0u;
  out->owner = b.owner;
  out->reserved_ = 0;
  return PS_OK;
} PS_NO_THROW

int32_t ps_push(ps_ctx* c, ps_job_t job, int32_t block, int32_t worker, const float* grad_dev) try {
  if (!c || !grad_dev) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
  if (worker < 0 || worker >= j->W) return PS_ERR_BAD_WORKER;
  if (reinterpret_cast<uintptr_t>(grad_dev) % PS_GRAD_ALIGN_BYTES) return PS_ERR_ALIGN;
  Block& b = j->blocks[block];
  if (b.owner != PS_OWNER_HERE) return PS_ERR_NOT_OWNER;
  if ((b.mask >> worker) & 1u) return PS_ERR_DUP_PUSH;
  if (b.grad[worker] != grad_dev) c->ptr_gen += 1;
  b.grad[worker] = grad_dev;
  b.mask |= 1u << worker;
  return PS_OK;
} PS_NO_THROW

int32_t ps_push_flat(ps_ctx* c, ps_job_t job, int32_t worker, const float* grad_flat_dev) try {
  if (!c || !grad_flat_dev) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (worker < 0 || worker >= j->W) return PS_ERR_BAD_WORKER;
  if (reinterpret_cast<uintptr_t>(grad_flat_dev) % PS_ALIGN_BYTES) return PS_ERR_ALIGN;
  const uint32_t bit = 1u << worker;
  for (const Block& b : j->blocks)
    if (b.owner == PS_OWNER_HERE && (b.mask & bit)) return PS_ERR_DUP_PUSH;
  bool changed = false;
  for (Block& b : j->blocks) {
    if (b.owner != PS_OWNER_HERE) continue;  // pushed to whoever owns it
    if (b.grad[worker] != grad_flat_dev + b.flat_off) changed = true;
    b.grad[worker] = grad_flat_dev + b.flat_off;
    b.mask |= bit;
  }
  if (changed) c->ptr_gen += 1;
  return PS_OK;
} PS_NO_THROW

int32_t ps_pack_wave(ps_ctx* c, const ps_job_t* jobs, int32_t n_jobs, ps_block_ref* out, int64_t cap,
                     int64_t* out_n) try {
  if (!c || !out_n || n_jobs < 0 || (n_jobs > 0 && !jobs) || cap < 0 || (cap > 0 && !out))
    return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  // each job's arrival sequence, restricted to the blocks this context owns
  std::vector<std::vector<int32_t>> seq((size_t)n_jobs);
  int64_t total = 0;
  for (int32_t a = 0; a < n_jobs; ++a) {
    Job* j = find_job(c, jobs[a]);
    if (!j) return PS_ERR_BAD_JOB;
    for (int32_t b = 0; b < a; ++b)
      if (jobs[b] == jobs[a]) return PS_ERR_DUP_BLOCK;
    for (int32_t b : j->arrival)
      if (j->blocks[b].owner == PS_OWNER_HERE) seq[a].push_back(b);
    total += (int64_t)seq[a].size();
  }
  *out_n = total;
  if (total > cap) return PS_ERR_CAPACITY;
  // k-way merge by position (2k+1)/(2n), compared exactly by cross-multiplication
  std::vector<int64_t> head(n_jobs, 0);
  for (int64_t t = 0; t < total; ++t) {
    int32_t best = -1;
    int64_t bk = 0, bn = 1;
    for (int32_t a = 0; a < n_jobs; ++a) {
      const int64_t n = (int64_t)seq[a].size();
      const int64_t k = head[a];
      if (k >= n) continue;
      if (best < 0 || (unsigned __int128)(2 * k + 1) * (uint64_t)bn <
                          (unsigned __int128)(2 * bk + 1) * (uint64_t)n) {
        best = a; bk = k; bn = n;
      }
    }
    out[t].job = jobs[best];
    out[t].block = seq[best][bk];
    head[best] = bk + 1;
  }
  return PS_OK;
} PS_NO_THROW

int32_t ps_split_ready(ps_ctx* c, const ps_block_ref* list, int64_t n, ps_block_ref* out_ready,
                       int64_t* out_n_ready, ps_block_ref* out_late, int64_t* out_n_late) try {
  if (!c || !out_n_ready || !out_n_late) return PS_ERR_ARG;
  if (n > 0 && (!out_ready || !out_late)) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  const int32_t st = validate_list(c, list, n, /*need_pushes=*/false);
  if (st != PS_OK) return st;
  int64_t nr = 0, nl = 0;
  for (int64_t i = 0; i < n; ++i) {
    const Job& j = c->jobs[list[i].job];
    if (j.blocks[list[i].block].mask == j.full_mask) out_ready[nr++] = list[i];
    else out_late[nl++] = list[i];
  }
  *out_n_ready = nr;
  *out_n_late = nl;
  return PS_OK;
} PS_NO_THROW

int32_t ps_migrate_begin(ps_ctx* c, ps_job_t job, int32_t block) try {
  if (!c) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
  Block& b = j->blocks[block];
  if (b.owner != PS_OWNER_HERE) return PS_ERR_NOT_OWNER;
  if (b.mask != 0) return PS_ERR_BUSY;  // pushes of the coming round are already in
  b.owner = PS_OWNER_LEAVING;
  return PS_OK;
} PS_NO_THROW

int32_t ps_migrate_cancel(ps_ctx* c, ps_job_t job, int32_t block) try {
  if (!c) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
  Block& b = j->blocks[block];
  if (b.owner != PS_OWNER_LEAVING) return PS_ERR_NOT_OWNER;
  b.owner = PS_OWNER_HERE;
  return PS_OK;
} PS_NO_THROW

int32_t ps_migrate_copy(ps_ctx* src, ps_job_t src_job, int32_t block, ps_ctx* dst, ps_job_t dst_job,
                        void* stream) try {
  if (!src || !dst || src == dst) return PS_ERR_ARG;
  // both contexts change: take their locks in address order
  std::mutex& m1 = src < dst ? src->mu : dst->mu;
  std::mutex& m2 = src < dst ? dst->mu : src->mu;
  std::lock_guard<std::mutex> g1(m1);
  std::lock_guard<std::mutex> g2(m2);
  Job* js = find_job(src, src_job);
  Job* jd = find_job(dst, dst_job);
  if (!js || !jd) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= js->blocks.size() || (size_t)block >= jd->blocks.size())
    return PS_ERR_BAD_BLOCK;
  Block& bs = js->blocks[block];
  Block& bd = jd->blocks[block];
  if (bs.owner != PS_OWNER_LEAVING || bd.owner != PS_OWNER_ELSEWHERE) return PS_ERR_NOT_OWNER;
  if (bs.numel != bd.numel || js->W != jd->W) return PS_ERR_ARG;
  if (!js->p || !jd->p) return PS_ERR_NO_DEVICE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  // the copy must see the source's last update of the shard, whatever stream ran it
  for (Slot& s : src->slots)
    if (s.in_flight && s.stream != hs) PS_HIP(src, hipStreamWaitEvent(hs, s.done, 0));
  // ... and, if the shard itself came here by a copy nobody has waited for yet, that copy
  if (bs.ready) {
    PS_HIP(src, hipStreamWaitEvent(hs, bs.ready->ev, 0));
    arrival_drop(src, bs);
  }
  {
    const int le = ps_launch_copy(js->p + bs.flat_off, jd->p + bd.flat_off, js->v + bs.flat_off,
                                  jd->v + bd.flat_off, (uint64_t)bs.numel, stream, src->copy_resident,
                                  copy_hold_ticks_per_tile(src), copy_stagger_q16(src));
    if (le != 0) return hip_fail(dst, (hipError_t)le, "launching the migration copy");
  }
  Arrival* a = arrival_get(dst);
  if (!a) return PS_ERR_NOMEM;
  const hipError_t er = hipEventRecord(a->ev, hs);
  if (er != hipSuccess) {
    dst->arrivals_free.push_back(a);
    return hip_fail(dst, er, "recording the arrival of a migrated block");
  }
  // the new owner may take pushes at once; its first update waits for the copy
  arrival_attach(dst, bd, a);
  bd.owner = PS_OWNER_HERE;
  bd.round = bs.round;
  bd.mask = 0;
  bs.owner = PS_OWNER_ELSEWHERE;
  return PS_OK;
} PS_NO_THROW

int32_t ps_migrate_many(ps_ctx* src, ps_job_t src_job, const int32_t* blocks, int32_t n, ps_ctx* dst,
                        ps_job_t dst_job, void* stream) try {
  if (!src || !dst || src == dst || n < 0 || (n > 0 && !blocks)) return PS_ERR_ARG;
  std::mutex& m1 = src < dst ? src->mu : dst->mu;
  std::mutex& m2 = src < dst ? dst->mu : src->mu;
  std::lock_guard<std::mutex> g1(m1);
  std::lock_guard<std::mutex> g2(m2);
  Job* js = find_job(src, src_job);
  Job* jd = find_job(dst, dst_job);
  if (!js || !jd) return PS_ERR_BAD_JOB;
  if (js->W != jd->W) return PS_ERR_ARG;
  // all or nothing: check every block before anything moves
  const uint64_t stamp = ++src->wave_counter;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t b = blocks[i];
    if (b < 0 || (size_t)b >= js->blocks.size() || (size_t)b >= jd->blocks.size()) return PS_ERR_BAD_BLOCK;
    Block& bs = js->blocks[b];
    const Block& bd = jd->blocks[b];
    if (bs.wave_stamp == stamp) return PS_ERR_DUP_BLOCK;
    bs.wave_stamp = stamp;
    if (bs.owner == PS_OWNER_ELSEWHERE || bd.owner != PS_OWNER_ELSEWHERE) return PS_ERR_NOT_OWNER;
    if (bs.owner == PS_OWNER_HERE && bs.mask != 0) return PS_ERR_BUSY;
    if (bs.numel != bd.numel || bs.flat_off != bd.flat_off) return PS_ERR_ARG;
  }
  if (n == 0) return PS_OK;
  if (!js->p || !jd->p) return PS_ERR_NO_DEVICE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  for (Slot& s : src->slots)
    if (s.in_flight && s.stream != hs) PS_HIP(src, hipStreamWaitEvent(hs, s.done, 0));
  for (int32_t i = 0; i < n && src->n_ready_pending > 0; ++i) {
    Block& bs = js->blocks[blocks[i]];
    if (!bs.ready) continue;  // else the shard came here by a copy nobody has waited for yet
    PS_HIP(src, hipStreamWaitEvent(hs, bs.ready->ev, 0));
    arrival_drop(src, bs);
  }
  // Blocks with consecutive ids are neighbours in the flat layout (between two
  // layers lies only padding that no block owns and that is zero on both sides):
  // each run of consecutive ids moves with one copy per array.
  std::vector<int32_t> ids(blocks, blocks + n);
  std::sort(ids.begin(), ids.end());
  for (size_t a = 0; a < ids.size();) {
    size_t z = a;
    while (z + 1 < ids.size() && ids[z + 1] == ids[z] + 1) ++z;
    const Block& first = js->blocks[ids[a]];
    const Block& last = js->blocks[ids[z]];
    const size_t bytes = (size_t)(last.flat_off + last.numel - first.flat_off) * 4;
    const int le = ps_launch_copy(js->p + first.flat_off, jd->p + first.flat_off, js->v + first.flat_off,
                                  jd->v + first.flat_off, bytes / 4, stream, src->copy_resident,
                                  copy_hold_ticks_per_tile(src), copy_stagger_q16(src));
    if (le != 0) return hip_fail(dst, (hipError_t)le, "launching the migration copy");
    a = z + 1;
  }
  Arrival* arr = arrival_get(dst);
  if (!arr) return PS_ERR_NOMEM;
  const hipError_t er = hipEventRecord(arr->ev, hs);
  if (er != hipSuccess) {
    dst->arrivals_free.push_back(arr);
    return hip_fail(dst, er, "recording the arrival of migrated blocks");
  }
  for (int32_t b : ids) {
    Block& bs = js->blocks[b];
    Block& bd = jd->blocks[b];
    arrival_attach(dst, bd, arr);
    bd.owner = PS_OWNER_HERE;
    bd.round = bs.round;
    bd.mask = 0;
    bs.owner = PS_OWNER_ELSEWHERE;
  }
  return PS_OK;
} PS_NO_THROW

int32_t ps_plan_wave(ps_ctx* c, const ps_block_ref* list, int64_t n, ps_wave_stats* out) try {
  if (!c || !out) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  const int32_t st = validate_list(c, list, n, /*need_pushes=*/true);
  if (st != PS_OK) return st;
  layout_plan(c, list, n, c->plan);
  *out = c->plan.stats;
  return PS_OK;
} PS_NO_THROW

int32_t ps_estimate_wave(ps_ctx* c, const ps_block_ref* list, int64_t n, ps_wave_stats* out) try {
  if (!c || !out) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  const int32_t st = validate_list(c, list, n, /*need_pushes=*/false);
  if (st != PS_OK) return st;
  layout_plan(c, list, n, c->plan);
  *out = c->plan.stats;
  return PS_OK;
} PS_NO_THROW

// The body of ps_aggregate and ps_aggregate_noalloc.  noalloc: the tables go
// into this GPU's static array through the staging buffer of ps_create instead
// of a slot that grows on demand, and no event is created.
static int32_t aggregate_impl(ps_ctx* c, const ps_block_ref* list, int64_t n, void* stream, bool noalloc) {
  if (!c) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  PsStaticScratch* ss = noalloc ? c->sscratch : nullptr;
  ScratchGuard scratch_guard(ss);

  // Steady-state training repeats the same wave with the same gradient buffers:
  // if the previous wave's tables still describe this one, they are used as they
  // are.  The candidate: the static array's tables, or the most recent slot's.
  Slot* cand = noalloc ? &c->static_slot : (c->last_slot >= 0 ? &c->slots[c->last_slot] : nullptr);
  if (cand && (!cand->valid || (noalloc && (!ss || cand->generation != ss->generation)))) cand = nullptr;
  // Same list and no push has recorded a new pointer since the tables were
  // built: the signature is the same without gathering it again.
  const bool same_list = cand && n > 0 && list && cand->plan.ptr_gen == c->ptr_gen &&
                         (int64_t)cand->plan.list.size() == n &&
                         std::memcmp(cand->plan.list.data(), list, (size_t)n * sizeof(ps_block_ref)) == 0;
  int32_t st = validate_list(c, list, n, /*need_pushes=*/true, /*gather_sig=*/!same_list);
  if (st != PS_OK) return st;
  if (n == 0) return PS_OK;
  if (!c->cfg.arena_dev) return PS_ERR_NO_DEVICE;
  if (noalloc && !ss) return PS_ERR_NO_DEVICE;
  bool sig_ready = !same_list;

  // A shard that arrived by migration must not be updated before its copy is
  // complete (the new owner's consistency rule): order this stream after it.
  if (c->n_ready_pending > 0) {
    const Arrival* waited = nullptr;  // blocks that came together sit together: skip repeats
    for (int64_t i = 0; i < n; ++i) {
      Block& b = c->jobs[list[i].job].blocks[list[i].block];
      if (!b.ready) continue;
      if (b.ready != waited) PS_HIP(c, hipStreamWaitEvent(hs, b.ready->ev, 0));
      waited = b.ready;
      arrival_drop(c, b);
    }
  }

  Slot* sp = nullptr;
  bool reuse = cand && (same_list || cand->plan.sig == c->sig);
  if (reuse) {
    // the tables carry each block's round as it was when they were built plus
    // the number of waves since: that must still be every block's round
    const Plan& P = cand->plan;
    for (int64_t i = 0; i < n && reuse; ++i)
      reuse = c->jobs[list[i].job].blocks[list[i].block].round == P.round_at_build[(size_t)i] + P.uses;
  }
  if (reuse) {
    sp = cand;
    if (noalloc) {
      // the array (tables and tile partials) is shared with whatever used it last
      if (ss->in_flight && ss->last_stream != stream)
        PS_HIP(c, hipStreamWaitEvent(hs, static_cast<hipEvent_t>(ss->last), 0));
    } else if (cand->in_flight && cand->stream != hs) {
      // tables and tile partials are shared with the slot's previous wave
      PS_HIP(c, hipStreamWaitEvent(hs, cand->done, 0));
    }
  } else {
    if (noalloc) sp = &c->static_slot;
    if (!sig_ready) gather_signature(c, list, n);
  }
  TimingSet* ts = nullptr;
  if (c->timing_level > 0 && !noalloc) {
    ts = &c->tsets[c->next_tset];
    c->next_tset = (c->next_tset + 1) % kTimingSets;
    st = timing_harvest(c, *ts);
    if (st != PS_OK) return st;
    for (hipEvent_t& e : ts->ev)
      if (!e) PS_HIP(c, hipEventCreate(&e));
    ts->all_phases = c->timing_level >= 2;
    if (ts->all_phases) PS_HIP(c, hipEventRecord(ts->ev[0], hs));
  }
  if (!reuse && noalloc) {
    Slot& s = *sp;
    s.valid = false;
    layout_plan(c, list, n, s.plan);
    const Offsets o = offsets_of(s.plan);
    if (o.total > PS_STATIC_SCRATCH_BYTES) {
      c->last_error = "ps_aggregate_noalloc: the wave's tables need " + std::to_string(o.total) +
                      " bytes of scratch, the static array holds " + std::to_string(PS_STATIC_SCRATCH_BYTES);
      return PS_ERR_CAPACITY;
    }
    // the staging buffer and the array may still be in use by the previous call
    if (ss->in_flight) PS_HIP(c, hipEventSynchronize(static_cast<hipEvent_t>(ss->last)));
    stage_tables(s.plan, o, s.host);
    ss->generation += 1;   // whatever happens next, older tables are gone
    PS_HIP(c, hipMemcpyAsync(ss->ptr, s.host, o.upload, hipMemcpyHostToDevice, hs));
    bind_tables(c, s, o, static_cast<char*>(ss->ptr));
    s.generation = ss->generation;
    s.plan.sig = c->sig;
  } else if (!reuse) {
    c->next_slot = (c->last_slot + 1) % kSlots;
    sp = &c->slots[c->next_slot];
    Slot& s = *sp;
    s.valid = false;
    layout_plan(c, list, n, s.plan);
    const Offsets o = offsets_of(s.plan);
    st = slot_reserve(c, s, o.upload, o.total);
    if (st != PS_OK) return st;
    stage_tables(s.plan, o, s.host);
    PS_HIP(c, hipMemcpyAsync(s.dev, s.host, o.upload, hipMemcpyHostToDevice, hs));
    bind_tables(c, s, o, s.dev);
    s.plan.sig = c->sig;
  }
  Slot& s = *sp;
  PsWaveTables t = s.tables;
  t.round_add = s.plan.uses;
  for (int i = 0; i < 3; ++i) t.ev[i] = ts ? ts->ev[i + 1] : nullptr;
  if (ts && !ts->all_phases) t.ev[2] = nullptr;
  uint32_t launched = 0;
  const int le = ps_launch_wave(t, stream, &launched);
  if (le != 0) {
    s.valid = false;
    if (launched > 0) {
      // Part of the wave is enqueued and will update its blocks: the pushes are
      // spent (a retry must not apply them again) and the wave cannot be taken
      // back.  Which blocks were reached is not known to the caller.
      for (int64_t i = 0; i < n; ++i) {
        Block& b = c->jobs[list[i].job].blocks[list[i].block];
        b.mask = 0;
        b.round += 1;
      }
      (void)hip_fail(c, (hipError_t)le, "launching the wave");
      c->last_error += " (after part of the wave was enqueued: its pushes are consumed, "
                       "the listed blocks' contents are undefined)";
      return PS_ERR_HIP;
    }
    return hip_fail(c, (hipError_t)le, "launching the wave");
  }
  // the wave is enqueued: consume the pushes (before anything else can fail, so
  // that a retry after an error below cannot apply them a second time)
  for (int64_t i = 0; i < n; ++i) {
    Job& j = c->jobs[list[i].job];
    Block& b = j.blocks[list[i].block];
    b.mask = 0;
    b.round += 1;
  }
  s.plan.uses += 1;
  if (ts) {
    ts->pending = true;
    ts->launches = s.plan.stats.n_launches;
  }
  // The tables stay trusted only once the event that guards them is recorded.
  s.valid = false;
  if (noalloc) {
    PS_HIP(c, hipEventRecord(static_cast<hipEvent_t>(ss->last), hs));
    ss->in_flight = true;
    ss->last_stream = stream;
  } else {
    PS_HIP(c, hipEventRecord(s.done, hs));
    s.in_flight = true;
    s.stream = hs;
    c->last_slot = (int)(sp - c->slots);
  }
  s.valid = true;
  return PS_OK;
}

int32_t ps_aggregate(ps_ctx* c, const ps_block_ref* list, int64_t n, void* stream) try {
  return aggregate_impl(c, list, n, stream, /*noalloc=*/false);
} PS_NO_THROW

int32_t ps_aggregate_noalloc(ps_ctx* c, const ps_block_ref* list, int64_t n, void* stream) try {
  return aggregate_impl(c, list, n, stream, /*noalloc=*/true);
} PS_NO_THROW

int32_t ps_pull(ps_ctx* c, ps_job_t job, int32_t block, const float** out_param_dev, int64_t* out_numel) try {
  if (!c || !out_param_dev) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
  if (j->blocks[block].owner == PS_OWNER_ELSEWHERE) return PS_ERR_NOT_OWNER;  // ask the new owner
  if (!j->p) return PS_ERR_NO_DEVICE;
  *out_param_dev = j->p + j->blocks[block].flat_off;
  if (out_numel) *out_numel = j->blocks[block].numel;
  return PS_OK;
} PS_NO_THROW

int32_t ps_pull_momentum(ps_ctx* c, ps_job_t job, int32_t block, const float** out_mom_dev,
                         int64_t* out_numel) try {
  if (!c || !out_mom_dev) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
  if (j->blocks[block].owner == PS_OWNER_ELSEWHERE) return PS_ERR_NOT_OWNER;
  if (!j->v) return PS_ERR_NO_DEVICE;
  *out_mom_dev = j->v + j->blocks[block].flat_off;
  if (out_numel) *out_numel = j->blocks[block].numel;
  return PS_OK;
} PS_NO_THROW

int32_t ps_pull_copy(ps_ctx* c, ps_job_t job, int32_t block, float* dst_dev, void* stream) try {
  if (!c || !dst_dev) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
  const Block& b = j->blocks[block];
  if (b.owner == PS_OWNER_ELSEWHERE) return PS_ERR_NOT_OWNER;
  if (!j->p) return PS_ERR_NO_DEVICE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  // a shard that came by migration and has not been updated here yet: its copy must have landed
  if (b.ready) PS_HIP(c, hipStreamWaitEvent(hs, b.ready->ev, 0));
  PS_HIP(c, hipMemcpyAsync(dst_dev, j->p + b.flat_off, (size_t)b.numel * 4, hipMemcpyDeviceToDevice, hs));
  return PS_OK;
} PS_NO_THROW

int32_t ps_pull_flat(ps_ctx* c, ps_job_t job, const float** out_param_dev, const float** out_mom_dev,
                     int64_t* out_flat_numel) try {
  if (!c) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (!j->p) return PS_ERR_NO_DEVICE;
  if (out_param_dev) *out_param_dev = j->p;
  if (out_mom_dev) *out_mom_dev = j->v;
  if (out_flat_numel) *out_flat_numel = j->flat_numel;
  return PS_OK;
} PS_NO_THROW

int32_t ps_rates(ps_ctx* c, ps_rates_info* out) try {
  if (!c || !out) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  out->read_bytes_per_sec = c->read_rate;
  out->write_bytes_per_sec = c->write_rate;
  out->reserved_[0] = 0;
  out->reserved_[1] = 0;
  return PS_OK;
} PS_NO_THROW

int32_t ps_timing_enable(ps_ctx* c, int32_t on) try {
  if (!c) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  if (!c->cfg.arena_dev) return PS_ERR_NO_DEVICE;
  for (TimingSet& t : c->tsets) {
    const int32_t st = timing_harvest(c, t);
    if (st != PS_OK) return st;
  }
  c->timing = ps_timing{};
  c->timing_level = on <= 0 ? 0 : (on >= 2 ? 2 : 1);
  return PS_OK;
} PS_NO_THROW

int32_t ps_timing_read(ps_ctx* c, ps_timing* out) try {
  if (!c || !out) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  for (TimingSet& t : c->tsets) {
    const int32_t st = timing_harvest(c, t);
    if (st != PS_OK) return st;
  }
  *out = c->timing;
  return PS_OK;
} PS_NO_THROW

int32_t ps_telemetry(ps_ctx* c, ps_job_t job, int32_t block, ps_block_stats* out) try {
  if (!c || !out) return PS_ERR_ARG;
  std::lock_guard<std::mutex> g(c->mu);
  Job* j = find_job(c, job);
  if (!j) return PS_ERR_BAD_JOB;
  if (block < 0 || (size_t)block >= j->blocks.size()) return PS_ERR_BAD_BLOCK;
  // The GPU writes value and round with one 16-byte store; read until two
  // readings agree so that the halves belong together.
  const volatile PsStat* at = j->stat + block;
  PsStat a{at->norm2, at->round};
  for (int tries = 0; tries < 8; ++tries) {
    const PsStat b{at->norm2, at->round};
    const bool same = std::memcmp(&a, &b, sizeof(a)) == 0;
    a = b;
    if (same) break;
  }
  out->grad_norm2 = a.norm2;
  out->round = a.round;
  return PS_OK;
} PS_NO_THROW

}  // extern "C"
