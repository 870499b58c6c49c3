// Tables shared by the host-side service and the gfx950 kernels of one wave.
// Everything here is plain data laid out for scalar (wave-uniform) loads.
#ifndef PS_INTERNAL_H_
#define PS_INTERNAL_H_

#include <stddef.h>
#include <stdint.h>

// One block of one job as the kernels see it: a 64-byte header followed
// directly by the block's W gradient pointers (worker order).  Header and
// pointers are fetched together once a tile names the record.
// Telemetry of one block as the GPU leaves it in host-visible memory: the value
// and the round it belongs to, written together with one 16-byte store.
struct PsStat {
  double norm2;   // sum S^2 of the block's last aggregation
  int64_t round;  // the block's round counter after that aggregation
};
static_assert(sizeof(PsStat) == 16, "value and round travel in one 16-byte store");

struct PsBlockRec {
  float* p;          // parameter shard (device, 256-byte aligned)
  float* v;          // momentum shard
  PsStat* stat;      // where this block's telemetry goes (host-visible memory, 16-byte aligned)
  uint32_t n;        // elements in the block
  uint32_t W;        // workers
  uint32_t tile0;    // large path: first of this block's entries in the tile-partials array
  uint32_t ntiles;   // large path: number of tiles
  float lr, mu, wd;
  uint32_t pad_;
  int64_t round0;    // round the block reaches in the wave these tables were built for;
                     // a later wave that reuses the tables adds the number of reuses
  // const float* grad[W] follows
};
static_assert(sizeof(PsBlockRec) == 64, "record header must stay 64 bytes");

// Records live in one byte array; they are named by their offset in 8-byte units.
constexpr uint32_t PS_REC_UNIT = 8;

// Large path: one workgroup per tile = (record, first element of the tile).
struct PsTile {
  uint32_t rec;
  uint32_t off;
};

// Small path: one workgroup per bin of consecutive entries.  An entry names a
// record and the position of the block's first 16-byte quad in the bin.
struct PsSmallEntry {
  uint32_t rec;
  uint32_t qstart;  // first quad of the block in the bin
  uint32_t pstart;  // first gradient pointer of the block in the bin's pointer list
  uint32_t pad_;
};
struct PsBin {
  uint32_t first;   // first entry
  uint32_t count;   // entries in the bin (<= PS_BIN_MAX_BLOCKS)
  uint32_t quads;   // total quads (<= PS_BIN_MAX_QUADS)
  uint32_t nptrs;   // gradient pointers of all entries together (<= PS_BIN_MAX_PTRS)
};

// A contiguous run of tiles, all of blocks with the same worker count W,
// launched as one kernel.
struct PsChunk {
  uint32_t begin, end;
  uint32_t W;
  uint32_t hold_ticks;  // wall-clock ticks a workgroup keeps its results before storing them
  uint32_t stagger_q16; // extra hold per workgroup index, in 1/65536 ticks
  uint32_t pad_;
  uint64_t read_bytes;  // bytes the launch reads: sum over its tiles of (4W + 8) * elements
};

constexpr uint32_t PS_WG = 256;                 // threads per workgroup (4 wavefronts)
#ifndef PS_TILE_U
#define PS_TILE_U 4
#endif
#ifndef PS_LOAD_G
#define PS_LOAD_G 2   // workers whose loads are in flight together: 62 VGPRs, 8 waves per SIMD
#endif
constexpr uint32_t PS_TILE_QUADS_PER_LANE = PS_TILE_U;  // 16-byte accesses per lane per stream in a tile
constexpr uint32_t PS_TILE_ELEMS = PS_WG * 4 * PS_TILE_QUADS_PER_LANE;
constexpr uint32_t PS_BIN_MAX_BLOCKS = 64;
constexpr uint32_t PS_BIN_MAX_QUADS = 1024;  // >= quads of the largest small-path block
// The bin tables sit in LDS (19 264 bytes a workgroup with these sizes); 8
// workgroups per CU must fit in the CU's 160 KiB, or the large path loses residency.
constexpr uint32_t PS_BIN_MAX_PTRS = 768;
constexpr uint32_t PS_SMALL_MAX_ELEMS = 4096;   // largest block the small path accepts

// Tiles per launch of the large path, by worker count.  HBM serves pure reads
// and pure writes much faster than a fine interleaving of many read streams with
// a few write streams, so a wave is cut into launches small enough to be resident
// on the chip all at once: their workgroups start together, read together, keep
// their results in registers until most of the launch's reads are done
// (hold_ticks) and then write, one after the other in address order.
inline uint32_t ps_chunk_tiles(uint32_t W) { (void)W; return 1u << 20; }  // i.e. whatever is resident

// Rates of the two phases of a launch, fitted on MI355X to the launch times of
// the aggregation kernel (time = bytes read / READ + bytes written / WRITE +
// a fixed cost; full launches of W = 2, 4, 8, 16 measure 30.3, 39.8, 59.5, 97.7
// us, the fit gives 30.2, 39.7, 58.9, 97.3): they predict when a launch's reads
// end, and how long a wave takes (ps_wave_stats.est_seconds).  The first workgroup of a launch starts to
// store when PS_DEFAULT_HOLD_PERMILLE / 1000 of the launch's predicted read
// time has passed, a little before the last reads are in; workgroup i (index
// order = address order) waits i * (the time one tile's stores take at the READ
// rate) * PS_DEFAULT_STAGGER_PERMILLE / 1000 longer, so the launch's writes
// arrive as one paced ascending sweep over about the time they need anyway
// instead of as one burst.  Measured on the 12-job wave (kernel GB/s; hold x
// stagger): all at once 960: 6550; 940/960/980/1000/1020 with 835: 6599 / 6673 /
// 6728 / 6693 / 6632; 980 with 750/800/870/900/950: 6650 / 6694 / 6713 / 6698 / 6664;
// a spread of 1200 or more loses 5 % and more.
constexpr double PS_READ_BYTES_PER_SEC = 7.0e12;
constexpr uint32_t PS_DEFAULT_HOLD_PERMILLE = 980;
constexpr double PS_WRITE_BYTES_PER_SEC = 7.0e12;
constexpr uint32_t PS_DEFAULT_STAGGER_PERMILLE = 835;
constexpr uint32_t PS_COPY_STAGGER_PERMILLE = 835;
constexpr double PS_EST_LAUNCH_SECONDS = 1.4e-6;
// A copy's launches write as much as they read; measured on MI355X they are
// fastest when the stores start at 900/1000 of the predicted read time (800:
// -3 %, 1000: -2 %, 1100: -6 %, no hold: -10 %).
constexpr uint32_t PS_COPY_HOLD_PERMILLE = 900;
constexpr double PS_EST_WAVE_SECONDS = 5.0e-6;

struct PsWaveTables {
  const unsigned char* recs;     // PsBlockRec records
  const PsTile* tiles;           // sorted so that tiles of one worker count are adjacent
  uint32_t n_tiles;
  const PsChunk* chunks;         // HOST array: launch ranges over tiles
  uint32_t n_chunks;
  double* tile_part;             // n_tiles doubles, device scratch
  const PsSmallEntry* small_entries;
  const PsBin* bins;
  uint32_t n_bins;
  const uint32_t* large_recs;    // record offsets of large-path blocks
  uint32_t n_large_blocks;
  bool fp_contract;
  int64_t round_add;             // waves launched with these tables before this one
  // optional hipEvent_t handles recorded before the first launch, after the
  // aggregation launches, and after the telemetry reduction (NULL = no timing)
  void* ev[3];
};

// Workgroups of the aggregation kernel for worker count W that the current
// device holds at once; 0 if it cannot be queried.
uint32_t ps_resident_workgroups(uint32_t W);

// Enqueue the kernels of one wave on stream (a hipStream_t).  Returns a
// hipError_t value (0 = success); stops at the first launch the runtime
// refuses.  *launched = kernels enqueued before that.
int ps_launch_wave(const PsWaveTables& t, void* stream, uint32_t* launched);

// Enqueue on stream the copy of n floats of parameters and n floats of momentum
// (both pairs 16-byte aligned) from one context's shards to another's: the
// TENSOR_COPY of a migration.  The copy is cut into launches of launch_tiles
// workgroups (what the chip holds at once; 0 = unknown: one launch); a launch
// of m tiles keeps what it read for hold_ticks_per_tile * m ticks of the wall
// clock before it stores (0 = no hold), workgroup i for i * stagger_q16 / 65536
// ticks longer.  Returns a hipError_t value (0 = success).
int ps_launch_copy(const float* src_p, float* dst_p, const float* src_v, float* dst_v, uint64_t n,
                   void* stream, uint32_t launch_tiles, double hold_ticks_per_tile, uint32_t stagger_q16);
// Workgroups of the copy kernel the current device holds at once; 0 if unknown.
uint32_t ps_resident_copy_workgroups();

// Enqueue on stream the zeroing of n floats at p (16-byte aligned) with a fill
// kernel (no memset node, so the call may sit inside a captured graph).
int ps_launch_zero(float* p, uint64_t n, void* stream);

// ---------------------------------------------------------------------------
// Scratch memory that exists without any allocation: one file-scope device
// array per GPU, for callers that may not allocate (ps_aggregate_noalloc).  It
// holds what a slot's device buffer holds: the wave's tables and the tile
// partials.  Every use on a GPU, from whatever context or stream, is ordered
// after the previous use through `last` (an event created at set-up).
// ---------------------------------------------------------------------------
constexpr size_t PS_STATIC_SCRATCH_BYTES = 8u << 20;
struct PsStaticScratch {
  void* ptr;          // device address of this GPU's copy of the array
  void* last;         // hipEvent_t recorded after the most recent use
  void* last_stream;  // stream of that use
  bool in_flight;     // `last` has been recorded at least once
  uint64_t generation;  // bumped whenever new tables are copied into the array
  void* use_mutex;    // std::mutex held for the length of one call that uses the array
};
// The scratch of the current device, set up on first use per device (address
// looked up with the device current, event created).  Returns a hipError_t
// value (0 = success).  Guard every use with ps_static_scratch_lock/unlock.
int ps_static_scratch(PsStaticScratch** out);
void ps_static_scratch_lock(PsStaticScratch* s);
void ps_static_scratch_unlock(PsStaticScratch* s);

#endif  // PS_INTERNAL_H_
