// Tables shared by the host-side service and the gfx950 kernels of one wave.
// Everything here is plain data laid out for scalar (wave-uniform) loads.
#ifndef PS_INTERNAL_H_
#define PS_INTERNAL_H_

#include <stdint.h>

// One block of one job as the kernels see it.  64 bytes so that a descriptor
// never straddles a cache line and can be fetched with four s_load_dwordx4.
struct PsBlockDesc {
  float* p;          // parameter shard (device, 256-byte aligned)
  float* v;          // momentum shard
  double* stat;      // where sum S^2 of this block goes (host-visible memory)
  uint32_t gofs;     // index of worker 0's pointer in the wave's gradient-pointer table
  uint32_t n;        // elements in the block
  uint32_t W;        // workers
  uint32_t tile0;    // large path: first of this block's entries in the tile-partials array
  uint32_t ntiles;   // large path: number of tiles
  float lr, mu, wd;
  uint32_t pad_[2];
};
static_assert(sizeof(PsBlockDesc) == 64, "descriptor must stay 64 bytes");

// Large path: one workgroup per tile = (descriptor, first element).
struct PsTile {
  uint32_t desc;
  uint32_t off;
};

// Small path: one workgroup per bin of consecutive entries.  An entry names a
// descriptor and the position of the block's first 16-byte quad in the bin.
struct PsSmallEntry {
  uint32_t desc;
  uint32_t qstart;
};
struct PsBin {
  uint32_t first;   // first entry
  uint32_t count;   // entries in the bin (<= PS_BIN_MAX_BLOCKS)
  uint32_t quads;   // total quads (<= PS_BIN_MAX_QUADS)
  uint32_t pad_;
};

constexpr uint32_t PS_WG = 256;                 // threads per workgroup (4 wavefronts)
constexpr uint32_t PS_TILE_QUADS_PER_LANE = 4;  // 16-byte loads per lane per stream in a full tile
constexpr uint32_t PS_TILE_ELEMS = PS_WG * 4 * PS_TILE_QUADS_PER_LANE;  // 4096
constexpr uint32_t PS_BIN_MAX_BLOCKS = 64;
constexpr uint32_t PS_BIN_MAX_QUADS = 2048;

struct PsWaveTables {
  const PsBlockDesc* desc;
  const float* const* gptr;
  const PsTile* tiles;
  uint32_t n_tiles;
  double* tile_part;             // n_tiles doubles, device scratch
  const PsSmallEntry* small_entries;
  const PsBin* bins;
  uint32_t n_bins;
  const uint32_t* large_blocks;  // descriptor indices of large-path blocks
  uint32_t n_large_blocks;
  bool fp_contract;
  // optional hipEvent_t handles recorded before the large kernel and after each
  // of the three kernels (all NULL = no timing)
  void* ev[4];
};

// Enqueue the kernels of one wave on stream (a hipStream_t).  Returns a
// hipError_t value (0 = success).
int ps_launch_wave(const PsWaveTables& t, void* stream);

#endif  // PS_INTERNAL_H_
