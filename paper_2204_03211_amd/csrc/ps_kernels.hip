// gfx950 kernels of one aggregation wave.
//
// Per element of a block (paper, Section 2: the server sums the workers' pushes
// and updates the master copy with the aggregated result):
//     S = ((g_0 + g_1) + ...) + g_{W-1}       binary32, fixed worker order
//     d = S + wd*p ; v' = mu*v + d ; p' = p - lr*v'
// every operation rounded on its own.  The work is a streaming reduction:
// (4W + 16) bytes of HBM traffic per parameter against W + 7 flops, so the
// kernels are built around 16-byte coalesced accesses with many of them in
// flight per lane; there is no contraction here for the matrix cores to do.
//
// Build with -ffp-contract=off; the pragma below says the same to the compiler
// for this translation unit regardless of the command line.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "ps_internal.h"

#pragma clang fp contract(off)

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// Cache policy of every streaming access: non-temporal.  Gradients, parameters
// and momentum are touched once per wave; measured on MI355X the hint is worth
// about 10 % of bandwidth on loads and on stores alike.
constexpr int kStream = 2;  // the "nt" bit of the buffer instructions' cache-policy field

// A raw buffer descriptor over `bytes` bytes at p.  Dword-x4 buffer accesses are
// range-checked per component: components past the end load as zero and are not
// stored, which is how a block's ragged tail is handled without a scalar path.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t span(const float* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ f32x4 load4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kStream));
}
__device__ __forceinline__ void store4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, f32x4 x) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(i32x4, x), r, byte_off, 0, kStream);
}

template <bool FMA>
__device__ __forceinline__ void update1(float s, float& p, float& v, float lr, float mu, float wd) {
  if constexpr (FMA) {
    const float d = __builtin_fmaf(wd, p, s);
    const float vn = __builtin_fmaf(mu, v, d);
    p = __builtin_fmaf(-lr, vn, p);
    v = vn;
  } else {
    const float t = wd * p;
    const float d = s + t;
    const float u = mu * v;
    const float vn = u + d;
    const float q = lr * vn;
    p = p - q;
    v = vn;
  }
}

template <bool FMA>
__device__ __forceinline__ double update4(f32x4 s, f32x4& p, f32x4& v, float lr, float mu,
                                          float wd, double a) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float pk = p[k], vk = v[k];
    update1<FMA>(s[k], pk, vk, lr, mu, wd);
    p[k] = pk;
    v[k] = vk;
    const double sd = (double)s[k];
    a = __builtin_fma(sd, sd, a);  // sd*sd is exact in binary64: same as mul then add
  }
  return a;
}

// Value and round leave together in one 16-byte store, so that a reader never
// pairs a new round with an old value.
__device__ __forceinline__ void put_stat(PsStat* dst, double norm2, int64_t round) {
  const PsStat s{norm2, round};
  *reinterpret_cast<i32x4*>(dst) = __builtin_bit_cast(i32x4, s);
}

__device__ __forceinline__ double wave_sum(double a) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) a += __shfl_xor(a, m, 64);
  return a;
}

// ---------------------------------------------------------------------------
// Large path: one tile (up to PS_TILE_ELEMS elements of one block) per
// workgroup.  W > 0: worker count known at compile time, so the loads of all
// W + 2 streams are issued before the first add.  W == 0: run-time count.
// ---------------------------------------------------------------------------
template <int W, bool FMA>
__device__ __forceinline__ double tile_body(const PsBlockRec* __restrict__ r,
                                            const float* const* __restrict__ gp, uint32_t w_rt,
                                            uint32_t off, uint32_t bytes, uint32_t tid,
                                            unsigned long long t_start, uint32_t hold_ticks) {
  constexpr int U = PS_TILE_QUADS_PER_LANE;
  constexpr int G = PS_LOAD_G;  // workers whose loads are in flight together (bounds VGPR use)
  const float lr = r->lr, mu = r->mu, wd = r->wd;
  f32x4 acc[U];
  {
    const __amdgpu_buffer_rsrc_t g0 = span(gp[0] + off, bytes);
#pragma unroll
    for (int u = 0; u < U; ++u) acc[u] = load4(g0, (u * PS_WG + tid) * 16);
  }
  if constexpr (W > 0) {
#pragma unroll
    for (int w0 = 1; w0 < W; w0 += G) {
      f32x4 x[G][U];
#pragma unroll
      for (int g = 0; g < G; ++g)
        if (w0 + g < W) {
          const __amdgpu_buffer_rsrc_t gw = span(gp[w0 + g] + off, bytes);
#pragma unroll
          for (int u = 0; u < U; ++u) x[g][u] = load4(gw, (u * PS_WG + tid) * 16);
        }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < G; ++g)
        if (w0 + g < W) {
#pragma unroll
          for (int u = 0; u < U; ++u) acc[u] = acc[u] + x[g][u];  // worker order: w0, w0+1, ...
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    for (uint32_t w = 1; w < w_rt; ++w) {
      const __amdgpu_buffer_rsrc_t gw = span(gp[w] + off, bytes);
#pragma unroll
      for (int u = 0; u < U; ++u) acc[u] = acc[u] + load4(gw, (u * PS_WG + tid) * 16);
    }
  }
  const __amdgpu_buffer_rsrc_t rp = span(r->p + off, bytes), rv = span(r->v + off, bytes);
  f32x4 pp[U], vv[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    pp[u] = load4(rp, (u * PS_WG + tid) * 16);
    vv[u] = load4(rv, (u * PS_WG + tid) * 16);
  }
  double a = 0.0;
#pragma unroll
  for (int u = 0; u < U; ++u) a = update4<FMA>(acc[u], pp[u], vv[u], lr, mu, wd, a);
  // The results now sit in registers.  Every workgroup of the launch started at
  // about t_start; waiting until hold_ticks later lets the launch's reads drain
  // before its writes begin (the caller has added this workgroup's place in
  // the launch's release order).  The clock always advances, so the wait ends.
#pragma unroll
  for (int u = 0; u < U; ++u) asm volatile("" : "+v"(pp[u]), "+v"(vv[u]));  // no sinking past the wait
  while ((uint32_t)(wall_clock64() - t_start) < hold_ticks) __builtin_amdgcn_s_sleep(8);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    store4(rp, (u * PS_WG + tid) * 16, pp[u]);
    store4(rv, (u * PS_WG + tid) * 16, vv[u]);
  }
  return a;
}

template <int W, bool FMA>
__device__ __forceinline__ void large_tile(const unsigned char* __restrict__ recs, PsTile te,
                                           uint32_t slot, double* __restrict__ tile_part,
                                           uint32_t hold_ticks) {
  const unsigned long long t_start = wall_clock64();
  const uint32_t tid = threadIdx.x;
  const uint32_t ro = __builtin_amdgcn_readfirstlane(te.rec);
  const uint32_t off = __builtin_amdgcn_readfirstlane(te.off);
  const PsBlockRec* __restrict__ r =
      reinterpret_cast<const PsBlockRec*>(recs + (size_t)ro * PS_REC_UNIT);
  const float* const* __restrict__ gp = reinterpret_cast<const float* const*>(r + 1);
  const uint32_t left = r->n - off;
  const uint32_t bytes = (left < PS_TILE_ELEMS ? left : PS_TILE_ELEMS) * 4;

  double a = tile_body<W, FMA>(r, gp, r->W, off, bytes, tid, t_start, hold_ticks);

  a = wave_sum(a);
  __shared__ double red[PS_WG / 64];
  if ((tid & 63) == 0) red[tid >> 6] = a;
  __syncthreads();
  if (tid == 0) tile_part[slot] = ((red[0] + red[1]) + red[2]) + red[3];
}

// ---------------------------------------------------------------------------
// Small path: one workgroup per bin of tiny blocks.  Record headers, the bin's
// quad prefix and all gradient pointers of the bin are staged in LDS; lanes are
// spread over the concatenated 16-byte quads of all blocks in the bin, so a
// 64-element bias next to a 1000-element one still fills whole wavefronts with
// 16-byte accesses.  Per-quad telemetry partials go through LDS and are reduced
// per block in a fixed order.
// ---------------------------------------------------------------------------
__device__ __forceinline__ f32x4 gload4(const float* a) {
  return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a));
}

template <bool FMA>
__device__ __forceinline__ void small_bin(const unsigned char* __restrict__ recs,
                                          const PsSmallEntry* __restrict__ entries, PsBin bin,
                                          long long round_add) {
  __shared__ PsBlockRec sd[PS_BIN_MAX_BLOCKS];
  __shared__ uint32_t srec[PS_BIN_MAX_BLOCKS];
  __shared__ uint32_t qs[PS_BIN_MAX_BLOCKS + 1];   // first quad of each entry
  __shared__ uint32_t ps[PS_BIN_MAX_BLOCKS + 1];   // first pointer of each entry
  __shared__ const float* sptr[PS_BIN_MAX_PTRS];
  __shared__ double qpart[PS_BIN_MAX_QUADS];
  static_assert(sizeof(PsBlockRec) * PS_BIN_MAX_BLOCKS + 4 * PS_BIN_MAX_BLOCKS + 8 * (PS_BIN_MAX_BLOCKS + 1) +
                        8 * PS_BIN_MAX_PTRS + 8 * PS_BIN_MAX_QUADS + 8 * (PS_WG / 64) <= 160 * 1024 / 8,
                "eight workgroups of this kernel must fit in one CU's LDS");

  const uint32_t tid = threadIdx.x;
  const uint32_t count = bin.count, quads = bin.quads, nptrs = bin.nptrs;
  if (tid < count) {
    const PsSmallEntry e = entries[bin.first + tid];
    const PsBlockRec* r = reinterpret_cast<const PsBlockRec*>(recs + (size_t)e.rec * PS_REC_UNIT);
    sd[tid] = *r;
    srec[tid] = e.rec;
    qs[tid] = e.qstart;
    ps[tid] = e.pstart;
  }
  if (tid == 0) {
    qs[count] = quads;
    ps[count] = nptrs;
  }
  __syncthreads();
  for (uint32_t i = tid; i < nptrs; i += PS_WG) {
    uint32_t lo = 0, hi = count;  // largest lo with ps[lo] <= i
    while (hi - lo > 1) {
      const uint32_t mid = (lo + hi) >> 1;
      if (ps[mid] <= i) lo = mid; else hi = mid;
    }
    const float* const* gp = reinterpret_cast<const float* const*>(
        recs + (size_t)srec[lo] * PS_REC_UNIT + sizeof(PsBlockRec));
    sptr[i] = gp[i - ps[lo]];
  }
  __syncthreads();

  for (uint32_t q = tid; q < quads; q += PS_WG) {
    uint32_t lo = 0, hi = count;  // largest lo with qs[lo] <= q
    while (hi - lo > 1) {
      const uint32_t mid = (lo + hi) >> 1;
      if (qs[mid] <= q) lo = mid; else hi = mid;
    }
    const PsBlockRec& d = sd[lo];
    const float* const* gp = sptr + ps[lo];
    const uint32_t e = (q - qs[lo]) * 4;
    const uint32_t rem = d.n - e;
    const uint32_t nw = d.W;
    const float lr = d.lr, mu = d.mu, wd = d.wd;
    double a = 0.0;
    if (rem >= 4) {
      f32x4 s = gload4(gp[0] + e);
      uint32_t w = 1;
      for (; w + 4 <= nw; w += 4) {  // four loads in flight, added in worker order
        const f32x4 x0 = gload4(gp[w] + e), x1 = gload4(gp[w + 1] + e);
        const f32x4 x2 = gload4(gp[w + 2] + e), x3 = gload4(gp[w + 3] + e);
        s = s + x0; s = s + x1; s = s + x2; s = s + x3;
      }
      for (; w < nw; ++w) s = s + gload4(gp[w] + e);
      f32x4 pp = gload4(d.p + e), vv = gload4(d.v + e);
      a = update4<FMA>(s, pp, vv, lr, mu, wd, a);
      __builtin_nontemporal_store(pp, reinterpret_cast<f32x4*>(d.p + e));
      __builtin_nontemporal_store(vv, reinterpret_cast<f32x4*>(d.v + e));
    } else {
      for (uint32_t k = 0; k < rem; ++k) {
        float s = gp[0][e + k];
        for (uint32_t w = 1; w < nw; ++w) s = s + gp[w][e + k];
        float pk = d.p[e + k], vk = d.v[e + k];
        update1<FMA>(s, pk, vk, lr, mu, wd);
        d.p[e + k] = pk;
        d.v[e + k] = vk;
        const double sdb = (double)s;
        a = __builtin_fma(sdb, sdb, a);
      }
    }
    qpart[q] = a;
  }
  __syncthreads();

  const uint32_t lane = tid & 63, wave = tid >> 6;
  for (uint32_t j = wave; j < count; j += PS_WG / 64) {
    double a = 0.0;
    for (uint32_t q = qs[j] + lane; q < qs[j + 1]; q += 64) a += qpart[q];
    a = wave_sum(a);
    if (lane == 0) put_stat(sd[j].stat, a, sd[j].round0 + round_add);
  }
}

#ifndef PS_MIN_WAVES
#define PS_MIN_WAVES 1
#endif
// One launch: workgroups [0, n_bins) take small-path bins, the rest take tiles
// tile_begin .. of the large path.  All tiles of one launch belong to blocks with
// the same worker count; W > 0 names it at compile time (every gradient load of
// a tile is then issued before the first add), W == 0 reads it from the record.
template <int W, bool FMA>
__global__ __launch_bounds__(PS_WG, PS_MIN_WAVES) void ps_agg_wave(const unsigned char* __restrict__ recs,
                                                     const PsTile* __restrict__ tiles,
                                                     uint32_t tile_begin,
                                                     double* __restrict__ tile_part,
                                                     const PsSmallEntry* __restrict__ entries,
                                                     const PsBin* __restrict__ bins,
                                                     uint32_t n_bins, uint32_t hold_ticks,
                                                     uint32_t stagger_q16, long long round_add) {
  const uint32_t b = blockIdx.x;
  if (b < n_bins) {
    small_bin<FMA>(recs, entries, bins[b], round_add);
  } else {
    const uint32_t i = b - n_bins;
    const uint32_t t = tile_begin + i;
    // Stores are released in index order, which is address order: workgroup i
    // waits stagger_q16 / 65536 ticks longer than workgroup i - 1, so that the
    // launch's writes reach HBM as one paced sweep instead of one burst.
    const uint32_t hold = hold_ticks ? hold_ticks + ((i * stagger_q16) >> 16) : 0u;
    large_tile<W, FMA>(recs, tiles[t], t, tile_part, hold);
  }
}

// ---------------------------------------------------------------------------
// Telemetry of large-path blocks: one wavefront adds up a block's tile partials.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(PS_WG) void ps_block_norms(const unsigned char* __restrict__ recs,
                                                        const uint32_t* __restrict__ large_recs,
                                                        uint32_t n_large,
                                                        const double* __restrict__ tile_part,
                                                        long long round_add) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t b = blockIdx.x * (PS_WG / 64) + (threadIdx.x >> 6);
  if (b >= n_large) return;  // whole wavefront leaves together
  const PsBlockRec* d =
      reinterpret_cast<const PsBlockRec*>(recs + (size_t)large_recs[b] * PS_REC_UNIT);
  double a = 0.0;
  for (uint32_t t = lane; t < d->ntiles; t += 64) a += tile_part[d->tile0 + t];
  a = wave_sum(a);
  if (lane == 0) put_stat(d->stat, a, d->round0 + round_add);
}

// ---------------------------------------------------------------------------
// Migration copy: a workgroup moves one tile (PS_TILE_ELEMS floats) of the
// parameter array and the same tile of the momentum array.  All eight loads of
// a lane are issued before its first store; ragged ends are left to the buffer
// range check.  Launched like the aggregation: no more workgroups than the chip
// holds at once, and every workgroup keeps what it has read in registers until
// the launch's reads are due to be over (hold_ticks of the wall clock after its
// own start, plus its place in the release order as in the aggregation; the
// clock always advances, so the wait ends).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(PS_WG) void ps_copy_shards(const float* __restrict__ src_p,
                                                        float* __restrict__ dst_p,
                                                        const float* __restrict__ src_v,
                                                        float* __restrict__ dst_v,
                                                        unsigned long long n, uint32_t first_tile,
                                                        uint32_t hold_ticks, uint32_t stagger_q16) {
  const unsigned long long t_start = wall_clock64();
  const uint32_t hold = hold_ticks ? hold_ticks + ((blockIdx.x * stagger_q16) >> 16) : 0u;
  constexpr int U = PS_TILE_QUADS_PER_LANE;
  // < n by the grid's size
  const unsigned long long at = ((unsigned long long)first_tile + blockIdx.x) * PS_TILE_ELEMS;
  const unsigned long long left = n - at;
  const uint32_t bytes = (uint32_t)(left < PS_TILE_ELEMS ? left : PS_TILE_ELEMS) * 4;
  const uint32_t tid = threadIdx.x;
  const __amdgpu_buffer_rsrc_t sp = span(src_p + at, bytes), sv = span(src_v + at, bytes);
  const __amdgpu_buffer_rsrc_t dp = span(dst_p + at, bytes), dv = span(dst_v + at, bytes);
  f32x4 a[U], b[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    a[u] = load4(sp, (u * PS_WG + tid) * 16);
    b[u] = load4(sv, (u * PS_WG + tid) * 16);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) asm volatile("" : "+v"(a[u]), "+v"(b[u]));  // loaded before the wait
  while ((uint32_t)(wall_clock64() - t_start) < hold) __builtin_amdgcn_s_sleep(8);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    store4(dp, (u * PS_WG + tid) * 16, a[u]);
    store4(dv, (u * PS_WG + tid) * 16, b[u]);
  }
}

// Zero n floats at p (16-byte aligned): a job's shards at registration.
__global__ __launch_bounds__(PS_WG) void ps_zero_shards(float* __restrict__ p, unsigned long long n) {
  constexpr int U = PS_TILE_QUADS_PER_LANE;
  const unsigned long long at = (unsigned long long)blockIdx.x * PS_TILE_ELEMS;  // < n by the grid's size
  const unsigned long long left = n - at;
  const uint32_t bytes = (uint32_t)(left < PS_TILE_ELEMS ? left : PS_TILE_ELEMS) * 4;
  const __amdgpu_buffer_rsrc_t d = span(p + at, bytes);
  const f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int u = 0; u < U; ++u) store4(d, (u * PS_WG + threadIdx.x) * 16, z);
}

template <int W, bool FMA>
hipError_t launch_one(const PsWaveTables& t, hipStream_t stream, uint32_t tile_begin, uint32_t n_tiles,
                      uint32_t n_bins, uint32_t hold_ticks, uint32_t stagger_q16 = 0) {
  hipLaunchKernelGGL((ps_agg_wave<W, FMA>), dim3(n_tiles + n_bins), dim3(PS_WG), 0, stream, t.recs,
                     t.tiles, tile_begin, t.tile_part, t.small_entries, t.bins, n_bins, hold_ticks,
                     stagger_q16, (long long)t.round_add);
  return hipGetLastError();
}

// Returns the first launch error; *launched counts the launches that went in before it.
template <bool FMA>
hipError_t launch_agg(const PsWaveTables& t, hipStream_t stream, uint32_t* launched) {
  uint32_t bins_left = t.n_bins;
  if (t.n_chunks == 0 && bins_left) {
    const hipError_t e = launch_one<0, FMA>(t, stream, 0, 0, bins_left, 0);
    if (e == hipSuccess) *launched += 1;
    return e;
  }
  for (uint32_t c = 0; c < t.n_chunks; ++c) {
    const PsChunk& ch = t.chunks[c];
    const uint32_t nt = ch.end - ch.begin;
    hipError_t e;
    // the bins ride with the first launch so that they overlap with tile work
    switch (ch.W) {
      case 1: e = launch_one<1, FMA>(t, stream, ch.begin, nt, bins_left, ch.hold_ticks, ch.stagger_q16); break;
      case 2: e = launch_one<2, FMA>(t, stream, ch.begin, nt, bins_left, ch.hold_ticks, ch.stagger_q16); break;
      case 4: e = launch_one<4, FMA>(t, stream, ch.begin, nt, bins_left, ch.hold_ticks, ch.stagger_q16); break;
      case 8: e = launch_one<8, FMA>(t, stream, ch.begin, nt, bins_left, ch.hold_ticks, ch.stagger_q16); break;
      case 16: e = launch_one<16, FMA>(t, stream, ch.begin, nt, bins_left, ch.hold_ticks, ch.stagger_q16); break;
      default: e = launch_one<0, FMA>(t, stream, ch.begin, nt, bins_left, ch.hold_ticks, ch.stagger_q16); break;
    }
    if (e != hipSuccess) return e;
    *launched += 1;
    bins_left = 0;
  }
  return hipSuccess;
}

}  // namespace

template <int W>
static uint32_t resident_of(int cus) {
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, ps_agg_wave<W, false>, PS_WG, 0) != hipSuccess)
    return 0;
  return per_cu > 0 ? (uint32_t)(per_cu * cus) : 0;
}

uint32_t ps_resident_workgroups(uint32_t W) {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return 0;
  switch (W) {
    case 1: return resident_of<1>(cus);
    case 2: return resident_of<2>(cus);
    case 4: return resident_of<4>(cus);
    case 8: return resident_of<8>(cus);
    case 16: return resident_of<16>(cus);
    default: return resident_of<0>(cus);
  }
}

// ---------------------------------------------------------------------------
// Static scratch.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the device address is looked up once per device, with
// that device current, and everything else uses that address.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
struct StaticScratchSlot {
  PsStaticScratch pub{};
  std::mutex use;      // held for the length of one call that uses the array
  bool ready = false;
};
StaticScratchSlot g_static[kMaxDevices];
std::mutex g_static_setup;
}  // namespace

int ps_static_scratch(PsStaticScratch** out) {
  *out = nullptr;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> g(g_static_setup);
  StaticScratchSlot& s = g_static[dev];
  if (!s.ready) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!ptr) return (int)hipErrorInvalidSymbol;
    hipEvent_t ev = nullptr;
    e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e != hipSuccess) return (int)e;
    s.pub.ptr = ptr;
    s.pub.last = ev;
    s.pub.last_stream = nullptr;
    s.pub.in_flight = false;
    s.pub.generation = 0;
    s.pub.use_mutex = &s.use;
    s.ready = true;
  }
  *out = &s.pub;
  return 0;
}

void ps_static_scratch_lock(PsStaticScratch* s) {
  static_cast<std::mutex*>(s->use_mutex)->lock();
}
void ps_static_scratch_unlock(PsStaticScratch* s) {
  static_cast<std::mutex*>(s->use_mutex)->unlock();
}

uint32_t ps_resident_copy_workgroups() {
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0 ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, ps_copy_shards, PS_WG, 0) != hipSuccess || per_cu <= 0)
    return 0;
  return (uint32_t)(per_cu * cus);
}

int ps_launch_copy(const float* src_p, float* dst_p, const float* src_v, float* dst_v, uint64_t n,
                   void* stream_, uint32_t launch_tiles, double hold_ticks_per_tile, uint32_t stagger_q16) {
  if (n == 0) return 0;
  const uint64_t tiles = (n + PS_TILE_ELEMS - 1) / PS_TILE_ELEMS;
  if (tiles > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
  const bool resident_known = launch_tiles != 0;
  if (!resident_known) launch_tiles = 0x7FFFFFFFu;   // one launch, and no hold: later generations would wait again
  (void)hipGetLastError();
  for (uint64_t t = 0; t < tiles; t += launch_tiles) {
    const uint32_t m = (uint32_t)std::min<uint64_t>(launch_tiles, tiles - t);
    // never longer than half a millisecond at the clock's nominal 100 MHz
    const uint32_t hold = resident_known ? (uint32_t)std::min(hold_ticks_per_tile * m, 5.0e4) : 0u;
    hipLaunchKernelGGL(ps_copy_shards, dim3(m), dim3(PS_WG), 0, static_cast<hipStream_t>(stream_),
                       src_p, dst_p, src_v, dst_v, (unsigned long long)n, (uint32_t)t, hold,
                       resident_known ? stagger_q16 : 0u);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

int ps_launch_zero(float* p, uint64_t n, void* stream_) {
  if (n == 0) return 0;
  const uint64_t tiles = (n + PS_TILE_ELEMS - 1) / PS_TILE_ELEMS;
  if (tiles > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(ps_zero_shards, dim3((uint32_t)tiles), dim3(PS_WG), 0, static_cast<hipStream_t>(stream_), p,
                     (unsigned long long)n);
  return (int)hipGetLastError();
}

int ps_launch_wave(const PsWaveTables& t, void* stream_, uint32_t* launched) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  auto mark = [&](int i) {
    if (t.ev[i]) (void)hipEventRecord(static_cast<hipEvent_t>(t.ev[i]), stream);
  };
  *launched = 0;
  (void)hipGetLastError();  // an error left behind by an earlier, unrelated call is not this wave's
  mark(0);
  hipError_t e = t.fp_contract ? launch_agg<true>(t, stream, launched) : launch_agg<false>(t, stream, launched);
  if (e != hipSuccess) return (int)e;
  mark(1);
  if (t.n_large_blocks) {
    const uint32_t per = PS_WG / 64;
    hipLaunchKernelGGL(ps_block_norms, dim3((t.n_large_blocks + per - 1) / per), dim3(PS_WG), 0,
                       stream, t.recs, t.large_recs, t.n_large_blocks, t.tile_part, (long long)t.round_add);
    e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    *launched += 1;
  }
  mark(2);
  return 0;
}
