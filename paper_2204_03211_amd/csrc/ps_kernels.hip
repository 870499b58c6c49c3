// gfx950 kernels of one aggregation wave.
//
// Per element of a block (paper, Section 2: the server sums the workers' pushes
// and updates the master copy with the aggregated result):
//     S = ((g_0 + g_1) + ...) + g_{W-1}       binary32, fixed worker order
//     d = S + wd*p ; v' = mu*v + d ; p' = p - lr*v'
// every operation rounded on its own.  The work is a streaming reduction:
// (4W + 16) bytes of HBM traffic per parameter against W + 7 flops, so the
// kernels are built around 16-byte coalesced loads with many of them in flight
// per lane; there is no contraction here for the matrix cores to do.
//
// Build with -ffp-contract=off; the pragma below says the same to the compiler
// for this translation unit regardless of the command line.
#include <hip/hip_runtime.h>

#include "ps_internal.h"

#pragma clang fp contract(off)

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int PS_MAX_W_UNROLLED = 16;  // largest worker count with a fully unrolled tile body

__device__ __forceinline__ f32x4 load_stream(const float* a) {
  // gradients, parameters and momentum are touched once per wave: keep them
  // from displacing anything useful in L2
  return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a));
}
__device__ __forceinline__ void store_stream(float* a, f32x4 x) {
  __builtin_nontemporal_store(x, reinterpret_cast<f32x4*>(a));
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

__device__ __forceinline__ double wave_sum(double a) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) a += __shfl_xor(a, m, 64);
  return a;
}

// A full tile: PS_TILE_ELEMS elements, no bounds checks.  W > 0 is a
// compile-time worker count (loads of all streams can be issued up front);
// W == 0 takes the count at run time.
template <int W, bool FMA>
__device__ __forceinline__ double tile_full(const float* const* __restrict__ gp, uint32_t w_rt,
                                            float* __restrict__ p, float* __restrict__ v, float lr,
                                            float mu, float wd, uint32_t tid) {
  constexpr int U = PS_TILE_QUADS_PER_LANE;
  f32x4 acc[U];
  const uint32_t nw = W > 0 ? (uint32_t)W : w_rt;
  {
    const float* g0 = gp[0];
#pragma unroll
    for (int u = 0; u < U; ++u) acc[u] = load_stream(g0 + (u * PS_WG + tid) * 4);
  }
  if constexpr (W > 0) {
#pragma unroll
    for (int w = 1; w < W; ++w) {
      const float* gw = gp[w];
#pragma unroll
      for (int u = 0; u < U; ++u) acc[u] = acc[u] + load_stream(gw + (u * PS_WG + tid) * 4);
    }
  } else {
    for (uint32_t w = 1; w < nw; ++w) {
      const float* gw = gp[w];
#pragma unroll
      for (int u = 0; u < U; ++u) acc[u] = acc[u] + load_stream(gw + (u * PS_WG + tid) * 4);
    }
  }
  double a = 0.0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t e = (u * PS_WG + tid) * 4;
    f32x4 pp = load_stream(p + e);
    f32x4 vv = load_stream(v + e);
    a = update4<FMA>(acc[u], pp, vv, lr, mu, wd, a);
    store_stream(p + e, pp);
    store_stream(v + e, vv);
  }
  return a;
}

// Any run of len elements starting at a 16-byte aligned address: whole quads
// with 16-byte accesses, the last 1..3 elements one by one.
template <bool FMA>
__device__ __forceinline__ double quad_any(const float* const* __restrict__ gp, uint32_t nw,
                                           float* __restrict__ p, float* __restrict__ v, float lr,
                                           float mu, float wd, uint32_t e, uint32_t rem) {
  double a = 0.0;
  if (rem >= 4) {
    f32x4 s = load_stream(gp[0] + e);
    for (uint32_t w = 1; w < nw; ++w) s = s + load_stream(gp[w] + e);
    f32x4 pp = load_stream(p + e);
    f32x4 vv = load_stream(v + e);
    a = update4<FMA>(s, pp, vv, lr, mu, wd, a);
    store_stream(p + e, pp);
    store_stream(v + e, vv);
  } else {
    for (uint32_t k = 0; k < rem; ++k) {
      float s = gp[0][e + k];
      for (uint32_t w = 1; w < nw; ++w) s = s + gp[w][e + k];
      float pk = p[e + k], vk = v[e + k];
      update1<FMA>(s, pk, vk, lr, mu, wd);
      p[e + k] = pk;
      v[e + k] = vk;
      const double sd = (double)s;
      a = __builtin_fma(sd, sd, a);
    }
  }
  return a;
}

// ---------------------------------------------------------------------------
// Large path: one workgroup per tile of a block.
// ---------------------------------------------------------------------------
template <bool FMA>
__global__ __launch_bounds__(PS_WG) void ps_agg_large(const PsBlockDesc* __restrict__ desc,
                                                      const float* const* __restrict__ gptr,
                                                      const PsTile* __restrict__ tiles,
                                                      double* __restrict__ tile_part) {
  const uint32_t t = blockIdx.x;
  const uint32_t tid = threadIdx.x;
  const PsTile te = tiles[t];
  const uint32_t di = __builtin_amdgcn_readfirstlane(te.desc);
  const uint32_t off = __builtin_amdgcn_readfirstlane(te.off);
  const PsBlockDesc* __restrict__ d = desc + di;
  const uint32_t n = d->n, W = d->W;
  const float lr = d->lr, mu = d->mu, wd = d->wd;
  float* __restrict__ p = d->p + off;
  float* __restrict__ v = d->v + off;
  const float* const* __restrict__ gp0 = gptr + d->gofs;
  const uint32_t len = min(PS_TILE_ELEMS, n - off);

  double a = 0.0;
  if (len == PS_TILE_ELEMS) {
    // the tile's W gradient pointers, advanced to the tile (uniform: SGPRs)
    const float* gp[PS_MAX_W_UNROLLED];
    switch (W) {
#define PS_CASE(WW)                                                            \
  case WW: {                                                                   \
    _Pragma("unroll") for (int w = 0; w < WW; ++w) gp[w] = gp0[w] + off;       \
    a = tile_full<WW, FMA>(gp, WW, p, v, lr, mu, wd, tid);                     \
  } break;
      PS_CASE(1)
      PS_CASE(2)
      PS_CASE(4)
      PS_CASE(8)
      PS_CASE(16)
#undef PS_CASE
      default: {
        // any other worker count: run-time loop over a pointer table advanced on the fly
        constexpr int U = PS_TILE_QUADS_PER_LANE;
        f32x4 acc[U];
        const float* g0 = gp0[0] + off;
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = load_stream(g0 + (u * PS_WG + tid) * 4);
        for (uint32_t w = 1; w < W; ++w) {
          const float* gw = gp0[w] + off;
#pragma unroll
          for (int u = 0; u < U; ++u) acc[u] = acc[u] + load_stream(gw + (u * PS_WG + tid) * 4);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t e = (u * PS_WG + tid) * 4;
          f32x4 pp = load_stream(p + e);
          f32x4 vv = load_stream(v + e);
          a = update4<FMA>(acc[u], pp, vv, lr, mu, wd, a);
          store_stream(p + e, pp);
          store_stream(v + e, vv);
        }
      }
    }
  } else {
    // ragged last tile of a block
    for (uint32_t q = tid; q * 4 < len; q += PS_WG) {
      const uint32_t e = q * 4;
      // quad_any indexes the gradient streams from the block start
      a += quad_any<FMA>(gp0, W, d->p, d->v, lr, mu, wd, off + e, len - e);
    }
  }

  a = wave_sum(a);
  __shared__ double red[PS_WG / 64];
  if ((tid & 63) == 0) red[tid >> 6] = a;
  __syncthreads();
  if (tid == 0) tile_part[t] = ((red[0] + red[1]) + red[2]) + red[3];
}

// ---------------------------------------------------------------------------
// Small path: one workgroup per bin of tiny blocks.  Descriptors and the bin's
// quad prefix are staged in LDS; lanes are spread over the concatenated quads of
// all blocks in the bin, so a 64-element bias next to a 1000-element one still
// fills whole wavefronts with 16-byte accesses.  Per-quad telemetry partials go
// through LDS and are reduced per block in a fixed order.
// ---------------------------------------------------------------------------
template <bool FMA>
__global__ __launch_bounds__(PS_WG) void ps_agg_small(const PsBlockDesc* __restrict__ desc,
                                                      const float* const* __restrict__ gptr,
                                                      const PsSmallEntry* __restrict__ entries,
                                                      const PsBin* __restrict__ bins) {
  __shared__ PsBlockDesc sd[PS_BIN_MAX_BLOCKS];
  __shared__ uint32_t qs[PS_BIN_MAX_BLOCKS + 1];
  __shared__ double qpart[PS_BIN_MAX_QUADS];

  const uint32_t tid = threadIdx.x;
  const PsBin bin = bins[blockIdx.x];
  const uint32_t count = bin.count, quads = bin.quads;
  if (tid < count) {
    const PsSmallEntry e = entries[bin.first + tid];
    sd[tid] = desc[e.desc];
    qs[tid] = e.qstart;
  }
  if (tid == 0) qs[count] = quads;
  __syncthreads();

  for (uint32_t q = tid; q < quads; q += PS_WG) {
    uint32_t lo = 0, hi = count;  // largest lo with qs[lo] <= q
    while (hi - lo > 1) {
      const uint32_t mid = (lo + hi) >> 1;
      if (qs[mid] <= q) lo = mid; else hi = mid;
    }
    const PsBlockDesc& d = sd[lo];
    const uint32_t e = (q - qs[lo]) * 4;
    qpart[q] = quad_any<FMA>(gptr + d.gofs, d.W, d.p, d.v, d.lr, d.mu, d.wd, e, d.n - e);
  }
  __syncthreads();

  const uint32_t lane = tid & 63, wave = tid >> 6;
  for (uint32_t j = wave; j < count; j += PS_WG / 64) {
    double a = 0.0;
    for (uint32_t q = qs[j] + lane; q < qs[j + 1]; q += 64) a += qpart[q];
    a = wave_sum(a);
    if (lane == 0) *sd[j].stat = a;
  }
}

// ---------------------------------------------------------------------------
// Telemetry of large-path blocks: one wavefront adds up a block's tile partials.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(PS_WG) void ps_block_norms(const PsBlockDesc* __restrict__ desc,
                                                        const uint32_t* __restrict__ large_blocks,
                                                        uint32_t n_large,
                                                        const double* __restrict__ tile_part) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t b = blockIdx.x * (PS_WG / 64) + (threadIdx.x >> 6);
  if (b >= n_large) return;  // whole wavefront leaves together
  const PsBlockDesc* d = desc + large_blocks[b];
  double a = 0.0;
  for (uint32_t t = lane; t < d->ntiles; t += 64) a += tile_part[d->tile0 + t];
  a = wave_sum(a);
  if (lane == 0) *d->stat = a;
}

}  // namespace

int ps_launch_wave(const PsWaveTables& t, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  auto mark = [&](int i) {
    if (t.ev[i]) (void)hipEventRecord(static_cast<hipEvent_t>(t.ev[i]), stream);
  };
  mark(0);
  if (t.n_tiles) {
    if (t.fp_contract)
      hipLaunchKernelGGL(ps_agg_large<true>, dim3(t.n_tiles), dim3(PS_WG), 0, stream, t.desc, t.gptr,
                         t.tiles, t.tile_part);
    else
      hipLaunchKernelGGL(ps_agg_large<false>, dim3(t.n_tiles), dim3(PS_WG), 0, stream, t.desc, t.gptr,
                         t.tiles, t.tile_part);
  }
  mark(1);
  if (t.n_bins) {
    if (t.fp_contract)
      hipLaunchKernelGGL(ps_agg_small<true>, dim3(t.n_bins), dim3(PS_WG), 0, stream, t.desc, t.gptr,
                         t.small_entries, t.bins);
    else
      hipLaunchKernelGGL(ps_agg_small<false>, dim3(t.n_bins), dim3(PS_WG), 0, stream, t.desc, t.gptr,
                         t.small_entries, t.bins);
  }
  mark(2);
  if (t.n_large_blocks) {
    const uint32_t per = PS_WG / 64;
    hipLaunchKernelGGL(ps_block_norms, dim3((t.n_large_blocks + per - 1) / per), dim3(PS_WG), 0,
                       stream, t.desc, t.large_blocks, t.n_large_blocks, t.tile_part);
  }
  mark(3);
  return (int)hipGetLastError();
}
