// Oracle for model aggregation in a parameter service -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, single-threaded CPU statement of what the aggregation path
// computes.  It exists so that tests can check the GPU library against it and
// so that the benchmark can time it as a CPU baseline.  It shares no code with
// the GPU library and nothing in the product path may call it.
//
// What is computed (paper, Section 2 "Background and Motivation": the server
// holds the master copy of the parameters and updates it with the aggregated
// result of the workers' pushes; Section 2.2 "Tensor-Based Model Structure":
// tensors are aggregated independently of each other; Section 2.1: a tensor's
// aggregation can start only when its backward pass is done, so gradients
// arrive last layer first).  The paper leaves the optimizer, the precision and
// the order of summation open.  The readings taken here:
//   * gradients, parameters, momentum are IEEE-754 binary32;
//   * the aggregate is the SUM over workers, taken strictly left to right in
//     worker index starting from worker 0's value;
//   * the update is heavy-ball momentum SGD with weight decay folded into the
//     gradient:  d = S + wd*p ;  v' = mu*v + d ;  p' = p - lr*v' ;
//   * every operation is a separately rounded binary32 operation (no fused
//     multiply-add);  build with -ffp-contract=off and without fast-math;
//   * the telemetry value of a block is sum_i S[i]^2, accumulated in binary64.
//
// Pins: tests/test_oracle_*.py check these functions against closed forms of
// the momentum recurrence, hand-derived IEEE rounding cases, torch.optim.SGD,
// published parameter counts and block-independence invariants.

#include <cstdint>

extern "C" {

// ---------------------------------------------------------------------------
// Splitting a layer (tensor) into blocks: as many full blocks of cap elements
// as fit, then one remainder block.  Writes (layer, offset in layer, numel) for
// every block of every layer in registration order.  Returns the number of
// blocks, or -1 if out_cap is too small or an argument is invalid.
// ---------------------------------------------------------------------------
int64_t orc_split_layers(const int64_t* layer_numel, int32_t n_layers, int64_t cap_elems,
                         int32_t* out_layer, int64_t* out_offset, int64_t* out_numel,
                         int64_t out_cap) {
  if (cap_elems <= 0 || n_layers < 0) return -1;
  int64_t nb = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    int64_t n = layer_numel[l];
    if (n <= 0) return -1;
    int64_t off = 0;
    while (off < n) {
      int64_t len = n - off;
      if (len > cap_elems) len = cap_elems;
      if (nb >= out_cap) return -1;
      out_layer[nb] = l;
      out_offset[nb] = off;
      out_numel[nb] = len;
      ++nb;
      off += len;
    }
  }
  return nb;
}

// ---------------------------------------------------------------------------
// Arrival order of one job's blocks within an iteration: back-propagation
// finishes the last registered layer first; the blocks of one layer keep
// ascending offset.  block_layer[b] is the layer of block b (blocks numbered in
// registration order).  Writes the block ids in arrival order.
// ---------------------------------------------------------------------------
void orc_arrival_order(const int32_t* block_layer, int32_t n_blocks, int32_t* out_order) {
  int32_t k = 0;
  int32_t end = n_blocks;  // one past the last block of the current layer
  while (end > 0) {
    int32_t begin = end - 1;
    while (begin > 0 && block_layer[begin - 1] == block_layer[end - 1]) --begin;
    for (int32_t b = begin; b < end; ++b) out_order[k++] = b;
    end = begin;
  }
}

// ---------------------------------------------------------------------------
// Interleaving several jobs' arrival sequences into one wave.  The k-th block
// (0-based) of a job with n blocks sits at fractional position (k + 1/2) / n of
// the iteration; the wave lists all (job, k) by ascending position, ties by job
// index.  Positions are compared as exact fractions.  Selection is done the
// slow way: repeatedly take the smallest head among the jobs.
// ---------------------------------------------------------------------------
void orc_interleave(const int32_t* n_blocks_per_job, int32_t n_jobs, int32_t* out_job,
                    int32_t* out_k) {
  int64_t total = 0;
  for (int32_t j = 0; j < n_jobs; ++j) total += n_blocks_per_job[j];
  // head[j] = next k of job j; kept in the output arrays' tail is not needed
  int32_t* head = new int32_t[n_jobs > 0 ? n_jobs : 1];
  for (int32_t j = 0; j < n_jobs; ++j) head[j] = 0;
  for (int64_t t = 0; t < total; ++t) {
    int32_t best = -1;
    for (int32_t j = 0; j < n_jobs; ++j) {
      if (head[j] >= n_blocks_per_job[j]) continue;
      if (best < 0) { best = j; continue; }
      // (2*kj+1)/(2*nj) < (2*kb+1)/(2*nb)  <=>  (2*kj+1)*nb < (2*kb+1)*nj
      __int128 lhs = (__int128)(2 * (int64_t)head[j] + 1) * n_blocks_per_job[best];
      __int128 rhs = (__int128)(2 * (int64_t)head[best] + 1) * n_blocks_per_job[j];
      if (lhs < rhs) best = j;  // strict: ties keep the lower job index
    }
    out_job[t] = best;
    out_k[t] = head[best]++;
  }
  delete[] head;
}

// ---------------------------------------------------------------------------
// One aggregation of one block: W gradient arrays g[0..W-1], each n floats;
// p and v are updated in place; *norm2 receives sum_i S[i]^2.
// ---------------------------------------------------------------------------
void orc_aggregate_block(int32_t W, int64_t n, const float* const* g, float* p, float* v,
                         float lr, float mu, float wd, double* norm2) {
  double acc = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    float s = g[0][i];
    for (int32_t w = 1; w < W; ++w) s = s + g[w][i];
    float t = wd * p[i];
    float d = s + t;
    float u = mu * v[i];
    float vn = u + d;
    float q = lr * vn;
    float pn = p[i] - q;
    v[i] = vn;
    p[i] = pn;
    acc += (double)s * (double)s;
  }
  if (norm2) *norm2 = acc;
}

// The aggregate alone (the sum step), for tests that pin the summation order.
void orc_sum_block(int32_t W, int64_t n, const float* const* g, float* out) {
  for (int64_t i = 0; i < n; ++i) {
    float s = g[0][i];
    for (int32_t w = 1; w < W; ++w) s = s + g[w][i];
    out[i] = s;
  }
}

}  // extern "C"
