// Grid-wise keep-set sampler: one thread per 2x2 cell (plus one per prefix row).
//
// The paper ("How to sample the gradient keep mask?") asks for a structured sample that is
// drawn afresh every step and visits every position equally often; it gives no algorithm.
// Here every 2x2 cell keeps k of its 4 slots, the slot permutation coming from a
// SplitMix64-style counter hash of (seed, stream_id, sample, cell).  Integer arithmetic
// only; the position of every cell's output in idx is a closed form, so no scan is needed.
#include "sbp_internal.h"

namespace sbp {

static constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

__host__ __device__ static inline uint64_t splitmix_out(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__host__ __device__ static inline uint64_t absorb(uint64_t h, uint64_t v) { return splitmix_out(h + v + kGamma); }

// kept slots of an edge cell with c valid slots: round-half-up(k*c/4), at least 1
__host__ __device__ static inline int k_partial(int k, int c) {
  int v = (k * c + 2) >> 2;
  return v < 1 ? 1 : v;
}

struct SampleGeom {
  int B, P, H, W, k, shared, per_sample;
  int ch, cw;         // cells per column / row (partial cells included)
  int fh, fw;         // full cells per column / row
  int k2, k1;         // kept slots of 2-slot and 1-slot edge cells
  int row_full;       // idx entries produced by one row of cells with two valid grid rows
  int per_sample_K;   // idx entries per sample
  int N;              // rows per sample
  uint64_t base;      // hash of (seed, stream_id)
};

static SampleGeom make_geom(const sbp_sample_desc& d) {
  SampleGeom g;
  g.B = d.B; g.P = d.P; g.H = d.H; g.W = d.W; g.k = d.k;
  g.shared = d.mode == SBP_GRID_SHARED; g.per_sample = d.per_sample;
  g.ch = (d.H + 1) / 2; g.cw = (d.W + 1) / 2; g.fh = d.H / 2; g.fw = d.W / 2;
  g.k2 = k_partial(d.k, 2); g.k1 = k_partial(d.k, 1);
  g.row_full = d.k * g.fw + (d.W & 1) * g.k2;
  int row_last = g.k2 * g.fw + (d.W & 1) * g.k1;
  g.per_sample_K = d.P + g.fh * g.row_full + (d.H & 1) * row_last;
  g.N = d.P + d.H * d.W;
  g.base = absorb(absorb(0, d.seed), d.stream_id);
  return g;
}

int64_t keep_count_host(const sbp_sample_desc& d) {
  SampleGeom g = make_geom(d);
  return (int64_t)g.B * g.per_sample_K;
}

// One work item: a prefix row or a cell of sample b.
__host__ __device__ static inline void sample_unit(const SampleGeom& g, long long t, int32_t* __restrict__ idx,
                                                   int32_t* __restrict__ inv) {
  const int units = g.P + g.ch * g.cw;              // work items per sample
  {
    const int b = (int)((unsigned)t / (unsigned)units);       // t < B * units < 2^31 (row ids are int32)
    const int u = (int)t - b * units;
    const int row0 = b * g.N;
    const int out0 = b * g.per_sample_K;
    if (u < g.P) {                                   // always-kept prefix row
      idx[out0 + u] = row0 + u;
      if (inv) inv[row0 + u] = out0 + u;
      return;
    }
    const int c = u - g.P;
    const int cy = c / g.cw, cx = c - cy * g.cw;
    const bool two_rows = cy < g.fh, two_cols = cx < g.fw;
    // position of this cell's first entry inside the sample's part of idx
    const int per_cell = two_rows ? g.k : g.k2;      // entries of each full-width cell in this cell row
    const int off = g.P + cy * g.row_full + cx * per_cell;   // rows above are all two-row rows
    uint64_t h = absorb(g.base, g.per_sample ? (uint64_t)b : 0ull);
    h = absorb(h, g.shared ? 0ull : (uint64_t)c);
    const uint32_t p = (uint32_t)(((h >> 32) * 24ull) >> 32);        // [0, 24)
    const uint32_t dig[3] = {p / 6u, (p % 6u) >> 1, p & 1u};
    // Lehmer decode: the t-th placed slot is the dig[t]-th slot still free
    uint32_t freem = 0xFu, order = 0;                 // order: 2 bits per rank -> slot
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      uint32_t want = r < 3 ? dig[r] : 0u, seen = 0, pick = 0;
#pragma unroll
      for (uint32_t s = 0; s < 4; ++s) {
        bool isfree = (freem >> s) & 1u;
        if (isfree && seen == want) pick = s;
        seen += isfree ? 1u : 0u;
      }
      freem &= ~(1u << pick);
      order |= pick << (2 * r);
    }
    const uint32_t valid = (two_rows ? 0xFu : 0x3u) & (two_cols ? 0xFu : 0x5u);
    const int nvalid = (two_rows ? 2 : 1) * (two_cols ? 2 : 1);
    const int kc = nvalid == 4 ? g.k : (nvalid == 2 ? g.k2 : g.k1);
    uint32_t keepm = 0;
    int taken = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {                     // walk slots by increasing rank
      uint32_t s = (order >> (2 * r)) & 3u;
      if (((valid >> s) & 1u) && taken < kc) { keepm |= 1u << s; ++taken; }
    }
    int pos = out0 + off;
#pragma unroll
    for (uint32_t s = 0; s < 4; ++s) {                // emit in ascending slot number
      if (!((valid >> s) & 1u)) continue;
      const int row = row0 + g.P + (2 * cy + (int)(s >> 1)) * g.W + 2 * cx + (int)(s & 1u);
      if ((keepm >> s) & 1u) {
        idx[pos] = row;
        if (inv) inv[row] = pos;
        ++pos;
      } else if (inv) {
        inv[row] = -1;
      }
    }
  }
}

__global__ void __launch_bounds__(256) sample_kernel(SampleGeom g, int32_t* __restrict__ idx,
                                                     int32_t* __restrict__ inv) {
  const long long total = (long long)g.B * (g.P + g.ch * g.cw);
  for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < total;
       t += (long long)gridDim.x * blockDim.x)
    sample_unit(g, t, idx, inv);
}

int32_t launch_sample(const sbp_sample_desc& d, int32_t* idx, int32_t* inv, hipStream_t s) {
  SampleGeom g = make_geom(d);
  long long total = (long long)g.B * (g.P + g.ch * g.cw);
  int blocks = (int)((total + 255) / 256);
  if (blocks > 65535) blocks = 65535;
  SBP_LAUNCH(SBP_PROF_SAMPLE, s, sample_kernel, dim3(blocks), dim3(256), 0, s, g, idx, inv);
  return check_launch("sample_kernel");
}

}  // namespace sbp
