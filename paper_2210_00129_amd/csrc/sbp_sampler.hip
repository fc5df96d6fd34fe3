// Grid-wise keep-set sampler: one thread per cell (plus one per prefix row); 2 x 2 cells, and 3 x 3 / 4 x 4 further down.
//
// The paper ("How to sample the gradient keep mask?") asks for a structured sample that is
// drawn afresh every step and visits every position equally often; it gives no algorithm.
// Here every 2x2 cell keeps k of its 4 slots, the slot permutation coming from a
// SplitMix64-style counter hash of (seed, stream_id, sample, cell).  Integer arithmetic
// only; the position of every cell's output in idx is a closed form, so no scan is needed.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <mutex>

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

// ---- cells of 3 x 3 and 4 x 4 slots (keep ratios k/9 and k/16) ---------------------------------------
// Same hash chain, same canonical order.  The permutation of the n = cell^2 slots is Lehmer-decoded from
// p = floor(h n! / 2^64) (digit t, most significant first, picks the d_t-th slot not yet placed); the k slots of
// smallest rank are kept; an edge cell with v valid slots keeps max(1, round-half-up(k v / n)) of them.
struct CellGeom {
  int B, P, H, W, k, cell, shared, per_sample;
  int cw, fh, fw, rh, rw;     // cells per row; full cells per column / row; rows / columns of the partial cells
  int k_fe, k_ef, k_ee;       // kept slots of right-edge, bottom-edge and corner cells
  int row_full, row_last;     // idx entries of a row of full-height cells / of the partial last row
  int units;                  // work items per sample: prefix rows + cells
  int per_sample_K, N;
  uint64_t base;
};
__host__ __device__ static inline int k_partial_cell(int k, int valid, int slots) {
  const int v = (2 * k * valid + slots) / (2 * slots);
  return v < 1 ? 1 : v;
}
static CellGeom make_cell_geom(const sbp_sample_desc& d) {
  CellGeom g;
  const int c = d.cell, n = c * c;
  g.B = d.B; g.P = d.P; g.H = d.H; g.W = d.W; g.k = d.k; g.cell = c;
  g.shared = d.mode == SBP_GRID_SHARED; g.per_sample = d.per_sample;
  g.cw = (d.W + c - 1) / c; g.fh = d.H / c; g.fw = d.W / c; g.rh = d.H % c; g.rw = d.W % c;
  g.k_fe = g.rw ? k_partial_cell(d.k, c * g.rw, n) : 0;
  g.k_ef = g.rh ? k_partial_cell(d.k, g.rh * c, n) : 0;
  g.k_ee = (g.rh && g.rw) ? k_partial_cell(d.k, g.rh * g.rw, n) : 0;
  g.row_full = d.k * g.fw + g.k_fe;
  g.row_last = g.k_ef * g.fw + g.k_ee;
  const int ch = (d.H + c - 1) / c;
  g.units = d.P + ch * g.cw;
  g.per_sample_K = d.P + g.fh * g.row_full + (g.rh ? g.row_last : 0);
  g.N = d.P + d.H * d.W;
  g.base = absorb(absorb(0, d.seed), d.stream_id);
  return g;
}

// ---- the other samplers: same row numbering, same hash --------------------------------------------------
// random mask: exactly n_keep of the H*W grid positions of a sample, those with the smallest (key, position),
// key = absorb(h_sample, position); temporal subsets: H frames of W positions, k of every `cell` frames kept whole.
static inline int random_keep(const sbp_sample_desc& d) {
  const long long v = ((long long)d.k * d.H * d.W + 2) / 4;
  return (int)(v < 1 ? 1 : v);
}
static inline int temporal_tail_keep(int k, int tail, int c) {
  const int v = (2 * k * tail + c) / (2 * c);
  return v < 1 ? 1 : v;
}
static inline int temporal_keep_frames(const sbp_sample_desc& d) {
  const int tail = d.H % d.cell;
  return d.k * (d.H / d.cell) + (tail ? temporal_tail_keep(d.k, tail, d.cell) : 0);
}

int64_t keep_count_host(const sbp_sample_desc& d) {
  if (d.mode == SBP_RANDOM_MASK) return (int64_t)d.B * (d.P + random_keep(d));
  if (d.mode == SBP_TEMPORAL) return (int64_t)d.B * (d.P + (int64_t)temporal_keep_frames(d) * d.W);
  if (d.cell != 2) {
    const CellGeom c = make_cell_geom(d);
    return (int64_t)c.B * c.per_sample_K;
  }
  SampleGeom g = make_geom(d);
  return (int64_t)g.B * g.per_sample_K;
}

struct VariantGeom {
  int B, P, H, W, k, cell, per_sample;
  int N;              // rows per sample
  int n_keep;         // random mask: kept grid positions per sample; temporal: kept frames per sample
  int tail_keep;      // temporal: kept frames of the partial last cell
  uint64_t base;
  uint64_t win_lo, win_hi;   // random mask on large maps: the n_keep-th smallest key is expected in [win_lo, win_hi)
  int mask_chunks;           // random mask on large maps: chunks of 64 positions whose keep bits fit the dynamic LDS (0: none)
};

// Random mask: one block per sample.  The n_keep-th smallest key is found by a radix select over the 64-bit
// keys, 8 bits per pass from the top, the keys being recomputed from the hash in every pass (nothing is
// stored); a last pass writes the kept positions in ascending order with a block-wide running count.
// Equal keys (never seen in practice, but possible) are broken by position, smallest first.
// WINDOW (large maps): the keys are uniform, so that key lies near n_keep / n * 2^64.  One pass over the positions
// counts the keys below a window around that value and collects the keys inside it in LDS; if the wanted rank
// falls into the window (it does unless the hash misbehaves by many standard deviations) the radix select runs
// over those few keys instead of recomputing all hashes eight times; otherwise the full select runs as before.
// The ordered write-out of a large map keeps one 64-bit "below" and one "equal" mask per chunk of 64 positions in
// LDS (one hash pass, a ballot per chunk), scans the chunk counts once, and every wavefront then writes its chunks
// without further barriers; where the masks do not fit (mask_chunks == 0) the chunked loop of the small maps runs.
template <int NT, bool WINDOW>
__global__ void __launch_bounds__(NT) sample_random_kernel(VariantGeom g, int32_t* __restrict__ idx,
                                                           int32_t* __restrict__ inv) {
  constexpr int NWAVE = NT / 64, CAP = WINDOW ? 4096 : 1;
  __shared__ uint64_t cand[CAP];
  __shared__ int cand_pos[CAP];                      // position of every collected key (large maps with keep bits in LDS)
  __shared__ int s_ncand, s_below;
  __shared__ int hist[256];
  __shared__ uint64_t s_prefix;
  __shared__ int s_remaining;
  __shared__ int s_wave_lt[NWAVE], s_wave_eq[NWAVE];
  __shared__ int s_run_lt, s_run_eq;
  const int b = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int n = g.H * g.W;
  const uint64_t hb = absorb(g.base, g.per_sample ? (uint64_t)b : 0ull);
  const int row0 = b * g.N, out0 = b * (g.P + g.n_keep);
  for (int p = t; p < g.P; p += NT) {
    idx[out0 + p] = row0 + p;
    if (inv) inv[row0 + p] = out0 + p;
  }
  bool windowed = false;                             // uniform over the block
  int ncand = 0, want = g.n_keep;
  if (WINDOW) {
    if (t == 0) { s_ncand = 0; s_below = 0; }
    __syncthreads();
    int below = 0;
    if (g.mask_chunks > 0) {
      // chunk by chunk: the keys below the window are kept whatever the threshold turns out to be - their keep bits
      // are written now, the collected keys remember their positions, and no second pass over the hash is needed
      extern __shared__ __attribute__((aligned(16))) unsigned long long dyn0[];
      unsigned long long* m_lt0 = dyn0;
      unsigned long long* m_eq0 = dyn0 + g.mask_chunks;
      for (int c = wave; c < g.mask_chunks; c += NWAVE) {
        const int p = 64 * c + lane;
        bool lt = false;
        if (p < n) {
          const uint64_t key = absorb(hb, (uint64_t)p);
          lt = key < g.win_lo;
          if (!lt && key < g.win_hi) {
            const int slot = atomicAdd(&s_ncand, 1);
            if (slot < CAP) { cand[slot] = key; cand_pos[slot] = p; }
          }
        }
        const unsigned long long mlt = __ballot(lt);
        if (lane == 0) { m_lt0[c] = mlt; m_eq0[c] = 0ull; }
        below += lt ? 1 : 0;
      }
    } else {
      for (int p = t; p < n; p += NT) {
        const uint64_t key = absorb(hb, (uint64_t)p);
        if (key < g.win_lo) {
          ++below;
        } else if (key < g.win_hi) {
          const int slot = atomicAdd(&s_ncand, 1);
          if (slot < CAP) cand[slot] = key;
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) below += __shfl_xor(below, o, 64);
    if (lane == 0) atomicAdd(&s_below, below);
    __syncthreads();
    ncand = s_ncand;
    const int rank = g.n_keep - s_below;             // 1-based rank of the wanted key among the collected ones
    windowed = ncand <= CAP && rank >= 1 && rank <= ncand;
    if (windowed) want = rank;
  }
  if (t == 0) { s_prefix = 0; s_remaining = want; }
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
    if (t < 256) hist[t] = 0;
    __syncthreads();
    const uint64_t prefix = s_prefix;
    if (windowed) {
      for (int i = t; i < ncand; i += NT) {
        const uint64_t key = cand[i];
        if (pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(int)((key >> shift) & 255u)], 1);
      }
    } else {
      for (int p = t; p < n; p += NT) {
        const uint64_t key = absorb(hb, (uint64_t)p);
        if (pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(int)((key >> shift) & 255u)], 1);
      }
    }
    __syncthreads();
    // bucket in which the running count reaches what is still wanted: inclusive scan of the 256 counts
    // by the first four wavefronts
    const int rem = s_remaining;
    int incl = t < 256 ? hist[t] : 0;
    const int mine = incl;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, 64);
      if (lane >= o) incl += v;
    }
    if (lane == 63 && wave < 4) s_wave_lt[wave] = incl;     // (scratch reuse: totals of the four wavefronts)
    __syncthreads();
    for (int w = 0; w < wave && w < 4; ++w) incl += s_wave_lt[w];
    const int excl = incl - mine;
    __syncthreads();                                // everyone has read s_remaining / s_prefix / s_wave_lt
    if (t < 256 && excl < rem && rem <= incl) {     // exactly one thread
      s_remaining = rem - excl;                     // keys still to take inside the chosen bucket
      s_prefix = prefix | ((uint64_t)t << shift);
    }
    __syncthreads();
  }
  const uint64_t thr = s_prefix;                    // the n_keep-th smallest key
  const int take_eq = s_remaining;                  // how many keys equal to it are kept (smallest positions first)
  if (WINDOW && g.mask_chunks > 0) {
    extern __shared__ __attribute__((aligned(16))) unsigned long long dyn[];
    const int nchunks = g.mask_chunks;              // = ceil(n / 64)
    unsigned long long* m_lt = dyn;
    unsigned long long* m_eq = dyn + nchunks;
    int* pre_lt = reinterpret_cast<int*>(dyn + 2 * nchunks);
    int* pre_eq = pre_lt + nchunks;
    __syncthreads();                                // s_prefix / s_remaining read by everyone
    if (windowed) {
      // the keys below the window already have their bits; of the collected keys those below the threshold get theirs
      // now, those equal to it go to the "equal" mask (the write-out keeps the take_eq smallest positions of them)
      for (int i = t; i < ncand; i += NT) {
        const uint64_t key = cand[i];
        const int p = cand_pos[i];
        if (key < thr) atomicOr(&m_lt[p >> 6], 1ull << (p & 63));
        else if (key == thr) atomicOr(&m_eq[p >> 6], 1ull << (p & 63));
      }
    } else {
      for (int c = wave; c < nchunks; c += NWAVE) {
        const int p = 64 * c + lane;
        bool lt = false, eq = false;
        if (p < n) {
          const uint64_t key = absorb(hb, (uint64_t)p);
          lt = key < thr;
          eq = key == thr;
        }
        const unsigned long long mlt = __ballot(lt), meq = __ballot(eq);
        if (lane == 0) { m_lt[c] = mlt; m_eq[c] = meq; }
      }
    }
    __syncthreads();
    // exclusive scan of the chunk counts: a thread owns a contiguous run of chunks
    const int per = (nchunks + NT - 1) / NT, c0 = min(nchunks, t * per), c1 = min(nchunks, c0 + per);
    int sum_lt = 0, sum_eq = 0;
    for (int c = c0; c < c1; ++c) { sum_lt += __popcll(m_lt[c]); sum_eq += __popcll(m_eq[c]); }
    int inc_lt = sum_lt, inc_eq = sum_eq;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int a = __shfl_up(inc_lt, o, 64), e = __shfl_up(inc_eq, o, 64);
      if (lane >= o) { inc_lt += a; inc_eq += e; }
    }
    if (lane == 63) { s_wave_lt[wave] = inc_lt; s_wave_eq[wave] = inc_eq; }
    __syncthreads();
    int run_lt = inc_lt - sum_lt, run_eq = inc_eq - sum_eq;
    for (int w = 0; w < wave; ++w) { run_lt += s_wave_lt[w]; run_eq += s_wave_eq[w]; }
    for (int c = c0; c < c1; ++c) {
      pre_lt[c] = run_lt; pre_eq[c] = run_eq;
      run_lt += __popcll(m_lt[c]); run_eq += __popcll(m_eq[c]);
    }
    __syncthreads();
    const unsigned long long lower = (1ull << lane) - 1ull;
    for (int c = wave; c < nchunks; c += NWAVE) {
      const int p = 64 * c + lane;
      if (p >= n) continue;
      const unsigned long long mlt = m_lt[c], meq = m_eq[c];
      const bool lt = (mlt >> lane) & 1ull, eq = (meq >> lane) & 1ull;
      const int lt_before = pre_lt[c] + __popcll(mlt & lower), eq_before = pre_eq[c] + __popcll(meq & lower);
      const bool keep = lt || (eq && eq_before < take_eq);
      const int row = row0 + g.P + p;
      if (keep) {
        const int pos = out0 + g.P + lt_before + min(eq_before, take_eq);
        idx[pos] = row;
        if (inv) inv[row] = pos;
      } else if (inv) {
        inv[row] = -1;
      }
    }
    return;
  }
  if (t == 0) { s_run_lt = 0; s_run_eq = 0; }
  __syncthreads();
  for (int p0 = 0; p0 < n; p0 += NT) {
    const int p = p0 + t;
    bool lt = false, eq = false;
    if (p < n) {
      const uint64_t key = absorb(hb, (uint64_t)p);
      lt = key < thr;
      eq = key == thr;
    }
    const unsigned long long mlt = __ballot(lt), meq = __ballot(eq);
    const unsigned long long below = (1ull << lane) - 1ull;
    if (lane == 0) { s_wave_lt[wave] = __popcll(mlt); s_wave_eq[wave] = __popcll(meq); }
    __syncthreads();
    int lt_before = s_run_lt + __popcll(mlt & below), eq_before = s_run_eq + __popcll(meq & below);
    for (int w = 0; w < wave; ++w) { lt_before += s_wave_lt[w]; eq_before += s_wave_eq[w]; }
    if (p < n) {
      const bool keep = lt || (eq && eq_before < take_eq);
      const int row = row0 + g.P + p;
      if (keep) {
        const int pos = out0 + g.P + lt_before + min(eq_before, take_eq);
        idx[pos] = row;
        if (inv) inv[row] = pos;
      } else if (inv) {
        inv[row] = -1;
      }
    }
    __syncthreads();
    if (t == 0) {
      int a = 0, e = 0;
      for (int w = 0; w < NWAVE; ++w) { a += s_wave_lt[w]; e += s_wave_eq[w]; }
      s_run_lt += a;
      s_run_eq += e;
    }
    __syncthreads();
  }
}

// Temporal subsets: one thread per row.  A frame's fate is a closed form of its cell: frame s of the cell draws
// the key absorb(h_cell, s); its rank among the cell's frames decides, and the kept frames before it are
// cell * k + (kept frames of the cell with a smaller slot number).
__global__ void __launch_bounds__(256) sample_temporal_kernel(VariantGeom g, int32_t* __restrict__ idx,
                                                              int32_t* __restrict__ inv) {
  const long long total = (long long)g.B * g.N;
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total; e += (long long)gridDim.x * blockDim.x) {
    const int b = (int)(e / g.N), r = (int)(e - (long long)b * g.N);
    const int out0 = b * (g.P + g.n_keep * g.W);
    if (r < g.P) {
      idx[out0 + r] = (int)e;
      if (inv) inv[e] = out0 + r;
      continue;
    }
    const int f = (r - g.P) / g.W, p = (r - g.P) - f * g.W;
    const int cell = f / g.cell, s = f - cell * g.cell;
    const int nvalid = min(g.cell, g.H - cell * g.cell);
    const int kc = nvalid == g.cell ? g.k : g.tail_keep;
    const uint64_t hc = absorb(absorb(g.base, g.per_sample ? (uint64_t)b : 0ull), (uint64_t)cell);
    uint64_t key[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) key[q] = absorb(hc, (uint64_t)q);
    int kept_before = 0;
    bool mine = false;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (q >= nvalid) continue;
      int rank = 0;
#pragma unroll
      for (int o = 0; o < 4; ++o)
        if (o < nvalid && (key[o] < key[q] || (key[o] == key[q] && o < q))) ++rank;
      const bool kq = rank < kc;
      if (q < s && kq) ++kept_before;
      if (q == s) mine = kq;
    }
    if (mine) {
      const int pos = out0 + g.P + (cell * g.k + kept_before) * g.W + p;
      idx[pos] = (int)e;
      if (inv) inv[e] = pos;
    } else if (inv) {
      inv[e] = -1;
    }
  }
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

__global__ void __launch_bounds__(256) sample_cells_kernel(CellGeom g, int32_t* __restrict__ idx, int32_t* __restrict__ inv) {
  const long long total = (long long)g.B * g.units;
  const int c = g.cell, n = c * c;
  for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
    const int b = (int)(t / g.units), u = (int)(t - (long long)b * g.units);
    const int row0 = b * g.N, out0 = b * g.per_sample_K;
    if (u < g.P) {
      idx[out0 + u] = row0 + u;
      if (inv) inv[row0 + u] = out0 + u;
      continue;
    }
    const int ci = u - g.P, cy = ci / g.cw, cx = ci - cy * g.cw;
    const bool full_h = cy < g.fh, full_w = cx < g.fw;
    const int vh = full_h ? c : g.rh, vw = full_w ? c : g.rw;
    const int kc = full_h ? (full_w ? g.k : g.k_fe) : (full_w ? g.k_ef : g.k_ee);
    const int off = g.P + (full_h ? cy * g.row_full : g.fh * g.row_full) + cx * (full_h ? g.k : g.k_ef);
    uint64_t h = absorb(g.base, g.per_sample ? (uint64_t)b : 0ull);
    h = absorb(h, g.shared ? 0ull : (uint64_t)ci);
    // p = floor(h * n! / 2^64), the index of the cell's slot permutation
    uint64_t fact = 1;
    for (int i = 2; i <= n; ++i) fact *= (uint64_t)i;
    const uint64_t p = __umul64hi(h, fact);
    // The factorial-base digits of p, least significant first: the digit of weight (i - 1)! is the remainder of
    // the i-th division by i.  The divisors are compile-time constants here (multiply-and-shift code), where taking
    // the digits from the top costs two 64-bit divisions by run-time values per digit.  Four bits per digit.
    uint64_t q = p, digits = 0;
#pragma unroll
    for (int i = 2; i <= 16; ++i)
      if (i <= n) {
        const uint64_t qq = q / (uint64_t)i;
        digits |= (q - qq * (uint64_t)i) << (4 * (i - 1));
        q = qq;
      }
    uint32_t freem = (1u << n) - 1u, keepm = 0;
    int taken = 0;
    for (int r = 0; r < n && taken < kc; ++r) {       // slots by increasing rank, until kc valid ones are kept
      const uint32_t d = (uint32_t)(digits >> (4 * (n - 1 - r))) & 15u;   // digit of weight (n - 1 - r)!
      uint32_t m = freem;                              // the d-th set bit of freem
      for (uint32_t q = 0; q < d; ++q) m &= m - 1u;
      const uint32_t slot = (uint32_t)__ffs((int)m) - 1u;
      freem &= ~(1u << slot);
      const int sy = (int)slot / c, sx = (int)slot - sy * c;
      if (sy < vh && sx < vw) { keepm |= 1u << slot; ++taken; }
    }
    int pos = out0 + off;
    for (int sy = 0; sy < vh; ++sy)
      for (int sx = 0; sx < vw; ++sx) {                // ascending slot number
        const int row = row0 + g.P + (c * cy + sy) * g.W + c * cx + sx;
        if ((keepm >> (sy * c + sx)) & 1u) {
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

// several draws of the 2 x 2 grid sampler in one launch: blockIdx.y = draw
static constexpr int kMaxDrawsPerLaunch = 16;
struct SampleBatchArgs {
  SampleGeom g[kMaxDrawsPerLaunch];
  int32_t* idx[kMaxDrawsPerLaunch];
  int32_t* inv[kMaxDrawsPerLaunch];
};
__global__ void __launch_bounds__(256) sample_batch_kernel(const SampleBatchArgs a) {
  const SampleGeom& g = a.g[blockIdx.y];
  const long long total = (long long)g.B * (g.P + g.ch * g.cw);
  for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < total;
       t += (long long)gridDim.x * blockDim.x)
    sample_unit(g, t, a.idx[blockIdx.y], a.inv[blockIdx.y]);
}

int32_t launch_sample_batch(const sbp_sample_desc* d, int32_t n, int32_t* const* idx, int32_t* const* inv, hipStream_t s) {
  int i = 0;
  while (i < n) {
    const bool grid2 = (d[i].mode == SBP_GRID_PER_CELL || d[i].mode == SBP_GRID_SHARED) && d[i].cell == 2;
    if (!grid2) {                      // the other samplers: one launch per draw
      const int32_t st = launch_sample(d[i], idx[i], inv ? inv[i] : nullptr, s);
      if (st != SBP_OK) return st;
      ++i;
      continue;
    }
    SampleBatchArgs a{};
    int m = 0;
    long long most = 1;
    while (i < n && m < kMaxDrawsPerLaunch && (d[i].mode == SBP_GRID_PER_CELL || d[i].mode == SBP_GRID_SHARED) && d[i].cell == 2) {
      a.g[m] = make_geom(d[i]);
      a.idx[m] = idx[i];
      a.inv[m] = inv ? inv[i] : nullptr;
      most = std::max(most, (long long)a.g[m].B * (a.g[m].P + a.g[m].ch * a.g[m].cw));
      ++m; ++i;
    }
    const unsigned blocks = (unsigned)std::min<long long>((most + 255) / 256, 65535);
    SBP_LAUNCH(SBP_PROF_SAMPLE, s, sample_batch_kernel, dim3(blocks, (unsigned)m), dim3(256), 0, s, a);
  }
  return check_launch("sample_batch_kernel");
}

int32_t launch_sample(const sbp_sample_desc& d, int32_t* idx, int32_t* inv, hipStream_t s) {
  if (d.mode == SBP_RANDOM_MASK || d.mode == SBP_TEMPORAL) {
    VariantGeom v{};
    v.B = d.B; v.P = d.P; v.H = d.H; v.W = d.W; v.k = d.k; v.cell = d.cell; v.per_sample = d.per_sample;
    v.N = d.P + d.H * d.W;
    v.base = absorb(absorb(0, d.seed), d.stream_id);
    if (d.mode == SBP_RANDOM_MASK) {
      v.n_keep = random_keep(d); v.tail_keep = 0;
      v.win_lo = v.win_hi = 0; v.mask_chunks = 0;
      if (d.H * d.W > 2048) {
        // window of +-(6 standard deviations + 16) ranks around the expected key n_keep / n * 2^64
        const double n = (double)d.H * d.W, q = v.n_keep / n;
        const double half = (6.0 * std::sqrt(n * q * (1.0 - q)) + 16.0) / n;
        const double two64 = 18446744073709551616.0;
        const double lo = std::max(0.0, q - half), hi = q + half;
        v.win_lo = (uint64_t)(lo * two64);
        v.win_hi = hi >= 1.0 ? ~0ull : (uint64_t)(hi * two64);
        const Options opt = options();
        if (opt.sampler_no_window) v.win_lo = v.win_hi = 0;   // override: an empty window, i.e. the full select
        // keep bits and chunk prefixes of the ordered write-out: 24 bytes per 64 positions, next to 50 KB of static LDS
        const int64_t chunks = ceil_div((int64_t)d.H * d.W, 64);
        size_t lds = (size_t)chunks * 24;
        static std::once_flag big_lds_once;             // more than 64 KB in all: granted per kernel, asked for once
        static bool big_lds_ok = false;
        if (lds > 12 * 1024)
          std::call_once(big_lds_once, [] {
            big_lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(sample_random_kernel<1024, true>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 104 * 1024) == hipSuccess;
          });
        v.mask_chunks = (int)chunks;
        if (lds > 104 * 1024 || (lds > 12 * 1024 && !big_lds_ok) || opt.sampler_no_masks) { v.mask_chunks = 0; lds = 0; }
        SBP_LAUNCH(SBP_PROF_SAMPLE, s, (sample_random_kernel<1024, true>), dim3(d.B), dim3(1024), lds, s, v, idx, inv);
      } else {
        SBP_LAUNCH(SBP_PROF_SAMPLE, s, (sample_random_kernel<256, false>), dim3(d.B), dim3(256), 0, s, v, idx, inv);
      }
      return check_launch("sample_random_kernel");
    }
    v.n_keep = temporal_keep_frames(d);
    v.tail_keep = d.H % d.cell ? temporal_tail_keep(d.k, d.H % d.cell, d.cell) : 0;
    const long long total = (long long)v.B * v.N;
    const unsigned blocks = (unsigned)std::max<long long>(1, std::min<long long>((total + 255) / 256, 65535));
    SBP_LAUNCH(SBP_PROF_SAMPLE, s, sample_temporal_kernel, dim3(blocks), dim3(256), 0, s, v, idx, inv);
    return check_launch("sample_temporal_kernel");
  }
  if (d.cell != 2) {
    const CellGeom c = make_cell_geom(d);
    const long long total = (long long)c.B * c.units;
    const unsigned blocks = (unsigned)std::max<long long>(1, std::min<long long>((total + 255) / 256, 65535));
    SBP_LAUNCH(SBP_PROF_SAMPLE, s, sample_cells_kernel, dim3(blocks), dim3(256), 0, s, c, idx, inv);
    return check_launch("sample_cells_kernel");
  }
  SampleGeom g = make_geom(d);
  long long total = (long long)g.B * (g.P + g.ch * g.cw);
  int blocks = (int)((total + 255) / 256);
  if (blocks > 65535) blocks = 65535;
  SBP_LAUNCH(SBP_PROF_SAMPLE, s, sample_kernel, dim3(blocks), dim3(256), 0, s, g, idx, inv);
  return check_launch("sample_kernel");
}

}  // namespace sbp
