// SBP backward of a linear / pointwise-conv layer on the kept rows only
// (paper, section "Calculation of Linear Layers", eq:backward_fc_sbp with the dropped terms removed):
//   dW[o,i] = sum_j dY[idx[j],o] X_k[j,i]      db[o] = sum_j dY[idx[j],o]
//   dX[idx[j],:] = dY[idx[j],:] W              every other row of dX = +0
// W is stored [Cout, Cin].
//
// bf16 path: both contractions run on the gfx950 matrix cores, in one launch per layer together with
// the zero fill of the dropped rows and the column sums for db: linear_big_kernel (256-wide tiles,
// sbp_mfma_big.h) where the layer is large enough to keep the CUs busy with them, linear_bwd_kernel
// (128 x 128 tiles, sbp_mfma_gemm.h) otherwise.  dW is split along the kept rows into fp32 partial
// sums that a second kernel adds in a fixed order (deterministic, no floating-point atomics).
// fp32 and odd shapes take plain kernels.
#include <cstdio>
#include <cstdlib>

#include <algorithm>
#include <cstddef>
#include <functional>
#include <mutex>
#include <queue>
#include <string>
#include <vector>

#include "sbp_mfma_big.h"
#include "sbp_mfma_gemm.h"

namespace sbp {

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by workgroup id.  This
// maps the id so that every XCD works on one contiguous chunk of the tile list: neighbouring tiles,
// which share operand panels, then meet in the same L2.  The grid is padded to a multiple of 8;
// ids that map beyond the list are idle.
static constexpr int kNumXCD = 8;
__device__ __forceinline__ int xcd_chunked_id(int wg, int ntiles) {
  const int per = (ntiles + kNumXCD - 1) / kNumXCD;
  return (wg % kNumXCD) * per + wg / kNumXCD;
}

static constexpr int kDbSliceRows = 128;      // smallest row slice of a column-sum block (general engine)
static constexpr int kDbSliceRowsBig = 512;   // large-tile engine: fewer, longer blocks with 16 row loads in flight per thread
static constexpr int kMaxDbSlices = 64;      // at most this many partial sums per channel
static constexpr int kMaxRowsPerSplit = 2048;   // kept rows per dW split (their ids are staged in LDS)

// Everything one linear layer's backward needs, in one launch.  The grid is four segments of
// workgroups, each doing one kind of work:
//   [zero]  write +0 to the rows of dX that are not kept (row m is kept iff idx[inv[m]] == m)
//   [db]    column sums of the kept rows of dY, one block per (row slice, 256 channels)
//   [dX]    BM x BN tiles of dX = dY_k W, scattered to the kept rows
//   [dW]    BM x BN tiles of the per-split partial sums of dW = dY_k^T X_k
// The host orders the segments [zero + db], [dX], [dW] by the expected length of their workgroups, longest
// first (seg_order): the CUs take workgroups in grid order, and a long kind dispatched last would run on alone
// when everything else is done.  zero + db is padded to a multiple of 8 and each tile segment is a multiple of
// 8, so the XCD chunking of a segment is exact wherever it starts.
struct LinArgs {
  const uint16_t* dY;
  const int32_t* idx_in;    // rows of dY (NULL: dY is compact)
  const int32_t* idx_out;   // rows of dX (NULL: dX is compact)
  const int32_t* idx;       // the keep list itself (for the kept-row test)
  const int32_t* inv;
  const uint16_t* Xk;
  const uint16_t* W;
  uint16_t* dX;
  float* part;
  float* dbp;
  int K, M, Cin, Cout, rows_per_split, db_slice_rows;
  int n_zero, n_helper, n_dx, n_dw;   // n_helper = zero + db blocks rounded up to a multiple of 8
  int n_big, rows_small, n_dw_big;     // large-tile kernel: long and short dW splits; n_dw_big of the n_dw units are long
  int seg_order[3];                   // dispatch order: large-tile kernel 0 = dX tiles, 1 = long dW, 2 = short dW units;
                                      // general kernel 0 = dX tiles, 1 = dW units, 2 = zero-fill and column-sum blocks
  int dx_bm;                          // large-tile kernel: rows of a dX tile (256 or 128)
  int db_in_dw;                       // large-tile kernel: the dW units also produce db, each from its share of the rows (one
                                      // partial per split and tile column in dbp); no column-sum blocks then
  int xk_kmajor;                      // large-tile kernel: Xk is in the row-group layout [K / 8][Cin][8]
};

// Zero fill of the dropped rows.  A wavefront takes 64 consecutive rows: every lane looks one row up
// (row m is kept iff idx[inv[m]] == m: two dependent loads, once per 64 rows), a ballot collects the
// dropped rows, and all lanes together write each of them.
__device__ __forceinline__ void zero_rows_block(const LinArgs& a, int blk) {
  const int ppr = a.Cin / 8;                                   // 16-byte pieces per row
  const int lane = threadIdx.x & 63;
  const int wpb = blockDim.x >> 6;                             // wavefronts per block
  const int gw = blk * wpb + (threadIdx.x >> 6);
  uint4* out = reinterpret_cast<uint4*>(a.dX);
  for (int base = gw * 64; base < a.M; base += a.n_zero * wpb * 64) {
    const int m = base + lane;
    bool dropped = false;
    if (m < a.M) {
      const int j = a.inv[m];
      dropped = !((unsigned)j < (unsigned)a.K && a.idx[j] == m);
    }
    unsigned long long mask = __ballot(dropped);
    while (mask) {
      const int b = __ffsll((long long)mask) - 1;
      mask &= mask - 1;
      uint4* row = out + (long long)(base + b) * ppr;
      for (int p = lane; p < ppr; p += 64) row[p] = make_uint4(0, 0, 0, 0);
    }
  }
}

// BMX, NSX: rows and ring depth of the dX tiles (the dW units use BM and NSTAGE)
template <int BM, int BN, int NW, int KB, int NSTAGE, int BMX, int NSX>
__device__ __forceinline__ void linear_bwd_body(char* smem, const LinArgs& a, int wg) {
  int kind = 0;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    kind = a.seg_order[q];
    const int n = kind == 0 ? a.n_dx : (kind == 1 ? a.n_dw : a.n_helper);
    if (wg < n) break;
    wg -= n;
  }
  if (kind == 2) {
    if (wg < a.n_zero) {
      zero_rows_block(a, wg);
    } else {
      const int b = wg - a.n_zero;
      const int nslice = (a.K + a.db_slice_rows - 1) / a.db_slice_rows;
      const int slice = b % nslice, chunk = b / nslice;
      if (a.dbp && chunk * 256 < a.Cout) {
        const int j0 = slice * a.db_slice_rows, j1 = min(a.K, j0 + a.db_slice_rows);
        colsum_block<8>(smem, a.dY, a.idx_in, a.Cout, j0, j1, chunk * 256, a.dbp + (long long)slice * a.Cout);
      }
    }
    return;
  }
  const int tiles_n = (a.Cin + BN - 1) / BN;
  if (kind == 0) {
    const int ntiles = ((a.K + BMX - 1) / BMX) * tiles_n;
    const int L = xcd_chunked_id(wg, ntiles);
    if (L >= ntiles) return;
    const int tile_m = L / tiles_n, tile_n = L - tile_m * tiles_n;
    dx_tile<BMX, BN, NW, KB, NSX>(smem, a.dY, a.idx_in, a.idx_out, a.W, a.K, a.Cin, a.Cout, a.dX, tile_m * BMX, tile_n * BN);
    return;
  }
  const int tiles_m = (a.Cout + BM - 1) / BM;
  const int nsplit = (a.K + a.rows_per_split - 1) / a.rows_per_split;
  const int ntiles = tiles_m * tiles_n * nsplit;
  const int L = xcd_chunked_id(wg, ntiles);
  if (L >= ntiles) return;
  const int split = L / (tiles_m * tiles_n);
  const int rem = L - split * tiles_m * tiles_n;
  const int tile_m = rem / tiles_n, tile_n = rem - tile_m * tiles_n;
  const int j0 = split * a.rows_per_split, j1 = min(a.K, j0 + a.rows_per_split);
  dw_tile<BM, BN, NW, KB, NSTAGE>(smem, a.dY, a.idx_in, a.Xk, a.Cin, a.Cout, j0, j1, a.part + (long long)split * a.Cout * a.Cin,
                      tile_m * BM, tile_n * BN);
}

template <int BM, int BN, int NW, int KB, int NSTAGE, int BMX, int NSX>
__global__ void __launch_bounds__(64 * NW, (BM + BN) <= 256 ? 2 : 1) linear_bwd_kernel(const LinArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  linear_bwd_body<BM, BN, NW, KB, NSTAGE, BMX, NSX>(smem, a, blockIdx.x);
}

// Several small layers in one launch of the general engine (128 x 128 tiles, stages of 64): the grids of the layers
// one behind the other, every layer with its own order of segments.  A ViT-Tiny-class layer is a few hundred
// workgroups that all find a slot at once; two such layers side by side fill the chip better than one after the other
// and save a launch.
struct SmallMultiArgs { int n; int start[SBP_MAX_BATCH_LAYERS + 1]; LinArgs lay[SBP_MAX_BATCH_LAYERS]; };
static_assert(sizeof(SmallMultiArgs) <= 4096, "kernel arguments are limited to 4 KB");

__global__ void __launch_bounds__(256, 2) linear_bwd_multi_kernel(const SmallMultiArgs m) {
#if defined(__HIP_DEVICE_COMPILE__)      // (address-space casts below: the host pass only needs the symbol)
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int li = 0, first = 0;
#pragma unroll
  for (int i = 1; i < SBP_MAX_BATCH_LAYERS; ++i)
    if (i < m.n && (int)blockIdx.x >= m.start[i]) { li = i; first = m.start[i]; }
  // the layer's arguments through the kernel-argument segment itself (constant address space, uniform index: scalar
  // loads into scalar registers); indexing the by-value struct made the compiler copy all of it to scratch memory
  typedef const __attribute__((address_space(4))) LinArgs* ConstLinArgsPtr;
  const __attribute__((address_space(4))) char* kargs =
      (const __attribute__((address_space(4))) char*)__builtin_amdgcn_kernarg_segment_ptr();
  const LinArgs a = *reinterpret_cast<ConstLinArgsPtr>(kargs + offsetof(SmallMultiArgs, lay) + (size_t)li * sizeof(LinArgs));
  const int wg = (int)blockIdx.x - first;
  if (a.dx_bm == 64) linear_bwd_body<128, 128, 4, 64, 2, 64, 3>(smem, a, wg);
  else linear_bwd_body<128, 128, 4, 64, 2, 128, 2>(smem, a, wg);
#endif
}

// Workgroups go to the 8 XCDs round robin by their index in the grid, and every XCD queues its own: a
// workgroup waits for a CU of its XCD although another XCD has one free.  segment_unit gives the workgroups of
// one XCD a contiguous run of the units of a grid segment [s, s + n) (they share operand panels in that XCD's
// L2); the runs differ by at most one unit and no workgroup is left without work.
__device__ __forceinline__ int congruent_below(int y, int t) { return (t - y + 7) >> 3; }   // #{i in [0,t): i % 8 == y}
__device__ __forceinline__ int segment_unit(int wg_global, int s, int n) {
  const int x = wg_global & 7;
  int before = 0;
  for (int y = 0; y < 8; ++y)
    if (y < x) before += congruent_below(y, s + n) - congruent_below(y, s);
  return before + congruent_below(x, wg_global) - congruent_below(x, s);
}

// One unit of the large-tile engine: kind 0 = dX tile number L, kind 1 / 2 = dW unit number L among the long /
// short splits (a tile of dW over the kept rows of one split, written as an fp32 partial sum; with db_in_dw also a
// partial of db: slice split * tiles_n + tile column of dbp).
__device__ __forceinline__ void big_unit(char* smem, const LinArgs& a, int kind, int L) {
  const int tiles_n = (a.Cin + big::BT - 1) / big::BT;
  if (kind == 0) {
    const int tile_m = L / tiles_n, tile_n = L - tile_m * tiles_n;
    if (a.dx_bm == 64)
      big::dx_tile<64>(smem, a.dY, a.idx_in, a.idx_out, a.W, a.K, a.Cin, a.Cout, a.dX, tile_m * 64, tile_n * big::BT);
    else if (a.dx_bm == 128)
      big::dx_tile<128>(smem, a.dY, a.idx_in, a.idx_out, a.W, a.K, a.Cin, a.Cout, a.dX, tile_m * 128, tile_n * big::BT);
    else
      big::dx_tile<256>(smem, a.dY, a.idx_in, a.idx_out, a.W, a.K, a.Cin, a.Cout, a.dX, tile_m * 256, tile_n * big::BT);
    return;
  }
  // the first n_big splits have rows_per_split rows each, the others rows_small
  const int tiles_m = (a.Cout + big::BT - 1) / big::BT, tiles_w = tiles_m * tiles_n;
  const int covered = min(a.K, a.n_big * a.rows_per_split);
  const int sl = L / tiles_w, rem = L - sl * tiles_w;          // sl: split within its kind
  const int tile_m = rem / tiles_n, tile_n = rem - tile_m * tiles_n;
  const int j0 = kind == 1 ? sl * a.rows_per_split : covered + sl * a.rows_small;
  const int j1 = min(a.K, j0 + (kind == 1 ? a.rows_per_split : a.rows_small));
  const int split = kind == 1 ? sl : a.n_big + sl;
  float* part = a.part + (long long)split * a.Cout * a.Cin;
  const int m0 = tile_m * big::BT, n0 = tile_n * big::BT;
  if (a.db_in_dw) {        // every unit sums its share of the columns of its dY panel: one slice of dbp per split and tile column
    float* dbp = a.dbp + ((long long)split * tiles_n + tile_n) * a.Cout;
    if (a.xk_kmajor) {
      if (a.idx_in) big::dw_tile<true, true, true>(smem, a.dY, a.idx_in, a.Xk, a.Cin, a.Cout, j0, j1, part, m0, n0, dbp, tile_n, tiles_n);
      else big::dw_tile<false, true, true>(smem, a.dY, nullptr, a.Xk, a.Cin, a.Cout, j0, j1, part, m0, n0, dbp, tile_n, tiles_n);
    } else {
      if (a.idx_in) big::dw_tile<true, true>(smem, a.dY, a.idx_in, a.Xk, a.Cin, a.Cout, j0, j1, part, m0, n0, dbp, tile_n, tiles_n);
      else big::dw_tile<false, true>(smem, a.dY, nullptr, a.Xk, a.Cin, a.Cout, j0, j1, part, m0, n0, dbp, tile_n, tiles_n);
    }
    return;
  }
  if (a.xk_kmajor) {
    if (a.idx_in) big::dw_tile<true, false, true>(smem, a.dY, a.idx_in, a.Xk, a.Cin, a.Cout, j0, j1, part, m0, n0);
    else big::dw_tile<false, false, true>(smem, a.dY, nullptr, a.Xk, a.Cin, a.Cout, j0, j1, part, m0, n0);
    return;
  }
  if (a.idx_in) big::dw_tile<true>(smem, a.dY, a.idx_in, a.Xk, a.Cin, a.Cout, j0, j1, part, m0, n0);
  else big::dw_tile<false>(smem, a.dY, nullptr, a.Xk, a.Cin, a.Cout, j0, j1, part, m0, n0);
}

// The same work with 256 x 256 tiles (sbp_mfma_big.h): one workgroup per CU, so the order of the grid
// is the order in which the CUs of an XCD pick work up: the longer kind of tile first, the shorter kind next,
// the streaming helpers (zero fill, column sums) last, where they fill the CUs that run out of tiles.
__global__ void __launch_bounds__(256, 1) linear_big_kernel(const LinArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int wg = blockIdx.x;
  if (wg >= a.n_dx + a.n_dw) {
    wg -= a.n_dx + a.n_dw;
    if (wg < a.n_zero) {
      zero_rows_block(a, wg);
    } else {
      const int b = wg - a.n_zero;
      const int nslice = (a.K + a.db_slice_rows - 1) / a.db_slice_rows;
      const int slice = b % nslice, chunk = b / nslice;
      if (a.dbp && chunk * 256 < a.Cout) {
        const int j0 = slice * a.db_slice_rows, j1 = min(a.K, j0 + a.db_slice_rows);
        colsum_block<16>(smem, a.dY, a.idx_in, a.Cout, j0, j1, chunk * 256, a.dbp + (long long)slice * a.Cout);
      }
    }
    return;
  }
  // which kind of unit: the three kinds lie in the grid in the order the host chose
  int kind = 0, seg_start = 0, seg_n = 0;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    kind = a.seg_order[q];
    seg_n = kind == 0 ? a.n_dx : (kind == 1 ? a.n_dw_big : a.n_dw - a.n_dw_big);
    if (wg < seg_start + seg_n) break;
    seg_start += seg_n;
  }
  big_unit(smem, a, kind, segment_unit(wg, seg_start, seg_n));
}

// ---- several layers in one launch ----------------------------------------------------------------------
// The backward of up to kMaxBatch independent layers as ONE grid: the units of all layers (dX tiles, dW units,
// zero-fill and column-sum blocks) lie in the grid as segments, longest kind of unit first whatever its layer,
// each segment spread over the eight XCD queues in contiguous runs (segment_unit).  A ViT block's four layers
// are about 1000 units: the CUs stay busy until the short helper blocks at the end of the grid even out the
// finish, where four separate launches each end with their longest unit and start with an empty chip.
static constexpr int kMaxBatch = 8;
static constexpr int kMaxEnt = 24;                  // entries of one XCD's queue
// Workgroup i of a grid runs on XCD i % 8, and every XCD hands its workgroups to its 32 CUs in order.  The host
// therefore writes one queue per XCD: entry = a run of consecutive units of one kind of one layer (kind 0 dX tiles,
// 1 dW units, 3 zero-fill blocks, 4 column-sum blocks), entries in the order they are to start.  A layer's tiles
// are kept on as few XCDs as the balance of work allows, as runs of neighbouring tiles: the operand panels they
// share are then fetched into one L2 instead of eight.
struct XcdEntry { int first_q, unit0; short layer; signed char kind, stride; };   // positions first_q .. next entry's first_q - 1 of the
                                                                                  // queue are units unit0, unit0 + stride, ...
struct MultiArgs {
  int nent[kNumXCD], nq[kNumXCD];     // entries and units of every queue
  int* counters;                      // [kNumXCD] in the workspace, zero at launch: next position of every queue
  int timeline_cap, pad_;
  unsigned long long* timeline;       // measurement aid (sbp_profile_timeline): 8 words per unit, or NULL
  XcdEntry ent[kNumXCD][kMaxEnt];
  LinArgs lay[kMaxBatch];
};
static_assert(sizeof(MultiArgs) <= 4096, "kernel arguments are limited to 4 KB");

// Grid = 8 x the longest queue; workgroup i serves position i / 8 of queue i % 8 (`dynamic` = 0), or (`dynamic` = 1)
// takes the next position of its XCD's queue from an atomic counter and, when that queue is empty, of the other
// queues, nearest first: XCDs that run out of their own units then help the others.  Workgroups that find nothing
// leave at once.
__global__ void __launch_bounds__(256, 1) linear_multi_kernel(const MultiArgs a, int dynamic) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int wg = blockIdx.x;
  const int home = wg & (kNumXCD - 1);
  int x = home, q = wg >> 3;
  if (dynamic) {
    int* ticket = reinterpret_cast<int*>(smem);
    if (threadIdx.x == 0) {
      int got = -1;
      for (int t = 0; t < kNumXCD && got < 0; ++t) {
        const int v = (home + t) & (kNumXCD - 1);
        const int p = __hip_atomic_fetch_add(a.counters + v, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (p < a.nq[v]) got = (v << 24) | p;
      }
      *ticket = got;
    }
    __syncthreads();
    const int got = __builtin_amdgcn_readfirstlane(*ticket);
    __syncthreads();                               // the unit may now overwrite the ticket's place in LDS
    if (got < 0) return;
    x = got >> 24; q = got & 0xffffff;
  } else if (q >= a.nq[x]) {
    return;
  }
  int e = 0;
  for (int i = 1; i < a.nent[x]; ++i)
    if (q >= a.ent[x][i].first_q) e = i;
  const int kind = a.ent[x][e].kind, layer = a.ent[x][e].layer;
  const int L = a.ent[x][e].unit0 + (q - a.ent[x][e].first_q) * a.ent[x][e].stride;
  const LinArgs& la = a.lay[layer];
  // measurement aid: the 100 MHz wall clock and the shader clock at the start and at the end of every unit
  int slot = q;
  for (int i = 0; i < x; ++i) slot += a.nq[i];
  const bool stamp = a.timeline != nullptr && slot < a.timeline_cap;
  unsigned long long t0 = 0, c0 = 0;
  if (stamp) { t0 = wall_clock64(); c0 = clock64(); }
  if (kind <= 2) {
    big_unit(smem, la, kind, L);
  } else if (kind == 3) {
    zero_rows_block(la, L);                        // la.n_zero = number of these blocks
  } else {
    const int nslice = (la.K + la.db_slice_rows - 1) / la.db_slice_rows;
    const int slice = L % nslice, chunk = L / nslice;
    const int j0 = slice * la.db_slice_rows, j1 = min(la.K, j0 + la.db_slice_rows);
    colsum_block<16>(smem, la.dY, la.idx_in, la.Cout, j0, j1, chunk * 256, la.dbp + (long long)slice * la.Cout);
  }
  if (stamp && threadIdx.x == 0) {
    unsigned long long* rec = a.timeline + 8ll * slot;
    rec[0] = t0; rec[1] = wall_clock64(); rec[2] = c0; rec[3] = clock64();
    rec[4] = (unsigned long long)kind | ((unsigned long long)layer << 8) | ((unsigned long long)L << 16);
    rec[5] = (unsigned long long)x | ((unsigned long long)home << 8) | ((unsigned long long)wg << 16);
  }
}

// dW = sum_s partial[s] (+ dW), db = sum_s dbp[s] (+ db): fixed summation order.  G lanes share an output: lane g
// adds a contiguous run of the splits (four loads in flight) and the G sums are added in lane order, so the order
// depends on G and the split count only.  G > 1 is for small weight matrices cut into many splits, where one thread
// per output would leave most CUs idle behind a long chain of dependent loads.
// dW in memory: fp32, or bf16 (BF16OUT: the fp32 sum rounded to nearest even; an old value is widened first)
template <bool BF16OUT>
__device__ __forceinline__ float4 load_dw4(const void* dW, long long e) {
  if (!BF16OUT) return reinterpret_cast<const float4*>(dW)[e];
  const uint2 w = reinterpret_cast<const uint2*>(dW)[e];
  return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                     __uint_as_float(w.y & 0xffff0000u));
}
template <bool BF16OUT>
__device__ __forceinline__ void store_dw4(void* dW, long long e, const float4& v) {
  if (!BF16OUT) reinterpret_cast<float4*>(dW)[e] = v;
  else reinterpret_cast<uint2*>(dW)[e] = make_uint2(bf16_pack(v.x, v.y), bf16_pack(v.z, v.w));
}

template <int G, bool BF16OUT>
__global__ void __launch_bounds__(NTHREADS) reduce_splits_kernel(const float* __restrict__ partial, int nsplit_w,
                                                                  long long nW, void* __restrict__ dW,
                                                                  const float* __restrict__ dbp, int nsplit_b, int Cout,
                                                                  float* __restrict__ db, int accumulate) {
  const long long nW4 = dW ? nW / 4 : 0;
  const long long nB = db ? Cout : 0;
  const long long total = nW4 + nB;
  const int g = threadIdx.x & (G - 1), lane = threadIdx.x & 63;
  for (long long e = (blockIdx.x * (long long)blockDim.x + threadIdx.x) / G; e < total;
       e += (long long)gridDim.x * blockDim.x / G) {
    if (e < nW4) {
      const int chunk = (nsplit_w + G - 1) / G, s_begin = g * chunk, s_end = min(nsplit_w, s_begin + chunk);
      float4 a = make_float4(0, 0, 0, 0);
      for (int s0 = s_begin; s0 < s_end; s0 += 4) {
        float4 p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          p[u] = s0 + u < s_end ? reinterpret_cast<const float4*>(partial + (long long)(s0 + u) * nW)[e]
                                : make_float4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < 4; ++u) { a.x += p[u].x; a.y += p[u].y; a.z += p[u].z; a.w += p[u].w; }
      }
      float4 t = a;
#pragma unroll
      for (int k = 1; k < G; ++k) {
        const int src = (lane & ~(G - 1)) + k;
        t.x += __shfl(a.x, src); t.y += __shfl(a.y, src); t.z += __shfl(a.z, src); t.w += __shfl(a.w, src);
      }
      if (g == 0) {
        if (accumulate) {
          const float4 old = load_dw4<BF16OUT>(dW, e);
          t.x = old.x + t.x; t.y = old.y + t.y; t.z = old.z + t.z; t.w = old.w + t.w;
        }
        store_dw4<BF16OUT>(dW, e, t);
      }
    } else {
      const long long o = e - nW4;
      const int chunk = (nsplit_b + G - 1) / G, s_begin = g * chunk, s_end = min(nsplit_b, s_begin + chunk);
      float a = 0.f;
      for (int s0 = s_begin; s0 < s_end; s0 += 8) {
        float p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) p[u] = s0 + u < s_end ? dbp[(long long)(s0 + u) * Cout + o] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) a += p[u];
      }
      float t = a;
#pragma unroll
      for (int k = 1; k < G; ++k) t += __shfl(a, (lane & ~(G - 1)) + k);
      if (g == 0) db[o] = accumulate ? db[o] + t : t;
    }
  }
}

// same, element by element, for weight matrices whose size is not a multiple of 4
template <bool BF16OUT>
__global__ void __launch_bounds__(NTHREADS) reduce_splits_scalar_kernel(const float* __restrict__ partial, int nsplit,
                                                                         long long nW, void* __restrict__ dW,
                                                                         const float* __restrict__ dbp, int Cout,
                                                                         float* __restrict__ db, int accumulate) {
  const long long nWe = dW ? nW : 0;
  const long long total = nWe + (db ? Cout : 0);
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
       e += (long long)gridDim.x * blockDim.x) {
    if (e < nWe) {
      float a = 0.f;
      for (int s = 0; s < nsplit; ++s) a += partial[(long long)s * nW + e];
      if (BF16OUT) {
        uint16_t* w = reinterpret_cast<uint16_t*>(dW);
        if (accumulate) a = __uint_as_float((uint32_t)w[e] << 16) + a;
        w[e] = (uint16_t)(bf16_pack(a, 0.f) & 0xffffu);
      } else {
        float* w = reinterpret_cast<float*>(dW);
        w[e] = accumulate ? w[e] + a : a;
      }
    } else {
      const long long o = e - nWe;
      float a = accumulate ? db[o] : 0.f;
      for (int s = 0; s < nsplit; ++s) a += dbp[(long long)s * Cout + o];
      db[o] = a;
    }
  }
}

// inv[idx[j]] = j.  inv needs no clearing: row m is kept iff 0 <= inv[m] < K and idx[inv[m]] == m.
__global__ void __launch_bounds__(NTHREADS) mark_rows_kernel(const int32_t* __restrict__ idx, int K,
                                                              int32_t* __restrict__ inv) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < K) inv[idx[j]] = j;
}

// Writes +0 to every row of dX that is not in idx (16-byte pieces).
__global__ void __launch_bounds__(NTHREADS) zero_dropped_rows_kernel(const int32_t* __restrict__ idx,
                                                                      const int32_t* __restrict__ inv, int K,
                                                                      long long M, int pieces_per_row,
                                                                      uint4* __restrict__ dX) {
  const long long total = M * pieces_per_row;
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
       e += (long long)gridDim.x * blockDim.x) {
    const long long m = e / pieces_per_row;
    const int j = inv[m];
    const bool kept = (unsigned)j < (unsigned)K && idx[j] == (int32_t)m;
    if (!kept) dX[e] = make_uint4(0, 0, 0, 0);
  }
}

// element-wise variant for rows whose byte length is not a multiple of 16
template <typename T>
__global__ void __launch_bounds__(NTHREADS) zero_dropped_rows_elem_kernel(const int32_t* __restrict__ idx,
                                                                           const int32_t* __restrict__ inv, int K,
                                                                           long long M, int C, T* __restrict__ dX) {
  const long long total = M * C;
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
       e += (long long)gridDim.x * blockDim.x) {
    const long long m = e / C;
    const int j = inv[m];
    const bool kept = (unsigned)j < (unsigned)K && idx[j] == (int32_t)m;
    if (!kept) dX[e] = (T)0;
  }
}

__global__ void __launch_bounds__(NTHREADS) fill_zero_kernel(uint32_t* __restrict__ p, long long n) {
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < n; e += (long long)gridDim.x * blockDim.x)
    p[e] = 0u;
}

// ------------------------------------------------------------------------------------------------
// Plain kernels (fp32 storage, or bf16 with channel counts that are not multiples of 8).
// ------------------------------------------------------------------------------------------------
template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {
  static __device__ __forceinline__ float ld(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
  static __device__ __forceinline__ void st(uint16_t* p, float v) { *p = (uint16_t)(bf16_pack(v, 0.f) & 0xffffu); }
};

// one thread per (kept row j, input channel i)
template <typename T>
__global__ void __launch_bounds__(NTHREADS) plain_dx_kernel(const T* __restrict__ dY, const int32_t* __restrict__ idx_in,
                                                             const int32_t* __restrict__ idx_out,
                                                             const T* __restrict__ W, long long K, int Cin, int Cout,
                                                             T* __restrict__ dX) {
  const long long total = K * Cin;
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
       e += (long long)gridDim.x * blockDim.x) {
    const long long j = e / Cin;
    const int i = (int)(e - j * Cin);
    const long long rin = idx_in ? (long long)idx_in[j] : j;
    const long long rout = idx_out ? (long long)idx_out[j] : j;
    const T* g = dY + rin * Cout;
    float a = 0.f;
    for (int o = 0; o < Cout; ++o) a = fmaf(Elem<T>::ld(g + o), Elem<T>::ld(W + (long long)o * Cin + i), a);
    Elem<T>::st(dX + rout * Cin + i, a);
  }
}

// one thread per (o, i) and row split; sums in chunks of 256 rows to keep fp32 rounding small
template <typename T>
__global__ void __launch_bounds__(NTHREADS) plain_dw_kernel(const T* __restrict__ dY, const int32_t* __restrict__ idx,
                                                             const T* __restrict__ Xk, int K, int Cin, int Cout,
                                                             int rows_per_split, float* __restrict__ partial) {
  const long long nW = (long long)Cin * Cout;
  const int j0 = blockIdx.y * rows_per_split, j1 = min(K, j0 + rows_per_split);
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < nW;
       e += (long long)gridDim.x * blockDim.x) {
    const int o = (int)(e / Cin), i = (int)(e - (long long)o * Cin);
    float total = 0.f;
    for (int jc = j0; jc < j1; jc += 256) {
      float a = 0.f;
      const int je = min(j1, jc + 256);
      for (int j = jc; j < je; ++j) {
        const long long r = idx ? (long long)idx[j] : (long long)j;
        a = fmaf(Elem<T>::ld(dY + r * Cout + o), Elem<T>::ld(Xk + (long long)j * Cin + i), a);
      }
      total += a;
    }
    partial[(long long)blockIdx.y * nW + e] = total;
  }
}

template <typename T>
__global__ void __launch_bounds__(NTHREADS) plain_db_kernel(const T* __restrict__ dY, const int32_t* __restrict__ idx,
                                                             int K, int Cout, int rows_per_split,
                                                             float* __restrict__ dbp) {
  const int j0 = blockIdx.y * rows_per_split, j1 = min(K, j0 + rows_per_split);
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= Cout) return;
  float total = 0.f;
  for (int jc = j0; jc < j1; jc += 256) {
    float a = 0.f;
    const int je = min(j1, jc + 256);
    for (int j = jc; j < je; ++j) {
      const long long r = idx ? (long long)idx[j] : (long long)j;
      a += Elem<T>::ld(dY + r * Cout + o);
    }
    total += a;
  }
  dbp[(long long)blockIdx.y * Cout + o] = total;
}

// ------------------------------------------------------------------------------------------------
// Host side: plan and launches.
// ------------------------------------------------------------------------------------------------
static constexpr int kNumCU = 256;

// ---- large-tile engine: tile height of dX and the dW splits ----------------------------------------
// Workgroup i of the grid goes to XCD i % 8, every XCD hands its workgroups in order to its 32 CUs, one per CU:
// list scheduling per XCD.  The host simulates it from unit costs and takes the cheapest schedule.
static constexpr int kBigMaxRowsPerSplit = 7936;   // row ids of a split in LDS next to the 128 KB ring (160 KB in all)
// Unit costs in nanoseconds: durations of the workgroups read from the device clock inside a training-like
// step (operands cold, all CUs busy) for the four ViT-Base layer shapes: a straight line through the units of
// 20 to 96 stages of 32.  The fixed part is the first stages' latency, the index tables and the epilogue (a
// dW unit stores 256 KB of partial sums).
static constexpr int64_t kNsStage256 = 750, kNsFixedDx256 = 6500;     // 256 x 256 dX tile
static constexpr int64_t kNsStage128 = 450, kNsFixedDx128 = 8000;     // 128 x 256 dX tile
static constexpr int64_t kNsStage64 = 365, kNsFixedDx64 = 8000;       // 64 x 256 dX tile
static constexpr int64_t kNsStageDw = 667, kNsFixedDw = 10000;        // 256 x 256 dW unit
static constexpr int64_t kNsFixedHelper = 1800;                       // zero-fill and column-sum blocks: fixed part
static constexpr int64_t kHelperBytesPerNs = 50;                      //   and the rate at which one CU streams
static constexpr double kReduceBytesPerNs = 2650;                     // the reduction streams the partials

struct BigChoice {
  int64_t M, K; int32_t Cin, Cout;
  int splits, rps, n_big, rows_small, dx_bm;
  int seg_order[3];
  double fill;      // work / (CUs x finish time) of the simulated schedule
};

static int64_t congruent_below_host(int64_t y, int64_t t) { return (t - y + 7) >> 3; }

// finish time of the grid: segments {count, unit length} in grid order
static int64_t simulate_grid(const int64_t* n, const int64_t* l, int nseg) {
  int64_t end = 0;
  for (int x = 0; x < kNumXCD; ++x) {
    std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> cu;
    for (int i = 0; i < kNumCU / kNumXCD; ++i) cu.push(0);
    int64_t start = 0;
    for (int q = 0; q < nseg; ++q) {
      const int64_t mine = congruent_below_host(x, start + n[q]) - congruent_below_host(x, start);
      for (int64_t i = 0; i < mine; ++i) {
        const int64_t t = cu.top() + l[q];
        cu.pop();
        cu.push(t);
        end = std::max(end, t);
      }
      start += n[q];
    }
  }
  return end;
}

static int big_zero_blocks(int64_t M) { return (int)std::min<int64_t>(128, std::max<int64_t>(8, ceil_div(M, 256))); }
static int db_slice_rows_for(int64_t K, bool big) {
  return (int)std::max<int64_t>(big ? kDbSliceRowsBig : kDbSliceRows, ceil_div(ceil_div(K, kMaxDbSlices), 8) * 8);
}

// The dW rows are cut into n_big long splits and, optionally, a few short ones: the short units are
// dispatched last and fill the CUs that finish early, which evens out schedules whose unit count just
// misses a multiple of the CU count.
static BigChoice choose_big(int64_t M, int64_t K, int32_t Cin, int32_t Cout) {
  thread_local BigChoice cache[32] = {};
  thread_local int next = 0;
  for (const BigChoice& c : cache)
    if (c.M == M && c.K == K && c.Cin == Cin && c.Cout == Cout && c.splits > 0) return c;
  const int64_t tiles_n = ceil_div(Cin, big::BT);
  const int64_t tiles_w = ceil_div(Cout, big::BT) * tiles_n;
  const int64_t nk_x = Cout / big::KB;
  // the helpers that share the launch (all of them assumed wanted)
  const int64_t n_zero = big_zero_blocks(M);
  const int64_t l_zero = kNsFixedHelper + (M - K) * Cin * 2 / n_zero / kHelperBytesPerNs;
  const int64_t slice_rows = db_slice_rows_for(K, true);
  const int64_t n_db = ceil_div(Cout, 256) * ceil_div(K, slice_rows);
  const int64_t l_db = kNsFixedHelper + slice_rows * 512 / kHelperBytesPerNs;
  BigChoice best{M, K, Cin, Cout, 0, 0, 0, 0, 256, {0, 1, 2}, 0.0};
  double best_cost = 0;
  auto l_dw = [](int64_t rows) { return kNsFixedDw + kNsStageDw * ceil_div(rows, big::KB); };
  static const int small_rows[] = {0, 256, 384, 512, 768, 1024, 1536};
  for (int bm : {256, 128, 64}) {
    const int64_t n_dx = ceil_div(K, bm) * tiles_n;
    const int64_t l_dx = bm == 256 ? kNsFixedDx256 + kNsStage256 * nk_x
                                   : (bm == 128 ? kNsFixedDx128 + kNsStage128 * nk_x : kNsFixedDx64 + kNsStage64 * nk_x);
    for (int64_t a : small_rows) {
      for (int64_t ns = (a ? 1 : 0); ns <= (a ? 4 : 0); ++ns) {
        if (ns * a >= K) break;
        for (int64_t nb = 1; nb <= 16; ++nb) {
          const int64_t A = ceil_div(ceil_div(K - ns * a, nb), 64) * 64;
          if (A > kBigMaxRowsPerSplit || A <= a) continue;
          const int64_t nb_real = a ? nb : ceil_div(K, A);
          const int64_t rest = K - std::min<int64_t>(K, nb_real * A);
          if (a && rest <= 0) continue;                        // the long splits already cover everything
          const int64_t ns_real = a ? ceil_div(rest, a) : 0;
          if (A < 512 && nb_real > 1) continue;                // splits shorter than 16 stages do not pay
          const int64_t kn[3] = {n_dx, tiles_w * nb_real, tiles_w * ns_real};
          const int64_t kl[3] = {l_dx, l_dw(std::min<int64_t>(A, K)), a ? l_dw(a) : 0};
          int order[3] = {0, 1, 2};
          std::sort(order, order + 3, [&](int x, int y) { return kl[x] > kl[y]; });   // longest kind first
          const int64_t n[5] = {kn[order[0]], kn[order[1]], kn[order[2]], n_zero, n_db};
          const int64_t l[5] = {kl[order[0]], kl[order[1]], kl[order[2]], l_zero, l_db};
          const int64_t end = simulate_grid(n, l, 5);
          const int64_t splits = nb_real + ns_real;
          // the reduction kernel that follows reads every split's fp32 copy of dW and writes dW
          const double cost = (double)end + 3000.0 + (double)(splits + 1) * Cout * Cin * 4.0 / kReduceBytesPerNs;
          if (best.splits == 0 || cost < best_cost) {
            best_cost = cost;
            best.splits = (int)splits; best.rps = (int)A; best.n_big = (int)nb_real; best.rows_small = (int)(ns_real ? a : 0);
            best.dx_bm = bm;
            for (int q = 0; q < 3; ++q) best.seg_order[q] = order[q];
            double work = 0;
            for (int q = 0; q < 5; ++q) work += (double)n[q] * (double)l[q];
            best.fill = work / ((double)kNumCU * (double)end);
          }
        }
      }
    }
  }
  if (options().debug_plan)
    std::fprintf(stderr, "sbp plan M=%lld K=%lld %d->%d: dx rows %d, %d long splits of %d rows, short splits of %d rows (%d splits), order %d%d%d, fill %.2f, cost %.1f us\n",
                 (long long)M, (long long)K, Cin, Cout, best.dx_bm, best.n_big, best.rps, best.rows_small, best.splits, best.seg_order[0],
                 best.seg_order[1], best.seg_order[2], best.fill, best_cost / 1e3);
  cache[next] = best;
  next = (next + 1) % 32;
  return best;
}

LinearPlan plan_linear(int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype, uint32_t flags) {
  LinearPlan p{};
  p.mfma = dtype == SBP_BF16 && Cin % 8 == 0 && Cout % 8 == 0;
  p.bm_w = p.bn_w = 128;
  p.nw_w = 4;
  p.kb = 64;
  int splits = 1;
  const Options opt = options();   // explicit overrides (sbp_set_option); every field is validated when it is set
  if (K > 0 && p.mfma) {
    const bool fits = Cout % big::KB == 0 && (uint64_t)M * (uint64_t)std::max(Cin, Cout) * 2u < (1ull << 32) &&
                      ceil_div(K, kBigMaxRowsPerSplit) <= 64;
    // it pays where whole 256-wide tiles exist and the simulated schedule keeps the CUs reasonably busy
    const bool pays = opt.tile_mode == 0 && Cin >= big::BT && Cout >= big::BT && K >= 1024 &&
                      choose_big(M, K, Cin, Cout).fill >= 0.45;
    p.big = fits && (opt.tile_mode == 2 || pays);
  }
  bool two_sizes = false;
  if (p.big) {
    const BigChoice c = choose_big(M, K, Cin, Cout);
    p.bm_w = p.bn_w = big::BT;
    p.kb = big::KB;
    p.dx_bm = c.dx_bm;
    splits = c.splits;
    p.rows_per_split = c.rps; p.n_big = c.n_big; p.rows_small = c.rows_small;
    for (int q = 0; q < 3; ++q) p.seg_order[q] = c.seg_order[q];
    two_sizes = true;
    if (c.splits == 0) {       // no simulated schedule fits (forced engine on an odd size): equal splits of the largest legal length
      splits = (int)ceil_div(K, kBigMaxRowsPerSplit);
      two_sizes = false;
      p.dx_bm = 256;
      p.seg_order[0] = 1; p.seg_order[1] = 0; p.seg_order[2] = 2;
    }
    if (opt.dxbm) p.dx_bm = opt.dxbm;
    const ShapePlan* sp = nullptr;                               // a schedule by hand: for this shape, else for all
    for (int i = 0; i < opt.nplans; ++i)
      if (opt.plans[i].cin == Cin && opt.plans[i].cout == Cout) sp = &opt.plans[i];
    if (!sp)
      for (int i = 0; i < opt.nplans; ++i)
        if (opt.plans[i].cin == 0) sp = &opt.plans[i];
    if (sp) {
      const int A = sp->rows_long, nb = sp->n_long, a = sp->rows_short;
      if (A <= kBigMaxRowsPerSplit && (int64_t)nb * A < K + A && (a > 0 || (int64_t)nb * A >= K)) {   // else: infeasible here, ignored
        p.dx_bm = sp->bm;
        p.rows_per_split = A; p.n_big = (int)std::min<int64_t>(nb, ceil_div(K, A)); p.rows_small = a;
        const int64_t rest = K - std::min<int64_t>(K, (int64_t)p.n_big * A);
        if (rest <= 0) p.rows_small = 0;
        splits = p.n_big + (p.rows_small ? (int)ceil_div(rest, p.rows_small) : 0);
        two_sizes = true;
        p.seg_order[0] = 1; p.seg_order[1] = 0; p.seg_order[2] = 2;
        if (opt.order_set) for (int q = 0; q < 3; ++q) p.seg_order[q] = opt.order[q];
      }
    }
    if (opt.splits) {                                          // equal splits, dW units first
      splits = std::max<int>(opt.splits, (int)ceil_div(K, kBigMaxRowsPerSplit));
      two_sizes = false;
      p.seg_order[0] = 1; p.seg_order[1] = 0; p.seg_order[2] = 2;
    }
  } else if (K > 0) {
    if (p.mfma) {
      if (opt.tile_mode == 1) { p.bm_w = opt.tile_bm; p.bn_w = opt.tile_bn; p.nw_w = opt.tile_nw; p.kb = opt.tile_kb; }
      // enough blocks to fill the chip's block slots once, each split at least 4 stages long
      const int64_t tiles = ceil_div(Cout, p.bm_w) * ceil_div(Cin, p.bn_w);
      const int64_t slots = (p.bm_w + p.bn_w <= 256) ? 2 * kNumCU : kNumCU;
      int64_t want = std::max<int64_t>(1, slots / tiles);
      int64_t max_by_len = std::max<int64_t>(1, K / (4 * 64));
      splits = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, max_by_len), 64));
      splits = (int)std::max<int64_t>(splits, ceil_div(K, kMaxRowsPerSplit));   // the split's row ids sit in LDS
      // Small layers, whose workgroups (nearly) all find a slot at once (two per CU): the launch then lasts as long as
      // its longest workgroup, a dX tile walking the whole of Cout with one stage in flight.  Tiles of 64 rows in a
      // ring of three keep two stages in flight in the same LDS (ViT-Tiny MLP: 52.9 -> 50.3 us per step); where the
      // tiles queue for slots the 128-row tiles move fewer bytes and win (detection shapes).
      p.dx_bm = 128;
      if (p.bm_w == 128 && p.kb == 64 && ceil_div(K, 128) * ceil_div(Cin, 128) + tiles * splits + 64 <= 700) p.dx_bm = 64;   // (measured: still ahead at 650 workgroups, behind at 770)
      if (opt.dxrows) p.dx_bm = opt.dxrows == 64 && p.bm_w == 128 && p.kb == 64 ? 64 : 128;
    } else {
      splits = (int)std::max<int64_t>(1, std::min<int64_t>(ceil_div(K, 512), 64));
    }
  }
  if (!two_sizes) {
    int64_t rps = K > 0 ? ceil_div(K, splits) : 0;
    rps = ceil_div(rps, 64) * 64;
    if (rps > 0) splits = (int)ceil_div(K, rps);
    p.rows_per_split = (int)rps;
    p.n_big = splits;
    p.rows_small = 0;
  }
  p.splits = splits;
  size_t off = 0;
  p.off_partial = off;
  p.db_slice_rows = db_slice_rows_for(K, p.big);
  p.db_slices = p.mfma ? (int)std::max<int64_t>(1, ceil_div(K, p.db_slice_rows)) : splits;
  // db partials: one per slice of the column-sum blocks, or (large tiles, db out of the dW units) per split and tile column
  const int64_t db_parts = std::max<int64_t>(p.db_slices, (int64_t)splits * (p.big ? ceil_div(Cin, big::BT) : 1));
  off += align_up(((size_t)splits * Cout * Cin + (size_t)db_parts * Cout) * sizeof(float), 256);
  p.off_inv = off;
  if (!(flags & SBP_FLAG_DX_COMPACT)) off += align_up((size_t)M * sizeof(int32_t), 256);
  p.off_xrows = off;      // X_k copied back to rows, for the engines that do not read the row-group layout
  if (flags & SBP_FLAG_XK_KMAJOR) off += align_up((size_t)K * Cin * 2, 256);
  p.bytes = off;
  return p;
}

template <typename T>
static int32_t launch_plain(const LinearPlan& p, const T* dY, const int32_t* idx_in, const int32_t* idx_out,
                            const T* Xk, const T* W, int64_t K, int32_t Cin, int32_t Cout, float* part,
                            float* dbp, bool want_dw, bool want_db, T* dX, hipStream_t s) {
  if (want_dw) {
    long long nW = (long long)Cin * Cout;
    dim3 grid((unsigned)std::min<long long>(ceil_div(nW, NTHREADS), 8192), p.splits);
    SBP_LAUNCH(SBP_PROF_DW_GEMM, s, (plain_dw_kernel<T>), grid, dim3(NTHREADS), 0, s, dY, idx_in, Xk, (int)K, Cin, Cout,
                       p.rows_per_split, part);
  }
  if (want_db) {
    dim3 grid((unsigned)ceil_div(Cout, NTHREADS), p.splits);
    SBP_LAUNCH(SBP_PROF_COLSUM, s, (plain_db_kernel<T>), grid, dim3(NTHREADS), 0, s, dY, idx_in, (int)K, Cout,
                       p.rows_per_split, dbp);
  }
  if (dX) {
    long long total = (long long)K * Cin;
    unsigned blocks = (unsigned)std::min<long long>(ceil_div(total, NTHREADS), 65535);
    SBP_LAUNCH(SBP_PROF_DX_GEMM, s, (plain_dx_kernel<T>), dim3(blocks), dim3(NTHREADS), 0, s, dY, idx_in, idx_out, W,
                       (long long)K, Cin, Cout, dX);
  }
  return SBP_OK;
}

// Dynamic LDS beyond 64 KB has to be granted per kernel; asked for once per kernel and size (one device per process).
template <typename KernelT>
static void allow_big_lds(KernelT kernel, size_t lds) {
  static std::mutex m;                          // one instance of these per kernel type
  static size_t granted = 0;
  static KernelT granted_for = nullptr;
  std::lock_guard<std::mutex> lock(m);
  if (lds <= 64 * 1024 || (granted_for == kernel && lds <= granted)) return;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess) {
    granted = lds;
    granted_for = kernel;
  }
}

// fills in the segment sizes and their order; returns the number of workgroups, *lds_out the LDS bytes a workgroup needs
template <int BM, int BN, int NW, int KB, int NSTAGE, int BMX = BM, int NSX = NSTAGE>
static unsigned prepare_linear_bwd(const LinearPlan& p, LinArgs& a, bool want_dx, bool want_dw, bool want_zero, size_t* lds_out) {
  // stage ring + the row-id table of a dW split (rows_per_split rounded up to the stage length), or the dX tiles' ring
  *lds_out = std::max((size_t)NSTAGE * (BM + BN) * KB * 2 + (size_t)(p.rows_per_split + KB) * sizeof(int),
                      (size_t)NSX * (BMX + BN) * KB * 2);
  const long long tiles_n = ceil_div(a.Cin, BN);
  a.n_zero = want_zero ? (int)std::min<long long>(128, std::max<long long>(8, ceil_div((long long)a.M, 64 * NW))) : 0;
  const int n_db = a.dbp ? (int)(ceil_div(a.Cout, 256) * p.db_slices) : 0;
  a.n_helper = (int)(8 * ceil_div(a.n_zero + n_db, 8));
  a.n_dx = want_dx ? (int)(8 * ceil_div(ceil_div(a.K, BMX) * tiles_n, 8)) : 0;
  a.n_dw = want_dw ? (int)(8 * ceil_div(ceil_div(a.Cout, BM) * tiles_n * p.splits, 8)) : 0;
  const unsigned grid = (unsigned)(a.n_helper + a.n_dx + a.n_dw);
  if (grid == 0) return 0;
  // Longest kind first.  Lengths in nanoseconds, read from the device clock on the detection and ViT-Tiny shapes: a
  // tile costs about 3 us plus 1 us per stage of 64 (two stages in flight do not hide the memory latency), a
  // streaming block 1.8 us plus its bytes at what one CU gets while the others stream too.
  const int64_t len[3] = {
      3000 + 1000 * ceil_div(a.Cout, 64), 3000 + 1000 * ceil_div(p.rows_per_split, 64),
      1800 + std::max<int64_t>(a.n_zero ? (int64_t)(a.M - a.K) * a.Cin * 2 / a.n_zero : 0, n_db ? (int64_t)a.db_slice_rows * 512 : 0) / 40};
  for (int q = 0; q < 3; ++q) a.seg_order[q] = q;
  std::sort(a.seg_order, a.seg_order + 3, [&](int x, int y) { return len[x] != len[y] ? len[x] > len[y] : x < y; });
  const Options opt = options();
  if (opt.order_set)                                // the order by hand (a permutation, checked when it was set)
    for (int q = 0; q < 3; ++q) a.seg_order[q] = opt.order[q];
  return grid;
}

template <int BM, int BN, int NW, int KB, int NSTAGE, int BMX = BM, int NSX = NSTAGE>
static void launch_linear_bwd(const LinearPlan& p, LinArgs a, bool want_dx, bool want_dw, bool want_zero,
                              hipStream_t s) {
  size_t lds = 0;
  const unsigned grid = prepare_linear_bwd<BM, BN, NW, KB, NSTAGE, BMX, NSX>(p, a, want_dx, want_dw, want_zero, &lds);
  if (grid == 0) return;
  allow_big_lds(linear_bwd_kernel<BM, BN, NW, KB, NSTAGE, BMX, NSX>, lds);
  SBP_LAUNCH(SBP_PROF_DW_GEMM, s, (linear_bwd_kernel<BM, BN, NW, KB, NSTAGE, BMX, NSX>), dim3(grid), dim3(64 * NW), lds, s, a);
}

// Writes +0 to the rows of out[M][row_bytes] that are not in idx (inv: inverse map, see mark_rows_kernel).
void launch_build_inverse(const int32_t* idx, int64_t K, int32_t* inv, hipStream_t s) {
  if (K > 0)
    SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, mark_rows_kernel, dim3((unsigned)ceil_div(K, NTHREADS)), dim3(NTHREADS), 0, s, idx,
               (int)K, inv);
}

void launch_zero_dropped_rows(const int32_t* idx, const int32_t* inv, int64_t K, int64_t M, int64_t row_bytes,
                              void* out, hipStream_t s) {
  if (row_bytes % 16 == 0 && (uintptr_t)out % 16 == 0) {
    const int ppr = (int)(row_bytes / 16);
    unsigned blocks = (unsigned)std::min<long long>(ceil_div(M * ppr, NTHREADS), 8192);
    SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, zero_dropped_rows_kernel, dim3(blocks), dim3(NTHREADS), 0, s, idx, inv, (int)K,
               (long long)M, ppr, (uint4*)out);
  } else if (row_bytes % 4 == 0 && (uintptr_t)out % 4 == 0) {
    const int C = (int)(row_bytes / 4);
    unsigned blocks = (unsigned)std::min<long long>(ceil_div(M * C, NTHREADS), 8192);
    SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, (zero_dropped_rows_elem_kernel<uint32_t>), dim3(blocks), dim3(NTHREADS), 0, s, idx, inv,
               (int)K, (long long)M, C, (uint32_t*)out);
  } else {
    const int C = (int)(row_bytes / 2);
    unsigned blocks = (unsigned)std::min<long long>(ceil_div(M * C, NTHREADS), 8192);
    SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, (zero_dropped_rows_elem_kernel<uint16_t>), dim3(blocks), dim3(NTHREADS), 0, s, idx, inv,
               (int)K, (long long)M, C, (uint16_t*)out);
  }
}

static void launch_linear_big(const LinearPlan& p, LinArgs a, bool want_dx, bool want_dw, bool want_zero, hipStream_t s) {
  // behind the ring: the row ids of a dW split (read one stage ahead) or the 256 output rows of a dX tile
  const size_t lds = (size_t)big::RING + std::max<size_t>((size_t)(std::max(p.rows_per_split, p.rows_small) + 2 * big::KB), big::BT) * sizeof(int);
  allow_big_lds(linear_big_kernel, lds);
  const long long tiles_n = ceil_div(a.Cin, big::BT);
  a.n_zero = want_zero ? big_zero_blocks(a.M) : 0;
  // with dW wanted, db comes out of the dW units (one slice per split and tile column); column-sum blocks
  // that read dY_k once more only where db is wanted alone
  a.db_in_dw = a.dbp && want_dw ? 1 : 0;
  const int n_db = a.dbp && !a.db_in_dw ? (int)(ceil_div(a.Cout, 256) * p.db_slices) : 0;
  a.n_helper = a.n_zero + n_db;
  a.dx_bm = p.dx_bm;
  a.n_dx = want_dx ? (int)(ceil_div(a.K, p.dx_bm) * tiles_n) : 0;
  const long long tiles_w = ceil_div(a.Cout, big::BT) * tiles_n;
  a.n_big = p.n_big; a.rows_small = p.rows_small;
  a.n_dw_big = want_dw ? (int)(tiles_w * p.n_big) : 0;
  a.n_dw = a.n_dw_big + (want_dw ? (int)(tiles_w * (p.splits - p.n_big)) : 0);
  for (int q = 0; q < 3; ++q) a.seg_order[q] = p.seg_order[q];
  const unsigned grid = (unsigned)(a.n_helper + a.n_dx + a.n_dw);
  if (grid == 0) return;
  SBP_LAUNCH(SBP_PROF_DW_GEMM, s, linear_big_kernel, dim3(grid), dim3(256), lds, s, a);
}

// lanes per output of the split reductions: small weight matrices cut into many splits get several
static int reduce_lanes(long long total, int deepest) { return total <= 20000 && deepest >= 16 ? 8 : (total <= 40000 && deepest >= 8 ? 4 : 1); }

int32_t launch_backward_linear(const LinearPlan& p, const void* dY, const int32_t* idx, const int32_t* inv_in,
                               const void* Xk, const void* W, int64_t M, int64_t K, int32_t Cin, int32_t Cout,
                               int32_t dtype, void* dW, float* db, void* dX, void* ws, uint32_t flags,
                               hipStream_t s) {
  const int eb = dtype == SBP_F32 ? 4 : 2;
  const bool dy_compact = flags & SBP_FLAG_DY_COMPACT, dx_compact = flags & SBP_FLAG_DX_COMPACT;
  const int accumulate = (flags & SBP_FLAG_ACCUMULATE_DW) ? 1 : 0;
  const bool dw_bf16 = flags & SBP_FLAG_DW_OUT_BF16;
  const int32_t* idx_in = dy_compact ? nullptr : idx;
  const int32_t* idx_out = dx_compact ? nullptr : idx;
  float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_partial);
  float* dbp = part + (size_t)p.splits * Cout * Cin;
  int32_t* inv_ws = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + p.off_inv);
  const int32_t* inv = inv_in;
  const long long nW = (long long)Cin * Cout;

  if (K == 0) {  // nothing kept: gradients are zero
    if (!accumulate) {   // a sum over no splits, written in dW's type
      const unsigned blocks = (unsigned)std::min<long long>(ceil_div(nW + Cout, NTHREADS), 4096);
      if (dw_bf16)
        SBP_LAUNCH(SBP_PROF_OTHER, s, reduce_splits_scalar_kernel<true>, dim3(blocks), dim3(NTHREADS), 0, s, nullptr, 0, nW, dW,
                   nullptr, Cout, db, 0);
      else
        SBP_LAUNCH(SBP_PROF_OTHER, s, reduce_splits_scalar_kernel<false>, dim3(blocks), dim3(NTHREADS), 0, s, nullptr, 0, nW, dW,
                   nullptr, Cout, db, 0);
    }
    if (dX && !dx_compact)
      SBP_LAUNCH(SBP_PROF_OTHER, s, fill_zero_kernel, dim3(1024), dim3(NTHREADS), 0, s, (uint32_t*)dX,
                         (long long)M * Cin * eb / 4);
    return check_launch("backward_linear (K = 0)");
  }

  const bool scatter = dX && !dx_compact;
  if (scatter && !inv) {   // no inverse map from the caller: build one (needs no clearing, see mark_rows_kernel)
    launch_build_inverse(idx, K, inv_ws, s);
    inv = inv_ws;
  }

  const bool aligned = ((uintptr_t)dY % 16 == 0) && ((uintptr_t)Xk % 16 == 0) && ((uintptr_t)W % 16 == 0) &&
                       ((uintptr_t)dX % 16 == 0);
  const bool use_mfma = p.mfma && aligned;
  bool kmajor = (flags & SBP_FLAG_XK_KMAJOR) && dW && Xk;
  if (kmajor && !(use_mfma && p.big && p.rows_per_split % 8 == 0 && p.rows_small % 8 == 0)) {
    void* rows = static_cast<char*>(ws) + p.off_xrows;
    const int32_t st = launch_kmajor_to_rows(Xk, K, Cin, rows, s);
    if (st != SBP_OK) return st;
    Xk = rows;
    kmajor = false;
  }
  if (use_mfma) {
    const uint16_t* dYh = static_cast<const uint16_t*>(dY);
    LinArgs a{};
    a.dY = dYh; a.idx_in = idx_in; a.idx_out = idx_out; a.idx = idx; a.inv = inv;
    a.Xk = static_cast<const uint16_t*>(Xk); a.W = static_cast<const uint16_t*>(W);
    a.dX = static_cast<uint16_t*>(dX); a.part = part; a.dbp = db ? dbp : nullptr;
    a.K = (int)K; a.M = (int)M; a.Cin = Cin; a.Cout = Cout;
    a.rows_per_split = p.rows_per_split; a.db_slice_rows = p.db_slice_rows;
    a.xk_kmajor = kmajor ? 1 : 0;
    const bool want_dx = dX != nullptr, want_dw = dW != nullptr;
    if (p.big)
      launch_linear_big(p, a, want_dx, want_dw, scatter, s);
    else if (p.bm_w == 256 && p.nw_w == 8 && p.kb == 32)
      launch_linear_bwd<256, 256, 8, 32, 4>(p, a, want_dx, want_dw, scatter, s);
    else if (p.bm_w == 256 && p.nw_w == 8)
      launch_linear_bwd<256, 256, 8, 64, 2>(p, a, want_dx, want_dw, scatter, s);
    else if (p.bm_w == 256 && p.kb == 32)
      launch_linear_bwd<256, 256, 4, 32, 4>(p, a, want_dx, want_dw, scatter, s);
    else if (p.bm_w == 256)
      launch_linear_bwd<256, 256, 4, 64, 2>(p, a, want_dx, want_dw, scatter, s);
    else if (p.kb == 32)
      launch_linear_bwd<128, 128, 4, 32, 4>(p, a, want_dx, want_dw, scatter, s);
    else if (p.dx_bm == 64)
      launch_linear_bwd<128, 128, 4, 64, 2, 64, 3>(p, a, want_dx, want_dw, scatter, s);
    else
      launch_linear_bwd<128, 128, 4, 64, 2>(p, a, want_dx, want_dw, scatter, s);
  } else if (dtype == SBP_F32) {
    launch_plain<float>(p, (const float*)dY, idx_in, idx_out, (const float*)Xk, (const float*)W, K, Cin, Cout, part,
                        dbp, dW != nullptr, db != nullptr, (float*)dX, s);
  } else {
    launch_plain<uint16_t>(p, (const uint16_t*)dY, idx_in, idx_out, (const uint16_t*)Xk, (const uint16_t*)W, K, Cin,
                           Cout, part, dbp, dW != nullptr, db != nullptr, (uint16_t*)dX, s);
  }

  if (dW || db) {
    if (nW % 4 == 0) {
      const long long total = (dW ? nW / 4 : 0) + (db ? Cout : 0);
      // (large tiles with dW: db partials come from the dW units, one per split and tile column)
      const int nsplit_b = use_mfma && !(p.big && dW) ? p.db_slices : (p.big ? p.splits * (int)ceil_div(Cin, big::BT) : p.splits);
      const int deepest = std::max(dW ? p.splits : 0, db ? nsplit_b : 0);
      const int G = reduce_lanes(total, deepest);
      unsigned blocks = (unsigned)std::min<long long>(ceil_div(total * G, NTHREADS), 4096);
      auto kernel = dw_bf16 ? (G == 8 ? reduce_splits_kernel<8, true> : (G == 4 ? reduce_splits_kernel<4, true> : reduce_splits_kernel<1, true>))
                            : (G == 8 ? reduce_splits_kernel<8, false> : (G == 4 ? reduce_splits_kernel<4, false> : reduce_splits_kernel<1, false>));
      SBP_LAUNCH(SBP_PROF_REDUCE, s, kernel, dim3(blocks), dim3(NTHREADS), 0, s, part, p.splits, nW, dW, dbp, nsplit_b, Cout, db,
                 accumulate);
    } else {
      const long long total = (dW ? nW : 0) + (db ? Cout : 0);
      unsigned blocks = (unsigned)std::min<long long>(ceil_div(total, NTHREADS), 4096);
      if (dw_bf16)   // plain path only: db partials follow the dW splits
        SBP_LAUNCH(SBP_PROF_REDUCE, s, reduce_splits_scalar_kernel<true>, dim3(blocks), dim3(NTHREADS), 0, s, part, p.splits, nW,
                   dW, dbp, Cout, db, accumulate);
      else
        SBP_LAUNCH(SBP_PROF_REDUCE, s, reduce_splits_scalar_kernel<false>, dim3(blocks), dim3(NTHREADS), 0, s, part, p.splits, nW,
                   dW, dbp, Cout, db, accumulate);
    }
  }

  if (scatter && !use_mfma)   // the MFMA launch zero-fills by itself
    launch_zero_dropped_rows(idx, inv, K, M, (int64_t)Cin * eb, dX, s);
  return check_launch("backward_linear");
}

// ------------------------------------------------------------------------------------------------
// Several independent layers in one launch (linear_multi_kernel) + one reduction launch.
// ------------------------------------------------------------------------------------------------
struct RedLayer {
  const float* part; const float* dbp; void* dW; float* db;
  long long nW;
  int nsplit_w, nsplit_b, Cout, accumulate, bf16out, blk_start, nblk;
  int G;       // lanes per output (1, 4 or 8): lane g adds a contiguous run of the splits, the G sums are added in lane order
};
struct RedMultiArgs { int n; RedLayer lay[kMaxBatch]; };

// the split reduction of every layer of a batch: blocks [blk_start, blk_start + nblk) serve layer i; per output the
// partial sums are added in a fixed order (as in reduce_splits_kernel)
__global__ void __launch_bounds__(NTHREADS) reduce_multi_kernel(const RedMultiArgs a) {
  int li = 0;
  for (int i = 1; i < a.n; ++i)
    if ((int)blockIdx.x >= a.lay[i].blk_start) li = i;
  const RedLayer& r = a.lay[li];
  const int G = r.G, g = threadIdx.x & (G - 1), lane = threadIdx.x & 63;
  const long long nW4 = r.dW ? r.nW / 4 : 0;
  const long long total = nW4 + (r.db ? r.Cout : 0);
  const int lg = G == 8 ? 3 : (G == 4 ? 2 : 0);          // G is 1, 4 or 8
  const long long first = (((long long)blockIdx.x - r.blk_start) * NTHREADS + threadIdx.x) >> lg;
  for (long long e = first; e < total; e += ((long long)r.nblk * NTHREADS) >> lg) {
    if (e < nW4) {
      const int chunk = (r.nsplit_w + G - 1) / G, s_begin = g * chunk, s_end = min(r.nsplit_w, s_begin + chunk);
      float4 acc = make_float4(0, 0, 0, 0);
      for (int s0 = s_begin; s0 < s_end; s0 += 4) {
        float4 p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          p[u] = s0 + u < s_end ? reinterpret_cast<const float4*>(r.part + (long long)(s0 + u) * r.nW)[e]
                                : make_float4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < 4; ++u) { acc.x += p[u].x; acc.y += p[u].y; acc.z += p[u].z; acc.w += p[u].w; }
      }
      if (G > 1) {
        const float4 own = acc;
        for (int k = 1; k < G; ++k) {
          const int src = (lane & ~(G - 1)) + k;
          acc.x += __shfl(own.x, src); acc.y += __shfl(own.y, src); acc.z += __shfl(own.z, src); acc.w += __shfl(own.w, src);
        }
      }
      if (g == 0) {
        if (r.bf16out) {
          if (r.accumulate) {
            const float4 old = load_dw4<true>(r.dW, e);
            acc.x = old.x + acc.x; acc.y = old.y + acc.y; acc.z = old.z + acc.z; acc.w = old.w + acc.w;
          }
          store_dw4<true>(r.dW, e, acc);
        } else {
          if (r.accumulate) {
            const float4 old = load_dw4<false>(r.dW, e);
            acc.x = old.x + acc.x; acc.y = old.y + acc.y; acc.z = old.z + acc.z; acc.w = old.w + acc.w;
          }
          store_dw4<false>(r.dW, e, acc);
        }
      }
    } else {
      const long long o = e - nW4;
      const int chunk = (r.nsplit_b + G - 1) / G, s_begin = g * chunk, s_end = min(r.nsplit_b, s_begin + chunk);
      float acc = 0.f;
      for (int s0 = s_begin; s0 < s_end; s0 += 8) {
        float p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) p[u] = s0 + u < s_end ? r.dbp[(long long)(s0 + u) * r.Cout + o] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += p[u];
      }
      if (G > 1) {
        const float own = acc;
        for (int k = 1; k < G; ++k) acc += __shfl(own, (lane & ~(G - 1)) + k);
      }
      if (g == 0) r.db[o] = r.accumulate ? r.db[o] + acc : acc;
    }
  }
}

// Is this layer one the multi-layer launch can take?  (bf16 on the matrix cores, the large-tile engine's limits,
// something kept, 16-byte aligned tensors; everything else runs layer by layer.)
static bool batch_layer_fits(const sbp_linear_layer& l, int32_t dtype) {
  if (dtype != SBP_BF16 || l.K < 1) return false;
  if (l.Cin % 8 || l.Cout % big::KB) return false;
  if ((uint64_t)l.M * (uint64_t)std::max(l.Cin, l.Cout) * 2u >= (1ull << 32)) return false;
  if (ceil_div(l.K, kBigMaxRowsPerSplit) > 64) return false;
  if (((uintptr_t)l.dY | (uintptr_t)l.X_k | (uintptr_t)l.W | (uintptr_t)l.dX) & 15) return false;
  if (l.dW && (l.flags & SBP_FLAG_DW_OUT_BF16) == 0 && ((uintptr_t)l.dW & 15)) return false;
  return true;
}

// Unit costs inside a batched launch, read from the per-unit time stamps of the ViT-Base block (sbp_profile_timeline) with
// the per-XCD queues in place: every CU is in matrix-core code for the whole launch and the chip then runs at 1.6-1.7 GHz
// (1.3 GHz before the queues cut the traffic between the L2s and memory by a third); dW units of 99 / 66 stages took
// 95 / 63 us, dX tiles of 96 / 72 / 24 stages 89 / 67 / 29 us.  The shorter dX tiles are scaled as in the single-layer costs.
static constexpr int64_t kNsStageBatchDb = 110;         // extra per stage in which a dW unit sums db columns
static constexpr int64_t kNsFixedBatchDw = 3000, kNsStageBatchDw = 930, kNsFixedBatch = 9000, kNsStageBatch256 = 830,
                         kNsStageBatch128 = 500, kNsStageBatch64 = 400;
struct BatchLayerChoice { int dx_bm, splits; };
static int64_t split_rows(int64_t K, int64_t splits) { return ceil_div(ceil_div(K, splits), 64) * 64; }   // rows of each equal split

// The jobs of a batch for given per-layer choices: {units, unit length, layer, kind}.
struct Job { int64_t n, len; int layer, kind; };
static constexpr int kMaxJobs = 4 * kMaxBatch;
static int batch_jobs(const sbp_linear_layer* L, int n, const BatchLayerChoice* c, Job* out, double* reduce_ns) {
  int nj = 0;
  double red = 0;
  for (int i = 0; i < n; ++i) {
    const sbp_linear_layer& l = L[i];
    const int64_t tiles_n = ceil_div(l.Cin, big::BT), tiles_w = ceil_div(l.Cout, big::BT) * tiles_n, nk_x = l.Cout / big::KB;
    if (l.dX) {
      const int bm = c[i].dx_bm;
      const int64_t len = kNsFixedBatch + (bm == 256 ? kNsStageBatch256 : (bm == 128 ? kNsStageBatch128 : kNsStageBatch64)) * nk_x;
      out[nj++] = Job{ceil_div(l.K, bm) * tiles_n, len, i, 0};
      if (!(l.flags & SBP_FLAG_DX_COMPACT) && l.M > l.K) {
        const int64_t nz = big_zero_blocks(l.M);
        out[nj++] = Job{nz, kNsFixedHelper + (l.M - l.K) * l.Cin * 2 / nz / kHelperBytesPerNs, i, 3};
      }
    }
    if (l.dW) {
      const int64_t rps = split_rows(l.K, c[i].splits);
      const int64_t nsp = ceil_div(l.K, rps);
      const int64_t stages = ceil_div(std::min<int64_t>(rps, l.K), big::KB);
      // with db wanted every dW unit sums the db columns of its panel in its share (1 / tiles_n) of the stages
      const int64_t db_stages = l.db ? ceil_div(stages, tiles_n) : 0;
      out[nj++] = Job{tiles_w * nsp, kNsFixedBatchDw + kNsStageBatchDw * stages + kNsStageBatchDb * db_stages, i, 1};
      const bool direct = nsp == 1 && !(l.flags & (SBP_FLAG_ACCUMULATE_DW | SBP_FLAG_DW_OUT_BF16));
      if (!direct) red += (double)(nsp + 1) * l.Cout * l.Cin * 4.0 / kReduceBytesPerNs;
    }
    if (l.db && !l.dW) {               // (with dW the column sums come out of the dW units)
      const int64_t slice_rows = db_slice_rows_for(l.K, true);
      out[nj++] = Job{ceil_div(l.Cout, 256) * ceil_div(l.K, slice_rows), kNsFixedHelper + slice_rows * 512 / kHelperBytesPerNs, i, 4};
    }
  }
  *reduce_ns = red;
  return nj;
}

// The eight queues, by simulated list scheduling: units in the order longest kind first (helpers last), each to the
// XCD whose next CU frees first - but the XCD that took the previous unit keeps taking units while one of its CUs is
// (nearly) as early: consecutive units of a job, which share operand panels, land in one L2 in runs of a round of 32
// or more, a job lies on as few XCDs as an even finish allows, and short units fill what the long ones leave.  The
// queues list the units of an XCD in the order of their simulated starts.  Returns the simulated finish time in ns,
// or -1 if a queue would need more than kMaxEnt entries.
struct XcdQueues {
  int nent[kNumXCD], nq[kNumXCD];
  XcdEntry ent[kNumXCD][kMaxEnt];
  int64_t len[kNumXCD][kMaxEnt];
  int cnt[kNumXCD][kMaxEnt];
};
static int64_t partition_xcd(const Job* jobs, int nj, XcdQueues* out) {
  XcdQueues& Q = *out;
  const bool spread = options().batch_spread;     // override: no affinity, consecutive units on consecutive XCDs
  int order[kMaxJobs];
  for (int j = 0; j < nj; ++j) order[j] = j;
  std::stable_sort(order, order + nj, [&](int u, int v) {
    const bool hu = jobs[u].kind == 3 || jobs[u].kind == 4, hv = jobs[v].kind == 3 || jobs[v].kind == 4;
    return hu != hv ? hv : jobs[u].len > jobs[v].len;
  });
  using MinHeap = std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>>;
  MinHeap cu[kNumXCD];
  for (int x = 0; x < kNumXCD; ++x) {
    Q.nent[x] = Q.nq[x] = 0;
    for (int i = 0; i < kNumCU / kNumXCD; ++i) cu[x].push(0);
  }
  int64_t end = 0;
  int cur = 0;
  for (int t = 0; t < nj; ++t) {
    const Job& jb = jobs[order[t]];
    const int64_t slack = spread ? 0 : jb.len / 4;
    for (int64_t u = 0; u < jb.n; ++u) {
      if (spread) cur = (cur + 1) & (kNumXCD - 1);
      int best = cur;
      for (int x = 0; x < kNumXCD; ++x)
        if (cu[x].top() + (x == cur ? 0 : slack) < cu[best].top() + (best == cur ? 0 : slack)) best = x;
      const int64_t fin = cu[best].top() + jb.len;
      cu[best].pop();
      cu[best].push(fin);
      end = std::max(end, fin);
      cur = best;
      int& ne = Q.nent[best];
      XcdEntry* last = ne > 0 ? &Q.ent[best][ne - 1] : nullptr;
      const bool same_job = last && last->layer == jb.layer && last->kind == jb.kind;
      if (same_job && Q.cnt[best][ne - 1] == 1 && u > last->unit0 && u - last->unit0 < 128) {
        last->stride = (signed char)(u - last->unit0);          // the second unit of a run fixes its stride
        ++Q.cnt[best][ne - 1];
      } else if (same_job && Q.cnt[best][ne - 1] > 1 && last->unit0 + (int64_t)Q.cnt[best][ne - 1] * last->stride == u) {
        ++Q.cnt[best][ne - 1];
      } else {
        if (ne == kMaxEnt) return -1;
        Q.ent[best][ne] = XcdEntry{Q.nq[best], (int)u, (short)jb.layer, (signed char)jb.kind, 1};
        Q.len[best][ne] = jb.len;
        Q.cnt[best][ne] = 1;
        ++ne;
      }
      ++Q.nq[best];
    }
  }
  return end;
}

static double batch_cost(const sbp_linear_layer* L, int n, const BatchLayerChoice* c) {
  Job jobs[kMaxJobs];
  double red = 0;
  const int nj = batch_jobs(L, n, c, jobs, &red);
  XcdQueues Q;
  const int64_t end = partition_xcd(jobs, nj, &Q);
  if (end < 0) return 1e30;
  return (double)end + (red > 0 ? 3000.0 + red : 0.0);
}

// Per-layer tile height and split count of a batch: coordinate descent on the simulated finish time of the whole
// grid plus the reduction's time, from tall tiles and two splits; cached per batch signature.
static void choose_batch(const sbp_linear_layer* L, int n, BatchLayerChoice* c) {
  struct Key { int64_t M, K; int32_t Cin, Cout; uint32_t flags; int want; };
  struct Entry { int n; Key k[kMaxBatch]; BatchLayerChoice c[kMaxBatch]; };
  thread_local Entry cache[8] = {};
  thread_local int next = 0;
  Key key[kMaxBatch];
  for (int i = 0; i < n; ++i)
    key[i] = Key{L[i].M, L[i].K, L[i].Cin, L[i].Cout, L[i].flags, (L[i].dW ? 1 : 0) | (L[i].db ? 2 : 0) | (L[i].dX ? 4 : 0)};
  const Options opt = options();
  int min_splits[kMaxBatch];
  for (int i = 0; i < n; ++i) min_splits[i] = (int)ceil_div(L[i].K, kBigMaxRowsPerSplit);
  auto overrides = [&]() {                        // explicit overrides (tests, sweeps) on top of the automatic choice
    for (int i = 0; i < n; ++i) {
      if (opt.dxbm) c[i].dx_bm = opt.dxbm;
      if (opt.splits) c[i].splits = std::max(opt.splits, min_splits[i]);
    }
  };
  for (const Entry& e : cache) {
    if (e.n != n) continue;
    bool same = true;
    for (int i = 0; i < n && same; ++i)
      same = e.k[i].M == key[i].M && e.k[i].K == key[i].K && e.k[i].Cin == key[i].Cin && e.k[i].Cout == key[i].Cout &&
             e.k[i].flags == key[i].flags && e.k[i].want == key[i].want;
    if (same) { for (int i = 0; i < n; ++i) c[i] = e.c[i]; overrides(); return; }
  }
  // start from what every layer would get on its own (a search over one layer at a time cannot leave a start in which
  // every layer has a few long units: the finish is the longest unit's, and shortening one layer's does not move it)
  for (int i = 0; i < n; ++i) {
    const BigChoice own = choose_big(L[i].M, L[i].K, L[i].Cin, L[i].Cout);
    c[i] = BatchLayerChoice{own.splits > 0 ? own.dx_bm : 256, std::max(min_splits[i], own.splits > 0 ? own.splits : 1)};
  }
  double best = batch_cost(L, n, c);
  for (int pass = 0; pass < 2; ++pass)
    for (int i = 0; i < n; ++i) {
      BatchLayerChoice arg = c[i];
      int cand[24], nc = 0;
      for (int sp = 1; sp <= 8; ++sp) cand[nc++] = std::max(sp, min_splits[i]);
      for (int m : {5, 6, 8, 10, 12, 16, 20, 24, 32}) cand[nc++] = std::max(min_splits[i] * m / 4, min_splits[i]);
      for (int d = -2; d <= 2; ++d) cand[nc++] = std::max(c[i].splits + d, min_splits[i]);
      std::sort(cand, cand + nc);
      nc = (int)(std::unique(cand, cand + nc) - cand);
      for (int bm : {256, 128, 64}) {
        if (!L[i].dX && bm != 256) continue;
        for (int q = 0; q < nc; ++q) {
          const int sp = cand[q];
          if (!L[i].dW && q > 0) break;
          if (sp > min_splits[i] && sp > 1 && ceil_div(L[i].K, sp) < 512) break;   // splits shorter than 16 stages do not pay
          c[i] = BatchLayerChoice{bm, sp};
          const double cost = batch_cost(L, n, c);
          if (cost < best) { best = cost; arg = c[i]; }
        }
      }
      c[i] = arg;
    }
  if (opt.debug_plan) {
    std::fprintf(stderr, "sbp batch plan (%d layers, simulated %.1f us):", n, best / 1e3);
    for (int i = 0; i < n; ++i) std::fprintf(stderr, " [%d->%d K=%lld: dx rows %d, %d splits]", L[i].Cin, L[i].Cout, (long long)L[i].K, c[i].dx_bm, c[i].splits);
    std::fprintf(stderr, "\n");
  }
  Entry& e = cache[next];
  next = (next + 1) % 8;
  e.n = n;
  for (int i = 0; i < n; ++i) { e.k[i] = key[i]; e.c[i] = c[i]; }
  overrides();
}

BatchPlan plan_linear_batch(const sbp_linear_layer* L, int32_t n, int32_t dtype) {
  BatchPlan p{};
  p.n = n;
  // one grid for all layers: where every layer is within the large-tile engine's limits and wide enough for its 256-wide
  // tiles to pay (narrower layers are better off with the 128-tile engine, layer by layer); override "tile" = "big"
  // takes the common grid wherever the limits allow
  const bool forced = options().tile_mode == 2;
  p.fused = n >= 1 && n <= kMaxBatch;
  for (int i = 0; i < n && p.fused; ++i)
    p.fused = batch_layer_fits(L[i], dtype) && (forced || (L[i].Cin >= big::BT && L[i].Cout >= big::BT && L[i].K >= 1024));
  // layer by layer: every layer gets its own piece of the workspace.  The size returned covers both modes, so that
  // a size query made with other (e.g. differently aligned) addresses than the call still holds.
  size_t off = 0, seq_bytes = 0;
  for (int i = 0; i < n; ++i) {
    if (!p.fused) p.lay[i].off = seq_bytes;
    seq_bytes += align_up(plan_linear(L[i].M, L[i].K, L[i].Cin, L[i].Cout, dtype, L[i].flags).bytes, 256);
  }
  p.bytes = seq_bytes;
  if (!p.fused) return p;
  BatchLayerChoice c[kMaxBatch];
  choose_batch(L, n, c);
  for (int i = 0; i < n; ++i) {
    const sbp_linear_layer& l = L[i];
    BatchLayer& b = p.lay[i];
    b.dx_bm = c[i].dx_bm;
    // (fewer splits than asked for may cover K once their length is rounded up: iterate to the fixed point, so that
    // the unit tables, which are rebuilt from `splits` at every launch, agree with these numbers)
    b.splits = c[i].splits;
    for (;;) {
      b.rows_per_split = (int)split_rows(l.K, b.splits);
      const int covered = (int)ceil_div(l.K, b.rows_per_split);
      if (covered == b.splits) break;
      b.splits = covered;
    }
    b.direct = l.dW && b.splits == 1 && !(l.flags & (SBP_FLAG_ACCUMULATE_DW | SBP_FLAG_DW_OUT_BF16));
    b.db_slice_rows = db_slice_rows_for(l.K, true);
    b.db_slices = (int)ceil_div(l.K, b.db_slice_rows);
    b.off = off;
    if (l.dW && !b.direct) off += align_up((size_t)b.splits * l.Cout * l.Cin * sizeof(float), 256);
    b.off_dbp = off;
    if (l.db) off += align_up((size_t)std::max<int64_t>(b.db_slices, b.splits * ceil_div(l.Cin, big::BT)) * l.Cout * sizeof(float), 256);
    b.off_inv = off;
    if (l.dX && !(l.flags & SBP_FLAG_DX_COMPACT) && !l.inv) off += align_up((size_t)l.M * sizeof(int32_t), 256);
  }
  p.off_counters = off;
  off += 256;
  p.bytes = std::max(off, seq_bytes);
  if (options().debug_plan) {
    Job jobs[kMaxJobs];
    double red = 0;
    const int nj = batch_jobs(L, n, c, jobs, &red);
    XcdQueues Q;
    const int64_t end = partition_xcd(jobs, nj, &Q);
    std::fprintf(stderr, "sbp batch queues: simulated end %.1f us, reduction %.1f us\n", end / 1e3, red / 1e3);
    for (int x = 0; x < kNumXCD && end >= 0; ++x) {
      std::fprintf(stderr, "  xcd %d (%d workgroups):", x, Q.nq[x]);
      for (int e = 0; e < Q.nent[x]; ++e)
        std::fprintf(stderr, " L%d.k%d[%d +%dx%d) %.0fus", Q.ent[x][e].layer, Q.ent[x][e].kind, Q.ent[x][e].unit0, Q.cnt[x][e], Q.ent[x][e].stride, Q.len[x][e] / 1e3);
      std::fprintf(stderr, "\n");
    }
  }
  return p;
}

// A batch that does not take the large-tile grid but whose layers all take the general engine in its default shape
// (bf16, 128 x 128 tiles, stages of 64): one launch of linear_bwd_multi_kernel + one reduction launch.  Every layer uses
// its own piece of the workspace exactly as a single call would.  Returns false if the batch is not of that kind.
static bool launch_small_batch(const BatchPlan& p, const sbp_linear_layer* L, int32_t dtype, char* wsb, hipStream_t s, int32_t* status) {
  if (p.n < 2 || dtype != SBP_BF16 || options().tile_mode != 0) return false;
  LinearPlan lp[kMaxBatch];
  for (int i = 0; i < p.n; ++i) {
    const sbp_linear_layer& l = L[i];
    lp[i] = plan_linear(l.M, l.K, l.Cin, l.Cout, dtype, l.flags);
    if (!lp[i].mfma || lp[i].big || lp[i].bm_w != 128 || lp[i].nw_w != 4 || lp[i].kb != 64 || l.K < 1) return false;
    if (l.flags & SBP_FLAG_XK_KMAJOR) return false;
    if (!l.dW && !l.db && !l.dX) return false;
    if (((uintptr_t)l.dY | (uintptr_t)l.X_k | (uintptr_t)l.W | (uintptr_t)l.dX) & 15) return false;
    if (l.dW && ((uintptr_t)l.dW & 15)) return false;
  }
  // the layers fill the chip together: each needs only its share of the dW splits a launch of its own would take (fewer
  // partial sums to write and to add); the workspace was sized for the larger number
  for (int i = 0; i < p.n; ++i) {
    const int64_t K = L[i].K;
    int splits = (int)std::max<int64_t>(ceil_div(lp[i].splits, p.n), ceil_div(K, kMaxRowsPerSplit));
    const int64_t rps = ceil_div(ceil_div(K, splits), 64) * 64;
    splits = (int)ceil_div(K, rps);
    if (splits < lp[i].splits) {
      lp[i].splits = splits;
      lp[i].rows_per_split = (int)rps;
    }
  }
  SmallMultiArgs m{};
  RedMultiArgs r{};
  m.n = r.n = p.n;
  size_t lds = 0;
  int blk = 0;
  bool any_reduce = false;
  for (int i = 0; i < p.n; ++i) {
    const sbp_linear_layer& l = L[i];
    char* w = wsb + p.lay[i].off;
    float* part = reinterpret_cast<float*>(w + lp[i].off_partial);
    float* dbp = part + (size_t)lp[i].splits * l.Cout * l.Cin;
    const bool dy_compact = l.flags & SBP_FLAG_DY_COMPACT, dx_compact = l.flags & SBP_FLAG_DX_COMPACT;
    const bool scatter = l.dX && !dx_compact;
    const int32_t* inv = l.inv;
    if (scatter && !inv) {
      int32_t* inv_ws = reinterpret_cast<int32_t*>(w + lp[i].off_inv);
      launch_build_inverse(l.idx, l.K, inv_ws, s);
      inv = inv_ws;
    }
    LinArgs& a = m.lay[i];
    a.dY = static_cast<const uint16_t*>(l.dY);
    a.idx_in = dy_compact ? nullptr : l.idx;
    a.idx_out = dx_compact ? nullptr : l.idx;
    a.idx = l.idx; a.inv = inv;
    a.Xk = static_cast<const uint16_t*>(l.X_k); a.W = static_cast<const uint16_t*>(l.W);
    a.dX = static_cast<uint16_t*>(l.dX); a.part = part; a.dbp = l.db ? dbp : nullptr;
    a.K = (int)l.K; a.M = (int)l.M; a.Cin = l.Cin; a.Cout = l.Cout;
    a.rows_per_split = lp[i].rows_per_split; a.db_slice_rows = lp[i].db_slice_rows;
    a.dx_bm = lp[i].dx_bm;
    size_t need = 0;
    const unsigned grid = lp[i].dx_bm == 64
        ? prepare_linear_bwd<128, 128, 4, 64, 2, 64, 3>(lp[i], a, l.dX != nullptr, l.dW != nullptr, scatter, &need)
        : prepare_linear_bwd<128, 128, 4, 64, 2>(lp[i], a, l.dX != nullptr, l.dW != nullptr, scatter, &need);
    lds = std::max(lds, need);
    m.start[i] = blk;
    blk += (int)grid;
    RedLayer& rl = r.lay[i];
    rl.part = part; rl.dbp = dbp; rl.dW = l.dW; rl.db = l.db;
    rl.nW = (long long)l.Cin * l.Cout;
    rl.nsplit_w = lp[i].splits; rl.nsplit_b = lp[i].db_slices; rl.Cout = l.Cout;
    rl.accumulate = (l.flags & SBP_FLAG_ACCUMULATE_DW) ? 1 : 0;
    rl.bf16out = (l.flags & SBP_FLAG_DW_OUT_BF16) ? 1 : 0;
    rl.G = reduce_lanes((rl.dW ? rl.nW / 4 : 0) + (rl.db ? rl.Cout : 0), std::max(rl.dW ? rl.nsplit_w : 0, rl.db ? rl.nsplit_b : 0));
    any_reduce = any_reduce || rl.dW || rl.db;
  }
  m.start[p.n] = blk;
  if (blk > 0) {
    allow_big_lds(linear_bwd_multi_kernel, lds);
    SBP_LAUNCH(SBP_PROF_DW_GEMM, s, linear_bwd_multi_kernel, dim3((unsigned)blk), dim3(256), lds, s, m);
  }
  if (any_reduce) {
    int rb = 0;
    for (int i = 0; i < p.n; ++i) {
      RedLayer& rl = r.lay[i];
      const long long total = (rl.dW ? rl.nW / 4 : 0) + (rl.db ? rl.Cout : 0);
      rl.blk_start = rb;
      rl.nblk = (int)std::min<long long>(ceil_div(total * rl.G, NTHREADS), 16384);
      rb += rl.nblk;
    }
    if (rb > 0) SBP_LAUNCH(SBP_PROF_REDUCE, s, reduce_multi_kernel, dim3((unsigned)rb), dim3(NTHREADS), 0, s, r);
  }
  *status = check_launch("backward_linear_batch (general engine)");
  return true;
}

int32_t launch_backward_linear_batch(const BatchPlan& p, const sbp_linear_layer* L, int32_t dtype, void* ws, hipStream_t s) {
  char* wsb = static_cast<char*>(ws);
  if (!p.fused) {
    int32_t st = SBP_OK;
    if (launch_small_batch(p, L, dtype, wsb, s, &st)) return st;
    for (int i = 0; i < p.n; ++i) {
      const sbp_linear_layer& l = L[i];
      if (!l.dW && !l.db && !l.dX) continue;
      const LinearPlan lp = plan_linear(l.M, l.K, l.Cin, l.Cout, dtype, l.flags);
      const int32_t st = launch_backward_linear(lp, l.dY, l.idx, l.inv, l.X_k, l.W, l.M, l.K, l.Cin, l.Cout, dtype, l.dW,
                                                l.db, l.dX, wsb + p.lay[i].off, l.flags, s);
      if (st != SBP_OK) return st;
    }
    return SBP_OK;
  }
  MultiArgs a{};
  RedMultiArgs r{};
  BatchLayerChoice c[kMaxBatch];
  size_t lds = 0;
  bool any = false, any_reduce = false;
  for (int i = 0; i < p.n; ++i) {
    const sbp_linear_layer& l = L[i];
    const BatchLayer& b = p.lay[i];
    c[i] = BatchLayerChoice{b.dx_bm, b.splits};
    const bool dy_compact = l.flags & SBP_FLAG_DY_COMPACT, dx_compact = l.flags & SBP_FLAG_DX_COMPACT;
    const bool scatter = l.dX && !dx_compact;
    const int32_t* inv = l.inv;
    if (scatter && !inv && l.M > l.K) {
      int32_t* inv_ws = reinterpret_cast<int32_t*>(wsb + b.off_inv);
      launch_build_inverse(l.idx, l.K, inv_ws, s);
      inv = inv_ws;
    }
    LinArgs& la = a.lay[i];
    la.dY = static_cast<const uint16_t*>(l.dY);
    la.idx_in = dy_compact ? nullptr : l.idx;
    la.idx_out = dx_compact ? nullptr : l.idx;
    la.idx = l.idx; la.inv = inv;
    la.Xk = static_cast<const uint16_t*>(l.X_k); la.W = static_cast<const uint16_t*>(l.W);
    la.dX = static_cast<uint16_t*>(l.dX);
    la.part = b.direct ? static_cast<float*>(l.dW) : reinterpret_cast<float*>(wsb + b.off);
    la.dbp = l.db ? reinterpret_cast<float*>(wsb + b.off_dbp) : nullptr;
    la.K = (int)l.K; la.M = (int)l.M; la.Cin = l.Cin; la.Cout = l.Cout;
    la.rows_per_split = b.rows_per_split; la.db_slice_rows = b.db_slice_rows;
    la.n_big = b.splits; la.rows_small = 0; la.dx_bm = b.dx_bm;
    la.n_zero = scatter && l.M > l.K ? big_zero_blocks(l.M) : 0;
    la.db_in_dw = l.db && l.dW ? 1 : 0;
    la.xk_kmajor = (l.flags & SBP_FLAG_XK_KMAJOR) ? 1 : 0;     // (equal splits of a multiple of 64 rows: every split starts on a row group)
    lds = std::max(lds, (size_t)big::RING + std::max<size_t>((size_t)(b.rows_per_split + 2 * big::KB), big::BT) * sizeof(int));
    lds = std::max<size_t>(lds, 16 * 1024);     // the column-sum blocks' staging
    any = any || l.dW || l.db || l.dX;
    RedLayer& rl = r.lay[i];
    rl.part = la.part; rl.dbp = la.dbp;
    rl.dW = b.direct ? nullptr : l.dW; rl.db = l.db;
    rl.nW = (long long)l.Cin * l.Cout;
    rl.nsplit_w = b.splits; rl.nsplit_b = la.db_in_dw ? b.splits * (int)ceil_div(l.Cin, big::BT) : b.db_slices; rl.Cout = l.Cout;
    rl.accumulate = (l.flags & SBP_FLAG_ACCUMULATE_DW) ? 1 : 0;
    rl.bf16out = (l.flags & SBP_FLAG_DW_OUT_BF16) ? 1 : 0;
    rl.G = 1;
    any_reduce = any_reduce || rl.dW || rl.db;
  }
  if (!any) return SBP_OK;
  Job jobs[kMaxJobs];
  double red_ns = 0;
  const int nj = batch_jobs(L, p.n, c, jobs, &red_ns);
  // the unit counts must describe exactly the work the per-layer arguments imply: checked here, on the host
  for (int j = 0; j < nj; ++j) {
    const LinArgs& la = a.lay[jobs[j].layer];
    const int64_t tiles_n = ceil_div(la.Cin, big::BT), tiles_w = ceil_div(la.Cout, big::BT) * tiles_n;
    const int64_t expect = jobs[j].kind == 0 ? ceil_div(la.K, la.dx_bm) * tiles_n
                         : jobs[j].kind == 1 ? tiles_w * la.n_big
                         : jobs[j].kind == 3 ? la.n_zero
                         : jobs[j].kind == 4 ? ceil_div(la.Cout, 256) * ceil_div(la.K, la.db_slice_rows) : -1;
    if (jobs[j].n != expect || (int64_t)la.n_big * la.rows_per_split < la.K || jobs[j].n <= 0)
      return fail(SBP_ERR_SHAPE, "backward_linear_batch: inconsistent unit table (layer %d, kind %d)", jobs[j].layer, jobs[j].kind);
  }
  XcdQueues Q;
  if (partition_xcd(jobs, nj, &Q) < 0) return fail(SBP_ERR_SHAPE, "backward_linear_batch: queue table overflow");
  int longest = 0;
  int64_t covered[kMaxJobs] = {};
  for (int x = 0; x < kNumXCD; ++x) {
    a.nent[x] = Q.nent[x]; a.nq[x] = Q.nq[x];
    longest = std::max(longest, Q.nq[x]);
    for (int e = 0; e < Q.nent[x]; ++e) {
      a.ent[x][e] = Q.ent[x][e];
      for (int j = 0; j < nj; ++j)      // every entry must lie inside its job's unit range
        if (jobs[j].layer == Q.ent[x][e].layer && jobs[j].kind == Q.ent[x][e].kind) {
          if (Q.ent[x][e].unit0 < 0 || Q.ent[x][e].stride < 1 ||
              Q.ent[x][e].unit0 + (int64_t)(Q.cnt[x][e] - 1) * Q.ent[x][e].stride >= jobs[j].n)
            return fail(SBP_ERR_SHAPE, "backward_linear_batch: queue entry outside its job");
          covered[j] += Q.cnt[x][e];
        }
    }
  }
  for (int j = 0; j < nj; ++j)
    if (covered[j] != jobs[j].n) return fail(SBP_ERR_SHAPE, "backward_linear_batch: queues do not cover job %d", j);
  timeline_target(&a.timeline, &a.timeline_cap);
  if (longest > 0) {
    a.counters = reinterpret_cast<int*>(wsb + p.off_counters);
    const int dynamic = options().batch_dynamic ? 1 : 0;
    int grid = kNumXCD * longest;
    if (dynamic) {          // the same number of workgroups on every XCD, a quarter more than an even share of the units
      int total = 0;
      for (int x = 0; x < kNumXCD; ++x) total += Q.nq[x];
      grid = kNumXCD * (int)ceil_div((int64_t)total * 5, 4 * kNumXCD);
      SBP_LAUNCH(SBP_PROF_OTHER, s, fill_zero_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(a.counters), (long long)kNumXCD);
    }
    allow_big_lds(linear_multi_kernel, lds);
    SBP_LAUNCH(SBP_PROF_DW_GEMM, s, linear_multi_kernel, dim3((unsigned)grid), dim3(256), lds, s, a, dynamic);
  }
  if (any_reduce) {
    r.n = p.n;
    int blk = 0;
    for (int i = 0; i < p.n; ++i) {
      RedLayer& rl = r.lay[i];
      const long long total = (rl.dW ? rl.nW / 4 : 0) + (rl.db ? rl.Cout : 0);
      rl.blk_start = blk;
      rl.nblk = (int)std::min<long long>(ceil_div(total, NTHREADS), 16384);   // (one output per thread up to 4 M of them: the partials of an output are all in flight at once)
      blk += rl.nblk;
    }
    if (blk > 0) SBP_LAUNCH(SBP_PROF_REDUCE, s, reduce_multi_kernel, dim3((unsigned)blk), dim3(NTHREADS), 0, s, r);
  }
  return check_launch("backward_linear_batch");
}

}  // namespace sbp
