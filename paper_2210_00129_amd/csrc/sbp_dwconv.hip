// Depthwise-conv backward restricted to the kept output positions (paper, section "Calculation of
// Convolutional Layers", eq:conv_grad_layer_before_sbp, with dY = 0 at dropped positions):
//   dWd[u,v,c] = sum_{(b,y,x) kept} dY[b,y,x,c] X[b,y+u-pad,x+v-pad,c]
//   db[c]      = sum_{(b,y,x) kept} dY[b,y,x,c]
//   dX[b,y,x,c]= sum_{u,v} [(b,y-u+pad,x-v+pad) kept] dY[b,y-u+pad,x-v+pad,c] Wd[u,v,c]
// Channels-last: a wavefront's lanes are adjacent channels, so "is this neighbour kept" is the same
// for the whole wavefront and dropped taps are skipped by a scalar branch.  bf16 or fp32 storage,
// fp32 arithmetic on the vector ALUs (a depthwise conv is no dense contraction: no MFMA).
#include "sbp_internal.h"

namespace sbp {

static constexpr int DW_THREADS = 256;

template <typename T> struct DwElem;
template <> struct DwElem<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct DwElem<uint16_t> {
  static __device__ __forceinline__ float ld(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
  static __device__ __forceinline__ void st(uint16_t* p, float v) {
    uint32_t u = __float_as_uint(v);
    uint32_t r = ((u & 0x7fffffffu) > 0x7f800000u) ? ((u >> 16) | 0x40u) : ((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    *p = (uint16_t)r;
  }
};

__global__ void __launch_bounds__(DW_THREADS) dw_fill_kernel(int32_t* __restrict__ p, long long n, int32_t v) {
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < n; e += (long long)gridDim.x * blockDim.x)
    p[e] = v;
}
__global__ void __launch_bounds__(DW_THREADS) dw_mark_kernel(const int32_t* __restrict__ idx, int K,
                                                              int32_t* __restrict__ inv) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < K) inv[idx[j]] = j;
}

// dX: one thread per (position, channel); block = positions_per_block x C threads (C fastest).
template <typename T, int KS>
__global__ void __launch_bounds__(DW_THREADS) dw_dx_kernel(const T* __restrict__ dY, const int32_t* __restrict__ inv,
                                                           const T* __restrict__ Wd, int B, int H, int W, int C,
                                                           T* __restrict__ dX) {
  constexpr int PAD = KS / 2;
  const long long total = (long long)B * H * W * C;
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
       e += (long long)gridDim.x * blockDim.x) {
    const int c = (int)(e % C);
    const long long pos = e / C;
    const int x = (int)(pos % W);
    const int y = (int)((pos / W) % H);
    const long long b = pos / ((long long)W * H);
    float a = 0.f;
#pragma unroll
    for (int u = 0; u < KS; ++u) {
      const int yy = y - u + PAD;
      if (yy < 0 || yy >= H) continue;
#pragma unroll
      for (int v = 0; v < KS; ++v) {
        const int xx = x - v + PAD;
        if (xx < 0 || xx >= W) continue;
        const long long q = (b * H + yy) * W + xx;
        if (inv[q] >= 0) a = fmaf(DwElem<T>::ld(dY + q * C + c), DwElem<T>::ld(Wd + (u * KS + v) * C + c), a);
      }
    }
    DwElem<T>::st(dX + e, a);
  }
}

// dWd / db partial sums: thread = (tap or bias, channel); blockIdx.y = slice of the kept list.
// part[slice][tap][c]; tap == KS*KS is the bias row.
template <typename T, int KS>
__global__ void __launch_bounds__(DW_THREADS) dw_dw_kernel(const T* __restrict__ dY, const int32_t* __restrict__ idx,
                                                           const T* __restrict__ X, int H, int W, int C, int K,
                                                           int per_slice, float* __restrict__ part) {
  constexpr int PAD = KS / 2;
  constexpr int NT = KS * KS + 1;
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= NT * C) return;
  const int tap = e / C, c = e - tap * C;
  const int u = tap / KS, v = tap - u * KS;
  const int j0 = blockIdx.y * per_slice, j1 = min(K, j0 + per_slice);
  float a = 0.f;
  for (int j = j0; j < j1; ++j) {
    const int q = idx[j];
    const float g = DwElem<T>::ld(dY + (long long)q * C + c);
    if (tap == KS * KS) { a += g; continue; }
    const int x = q % W, y = (q / W) % H;
    const int yy = y + u - PAD, xx = x + v - PAD;
    if (yy >= 0 && yy < H && xx >= 0 && xx < W)
      a = fmaf(g, DwElem<T>::ld(X + ((long long)q + (long long)(u - PAD) * W + (v - PAD)) * C + c), a);
  }
  part[((long long)blockIdx.y * NT + tap) * C + c] = a;
}

__global__ void __launch_bounds__(DW_THREADS) dw_reduce_kernel(const float* __restrict__ part, int nslices, int ntap,
                                                                int C, float* __restrict__ dWd, float* __restrict__ db) {
  // 32 outputs per block, 8 lanes per output: lane j adds slices j, j + 8, ... in order, then the 8 lane
  // sums are added in lane order -- a fixed order, whatever the launch looks like
  __shared__ float red[8][33];
  const int n = (ntap + 1) * C;
  const int o = threadIdx.x & 31, j = threadIdx.x >> 5;
  const int e = blockIdx.x * 32 + o;
  float a = 0.f;
  if (e < n) {
    for (int s0 = j; s0 < nslices; s0 += 32) {     // four independent loads in flight
      float p[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) p[u] = s0 + 8 * u < nslices ? part[(long long)(s0 + 8 * u) * n + e] : 0.f;
#pragma unroll
      for (int u = 0; u < 4; ++u) a += p[u];
    }
  }
  red[j][o] = a;
  __syncthreads();
  if (j == 0 && e < n) {
    float t = 0.f;
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) t += red[jj][o];
    if (e < ntap * C) { if (dWd) dWd[e] = t; }
    else if (db) db[e - ntap * C] = t;
  }
}

// ------------------------------------------------------------------------------------------------
// bf16 fast path (even channel count).  A lane owns two adjacent channels (one 32-bit word), so a
// wavefront reads 256 contiguous bytes per position and the "is this position kept" test is uniform
// over the block (a scalar load and a scalar branch).
//
// dX: a block produces TX consecutive positions of one row for 2 * blockDim.x channels.  The KS*KS
// weights of its channels sit in registers; it walks the KS x (TX + KS - 1) window of dY once, skips
// the dropped positions, and adds each kept gradient to the (up to KS) outputs it reaches.
// ------------------------------------------------------------------------------------------------
static constexpr int DW_TX = 8;

__device__ __forceinline__ float dw_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float dw_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t dw_round(float v) {
  uint32_t u = __float_as_uint(v);
  return ((u & 0x7fffffffu) > 0x7f800000u) ? ((u >> 16) | 0x40u) : ((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// kept-mask of a window of positions: lane p tests position p, the ballot makes it wave-uniform
template <int KS>
__device__ __forceinline__ void dw_window_masks(const int32_t* __restrict__ inv, int row, int y, int x0, int H, int W,
                                                unsigned long long (&mask)[2]) {
  constexpr int PAD = KS / 2, WIN = DW_TX + KS - 1;
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int p = lane + 64 * h;                 // window position p = r * WIN + col
    const int r = p / WIN, col = p - r * WIN;
    const int yy = y + r - PAD, xx = x0 + col - PAD;
    bool kept = false;
    if (p < KS * WIN && yy >= 0 && yy < H && xx >= 0 && xx < W) kept = inv[(long long)(row + r - PAD) * W + xx] >= 0;
    mask[h] = __ballot(kept);
  }
}
__device__ __forceinline__ bool dw_bit(const unsigned long long (&mask)[2], int p) {
  return (mask[p >> 6] >> (p & 63)) & 1ull;
}

template <int KS>
__global__ void __launch_bounds__(DW_THREADS) dw_dx_fast_kernel(const uint32_t* __restrict__ dY, const int32_t* __restrict__ inv,
                                                                const uint32_t* __restrict__ Wd, int H, int W, int C2,
                                                                uint32_t* __restrict__ dX, int tiles_x) {
  constexpr int PAD = KS / 2, WIN = DW_TX + KS - 1;
  static_assert(KS * WIN <= 128, "window must fit two ballots");
  const int cp_raw = blockIdx.y * blockDim.x + threadIdx.x;
  const bool active = cp_raw < C2;
  const int cp = active ? cp_raw : C2 - 1;
  const int tile = blockIdx.x;
  const int x0 = (tile % tiles_x) * DW_TX;
  const int row = tile / tiles_x;            // b * H + y
  const int y = row % H;
  unsigned long long mask[2];
  dw_window_masks<KS>(inv, row, y, x0, H, W, mask);
  float w0[KS * KS], w1[KS * KS];
#pragma unroll
  for (int tp = 0; tp < KS * KS; ++tp) {
    const uint32_t w = Wd[tp * C2 + cp];
    w0[tp] = dw_lo(w); w1[tp] = dw_hi(w);
  }
  float a0[DW_TX], a1[DW_TX];
#pragma unroll
  for (int ox = 0; ox < DW_TX; ++ox) { a0[ox] = 0.f; a1[ox] = 0.f; }
  // all loads of the window are issued together (clamped addresses; values of dropped or outside
  // positions are never used), then the kept positions are accumulated
  uint32_t g[KS][WIN];
#pragma unroll
  for (int r = 0; r < KS; ++r) {
    const long long prow = (long long)(row - y + min(max(y + r - PAD, 0), H - 1)) * W;
#pragma unroll
    for (int col = 0; col < WIN; ++col) g[r][col] = dY[(prow + min(max(x0 + col - PAD, 0), W - 1)) * C2 + cp];
  }
#pragma unroll
  for (int r = 0; r < KS; ++r) {
    const int u = KS - 1 - r;                // tap row that links output row y to gradient row y + r - PAD
#pragma unroll
    for (int col = 0; col < WIN; ++col) {
      if (!dw_bit(mask, r * WIN + col)) continue;     // dropped or outside: wave-uniform
      const float g0 = dw_lo(g[r][col]), g1 = dw_hi(g[r][col]);
#pragma unroll
      for (int ox = 0; ox < DW_TX; ++ox) {
        const int v = ox - col + 2 * PAD;
        if (v >= 0 && v < KS) {
          a0[ox] = fmaf(g0, w0[u * KS + v], a0[ox]);
          a1[ox] = fmaf(g1, w1[u * KS + v], a1[ox]);
        }
      }
    }
  }
  if (active) {
#pragma unroll
    for (int ox = 0; ox < DW_TX; ++ox)
      if (x0 + ox < W) dX[((long long)row * W + x0 + ox) * C2 + cp] = dw_round(a0[ox]) | (dw_round(a1[ox]) << 16);
  }
}

// dWd, db: blockDim = (channel pairs, GROUPS).  Every group walks its share of the row tiles, keeping
// KS*KS + 1 running sums per channel in registers: for a tile it issues all loads at once (the up to TX
// gradients of the row and the KS x (TX + KS - 1) inputs under the window), then adds g[x] * X[x + v] for
// the kept x only.  The groups of a block are then added in a fixed order through LDS and the block
// writes one partial; a second kernel adds the partials of all blocks.
template <int KS, int GROUPS>
__global__ void __launch_bounds__(DW_THREADS * GROUPS) dw_dw_fast_kernel(const uint32_t* __restrict__ dY,
                                                                         const int32_t* __restrict__ inv,
                                                                         const uint32_t* __restrict__ X, int H, int W,
                                                                         int C2, int tiles_x, int ntiles,
                                                                         float* __restrict__ part) {
  constexpr int PAD = KS / 2, WIN = DW_TX + KS - 1, NT = KS * KS + 1;
  extern __shared__ float red[];             // [GROUPS - 1][CHUNK][blockDim.x][2]
  const int cp_raw = blockIdx.y * blockDim.x + threadIdx.x;
  const bool active = cp_raw < C2;
  const int cp = active ? cp_raw : C2 - 1;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.y);   // a wavefront never spans two groups
  const int lane = threadIdx.x & 63;
  float s0[NT], s1[NT];
#pragma unroll
  for (int tp = 0; tp < NT; ++tp) { s0[tp] = 0.f; s1[tp] = 0.f; }

  for (int tile = blockIdx.x * GROUPS + grp; tile < ntiles; tile += gridDim.x * GROUPS) {
    const int x0 = (tile % tiles_x) * DW_TX;
    const int row = tile / tiles_x;          // b * H + y
    const int y = row % H;
    const long long prow = (long long)row * W;
    const unsigned long long keep =
        __ballot(lane < DW_TX && x0 + lane < W && inv[prow + min(x0 + lane, W - 1)] >= 0);   // wave-uniform
    if (keep == 0) continue;
    // every load of the tile is issued before the first use: clamped addresses, unused values ignored
    uint32_t g[DW_TX], xw[KS][WIN];
    {
      const uint32_t* grow = dY + prow * C2 + cp;
#pragma unroll
      for (int ox = 0; ox < DW_TX; ++ox) g[ox] = grow[(long long)min(x0 + ox, W - 1) * C2];
    }
#pragma unroll
    for (int u = 0; u < KS; ++u) {
      const uint32_t* xrow = X + (long long)(row - y + min(max(y + u - PAD, 0), H - 1)) * W * C2 + cp;
#pragma unroll
      for (int col = 0; col < WIN; ++col) xw[u][col] = xrow[(long long)min(max(x0 + col - PAD, 0), W - 1) * C2];
    }
    float g0[DW_TX], g1[DW_TX];
#pragma unroll
    for (int ox = 0; ox < DW_TX; ++ox) {
      const bool k = (keep >> ox) & 1ull;
      g0[ox] = k ? dw_lo(g[ox]) : 0.f;
      g1[ox] = k ? dw_hi(g[ox]) : 0.f;
      s0[KS * KS] += g0[ox]; s1[KS * KS] += g1[ox];
    }
#pragma unroll
    for (int u = 0; u < KS; ++u) {
      const int yy = y + u - PAD;
      if (yy < 0 || yy >= H) continue;               // zero padding: uniform
#pragma unroll
      for (int col = 0; col < WIN; ++col) {
        const int xx = x0 + col - PAD;
        if (xx < 0 || xx >= W) continue;             // zero padding: uniform
        const float xa = dw_lo(xw[u][col]), xb = dw_hi(xw[u][col]);
#pragma unroll
        for (int ox = 0; ox < DW_TX; ++ox) {
          const int v = col - ox;
          if (v < 0 || v >= KS) continue;            // compile time
          s0[u * KS + v] = fmaf(g0[ox], xa, s0[u * KS + v]);   // g is zero at dropped positions
          s1[u * KS + v] = fmaf(g1[ox], xb, s1[u * KS + v]);
        }
      }
    }
  }

  // add the groups (fixed order 0, 1, 2, ...) through LDS, CHUNK taps at a time
  constexpr int CHUNK = 10;
  const int ct = blockDim.x;
  float* out = part + ((long long)blockIdx.x * NT) * (2 * C2);
#pragma unroll
  for (int c0 = 0; c0 < NT; c0 += CHUNK) {
    if (grp > 0) {
#pragma unroll
      for (int j = 0; j < CHUNK; ++j)
        if (c0 + j < NT) {
          red[(((grp - 1) * CHUNK + j) * ct + threadIdx.x) * 2 + 0] = s0[c0 + j];
          red[(((grp - 1) * CHUNK + j) * ct + threadIdx.x) * 2 + 1] = s1[c0 + j];
        }
    }
    __syncthreads();
    if (grp == 0 && active) {
#pragma unroll
      for (int j = 0; j < CHUNK; ++j)
        if (c0 + j < NT) {
          float t0 = s0[c0 + j], t1 = s1[c0 + j];
          for (int g2 = 1; g2 < GROUPS; ++g2) {
            t0 += red[(((g2 - 1) * CHUNK + j) * ct + threadIdx.x) * 2 + 0];
            t1 += red[(((g2 - 1) * CHUNK + j) * ct + threadIdx.x) * 2 + 1];
          }
          out[(long long)(c0 + j) * (2 * C2) + 2 * cp + 0] = t0;
          out[(long long)(c0 + j) * (2 * C2) + 2 * cp + 1] = t1;
        }
    }
    __syncthreads();
  }
}

static constexpr int DW_GROUPS = 2;
static constexpr int DW_MAX_PARTS = 256;

DwPlan plan_dwconv(int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks, int64_t K, int32_t dtype) {
  DwPlan p{};
  (void)dtype;
  p.tiles_y = p.tiles_x = 0;
  // partial sums of dWd / db: one per block of the reduction kernel.  The fast path walks row tiles
  // (its parallelism does not depend on K), the plain path slices the kept list.
  const int64_t row_tiles = (int64_t)B * H * ceil_div(W, DW_TX);
  p.nparts = (int)std::max<int64_t>(1, std::min<int64_t>(DW_MAX_PARTS, std::max<int64_t>(ceil_div(row_tiles, 2 * DW_GROUPS), 1)));
  size_t off = 0;
  p.off_inv = off;
  off += align_up((size_t)B * H * W * sizeof(int32_t), 256);
  p.off_partial = off;
  off += align_up((size_t)p.nparts * (ks * ks + 1) * C * sizeof(float), 256);
  p.bytes = off;
  return p;
}

template <typename T, int KS>
static void launch_dw_typed(const DwPlan& p, const T* dY, const int32_t* idx, const int32_t* inv, const T* X,
                            const T* Wd, int B, int H, int W, int C, int64_t K, float* dWd, float* db, T* dX,
                            float* part, hipStream_t s) {
  if (dX) {
    const long long total = (long long)B * H * W * C;
    unsigned blocks = (unsigned)std::min<long long>(ceil_div(total, DW_THREADS), 1 << 20);
    SBP_LAUNCH(SBP_PROF_DWCONV_DX, s, (dw_dx_kernel<T, KS>), dim3(blocks), dim3(DW_THREADS), 0, s, dY, inv, Wd, B, H, W, C, dX);
  }
  if (dWd || db) {
    const int n = (KS * KS + 1) * C;
    const int per_slice = (int)ceil_div(std::max<int64_t>(K, 1), p.nparts);
    dim3 grid((unsigned)ceil_div(n, DW_THREADS), p.nparts);
    SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_dw_kernel<T, KS>), grid, dim3(DW_THREADS), 0, s, dY, idx, X, H, W, C, (int)K, per_slice,
                       part);
    SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, dw_reduce_kernel, dim3((unsigned)ceil_div(n, 32)), dim3(DW_THREADS), 0, s, part,
                       p.nparts, KS * KS, C, dWd, db);
  }
}

int32_t launch_backward_dwconv(const DwPlan& p, const void* dY, const int32_t* idx, const int32_t* inv_in,
                               const void* X, const void* Wd, int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks,
                               int32_t pad, int64_t K, int32_t dtype, float* dWd, float* db, void* dX, void* ws,
                               hipStream_t s) {
  (void)pad;
  int32_t* inv_ws = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + p.off_inv);
  float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_partial);
  const long long npos = (long long)B * H * W;
  const int32_t* inv = inv_in;
  if (!inv) {            // build the inverse map from idx
    SBP_LAUNCH(SBP_PROF_OTHER, s, dw_fill_kernel, dim3((unsigned)std::min<long long>(ceil_div(npos, DW_THREADS), 4096)),
                       dim3(DW_THREADS), 0, s, inv_ws, npos, -1);
    if (K > 0)
      SBP_LAUNCH(SBP_PROF_OTHER, s, dw_mark_kernel, dim3((unsigned)ceil_div(K, DW_THREADS)), dim3(DW_THREADS), 0, s, idx, (int)K,
                         inv_ws);
    inv = inv_ws;
  }
  const bool fast = dtype == SBP_BF16 && C % 2 == 0 && (ks == 7 || ks == 3) && ((uintptr_t)dY % 4 == 0) &&
                    ((uintptr_t)X % 4 == 0) && ((uintptr_t)Wd % 4 == 0) && ((uintptr_t)dX % 4 == 0);
  if (fast) {
    const int C2 = C / 2;
    const int ct = (int)std::min<int64_t>(DW_THREADS, ceil_div(C2, 64) * 64);
    const int cblocks = (int)ceil_div(C2, ct);
    const int tiles_x = (int)ceil_div(W, DW_TX);
    const int ntiles = tiles_x * B * H;
    if (dX) {
      dim3 grid((unsigned)ntiles, (unsigned)cblocks);
      if (ks == 7)
        SBP_LAUNCH(SBP_PROF_DWCONV_DX, s, (dw_dx_fast_kernel<7>), grid, dim3(ct), 0, s, (const uint32_t*)dY, inv,
                   (const uint32_t*)Wd, H, W, C2, (uint32_t*)dX, tiles_x);
      else
        SBP_LAUNCH(SBP_PROF_DWCONV_DX, s, (dw_dx_fast_kernel<3>), grid, dim3(ct), 0, s, (const uint32_t*)dY, inv,
                   (const uint32_t*)Wd, H, W, C2, (uint32_t*)dX, tiles_x);
    }
    if (dWd || db) {
      const int nblk = (int)std::min<int64_t>(p.nparts, ceil_div(ntiles, DW_GROUPS));
      dim3 grid((unsigned)nblk, (unsigned)cblocks);
      const size_t lds = (size_t)(DW_GROUPS - 1) * 10 * ct * 2 * sizeof(float);
      if (ks == 7)
        SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_dw_fast_kernel<7, DW_GROUPS>), grid, dim3(ct, DW_GROUPS), lds, s,
                   (const uint32_t*)dY, inv, (const uint32_t*)X, H, W, C2, tiles_x, ntiles, part);
      else
        SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_dw_fast_kernel<3, DW_GROUPS>), grid, dim3(ct, DW_GROUPS), lds, s,
                   (const uint32_t*)dY, inv, (const uint32_t*)X, H, W, C2, tiles_x, ntiles, part);
      const int n = (ks * ks + 1) * C;
      SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, dw_reduce_kernel, dim3((unsigned)ceil_div(n, 32)), dim3(DW_THREADS), 0,
                 s, part, nblk, ks * ks, C, dWd, db);
    }
    return check_launch("backward_dwconv");
  }
#define SBP_DW_CASE(T, KS)                                                                                      \
  launch_dw_typed<T, KS>(p, (const T*)dY, idx, inv, (const T*)X, (const T*)Wd, B, H, W, C, K, dWd, db, (T*)dX, \
                         part, s)
  if (dtype == SBP_F32) {
    switch (ks) { case 1: SBP_DW_CASE(float, 1); break; case 3: SBP_DW_CASE(float, 3); break;
                  case 5: SBP_DW_CASE(float, 5); break; default: SBP_DW_CASE(float, 7); break; }
  } else {
    switch (ks) { case 1: SBP_DW_CASE(uint16_t, 1); break; case 3: SBP_DW_CASE(uint16_t, 3); break;
                  case 5: SBP_DW_CASE(uint16_t, 5); break; default: SBP_DW_CASE(uint16_t, 7); break; }
  }
#undef SBP_DW_CASE
  return check_launch("backward_dwconv");
}

}  // namespace sbp
