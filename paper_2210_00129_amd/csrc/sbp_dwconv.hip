// Depthwise-conv backward restricted to the kept output positions (paper, section "Calculation of
// Convolutional Layers", eq:conv_grad_layer_before_sbp, with dY = 0 at dropped positions):
//   dWd[u,v,c] = sum_{(b,y,x) kept} dY[b,y,x,c] X[b,y+u-pad,x+v-pad,c]
//   db[c]      = sum_{(b,y,x) kept} dY[b,y,x,c]
//   dX[b,y,x,c]= sum_{u,v} [(b,y-u+pad,x-v+pad) kept] dY[b,y-u+pad,x-v+pad,c] Wd[u,v,c]
// Channels-last: a wavefront's lanes are adjacent channels, so "is this neighbour kept" is the same
// for the whole wavefront and dropped taps are skipped by a scalar branch.  bf16 or fp32 storage,
// fp32 arithmetic on the vector ALUs (a depthwise conv is no dense contraction: no MFMA).
#include <cstdlib>
#include <mutex>

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
// wavefront reads 256 contiguous bytes per position and "is this position kept" is uniform over the
// wavefront (a ballot over a row of inverse-map lookups).  Work is cut into strips of DW_TX columns.
// ------------------------------------------------------------------------------------------------
static constexpr int DW_TX = 8;

// Strip kernels: a workgroup (dX) or a group of a workgroup (dWd, db) walks down a strip of DW_TX columns over a
// chunk of rows: each row of the map is fetched once per strip instead of KS times, the weights once per chunk,
// the next row's loads (and its inverse-map lookups) are in flight while the current row is computed, and the
// row loops have no per-position branches: dropped and outside positions are zeroed when a row arrives.
typedef __bf16 dw_bf16x2 __attribute__((ext_vector_type(2)));
typedef float dw_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t dw_pack(float lo, float hi) {      // round to nearest even (v_cvt_pk_bf16_f32)
  const dw_f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, dw_bf16x2));
}

struct DwStrip {
  int b, x0, y0, y1;
};
__device__ __forceinline__ DwStrip dw_strip(int strip, int tiles_x, int chunks, int rows_per_chunk, int H) {
  DwStrip t;
  const int xt = strip % tiles_x, rest = strip / tiles_x;
  const int ch = rest % chunks;
  t.b = rest / chunks;
  t.x0 = xt * DW_TX;
  t.y0 = ch * rows_per_chunk;
  t.y1 = min(H, t.y0 + rows_per_chunk);
  return t;
}

// one window row of a [B, H, W, C2] tensor of channel pairs: columns x0 - PAD .. x0 + DW_TX + PAD - 1 of row yy,
// addresses clamped into the map (values outside are never used)
// (the element offsets of the window's columns inside a row are the same for every row of a strip: computed once,
// wave-uniform, so that a row costs one 64-bit row address and an add per column instead of a clamp and a 64-bit
// multiply per column - with one or two wavefronts per SIMD every scalar instruction takes an issue slot too)
template <int KS>
struct DwCols {
  int off[DW_TX + KS - 1];
  __device__ __forceinline__ void init(int x0, int W, int C2) {
#pragma unroll
    for (int col = 0; col < DW_TX + KS - 1; ++col) off[col] = min(max(x0 + col - KS / 2, 0), W - 1) * C2;
  }
};
template <int KS>
__device__ __forceinline__ void dw_load_row(const uint32_t* __restrict__ src, int b, int yy, const DwCols<KS>& cols, int H, int W,
                                            int C2, int cp, uint32_t (&dst)[DW_TX + KS - 1]) {
  constexpr int WIN = DW_TX + KS - 1;
  // wave-uniform column address + the lane's channel pair as an unsigned 32-bit offset: scalar base and vector offset
  // of one load instruction, no 64-bit vector arithmetic
  const uint32_t* rowp = src + ((long long)b * H + min(max(yy, 0), H - 1)) * W * C2;
  const uint32_t lane_off = (uint32_t)cp;
#pragma unroll
  for (int col = 0; col < WIN; ++col) dst[col] = (rowp + cols.off[col])[lane_off];
}
// dst[col] &= all-ones where bit col of `bits` is set, zero elsewhere (the mask is wave-uniform: scalar operands)
template <int N>
__device__ __forceinline__ void dw_mask_words(uint32_t (&dst)[N], unsigned bits) {
#pragma unroll
  for (int col = 0; col < N; ++col) dst[col] &= ((bits >> col) & 1u) ? 0xffffffffu : 0u;
}
// Lane c looks window column c of row yy up in the inverse map (-1: outside the map or dropped).  The ballot
// over (value >= 0) that turns it into a wave-uniform mask is taken later, by the caller, so that the lookup's
// latency overlaps the other loads instead of stopping the wavefront at every row.
template <int KS>
__device__ __forceinline__ int dw_row_lookup(const int32_t* __restrict__ inv, int b, int yy, int x0, int H, int W) {
  constexpr int PAD = KS / 2, WIN = DW_TX + KS - 1;
  const int lane = threadIdx.x & 63, xx = x0 + lane - PAD;
  const bool inside = lane < WIN && yy >= 0 && yy < H && xx >= 0 && xx < W;
  const int v = inv[((long long)b * H + min(max(yy, 0), H - 1)) * W + min(max(xx, 0), W - 1)];   // unconditional: no branch, no wait here
  return inside ? v : -1;
}

// Two bf16 values of ONE channel side by side (v_dot2c_f32_bf16 multiplies them pairwise and adds both products
// to an fp32 accumulator): a loaded word holds two channels of one position, so pairs along x are made with one
// byte permute per word.
typedef __bf16 dw_bf16x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t dw_pair_lo(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x05040100u); }  // (x.lo, y.lo)
__device__ __forceinline__ uint32_t dw_pair_hi(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x07060302u); }  // (x.hi, y.hi)
__device__ __forceinline__ float dw_dot2(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dw_bf16x2v, a), __builtin_bit_cast(dw_bf16x2v, b), acc, false);
}

// dX, gradient row by gradient row: the workgroup walks down its strip, every masked row of dY is fetched once,
// paired along x, and added to the KS output rows it reaches, whose DW_TX x 2 running sums each stay in registers
// (slot j holds output row yy - PAD + j; after gradient row yy slot 0 is complete, is stored, and the slots
// move up).  Products are exact (bf16 x bf16 in fp32), sums fp32.
// (strip: number of the strip chunk; the channel pair comes from blockIdx.y and threadIdx.x)
template <int KS>
__device__ __forceinline__ void dw_dx_strip_body(int strip, const uint32_t* __restrict__ dY, const int32_t* __restrict__ inv,
                                                 const uint32_t* __restrict__ Wd, int H, int W, int C2,
                                                 uint32_t* __restrict__ dX, int tiles_x, int chunks, int rows_per_chunk) {
  constexpr int PAD = KS / 2, WIN = DW_TX + KS - 1, NP = (KS + 1) / 2, NG = WIN / 2;
  static_assert(WIN % 2 == 0, "pairs along the window row");
  const int cp_raw = blockIdx.y * blockDim.x + threadIdx.x;
  const bool active = cp_raw < C2;
  const int cp = active ? cp_raw : C2 - 1;
  const DwStrip t = dw_strip(strip, tiles_x, chunks, rows_per_chunk, H);
  // weight pairs of tap row u: (w[u][KS-1-2m], w[u][KS-2-2m]) meet the gradients of columns (ox + 2m, ox + 2m + 1)
  uint32_t wp[KS][NP][2];
#pragma unroll
  for (int u = 0; u < KS; ++u)
#pragma unroll
    for (int m = 0; m < NP; ++m) {
      const uint32_t lo = Wd[(u * KS + KS - 1 - 2 * m) * C2 + cp];
      const uint32_t hi = KS - 2 - 2 * m >= 0 ? Wd[(u * KS + KS - 2 - 2 * m) * C2 + cp] : 0u;
      wp[u][m][0] = dw_pair_lo(lo, hi);
      wp[u][m][1] = dw_pair_hi(lo, hi);
    }
  float acc[KS][DW_TX][2];
#pragma unroll
  for (int j = 0; j < KS; ++j)
#pragma unroll
    for (int ox = 0; ox < DW_TX; ++ox) acc[j][ox][0] = acc[j][ox][1] = 0.f;
  uint32_t raw[WIN], nxt[WIN];
  DwCols<KS> cols;
  cols.init(t.x0, W, C2);
  dw_load_row<KS>(dY, t.b, t.y0 - PAD, cols, H, W, C2, cp, raw);
  int look = dw_row_lookup<KS>(inv, t.b, t.y0 - PAD, t.x0, H, W);
  for (int yy = t.y0 - PAD; yy < t.y1 + PAD; ++yy) {
    int lookn = -1;
    if (yy + 1 < t.y1 + PAD) {                 // the next gradient row: in flight during this one
      dw_load_row<KS>(dY, t.b, yy + 1, cols, H, W, C2, cp, nxt);
      lookn = dw_row_lookup<KS>(inv, t.b, yy + 1, t.x0, H, W);
    }
    dw_mask_words<WIN>(raw, (unsigned)__ballot(look >= 0));    // dropped and outside positions: zero
    uint32_t ge[2][NG], go[2][NG];             // (g[2k], g[2k+1]) and (g[2k+1], g[2k+2]) per channel
#pragma unroll
    for (int k = 0; k < NG; ++k) {
      const uint32_t r0 = raw[2 * k], r1 = raw[2 * k + 1], r2 = 2 * k + 2 < WIN ? raw[2 * k + 2] : 0u;
      ge[0][k] = dw_pair_lo(r0, r1); ge[1][k] = dw_pair_hi(r0, r1);
      go[0][k] = dw_pair_lo(r1, r2); go[1][k] = dw_pair_hi(r1, r2);
    }
#pragma unroll
    for (int j = 0; j < KS; ++j) {             // tap row j links this gradient row to output row yy - PAD + j
      const int y = yy - PAD + j;
      if (y < t.y0 || y >= t.y1) continue;     // another chunk's row: wave-uniform
#pragma unroll
      for (int ox = 0; ox < DW_TX; ++ox)
#pragma unroll
        for (int m = 0; m < NP; ++m) {
          const int col = ox + 2 * m;          // gradient columns col, col + 1 of the window
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            const uint32_t g = (col & 1) ? go[c][(col - 1) / 2] : ge[c][col / 2];
            acc[j][ox][c] = dw_dot2(g, wp[j][m][c], acc[j][ox][c]);
          }
        }
    }
    const int yo = yy - PAD;                   // slot 0 is complete
    if (yo >= t.y0 && active) {
      uint32_t* orow = dX + (((long long)t.b * H + yo) * W + t.x0) * C2 + cp;
#pragma unroll
      for (int ox = 0; ox < DW_TX; ++ox)
        if (t.x0 + ox < W) orow[(long long)ox * C2] = dw_pack(acc[0][ox][0], acc[0][ox][1]);
    }
#pragma unroll
    for (int j = 0; j + 1 < KS; ++j)
#pragma unroll
      for (int ox = 0; ox < DW_TX; ++ox) { acc[j][ox][0] = acc[j + 1][ox][0]; acc[j][ox][1] = acc[j + 1][ox][1]; }
#pragma unroll
    for (int ox = 0; ox < DW_TX; ++ox) acc[KS - 1][ox][0] = acc[KS - 1][ox][1] = 0.f;
#pragma unroll
    for (int col = 0; col < WIN; ++col) raw[col] = nxt[col];
    look = lookn;
  }
}

template <int KS>
__global__ void __launch_bounds__(DW_THREADS) dw_dx_strip_kernel(const uint32_t* __restrict__ dY, const int32_t* __restrict__ inv,
                                                                 const uint32_t* __restrict__ Wd, int H, int W, int C2,
                                                                 uint32_t* __restrict__ dX, int tiles_x, int chunks,
                                                                 int rows_per_chunk) {
  dw_dx_strip_body<KS>(blockIdx.x, dY, inv, Wd, H, W, C2, dX, tiles_x, chunks, rows_per_chunk);
}

// dWd, db: blockDim = (channel pairs, GROUPS); every group walks strips with the window of X in registers and
// KS*KS + 1 running sums per channel.  Groups are added through LDS in a fixed order, one partial per block.
// (blk of nblk: this block among those that share the strips; the whole workgroup calls this together)
template <int KS, int GROUPS>
__device__ __forceinline__ void dw_dw_strip_body(int blk, int nblk, float* red, const uint32_t* __restrict__ dY,
                                                 const int32_t* __restrict__ inv, const uint32_t* __restrict__ X, int H, int W,
                                                 int C2, int tiles_x, int chunks, int rows_per_chunk, int nstrips,
                                                 float* __restrict__ part) {
  constexpr int PAD = KS / 2, WIN = DW_TX + KS - 1, NT = KS * KS + 1;   // red: [GROUPS - 1][CHUNK][blockDim.x][2] in LDS
  const int cp_raw = blockIdx.y * blockDim.x + threadIdx.x;
  const bool active = cp_raw < C2;
  const int cp = active ? cp_raw : C2 - 1;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.y);   // a wavefront never spans two groups
  const int lane = threadIdx.x & 63;
  float s0[NT], s1[NT];
#pragma unroll
  for (int tp = 0; tp < NT; ++tp) { s0[tp] = 0.f; s1[tp] = 0.f; }

  for (int strip = blk * GROUPS + grp; strip < nstrips; strip += nblk * GROUPS) {
    const DwStrip t = dw_strip(strip, tiles_x, chunks, rows_per_chunk, H);
    unsigned colmask = 0;                     // window columns inside the map
#pragma unroll
    for (int col = 0; col < WIN; ++col)
      if (t.x0 + col - PAD >= 0 && t.x0 + col - PAD < W) colmask |= 1u << col;
    // window rows of X: positions outside the map are zeroed as a row enters the window (zero padding), the
    // gradients of dropped positions are zeroed too, and the row loop has no branches
    DwCols<KS> cols;
    cols.init(t.x0, W, C2);
    uint32_t win[KS][WIN], nxt[WIN], g[DW_TX], gn[DW_TX];
#pragma unroll
    for (int r = 0; r < KS; ++r) {
      const int yy = t.y0 + r - PAD;
      dw_load_row<KS>(X, t.b, yy, cols, H, W, C2, cp, win[r]);
      dw_mask_words<WIN>(win[r], (yy >= 0 && yy < H) ? colmask : 0u);
    }
    // gradients of row y and, per lane, the inverse-map entry of position x0 + lane (-1: outside or dropped);
    // the ballot that makes the kept mask is taken when the values are needed, a row later
    auto load_g = [&](int y, uint32_t (&dst)[DW_TX]) -> int {
      const long long prow = ((long long)t.b * H + y) * W;
      const uint32_t* rowp = dY + prow * C2;
#pragma unroll
      for (int ox = 0; ox < DW_TX; ++ox) dst[ox] = (rowp + cols.off[ox + PAD])[(uint32_t)cp];   // window column ox + PAD is map column x0 + ox
      const int v = inv[prow + min(t.x0 + lane, W - 1)];                 // unconditional: no branch, no wait here
      return (lane < DW_TX && t.x0 + lane < W) ? v : -1;
    };
    const int look0 = load_g(t.y0, g);
    dw_mask_words<DW_TX>(g, (unsigned)__ballot(look0 >= 0));
    for (int y = t.y0; y < t.y1; ++y) {
      int lookn = -1;
      if (y + 1 < t.y1) {
        dw_load_row<KS>(X, t.b, y + 1 + PAD, cols, H, W, C2, cp, nxt);
        lookn = load_g(y + 1, gn);
      }
      // pairs along x of one channel: gradients (g[2k], g[2k+1]) against window pairs (x[2k+v], x[2k+v+1]); one
      // v_dot2 adds two exact products to the fp32 sum of tap (u, v); the bias sum pairs the gradients with (1, 1)
      static_assert(DW_TX % 2 == 0, "gradient pairs");
      constexpr uint32_t kOnes = 0x3f803f80u;
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        uint32_t gp[DW_TX / 2];
#pragma unroll
        for (int k = 0; k < DW_TX / 2; ++k) {
          gp[k] = c == 0 ? dw_pair_lo(g[2 * k], g[2 * k + 1]) : dw_pair_hi(g[2 * k], g[2 * k + 1]);
          if (c == 0) s0[KS * KS] = dw_dot2(gp[k], kOnes, s0[KS * KS]);
          else s1[KS * KS] = dw_dot2(gp[k], kOnes, s1[KS * KS]);
        }
#pragma unroll
        for (int u = 0; u < KS; ++u) {
          uint32_t xe[WIN / 2], xo[WIN / 2];       // (x[2m], x[2m+1]) and (x[2m+1], x[2m+2])
#pragma unroll
          for (int m = 0; m < WIN / 2; ++m) {
            xe[m] = c == 0 ? dw_pair_lo(win[u][2 * m], win[u][2 * m + 1]) : dw_pair_hi(win[u][2 * m], win[u][2 * m + 1]);
            xo[m] = 2 * m + 2 < WIN ? (c == 0 ? dw_pair_lo(win[u][2 * m + 1], win[u][2 * m + 2]) : dw_pair_hi(win[u][2 * m + 1], win[u][2 * m + 2])) : 0u;
          }
#pragma unroll
          for (int v = 0; v < KS; ++v)
#pragma unroll
            for (int k = 0; k < DW_TX / 2; ++k) {
              const int m = 2 * k + v;                 // first window column of the pair (compile time)
              const uint32_t xp = (m & 1) ? xo[(m - 1) / 2] : xe[m / 2];
              if (c == 0) s0[u * KS + v] = dw_dot2(gp[k], xp, s0[u * KS + v]);
              else s1[u * KS + v] = dw_dot2(gp[k], xp, s1[u * KS + v]);
            }
        }
      }
#pragma unroll
      for (int r = 0; r + 1 < KS; ++r)
#pragma unroll
        for (int col = 0; col < WIN; ++col) win[r][col] = win[r + 1][col];
#pragma unroll
      for (int col = 0; col < WIN; ++col) win[KS - 1][col] = nxt[col];
      dw_mask_words<WIN>(win[KS - 1], (y + 1 + PAD < H) ? colmask : 0u);
#pragma unroll
      for (int ox = 0; ox < DW_TX; ++ox) g[ox] = gn[ox];
      dw_mask_words<DW_TX>(g, (unsigned)__ballot(lookn >= 0));
    }
  }

  // add the groups (fixed order 0, 1, 2, ...) through LDS, CHUNK taps at a time
  constexpr int CHUNK = 10;
  const int ct = blockDim.x;
  float* out = part + ((long long)blk * NT) * (2 * C2);
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

template <int KS, int GROUPS>
__global__ void __launch_bounds__(DW_THREADS * GROUPS) dw_dw_strip_kernel(const uint32_t* __restrict__ dY,
                                                                          const int32_t* __restrict__ inv,
                                                                          const uint32_t* __restrict__ X, int H, int W,
                                                                          int C2, int tiles_x, int chunks, int rows_per_chunk,
                                                                          int nstrips, float* __restrict__ part) {
  extern __shared__ float red[];
  dw_dw_strip_body<KS, GROUPS>(blockIdx.x, gridDim.x, red, dY, inv, X, H, W, C2, tiles_x, chunks, rows_per_chunk, nstrips, part);
}

// Both in one launch, for callers that want dX and the weight gradient (the usual case): on a small map each of the
// two kernels alone leaves the SIMDs with one wavefront, and neither can hide its latencies; side by side they
// share the CUs.  The first n_dw workgroups walk strips for dWd / db, the others take GROUPS dX strips each.
struct DwBothArgs {
  const uint32_t* dY; const int32_t* inv; const uint32_t* X; const uint32_t* Wd;
  int H, W, C2, tiles_x;
  int chunks_w, rows_w, nstrips_w, n_dw;     // weight-gradient role
  int chunks_x, rows_x, nstrips_x;           // dX role
  float* part; uint32_t* dX;
};
template <int KS, int GROUPS>
__global__ void __launch_bounds__(DW_THREADS * GROUPS) dw_both_strip_kernel(const DwBothArgs a) {
  extern __shared__ float red[];
  if ((int)blockIdx.x < a.n_dw) {
    dw_dw_strip_body<KS, GROUPS>(blockIdx.x, a.n_dw, red, a.dY, a.inv, a.X, a.H, a.W, a.C2, a.tiles_x, a.chunks_w, a.rows_w,
                                 a.nstrips_w, a.part);
  } else {
    const int strip = ((int)blockIdx.x - a.n_dw) * GROUPS + (int)threadIdx.y;
    if (strip < a.nstrips_x) dw_dx_strip_body<KS>(strip, a.dY, a.inv, a.Wd, a.H, a.W, a.C2, a.dX, a.tiles_x, a.chunks_x, a.rows_x);
  }
}

// ------------------------------------------------------------------------------------------------
// bf16, channel counts that are multiples of 8: LDS-tiled kernel.  A workgroup takes a tile of R rows x TS strips of 8
// columns and a slab of 32 channels, stages the gradient tile WITH its halo of KS - 1 rows and columns (dropped and
// outside positions as zeros: no mask is looked at afterwards) and the X tile (no halo) in LDS once, and computes from
// them both the dX of the tile and the tile's share of dWd and db:
//   dX[y][x]   = sum_{i,t} g[y - PAD + i][x - PAD + t] w[KS-1-i][KS-1-t]
//   dWd[u][v] += sum_{(y,x) in tile} X[y][x] g[y - u + PAD][x - v + PAD]      (summed over X positions: every pair of an
//                                                                              X and a gradient position lies in one tile)
// LDS lines are [row][channel][column]: 2-byte elements, columns contiguous, so a 4-byte word is two neighbouring
// columns of ONE channel - the operand shape of v_dot2_f32_bf16 (two exact products added to an fp32 sum).  A lane owns
// one channel and, per work item, one row of one strip: per gradient row it reads 8 words (two 16-byte reads), makes the
// 7 odd-aligned pairs with v_alignbit, and feeds 8 x 4 dot2 (dX) and 4 x KS dot2 (dWd) from them.  The two halves of a
// wavefront work on different strips; the 8 half-wavefronts of a workgroup are added through LDS at the end, one
// partial per workgroup (fixed order), and dw_reduce_kernel adds the workgroups' partials.
// ------------------------------------------------------------------------------------------------
static constexpr int DWF_SLAB = 32;      // channels per workgroup
static constexpr int DWF_THREADS = 256;  // two workgroups per CU (512 threads each were slower: the kernel is bound by its instruction count)
static constexpr int DWF_SLOTS = DWF_THREADS / DWF_SLAB;   // half-wavefronts = strips in flight
static constexpr int DWF_RED = DWF_SLOTS < 8 ? DWF_SLOTS : 8;        // slots of the LDS buffer the half-wavefronts' sums are added through

struct DwFusedArgs {
  const uint16_t* dY; const int32_t* inv; const uint16_t* X; const uint16_t* Wd;
  uint16_t* dX; float* part;   // part[workgroup x][KS*KS + 1][C]
  int B, H, W, C;
  int R, TS;                   // output rows and 8-column strips per tile
  int tiles_y, tiles_x, ntiles;
  int pitch;                   // bytes of one (row, channel) line of the LDS tiles
  int want_dx, want_dw;
};

__device__ __forceinline__ uint32_t dwf_alignbit(uint32_t hi, uint32_t lo) { return __builtin_amdgcn_alignbit(hi, lo, 16); }   // (lo.hi, hi.lo)

// the words (A.k, B.k) of 8 channels of two neighbouring positions into the 8 channel lines starting at dst
__device__ __forceinline__ void dwf_store_pairs(char* dst, int pitch, const uint4& A, const uint4& Bv) {
  *reinterpret_cast<uint32_t*>(dst + 0 * pitch) = dw_pair_lo(A.x, Bv.x);
  *reinterpret_cast<uint32_t*>(dst + 1 * pitch) = dw_pair_hi(A.x, Bv.x);
  *reinterpret_cast<uint32_t*>(dst + 2 * pitch) = dw_pair_lo(A.y, Bv.y);
  *reinterpret_cast<uint32_t*>(dst + 3 * pitch) = dw_pair_hi(A.y, Bv.y);
  *reinterpret_cast<uint32_t*>(dst + 4 * pitch) = dw_pair_lo(A.z, Bv.z);
  *reinterpret_cast<uint32_t*>(dst + 5 * pitch) = dw_pair_hi(A.z, Bv.z);
  *reinterpret_cast<uint32_t*>(dst + 6 * pitch) = dw_pair_lo(A.w, Bv.w);
  *reinterpret_cast<uint32_t*>(dst + 7 * pitch) = dw_pair_hi(A.w, Bv.w);
}

template <int KS>
__global__ void __launch_bounds__(DWF_THREADS, 2) dw_fused_kernel(const DwFusedArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int PAD = KS / 2, NP = (KS + 1) / 2, NT = KS * KS + 1;
  const int tid = threadIdx.x;
  const int slot = tid >> 5, ch = tid & 31;
  const int slab0 = blockIdx.y * DWF_SLAB;
  const int c = slab0 + ch;
  const bool active = c < a.C;
  const int cc = active ? c : a.C - 1;
  const int GR = a.R + KS - 1;                         // gradient rows of a tile
  const int ncw = a.pitch >> 2;                        // words per line
  char* gt = lds;                                      // [GR][32][pitch]
  char* xt = lds + (size_t)GR * DWF_SLAB * a.pitch;    // [R][32][pitch]
  unsigned char* mask = reinterpret_cast<unsigned char*>(xt + (size_t)a.R * DWF_SLAB * a.pitch);   // [GR][2 ncw] kept / dropped

  // flipped weight pairs of this lane's channel: pair m of gradient row i holds taps (KS-1-2m, KS-2-2m) of row KS-1-i
  uint32_t wp[KS][NP];
  if (a.want_dx) {
#pragma unroll
    for (int i = 0; i < KS; ++i)
#pragma unroll
      for (int m = 0; m < NP; ++m) {
        const int u = KS - 1 - i, v0 = KS - 1 - 2 * m, v1 = KS - 2 - 2 * m;
        const uint32_t lo = a.Wd[(u * KS + v0) * a.C + cc];
        const uint32_t hi = v1 >= 0 ? a.Wd[(u * KS + v1) * a.C + cc] : 0u;
        wp[i][m] = lo | (hi << 16);
      }
  }
  float accw[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) accw[t] = 0.f;

  for (int tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
    const int tx = tile % a.tiles_x, rest = tile / a.tiles_x;
    const int ty = rest % a.tiles_y, b = rest / a.tiles_y;
    const int y0 = ty * a.R, x0 = tx * a.TS * 8;
    __syncthreads();                                   // the previous tile's readers are done
    // ---- stage the gradient tile (halo, zeros where dropped or outside) and the X tile -----------------------------
    {
      // Order of the global loads (latency is what staging costs: every load here misses the caches of the CU):
      //   1. the inverse-map entries of the halo tile's positions (kept / dropped; up to 4 per thread),
      //   2. the thread's X rows (2 rows in flight; they depend on nothing),
      //   3. kept / dropped bytes into LDS (waits for 1 only: loads complete in order), barrier,
      //   4. the thread's gradient rows, kept positions only (3 rows in flight: more spill registers),
      //   5. X rows into LDS, gradient rows into LDS; further chunks of rows, if any, the same way.
      const int ncols = 2 * ncw;
      const int npos = GR * ncols;
      int mv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int p = tid + u * DWF_THREADS;
        mv[u] = -1;
        if (p < npos) {
          const int row = p / ncols, j = p - row * ncols;
          const int y = y0 - PAD + row, x = x0 - PAD + j;
          if (y >= 0 && y < a.H && x >= 0 && x < a.W) mv[u] = a.inv[((long long)b * a.H + y) * a.W + x];
        }
      }
      // thread <-> (8-channel group, word of the line, row phase): no divisions per item, rows advance by a fixed step
      const int per_row = ncw * 4, rstep = DWF_THREADS / per_row;     // (host: per_row <= DWF_THREADS)
      const int g8 = tid & 3, wj = (tid >> 2) % ncw, r0 = (tid >> 2) / ncw;
      const int c8 = min(slab0 + 8 * g8, a.C - 8);                     // (slabs beyond C: clamped, their lanes store nothing)
      const bool stager = r0 < rstep;
      const bool xstager = stager && a.want_dw && wj < a.TS * 4;
      const int x = x0 - PAD + 2 * wj, xx = x0 + 2 * wj;
      auto load_x = [&](int rb, uint4 (&A)[2], uint4 (&Bv)[2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int row = rb + u * rstep, y = y0 + row;
          A[u] = make_uint4(0, 0, 0, 0); Bv[u] = make_uint4(0, 0, 0, 0);
          if (row < a.R && y < a.H) {
            const long long prow = ((long long)b * a.H + y) * a.W;
            if (xx < a.W) A[u] = *reinterpret_cast<const uint4*>(a.X + (prow + xx) * a.C + c8);
            if (xx + 1 < a.W) Bv[u] = *reinterpret_cast<const uint4*>(a.X + (prow + xx + 1) * a.C + c8);
          }
        }
      };
      auto store_x = [&](int rb, const uint4 (&A)[2], const uint4 (&Bv)[2]) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int row = rb + u * rstep;
          if (row < a.R) dwf_store_pairs(xt + ((size_t)(row * DWF_SLAB + 8 * g8)) * a.pitch + wj * 4, a.pitch, A[u], Bv[u]);
        }
      };
      uint4 XA[2], XB[2];
      if (xstager) load_x(r0, XA, XB);
      for (int u = 0; u < 4; ++u) {
        const int p = tid + u * DWF_THREADS;
        if (p < npos) mask[p] = mv[u] >= 0 ? 1 : 0;
      }
      for (int p = tid + 4 * DWF_THREADS; p < npos; p += DWF_THREADS) {      // (tiles of more than 1024 positions)
        const int row = p / ncols, j = p - row * ncols;
        const int y = y0 - PAD + row, xq = x0 - PAD + j;
        bool kept = false;
        if (y >= 0 && y < a.H && xq >= 0 && xq < a.W) kept = a.inv[((long long)b * a.H + y) * a.W + xq] >= 0;
        mask[p] = kept ? 1 : 0;
      }
      __syncthreads();
      if (stager) {
        for (int rb = r0; rb < GR; rb += 3 * rstep) {
          uint4 A[3], Bv[3];
#pragma unroll
          for (int u = 0; u < 3; ++u) {
            const int row = rb + u * rstep;
            A[u] = make_uint4(0, 0, 0, 0); Bv[u] = make_uint4(0, 0, 0, 0);
            if (row < GR) {
              const unsigned m = *reinterpret_cast<const unsigned short*>(mask + row * ncols + 2 * wj);
              const long long prow = ((long long)b * a.H + (y0 - PAD + row)) * a.W;
              if (m & 0xffu) A[u] = *reinterpret_cast<const uint4*>(a.dY + (prow + x) * a.C + c8);
              if (m >> 8) Bv[u] = *reinterpret_cast<const uint4*>(a.dY + (prow + x + 1) * a.C + c8);
            }
          }
          if (rb == r0 && xstager) store_x(r0, XA, XB);          // (arrived long ago)
#pragma unroll
          for (int u = 0; u < 3; ++u) {
            const int row = rb + u * rstep;
            if (row < GR) dwf_store_pairs(gt + ((size_t)(row * DWF_SLAB + 8 * g8)) * a.pitch + wj * 4, a.pitch, A[u], Bv[u]);
          }
        }
        if (xstager)
          for (int rb = r0 + 2 * rstep; rb < a.R; rb += 2 * rstep) {
            load_x(rb, XA, XB);
            store_x(rb, XA, XB);
          }
      }
    }
    __syncthreads();
    // ---- work items: (row, strip) pairs, dealt to the 8 half-wavefronts -------------------------------------------
    for (int it = slot; it < a.R * a.TS; it += DWF_SLOTS) {
      const int row = it / a.TS, st = it - row * a.TS;
      const int y = y0 + row;
      if (y >= a.H) continue;
      float acc[8];
#pragma unroll
      for (int ox = 0; ox < 8; ++ox) acc[ox] = 0.f;
      uint32_t xw[4] = {0, 0, 0, 0};
      if (a.want_dw) {
        const uint4 v = *reinterpret_cast<const uint4*>(xt + ((size_t)(row * DWF_SLAB + ch)) * a.pitch + st * 16);
        xw[0] = v.x; xw[1] = v.y; xw[2] = v.z; xw[3] = v.w;
      }
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        const char* line = gt + ((size_t)((row + i) * DWF_SLAB + ch)) * a.pitch + st * 16;
        const uint4 lo4 = *reinterpret_cast<const uint4*>(line), hi4 = *reinterpret_cast<const uint4*>(line + 16);
        const uint32_t Wv[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};   // elements (2k, 2k+1) from tile column 8 st
        uint32_t Ov[7];                                                                    // elements (2k+1, 2k+2)
#pragma unroll
        for (int k = 0; k < 7; ++k) Ov[k] = dwf_alignbit(Wv[k + 1], Wv[k]);
        // (loop orders: consecutive instructions add to different sums)
        if (a.want_dx) {
#pragma unroll
          for (int m = 0; m < NP; ++m)
#pragma unroll
            for (int ox = 0; ox < 8; ++ox) {
              const uint32_t src = (ox & 1) ? Ov[(ox - 1) / 2 + m] : Wv[ox / 2 + m];
              acc[ox] = dw_dot2(src, wp[i][m], acc[ox]);
            }
        }
        if (a.want_dw) {
#pragma unroll
          for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int t = 0; t < KS; ++t) {
              const uint32_t src = (t & 1) ? Ov[p + (t - 1) / 2] : Wv[p + t / 2];
              accw[(KS - 1 - i) * KS + (KS - 1 - t)] = dw_dot2(xw[p], src, accw[(KS - 1 - i) * KS + (KS - 1 - t)]);
            }
          if (i == PAD) {               // the gradients at the strip's own positions: the bias sum
            constexpr uint32_t kOnes = 0x3f803f80u;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
              const uint32_t src = (PAD & 1) ? Ov[p + (PAD - 1) / 2] : Wv[p + PAD / 2];
              accw[KS * KS] = dw_dot2(src, kOnes, accw[KS * KS]);
            }
          }
        }
      }
      if (a.want_dx && active) {
        uint16_t* orow = a.dX + (((long long)b * a.H + y) * a.W + x0 + st * 8) * a.C + c;
#pragma unroll
        for (int ox = 0; ox < 8; ++ox)
          if (x0 + st * 8 + ox < a.W) orow[(long long)ox * a.C] = (uint16_t)(dw_pack(acc[ox], 0.f) & 0xffffu);
      }
    }
  }
  // ---- the workgroup's partial sums of dWd / db: the upper half-wavefronts hand theirs to the lower ones through LDS,
  // then the DWF_RED sums are added in slot order (a fixed order)
  if (a.want_dw) {
    __syncthreads();
    float* red = reinterpret_cast<float*>(lds);          // [DWF_RED][tap][32]
    if constexpr (DWF_SLOTS > DWF_RED) {
      if (slot >= DWF_RED) {
#pragma unroll
        for (int t = 0; t < NT; ++t) red[((slot - DWF_RED) * NT + t) * DWF_SLAB + ch] = accw[t];
      }
      __syncthreads();
      if (slot < DWF_RED) {
#pragma unroll
        for (int t = 0; t < NT; ++t) red[(slot * NT + t) * DWF_SLAB + ch] += accw[t];
      }
    } else {
#pragma unroll
      for (int t = 0; t < NT; ++t) red[(slot * NT + t) * DWF_SLAB + ch] = accw[t];
    }
    __syncthreads();
    for (int o = tid; o < NT * DWF_SLAB; o += DWF_THREADS) {
      float sum = 0.f;
#pragma unroll
      for (int sl = 0; sl < DWF_RED; ++sl) sum += red[sl * NT * DWF_SLAB + o];
      const int t = o / DWF_SLAB, cl = o - t * DWF_SLAB;
      if (slab0 + cl < a.C) a.part[((long long)blockIdx.x * NT + t) * a.C + slab0 + cl] = sum;
    }
  }
}

static constexpr int DW_GROUPS = 2;
static constexpr int DW_MAX_PARTS = 256;

// Tile shape of the LDS-tiled kernel: TS strips of 8 columns wide (line pitch 16 (TS + 1) bytes, rounded up to an odd
// number of 16-byte units so that the 16-byte reads of neighbouring channels fall into different banks), R rows high,
// at most 80 KB of LDS so that two workgroups share a CU; chosen for the fewest rounds of 2 x 256 workgroups, then
// for the least halo.
struct DwFusedShape { int R, TS, pitch, tiles_y, tiles_x, nwg_x; size_t lds; };
static DwFusedShape dw_fused_shape(int B, int H, int W, int C, int ks) {
  DwFusedShape best{};
  double best_cost = 0;
  const int nstrips = (int)ceil_div(W, 8), slabs = (int)ceil_div(C, DWF_SLAB);
  for (int TS = 1; TS <= 6; ++TS) {
    int units = TS + 1;
    if (units % 2 == 0) ++units;
    const int pitch = 16 * units;
    const int tiles_x = (int)ceil_div(nstrips, TS);
    const int ts_eff = (int)ceil_div(nstrips, tiles_x);           // strips really used per tile
    if (ts_eff < TS) continue;                                    // a narrower tile covers the row as well
    for (int R = 2; R <= 16; ++R) {
      const size_t lds = std::max((size_t)(2 * R + ks - 1) * DWF_SLAB * pitch + align_up((size_t)(R + ks - 1) * (pitch / 2), 16),
                                  (size_t)DWF_RED * (ks * ks + 1) * DWF_SLAB * sizeof(float));
      if (lds > 80 * 1024) break;
      const int tiles_y = (int)ceil_div(H, R);
      const int64_t nwg = (int64_t)B * tiles_y * tiles_x * slabs;
      const double rounds = (double)ceil_div(nwg, 2 * 256);
      // time of a round ~ items per workgroup (each with ks gradient rows) + the staging of the halo tile
      const double cost = rounds * ((double)R * TS * ks + 0.15 * (R + ks - 1) * (TS + 1) * 4);
      if (best.R == 0 || cost < best_cost) {
        best_cost = cost;
        best = DwFusedShape{R, TS, pitch, tiles_y, tiles_x, 0, lds};
      }
    }
  }
  best.nwg_x = (int)std::min<int64_t>((int64_t)B * best.tiles_y * best.tiles_x, DW_MAX_PARTS);
  return best;
}

DwPlan plan_dwconv(int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks, int64_t K, int32_t dtype) {
  DwPlan p{};
  (void)dtype;
  p.tiles_y = p.tiles_x = 0;
  // partial sums of dWd / db: one per block of the reduction kernel.  The fast path walks row tiles
  // (its parallelism does not depend on K), the plain path slices the kept list.
  const int64_t row_tiles = (int64_t)B * H * ceil_div(W, DW_TX);
  p.nparts = (int)std::max<int64_t>(1, std::min<int64_t>(DW_MAX_PARTS, std::max<int64_t>(ceil_div(row_tiles, 2 * DW_GROUPS), 1)));
  if (ks == 7 || ks == 3) p.nparts = std::max(p.nparts, dw_fused_shape(B, H, W, C, ks).nwg_x);   // the LDS-tiled kernel's workgroups
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
  const Options opt = options();                                             // explicit overrides for sweeps and tests
  const bool tiled = dtype == SBP_BF16 && C % 8 == 0 && (ks == 7 || ks == 3) && !opt.dw_strips &&
                     (((uintptr_t)dY | (uintptr_t)X | (uintptr_t)dX) % 16 == 0) && (int64_t)B * H * W * C < (1ll << 40);
  if (tiled) {
    const DwFusedShape f = dw_fused_shape(B, H, W, C, ks);
    DwFusedArgs a{};
    a.dY = (const uint16_t*)dY; a.inv = inv; a.X = (const uint16_t*)X; a.Wd = (const uint16_t*)Wd;
    a.dX = (uint16_t*)dX; a.part = part;
    a.B = B; a.H = H; a.W = W; a.C = C;
    a.R = f.R; a.TS = f.TS; a.tiles_y = f.tiles_y; a.tiles_x = f.tiles_x; a.ntiles = B * f.tiles_y * f.tiles_x;
    a.pitch = f.pitch;
    a.want_dx = dX != nullptr; a.want_dw = (dWd || db) ? 1 : 0;
    const dim3 grid((unsigned)f.nwg_x, (unsigned)ceil_div(C, DWF_SLAB));
    static std::once_flag once7, once3;
    if (f.lds > 64 * 1024) {
      if (ks == 7) std::call_once(once7, [] { (void)hipFuncSetAttribute(reinterpret_cast<const void*>(dw_fused_kernel<7>), hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024); });
      else std::call_once(once3, [] { (void)hipFuncSetAttribute(reinterpret_cast<const void*>(dw_fused_kernel<3>), hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024); });
    }
    if (ks == 7) SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_fused_kernel<7>), grid, dim3(DWF_THREADS), f.lds, s, a);
    else SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_fused_kernel<3>), grid, dim3(DWF_THREADS), f.lds, s, a);
    if (a.want_dw) {
      const int n = (ks * ks + 1) * C;
      SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, dw_reduce_kernel, dim3((unsigned)ceil_div(n, 32)), dim3(DW_THREADS), 0, s, part, f.nwg_x,
                 ks * ks, C, dWd, db);
    }
    return check_launch("backward_dwconv");
  }
  const bool fast = dtype == SBP_BF16 && C % 2 == 0 && (ks == 7 || ks == 3) && ((uintptr_t)dY % 4 == 0) &&
                    ((uintptr_t)X % 4 == 0) && ((uintptr_t)Wd % 4 == 0) && ((uintptr_t)dX % 4 == 0);
  if (fast) {
    const int C2 = C / 2;
    const int ct = (int)std::min<int64_t>(DW_THREADS, ceil_div(C2, 64) * 64);
    const int cblocks = (int)ceil_div(C2, ct);
    const int tiles_x = (int)ceil_div(W, DW_TX);
    // rows per strip chunk: a chunk pays for KS - 1 halo rows on top of its own, a short chunk for its start-up;
    // about one workgroup per CU for dX, somewhat more for the weight gradient (measured on the 50 x 84 x 512 map)
    const int64_t row_tiles = (int64_t)tiles_x * B * H * cblocks;
    auto pick_rows = [&](int64_t per) {
      int r = (int)std::min<int64_t>(16, std::max<int64_t>(3, ceil_div(row_tiles, per)));
      if (opt.dw_rows) r = opt.dw_rows;
      return std::min(r, H);
    };
    int rows = pick_rows(256);
    int chunks = (int)ceil_div(H, rows);
    int nstrips = tiles_x * chunks * B;
    if (dX && (dWd || db) && !opt.dw_separate) {   // (override "dw_separate": the two kernels one after the other)
      // one launch for both; strip heights chosen so that everything finds a CU at once where the map allows
      DwBothArgs a{};
      a.dY = (const uint32_t*)dY; a.inv = inv; a.X = (const uint32_t*)X; a.Wd = (const uint32_t*)Wd;
      a.H = H; a.W = W; a.C2 = C2; a.tiles_x = tiles_x;
      a.rows_x = rows; a.chunks_x = chunks; a.nstrips_x = nstrips;
      const int n_dx = (int)ceil_div(nstrips, DW_GROUPS);
      a.rows_w = pick_rows(288);
      a.chunks_w = (int)ceil_div(H, a.rows_w);
      a.nstrips_w = tiles_x * a.chunks_w * B;
      a.n_dw = (int)std::min<int64_t>(p.nparts, ceil_div(a.nstrips_w, DW_GROUPS));
      a.part = part; a.dX = (uint32_t*)dX;
      dim3 grid((unsigned)(a.n_dw + n_dx), (unsigned)cblocks);
      const size_t lds = (size_t)(DW_GROUPS - 1) * 10 * ct * 2 * sizeof(float);
      if (ks == 7) SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_both_strip_kernel<7, DW_GROUPS>), grid, dim3(ct, DW_GROUPS), lds, s, a);
      else SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_both_strip_kernel<3, DW_GROUPS>), grid, dim3(ct, DW_GROUPS), lds, s, a);
      const int n = (ks * ks + 1) * C;
      SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, dw_reduce_kernel, dim3((unsigned)ceil_div(n, 32)), dim3(DW_THREADS), 0,
                 s, part, a.n_dw, ks * ks, C, dWd, db);
      return check_launch("backward_dwconv");
    }
    if (dX) {
      dim3 grid((unsigned)nstrips, (unsigned)cblocks);
      if (ks == 7)
        SBP_LAUNCH(SBP_PROF_DWCONV_DX, s, (dw_dx_strip_kernel<7>), grid, dim3(ct), 0, s, (const uint32_t*)dY, inv,
                   (const uint32_t*)Wd, H, W, C2, (uint32_t*)dX, tiles_x, chunks, rows);
      else
        SBP_LAUNCH(SBP_PROF_DWCONV_DX, s, (dw_dx_strip_kernel<3>), grid, dim3(ct), 0, s, (const uint32_t*)dY, inv,
                   (const uint32_t*)Wd, H, W, C2, (uint32_t*)dX, tiles_x, chunks, rows);
    }
    if (dWd || db) {
      rows = pick_rows(400);
      chunks = (int)ceil_div(H, rows);
      nstrips = tiles_x * chunks * B;
      const int nblk = (int)std::min<int64_t>(p.nparts, ceil_div(nstrips, DW_GROUPS));
      dim3 grid((unsigned)nblk, (unsigned)cblocks);
      const size_t lds = (size_t)(DW_GROUPS - 1) * 10 * ct * 2 * sizeof(float);
      if (ks == 7)
        SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_dw_strip_kernel<7, DW_GROUPS>), grid, dim3(ct, DW_GROUPS), lds, s,
                   (const uint32_t*)dY, inv, (const uint32_t*)X, H, W, C2, tiles_x, chunks, rows, nstrips, part);
      else
        SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, (dw_dw_strip_kernel<3, DW_GROUPS>), grid, dim3(ct, DW_GROUPS), lds, s,
                   (const uint32_t*)dY, inv, (const uint32_t*)X, H, W, C2, tiles_x, chunks, rows, nstrips, part);
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
