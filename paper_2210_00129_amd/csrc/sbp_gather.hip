// Row gather X_k[j,:] = X[idx[j],:]: the forward-side cache of SBP (the paper's method keeps
// only a subset of each layer input for the backward pass).  Pure data movement, bound by
// HBM: every thread moves 16-byte pieces, several in flight, rows laid out so that a
// wavefront reads and writes whole contiguous row segments.
#include <algorithm>
#include <cstdlib>

#include "sbp_internal.h"

namespace sbp {

// rows whose byte length is a multiple of 16: 16-byte pieces, UNROLL in flight per thread.  Piece numbers fit 32 bits
// (the host cuts larger inputs into several launches), so row and column come from a multiply and a shift.
template <int UNROLL>
__global__ void __launch_bounds__(256) gather_rows_vec16(const uint4* __restrict__ X, const int32_t* __restrict__ idx,
                                                         uint32_t total, FastDiv pieces_per_row, uint4* __restrict__ Xk) {
  const uint32_t stride = gridDim.x * 256u;
  uint32_t t = blockIdx.x * 256u + threadIdx.x;
  const uint32_t ppr = pieces_per_row.d;
  for (; t < total && total - t > (UNROLL - 1) * stride; t += UNROLL * stride) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      uint32_t j, c;
      pieces_per_row.divmod(t + u * stride, j, c);
      v[u] = X[(long long)idx[j] * ppr + c];
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) Xk[t + u * stride] = v[u];
    if (UNROLL * stride > ~t) return;                       // the next step would wrap
  }
  for (; t < total; t += stride) {
    uint32_t j, c;
    pieces_per_row.divmod(t, j, c);
    Xk[t] = X[(long long)idx[j] * ppr + c];
    if (stride > ~t) return;
  }
}

// any row length: element-wise copy in units of `unit` bytes (2 or 4)
template <typename T>
__global__ void __launch_bounds__(256) gather_rows_elem(const T* __restrict__ X, const int32_t* __restrict__ idx,
                                                        long long K, int C, T* __restrict__ Xk) {
  const long long total = K * C;
  for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < total;
       t += (long long)gridDim.x * blockDim.x) {
    long long j = t / C;
    int c = (int)(t - j * C);
    Xk[t] = X[(long long)idx[j] * C + c];
  }
}

int32_t launch_gather_rows(const void* X, const int32_t* idx, int64_t K, int32_t C, int32_t elem_bytes, void* Xk,
                           hipStream_t s) {
  const long long row_bytes = (long long)C * elem_bytes;
  const bool vec = row_bytes % 16 == 0 && ((uintptr_t)X % 16 == 0) && ((uintptr_t)Xk % 16 == 0);
  if (vec) {
    const int ppr = (int)(row_bytes / 16);
    constexpr int U = 1;   // pieces per thread and pass: one, in many blocks (16 wavefronts per SIMD), ran ahead of 2 or 4 in flight
    const int64_t rows_per_launch = std::max<int64_t>(1, 0xFFFFFFFFll / ppr);   // piece numbers of a launch fit 32 bits
    for (int64_t j0 = 0; j0 < K; j0 += rows_per_launch) {
      const int64_t rows = std::min(rows_per_launch, K - j0);
      const uint32_t total = (uint32_t)(rows * ppr);
      long long blocks = ceil_div(total, 256LL * U);
      if (blocks > 256 * 64) blocks = 256 * 64;
      if (blocks < 1) blocks = 1;
      SBP_LAUNCH(SBP_PROF_GATHER, s, gather_rows_vec16<U>, dim3((unsigned)blocks), dim3(256), 0, s, (const uint4*)X, idx + j0,
                 total, FastDiv((uint32_t)ppr), (uint4*)Xk + j0 * ppr);
    }
  } else {
    const long long total = K * C;
    long long blocks = ceil_div(total, 256);
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (elem_bytes == 4)
      SBP_LAUNCH(SBP_PROF_GATHER, s, gather_rows_elem<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, s, (const uint32_t*)X,
                         idx, (long long)K, C, (uint32_t*)Xk);
    else
      SBP_LAUNCH(SBP_PROF_GATHER, s, gather_rows_elem<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, s, (const uint16_t*)X,
                         idx, (long long)K, C, (uint16_t*)Xk);
  }
  return check_launch("gather_rows");
}

// ---- several row gathers in one launch (the forward-side caches of all layers of a block) ----------------
static constexpr int kMaxGatherBatch = SBP_MAX_BATCH_LAYERS;
struct GatherItem {
  const uint4* X; const int32_t* idx; uint4* Xk;
  uint32_t total;            // 16-byte pieces of the item
  FastDiv ppr;               // pieces per row
  int blk_start, nblk;       // its blocks in the grid
};
struct GatherBatchArgs { int n; GatherItem it[kMaxGatherBatch]; };

__global__ void __launch_bounds__(256) gather_rows_batch_kernel(const GatherBatchArgs a) {
  int q = 0;
  for (int i = 1; i < a.n; ++i)
    if ((int)blockIdx.x >= a.it[i].blk_start) q = i;
  const GatherItem& g = a.it[q];
  const uint32_t stride = (uint32_t)g.nblk * 256u;
  const uint32_t ppr = g.ppr.d;
  for (uint32_t t = ((uint32_t)blockIdx.x - (uint32_t)g.blk_start) * 256u + threadIdx.x; t < g.total; t += stride) {
    uint32_t j, c;
    g.ppr.divmod(t, j, c);
    g.Xk[t] = g.X[(long long)g.idx[j] * ppr + c];
    if (stride > ~t) return;                                // the next step would wrap
  }
}

// ---- row-group layout [ceil(K / 8)][C][8] (bf16): the 8 kept rows of a group side by side for every channel ----
// A thread owns 8 rows x 2 channels: eight 4-byte loads along the rows (a wavefront reads 256 contiguous bytes of every
// row), one byte permute per output word, two 16-byte stores (32 contiguous bytes per thread, 2 KB per wavefront).
struct KmajorItem {
  const uint32_t* X; const int32_t* idx; uint32_t* Xk;
  uint32_t total;            // threads of the item: groups of 8 rows x pairs of channels
  FastDiv c2;                // pairs of channels per row
  int K;
  int blk_start, nblk;
};
struct KmajorBatchArgs { int n; KmajorItem it[kMaxGatherBatch]; };

// TO_ROWS = false: X_k(row groups) from X[idx[.]];  true: rows [K][C] back from row groups (idx unused)
template <bool TO_ROWS>
__global__ void __launch_bounds__(256) kmajor_batch_kernel(const KmajorBatchArgs a) {
  int qi = 0;
  for (int i = 1; i < a.n; ++i)
    if ((int)blockIdx.x >= a.it[i].blk_start) qi = i;
  const KmajorItem& g = a.it[qi];
  const uint32_t stride = (uint32_t)g.nblk * 256u;
  const uint32_t c2n = g.c2.d;
  for (uint32_t t = ((uint32_t)blockIdx.x - (uint32_t)g.blk_start) * 256u + threadIdx.x; t < g.total; t += stride) {
    uint32_t kg, c2;
    g.c2.divmod(t, kg, c2);
    uint32_t v[8];
    if (!TO_ROWS) {
      int row[8];           // (all eight row ids first, then all eight loads: nothing waits in between)
#pragma unroll
      for (int r = 0; r < 8; ++r) row[r] = g.idx[min((int)(8 * kg) + r, g.K - 1)];
#pragma unroll
      for (int r = 0; r < 8; ++r) v[r] = g.X[(long long)row[r] * c2n + c2];
#pragma unroll
      for (int r = 0; r < 8; ++r)
        if ((int)(8 * kg) + r >= g.K) v[r] = 0;
      uint4 lo, hi;     // the 8 rows of the even / odd channel of the pair
      lo.x = __builtin_amdgcn_perm(v[1], v[0], 0x05040100u); hi.x = __builtin_amdgcn_perm(v[1], v[0], 0x07060302u);
      lo.y = __builtin_amdgcn_perm(v[3], v[2], 0x05040100u); hi.y = __builtin_amdgcn_perm(v[3], v[2], 0x07060302u);
      lo.z = __builtin_amdgcn_perm(v[5], v[4], 0x05040100u); hi.z = __builtin_amdgcn_perm(v[5], v[4], 0x07060302u);
      lo.w = __builtin_amdgcn_perm(v[7], v[6], 0x05040100u); hi.w = __builtin_amdgcn_perm(v[7], v[6], 0x07060302u);
      uint4* dst = reinterpret_cast<uint4*>(g.Xk) + ((long long)kg * c2n + c2) * 2;
      dst[0] = lo;
      dst[1] = hi;
    } else {
      const uint4* src = reinterpret_cast<const uint4*>(g.X) + ((long long)kg * c2n + c2) * 2;
      const uint4 lo = src[0], hi = src[1];
      const uint32_t l[4] = {lo.x, lo.y, lo.z, lo.w}, h[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {     // word q: rows 2q, 2q + 1 of one channel
        v[2 * q] = __builtin_amdgcn_perm(h[q], l[q], 0x05040100u);
        v[2 * q + 1] = __builtin_amdgcn_perm(h[q], l[q], 0x07060302u);
      }
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int j = (int)(8 * kg) + r;
        if (j < g.K) g.Xk[(long long)j * c2n + c2] = v[r];
      }
    }
    if (stride > ~t) return;
  }
}

static int32_t launch_kmajor(bool to_rows, const sbp_gather_item* items, int32_t n, hipStream_t s) {
  KmajorBatchArgs a{};
  int blk = 0, m = 0;
  for (int i = 0; i < n; ++i) {
    if (items[i].K == 0) continue;
    const long long total = ceil_div(items[i].K, 8) * (long long)(items[i].C / 2);
    if (total >= 0xFFFFFFFFll || items[i].K > INT32_MAX) return fail(SBP_ERR_SHAPE, "tensor too large for the row-group layout");
    KmajorItem& g = a.it[m++];
    g.X = static_cast<const uint32_t*>(items[i].X); g.idx = items[i].idx; g.Xk = static_cast<uint32_t*>(items[i].X_k);
    g.total = (uint32_t)total;
    g.c2 = FastDiv((uint32_t)(items[i].C / 2));
    g.K = (int)items[i].K;
    g.blk_start = blk;
    g.nblk = (int)std::min<long long>(ceil_div(total, 256), 256 * 64);
    blk += g.nblk;
  }
  a.n = m;
  if (m == 0) return SBP_OK;
  if (to_rows) SBP_LAUNCH(SBP_PROF_GATHER, s, kmajor_batch_kernel<true>, dim3((unsigned)blk), dim3(256), 0, s, a);
  else SBP_LAUNCH(SBP_PROF_GATHER, s, kmajor_batch_kernel<false>, dim3((unsigned)blk), dim3(256), 0, s, a);
  return check_launch("kmajor_batch");
}

// rows [K][C] (bf16, C % 8 == 0, 16-byte aligned) back from the row-group layout: for the engines that read X_k by rows
int32_t launch_kmajor_to_rows(const void* Xt, int64_t K, int32_t C, void* Xrows, hipStream_t s) {
  sbp_gather_item it{};
  it.X = Xt; it.idx = nullptr; it.X_k = Xrows; it.M = K; it.K = K; it.C = C; it.layout = SBP_LAYOUT_KMAJOR;
  return launch_kmajor(true, &it, 1, s);
}

int32_t launch_gather_rows_batch(const sbp_gather_item* items, int32_t n, int32_t elem_bytes, hipStream_t s) {
  {  // items in the row-group layout share one launch of their own; the others go on below
    sbp_gather_item km[kMaxGatherBatch], rows[kMaxGatherBatch];
    int nk = 0, nr = 0;
    for (int i = 0; i < n; ++i) (items[i].layout == SBP_LAYOUT_KMAJOR ? km[nk++] : rows[nr++]) = items[i];
    if (nk > 0) {
      const int32_t st = launch_kmajor(false, km, nk, s);
      if (st != SBP_OK || nr == 0) return st;
      return launch_gather_rows_batch(rows, nr, elem_bytes, s);
    }
  }
  bool fused = n > 1 && n <= kMaxGatherBatch;
  for (int i = 0; i < n && fused; ++i) {
    const long long row_bytes = (long long)items[i].C * elem_bytes;
    fused = items[i].K > 0 && row_bytes % 16 == 0 && ((uintptr_t)items[i].X % 16 == 0) && ((uintptr_t)items[i].X_k % 16 == 0) &&
            items[i].K * (row_bytes / 16) < 0xFFFFFFFFll;
  }
  if (!fused) {
    for (int i = 0; i < n; ++i) {
      if (items[i].K == 0) continue;
      const int32_t st = launch_gather_rows(items[i].X, items[i].idx, items[i].K, items[i].C, elem_bytes, items[i].X_k, s);
      if (st != SBP_OK) return st;
    }
    return SBP_OK;
  }
  GatherBatchArgs a{};
  a.n = n;
  int blk = 0;
  for (int i = 0; i < n; ++i) {
    const uint32_t ppr = (uint32_t)((long long)items[i].C * elem_bytes / 16);
    GatherItem& g = a.it[i];
    g.X = static_cast<const uint4*>(items[i].X); g.idx = items[i].idx; g.Xk = static_cast<uint4*>(items[i].X_k);
    g.total = (uint32_t)(items[i].K * ppr);
    g.ppr = FastDiv(ppr);
    g.blk_start = blk;
    g.nblk = (int)std::min<long long>(ceil_div(g.total, 256), 256 * 64);
    blk += g.nblk;
  }
  SBP_LAUNCH(SBP_PROF_GATHER, s, gather_rows_batch_kernel, dim3((unsigned)blk), dim3(256), 0, s, a);
  return check_launch("gather_rows_batch");
}

// ------------------------------------------------------------------------------------------------
// Down-sampling layers (convolution with kernel p x p and stride p: the paper's case s >= k, where
// every output position owns its own patch of inputs and the layer behaves like a point-wise one).
// The forward-side cache holds, per kept output position, its p x p input patch as one row
// [p * p * C] in (dy, dx, c) order; the linear backward then runs on these rows, and the compact
// gradient rows are written back to the patches of the [B, H, W, C] input gradient in one pass that
// also writes the zeros of every other position.
// Unit = one element of `unit_t` (16 bytes when rows allow, else one value).
// ------------------------------------------------------------------------------------------------
struct PatchGeom {
  int H, W, Ho, Wo, p, seg;      // seg = units per pixel
};

template <typename U>
__global__ void __launch_bounds__(256) gather_patches_kernel(const U* __restrict__ X, const int32_t* __restrict__ idx,
                                                             long long K, PatchGeom g, U* __restrict__ Xk) {
  const int per_row = g.p * g.p * g.seg;
  const long long total = K * per_row;
  for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
    const long long j = t / per_row;
    const int rem = (int)(t - j * per_row);
    const int s = rem / g.seg, c = rem - s * g.seg;
    const int dy = s / g.p, dx = s - dy * g.p;
    const int f = idx[j];
    const int b = f / (g.Ho * g.Wo), r = f - b * (g.Ho * g.Wo);
    const int yo = r / g.Wo, xo = r - yo * g.Wo;
    const long long pix = ((long long)b * g.H + g.p * yo + dy) * g.W + g.p * xo + dx;
    Xk[t] = X[pix * g.seg + c];
  }
}

template <typename U>
__global__ void __launch_bounds__(256) scatter_patches_kernel(const U* __restrict__ dXp, const int32_t* __restrict__ idx,
                                                              const int32_t* __restrict__ inv, int K, long long npix,
                                                              PatchGeom g, U* __restrict__ dX) {
  const long long total = npix * g.seg;
  const int per_row = g.p * g.p * g.seg;
  U zero;
  __builtin_memset(&zero, 0, sizeof(U));
  for (long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
    const long long pix = t / g.seg;
    const int c = (int)(t - pix * g.seg);
    const int x = (int)(pix % g.W);
    const long long by = pix / g.W;
    const int y = (int)(by % g.H), b = (int)(by / g.H);
    const int f = (b * g.Ho + y / g.p) * g.Wo + x / g.p;
    const int j = inv[f];
    const bool kept = (unsigned)j < (unsigned)K && idx[j] == f;
    dX[t] = kept ? dXp[(long long)j * per_row + ((y % g.p) * g.p + x % g.p) * g.seg + c] : zero;
  }
}

// The same two kernels with 32-bit unit numbers and multiply-shift divisions, for tensors of fewer than 2^32 units
// (the plain versions above spend more time on their eight integer divisions per unit than on the memory accesses).
struct PatchGeomFast {
  FastDiv seg, W, H, p, per_row, Wo, HoWo;
  int Ho_;
};

template <typename U>
__global__ void __launch_bounds__(256) gather_patches_fast_kernel(const U* __restrict__ X, const int32_t* __restrict__ idx,
                                                                  uint32_t total, PatchGeomFast g, U* __restrict__ Xk) {
  const uint32_t stride = gridDim.x * 256u;
  for (uint32_t t = blockIdx.x * 256u + threadIdx.x; t < total; t += stride) {
    uint32_t j, rem, s, c, dy, dx, b, r, yo, xo;
    g.per_row.divmod(t, j, rem);
    g.seg.divmod(rem, s, c);
    g.p.divmod(s, dy, dx);
    g.HoWo.divmod((uint32_t)idx[j], b, r);
    g.Wo.divmod(r, yo, xo);
    const long long pix = ((long long)b * g.H.d + g.p.d * yo + dy) * g.W.d + g.p.d * xo + dx;
    Xk[t] = X[pix * g.seg.d + c];
    if (stride > ~t) return;
  }
}

// Three dependent loads stand behind every unit (inverse map, keep list, patch row): UNROLL units per thread, each
// kind of load issued for all of them before the next kind, keep enough of them in flight.
template <typename U, int UNROLL>
__global__ void __launch_bounds__(256) scatter_patches_fast_kernel(const U* __restrict__ dXp, const int32_t* __restrict__ idx,
                                                                   const int32_t* __restrict__ inv, int K, uint32_t total,
                                                                   PatchGeomFast g, U* __restrict__ dX) {
  const uint32_t stride = gridDim.x * 256u;
  U zero;
  __builtin_memset(&zero, 0, sizeof(U));
  for (uint32_t t0 = blockIdx.x * 256u + threadIdx.x; t0 < total; t0 += UNROLL * stride) {
    int f[UNROLL], j[UNROLL];
    uint32_t off[UNROLL];
    bool live[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const uint32_t t = t0 + u * stride;
      live[u] = t >= t0 && t < total;                     // t >= t0: no wrap-around
      uint32_t pix, c, by, x, b, y, yo, yi, xo, xi;
      g.seg.divmod(live[u] ? t : 0u, pix, c);
      g.W.divmod(pix, by, x);
      g.H.divmod(by, b, y);
      g.p.divmod(y, yo, yi);
      g.p.divmod(x, xo, xi);
      f[u] = (int)((b * (uint32_t)g.Ho_ + yo) * g.Wo.d + xo);
      off[u] = (yi * g.p.d + xi) * g.seg.d + c;
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) j[u] = inv[f[u]];
    int back[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      back[u] = (unsigned)j[u] < (unsigned)K ? idx[j[u]] : -1;   // (no load where nothing is kept: idx may be empty)
    }
    U v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const bool kept = back[u] == f[u];
      v[u] = kept ? dXp[(long long)j[u] * g.per_row.d + off[u]] : zero;
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (live[u]) dX[t0 + u * stride] = v[u];
    if (UNROLL * stride > ~t0) return;
  }
}

template <typename U>
static void launch_patches_t(bool scatter, const void* src, const int32_t* idx, const int32_t* inv, int64_t K, long long npix,
                             PatchGeom g, void* dst, hipStream_t s) {
  const long long total = scatter ? npix * g.seg : K * (long long)g.p * g.p * g.seg;
  const unsigned blocks = (unsigned)std::max<long long>(1, std::min<long long>(ceil_div(total, 256), 256 * 32));
  if (total < (1ll << 32) && !options().patch_wide) {   // (override "patch_wide": the 64-bit kernels on any size)
    PatchGeomFast f;
    f.seg = FastDiv((uint32_t)g.seg); f.W = FastDiv((uint32_t)g.W); f.H = FastDiv((uint32_t)g.H); f.p = FastDiv((uint32_t)g.p);
    f.per_row = FastDiv((uint32_t)(g.p * g.p * g.seg)); f.Wo = FastDiv((uint32_t)g.Wo); f.HoWo = FastDiv((uint32_t)(g.Ho * g.Wo));
    f.Ho_ = g.Ho;
    if (scatter)
      SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, (scatter_patches_fast_kernel<U, 4>), dim3(std::max(1u, blocks / 4)), dim3(256), 0, s, (const U*)src, idx, inv,
                 (int)K, (uint32_t)total, f, (U*)dst);
    else
      SBP_LAUNCH(SBP_PROF_GATHER, s, (gather_patches_fast_kernel<U>), dim3(blocks), dim3(256), 0, s, (const U*)src, idx,
                 (uint32_t)total, f, (U*)dst);
    return;
  }
  if (scatter)
    SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, (scatter_patches_kernel<U>), dim3(blocks), dim3(256), 0, s, (const U*)src, idx, inv, (int)K,
               npix, g, (U*)dst);
  else
    SBP_LAUNCH(SBP_PROF_GATHER, s, (gather_patches_kernel<U>), dim3(blocks), dim3(256), 0, s, (const U*)src, idx, (long long)K, g,
               (U*)dst);
}

int32_t launch_patches(bool scatter, const void* src, const int32_t* idx, const int32_t* inv, int32_t B, int32_t H, int32_t W,
                       int32_t C, int32_t p, int64_t K, int32_t elem_bytes, void* dst, hipStream_t s) {
  PatchGeom g{H, W, H / p, W / p, p, C};
  const long long npix = (long long)B * H * W;
  const long long pix_bytes = (long long)C * elem_bytes;
  if (pix_bytes % 16 == 0 && (uintptr_t)src % 16 == 0 && (uintptr_t)dst % 16 == 0) {
    g.seg = (int)(pix_bytes / 16);
    launch_patches_t<uint4>(scatter, src, idx, inv, K, npix, g, dst, s);
  } else if (elem_bytes == 4) {
    launch_patches_t<uint32_t>(scatter, src, idx, inv, K, npix, g, dst, s);
  } else {
    launch_patches_t<uint16_t>(scatter, src, idx, inv, K, npix, g, dst, s);
  }
  return check_launch(scatter ? "scatter_patches" : "gather_patches");
}

}  // namespace sbp
