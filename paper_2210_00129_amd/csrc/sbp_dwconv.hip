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
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  const int n = (ntap + 1) * C;
  if (e >= n) return;
  float a = 0.f;
  for (int s = 0; s < nslices; ++s) a += part[(long long)s * n + e];
  if (e < ntap * C) { if (dWd) dWd[e] = a; }
  else if (db) db[e - ntap * C] = a;
}

DwPlan plan_dwconv(int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks, int64_t K, int32_t dtype) {
  DwPlan p{};
  (void)dtype;
  p.tiles_y = p.tiles_x = 0;
  p.nparts = (int)std::max<int64_t>(1, std::min<int64_t>(64, ceil_div(K, 64)));
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
    SBP_LAUNCH(SBP_PROF_DWCONV_DW, s, dw_reduce_kernel, dim3((unsigned)ceil_div(n, DW_THREADS)), dim3(DW_THREADS), 0, s, part,
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
  if (!inv && dX) {      // build the inverse map from idx
    SBP_LAUNCH(SBP_PROF_OTHER, s, dw_fill_kernel, dim3((unsigned)std::min<long long>(ceil_div(npos, DW_THREADS), 4096)),
                       dim3(DW_THREADS), 0, s, inv_ws, npos, -1);
    if (K > 0)
      SBP_LAUNCH(SBP_PROF_OTHER, s, dw_mark_kernel, dim3((unsigned)ceil_div(K, DW_THREADS)), dim3(DW_THREADS), 0, s, idx, (int)K,
                         inv_ws);
    inv = inv_ws;
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
