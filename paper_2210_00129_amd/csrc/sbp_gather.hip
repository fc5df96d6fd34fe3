// Row gather X_k[j,:] = X[idx[j],:]: the forward-side cache of SBP (the paper's method keeps
// only a subset of each layer input for the backward pass).  Pure data movement, bound by
// HBM: every thread moves 16-byte pieces, several in flight, rows laid out so that a
// wavefront reads and writes whole contiguous row segments.
#include "sbp_internal.h"

namespace sbp {

// rows whose byte length is a multiple of 16: 16-byte pieces, UNROLL in flight per thread
template <int UNROLL>
__global__ void __launch_bounds__(256) gather_rows_vec16(const uint4* __restrict__ X, const int32_t* __restrict__ idx,
                                                         long long K, int pieces_per_row, uint4* __restrict__ Xk) {
  const long long total = K * pieces_per_row;
  const long long stride = (long long)gridDim.x * blockDim.x;
  long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x;
  for (; t + (UNROLL - 1) * stride < total; t += UNROLL * stride) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      long long e = t + u * stride;
      long long j = e / pieces_per_row;
      int c = (int)(e - j * pieces_per_row);
      v[u] = X[(long long)idx[j] * pieces_per_row + c];
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) Xk[t + u * stride] = v[u];
  }
  for (; t < total; t += stride) {
    long long j = t / pieces_per_row;
    int c = (int)(t - j * pieces_per_row);
    Xk[t] = X[(long long)idx[j] * pieces_per_row + c];
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
    const long long total = K * ppr;
    constexpr int U = 4;
    long long blocks = ceil_div(total, 256LL * U);
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    SBP_LAUNCH(SBP_PROF_GATHER, s, gather_rows_vec16<U>, dim3((unsigned)blocks), dim3(256), 0, s, (const uint4*)X, idx,
                       (long long)K, ppr, (uint4*)Xk);
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

}  // namespace sbp
