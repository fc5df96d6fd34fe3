// Row-wise steps between the linear layers, on the kept rows only.  The paper's implementation (Alg.
// alg:sbp_impl) wraps "an arbitrary operation f": kept rows pass through f with gradient, dropped rows
// without, and with one keep-set shared by a stack of layers the split passes through the chain
// unchanged (eq:backward_fc2_sbp_same_drop_loc).  For a row-wise f that is the ordinary backward of f on
// the K kept rows, which therefore stay compact ([K, C]) from the output of one linear backward to the
// input of the next; only the last step of a branch scatters to [M, C] and zero-fills.
//   activation (exact GELU, z Phi(z)):  H_k = gelu(Z_k),  dZ_k = dH_k * (Phi(Z_k) + Z_k phi(Z_k))
//   LayerNorm backward per kept row:    dx = (g - mean(g) - xhat mean(g xhat)) rstd,  g = dU gamma,
//                                       dgamma = sum_k dU xhat,  dbeta = sum_k dU
// All of it is streaming work bound by HBM: 16-byte accesses, fp32 arithmetic, rows in registers.
#include <algorithm>

#include "sbp_internal.h"

namespace sbp {

static constexpr int PW_THREADS = 256;

__device__ __forceinline__ float pw_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float pw_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
typedef float pw_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 pw_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pw_pack(float lo, float hi) {   // round to nearest even (v_cvt_pk_bf16_f32)
  const pw_f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, pw_bf16x2));
}

// The exact GELU, z Phi(z), and its derivative Phi(z) + z phi(z).  fp32 tensors: the library's erff / expf.
// bf16 tensors: erfc(x) = (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x), x >= 0 (Abramowitz and Stegun 7.1.26,
// absolute error below 1.5e-7: three orders of magnitude under the rounding step of the output), whose
// exponential exp(-z^2 / 2) is the one the density needs: one v_exp_f32 and one v_rcp_f32 per value instead of
// two library calls, which had made these kernels ALU-bound.
template <typename T> struct Gelu {
  static __device__ __forceinline__ float value(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
  static __device__ __forceinline__ float grad(float z) {
    const float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752f));
    return cdf + z * 0.39894228040143268f * expf(-0.5f * z * z);
  }
};
template <> struct Gelu<uint16_t> {
  // Phi(z), and exp(-z^2 / 2) through e
  static __device__ __forceinline__ float cdf(float z, float& e) {
    const float x = fabsf(z) * 0.70710678118654752f;
    e = __builtin_amdgcn_exp2f(z * z * -0.72134752044448170f);            // exp(-z^2 / 2) = 2^(-z^2 log2(e) / 2)
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    const float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f), -0.284496736f), 0.254829592f);
    const float tail = 0.5f * poly * e;                                    // Phi(-|z|)
    return z >= 0.f ? 1.0f - tail : tail;
  }
  static __device__ __forceinline__ float value(float z) {
    float e;
    return z * cdf(z, e);
  }
  static __device__ __forceinline__ float grad(float z) {
    float e;
    const float c = cdf(z, e);
    return fmaf(z * 0.39894228040143268f, e, c);
  }
};

// 8 values per thread and access.  T = uint16_t (bf16) or float.
template <typename T> struct Vec8;
template <> struct Vec8<uint16_t> {
  typedef uint4 Raw;                                   // 8 values as they lie in memory
  static __device__ __forceinline__ Raw load_raw(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  static __device__ __forceinline__ Raw zero_raw() { return make_uint4(0, 0, 0, 0); }
  static __device__ __forceinline__ void unpack(const Raw& w, float (&v)[8]) {
    v[0] = pw_lo(w.x); v[1] = pw_hi(w.x); v[2] = pw_lo(w.y); v[3] = pw_hi(w.y);
    v[4] = pw_lo(w.z); v[5] = pw_hi(w.z); v[6] = pw_lo(w.w); v[7] = pw_hi(w.w);
  }
  static __device__ __forceinline__ void load(const uint16_t* p, float (&v)[8]) { unpack(load_raw(p), v); }
  static __device__ __forceinline__ void store(uint16_t* p, const float (&v)[8]) {
    uint4 w;
    w.x = pw_pack(v[0], v[1]); w.y = pw_pack(v[2], v[3]); w.z = pw_pack(v[4], v[5]); w.w = pw_pack(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = w;
  }
  static __device__ __forceinline__ float load1(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
  static __device__ __forceinline__ void store1(uint16_t* p, float v) { *p = (uint16_t)(pw_pack(v, 0.f) & 0xffffu); }
};
template <> struct Vec8<float> {
  struct Raw { float4 a, b; };
  static __device__ __forceinline__ Raw load_raw(const float* p) {
    return Raw{reinterpret_cast<const float4*>(p)[0], reinterpret_cast<const float4*>(p)[1]};
  }
  static __device__ __forceinline__ Raw zero_raw() { return Raw{make_float4(0.f, 0.f, 0.f, 0.f), make_float4(0.f, 0.f, 0.f, 0.f)}; }
  static __device__ __forceinline__ void unpack(const Raw& r, float (&v)[8]) {
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w; v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
  }
  static __device__ __forceinline__ void load(const float* p, float (&v)[8]) { unpack(load_raw(p), v); }
  static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
    reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
  }
  static __device__ __forceinline__ float load1(const float* p) { return *p; }
  static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
};

// ---- activation ------------------------------------------------------------------------------------
// out = gelu(Z) (BACKWARD = false) or dH * gelu'(Z) (BACKWARD = true) over n values; groups of 8, two in flight.
template <typename T, bool BACKWARD, bool VEC>
__global__ void __launch_bounds__(PW_THREADS) act_rows_kernel(const T* dH, const T* __restrict__ Z,
                                                               long long n, T* out) {   // out may be dH
  const long long stride = (long long)gridDim.x * blockDim.x;
  long long t = blockIdx.x * (long long)blockDim.x + threadIdx.x;
  if (VEC) {
    const long long groups = n / 8;
    for (; t + stride < groups; t += 2 * stride) {       // two groups in flight per thread
      float z[2][8], g[2][8], o[8];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        Vec8<T>::load(Z + 8 * (t + u * stride), z[u]);
        if (BACKWARD) Vec8<T>::load(dH + 8 * (t + u * stride), g[u]);
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = BACKWARD ? g[u][i] * Gelu<T>::grad(z[u][i]) : Gelu<T>::value(z[u][i]);
        Vec8<T>::store(out + 8 * (t + u * stride), o);
      }
    }
    for (; t < groups; t += stride) {
      float z[8], g[8], o[8];
      Vec8<T>::load(Z + 8 * t, z);
      if (BACKWARD) Vec8<T>::load(dH + 8 * t, g);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = BACKWARD ? g[i] * Gelu<T>::grad(z[i]) : Gelu<T>::value(z[i]);
      Vec8<T>::store(out + 8 * t, o);
    }
  } else {
    for (; t < n; t += stride) {
      const float z = Vec8<T>::load1(Z + t);
      Vec8<T>::store1(out + t, BACKWARD ? Vec8<T>::load1(dH + t) * Gelu<T>::grad(z) : Gelu<T>::value(z));
    }
  }
}

template <typename T>
static void launch_act_t(const T* dH, const T* Z, long long n, bool backward, T* out, hipStream_t s) {
  const bool vec = n % 8 == 0 && (uintptr_t)Z % 16 == 0 && (uintptr_t)out % 16 == 0 && (!backward || (uintptr_t)dH % 16 == 0);
  const long long work = vec ? n / 8 : n;
  const unsigned blocks = (unsigned)std::max<long long>(1, std::min<long long>(ceil_div(work, PW_THREADS), 256 * 64));
  if (vec) {
    if (backward) SBP_LAUNCH(SBP_PROF_OTHER, s, (act_rows_kernel<T, true, true>), dim3(blocks), dim3(PW_THREADS), 0, s, dH, Z, n, out);
    else SBP_LAUNCH(SBP_PROF_OTHER, s, (act_rows_kernel<T, false, true>), dim3(blocks), dim3(PW_THREADS), 0, s, dH, Z, n, out);
  } else {
    if (backward) SBP_LAUNCH(SBP_PROF_OTHER, s, (act_rows_kernel<T, true, false>), dim3(blocks), dim3(PW_THREADS), 0, s, dH, Z, n, out);
    else SBP_LAUNCH(SBP_PROF_OTHER, s, (act_rows_kernel<T, false, false>), dim3(blocks), dim3(PW_THREADS), 0, s, dH, Z, n, out);
  }
}

int32_t launch_act_rows(const void* dH, const void* Z, int64_t n, int32_t dtype, int32_t, bool backward, void* out,
                        hipStream_t s) {
  if (n == 0) return SBP_OK;
  if (dtype == SBP_F32) launch_act_t<float>((const float*)dH, (const float*)Z, n, backward, (float*)out, s);
  else launch_act_t<uint16_t>((const uint16_t*)dH, (const uint16_t*)Z, n, backward, (uint16_t*)out, s);
  return check_launch(backward ? "act_backward_rows" : "act_forward_rows");
}

// ---- LayerNorm backward ----------------------------------------------------------------------------
// Sum over the 64 lanes, every lane gets it, fixed order.  Inside a row of 16 lanes the partners come through the
// data-parallel-primitive lane selects of the vector ALU (neighbour, pair, mirrored half row, mirrored row: four adds,
// no LDS crossbar - a 64-lane butterfly of cross-lane reads through LDS took six dependent round trips of about 100
// cycles each, four times per LayerNorm row); the four row sums are then read as scalars and added in row order.
template <int CTRL>
__device__ __forceinline__ float dpp_lane(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_lane<0xB1>(v);      // quad_perm [1, 0, 3, 2]
  v += dpp_lane<0x4E>(v);      // quad_perm [2, 3, 0, 1]
  v += dpp_lane<0x141>(v);     // row_half_mirror
  v += dpp_lane<0x140>(v);     // row_mirror
  const int iv = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
  return ((r0 + r1) + r2) + r3;
}

// Fast path: C a multiple of 8, C <= 64 * 8 * NV.  A wavefront owns a row: lane l holds the 8-value groups
// l, l + 64, ... of it in registers.  A block of 4 wavefronts walks the rows [r0, r1) of its slice and keeps
// per-lane sums of dU * xhat and dU for its columns; the four wavefronts' sums are added in a fixed order
// through LDS and written as the block's partial.
template <typename T, int NV>
__global__ void __launch_bounds__(PW_THREADS) ln_bwd_rows_kernel(const T* __restrict__ dU, const T* __restrict__ Xk,
                                                                  const float* __restrict__ gamma, float eps,
                                                                  const int32_t* __restrict__ idx_out, int K, int C,
                                                                  int rows_per_block, T* __restrict__ dX,
                                                                  float* __restrict__ partial, int row_blocks,
                                                                  const int32_t* __restrict__ inv, int M) {
  extern __shared__ float red[];                       // [4][C]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ngroups = C / 8;
  if ((int)blockIdx.x >= row_blocks) {
    // The blocks behind the row blocks write +0 to the rows of dX [M, C] that are not kept (scattered output
    // only): a wavefront looks 64 rows up at once (row m is kept iff idx[inv[m]] == m) and all lanes together
    // write each dropped row.
    constexpr int PPG = 8 * sizeof(T) / 16;            // 16-byte pieces per group of 8 values
    const int nz = gridDim.x - row_blocks, gw = ((int)blockIdx.x - row_blocks) * 4 + wave;
    uint4* out = reinterpret_cast<uint4*>(dX);
    for (int base = gw * 64; base < M; base += nz * 4 * 64) {
      const int m = base + lane;
      bool dropped = false;
      if (m < M) {
        const int j = inv[m];
        dropped = !((unsigned)j < (unsigned)K && idx_out[j] == m);
      }
      unsigned long long mask = __ballot(dropped);
      while (mask) {
        const int b = __ffsll((long long)mask) - 1;
        mask &= mask - 1;
        uint4* row = out + (long long)(base + b) * (ngroups * PPG);
        for (int q = lane; q < ngroups * PPG; q += 64) row[q] = make_uint4(0, 0, 0, 0);
      }
    }
    return;
  }
  const int r0 = blockIdx.x * rows_per_block, r1 = min(K, r0 + rows_per_block);
  float gam[NV][8], sg[NV][8], sb[NV][8];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int grp = lane + 64 * v;
#pragma unroll
    for (int i = 0; i < 8; ++i) { gam[v][i] = 0.f; sg[v][i] = 0.f; sb[v][i] = 0.f; }
    if (grp < ngroups) {
      const float4 ga = reinterpret_cast<const float4*>(gamma + 8 * grp)[0], gb = reinterpret_cast<const float4*>(gamma + 8 * grp)[1];
      gam[v][0] = ga.x; gam[v][1] = ga.y; gam[v][2] = ga.z; gam[v][3] = ga.w;
      gam[v][4] = gb.x; gam[v][5] = gb.y; gam[v][6] = gb.z; gam[v][7] = gb.w;
    }
  }
  const float invC = 1.0f / (float)C;
  // U rows of the wavefront side by side: their loads go out together and their reduction chains interleave
  constexpr int U = NV <= 2 ? 2 : 1;
  // ... and the rows of the next round are requested before this round's arithmetic starts
  typename Vec8<T>::Raw xr[U][NV], dr[U][NV];
  auto request = [&](int jb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = jb + 4 * u;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int grp = lane + 64 * v;
        if (grp < ngroups && j < r1) {
          xr[u][v] = Vec8<T>::load_raw(Xk + (long long)j * C + 8 * grp);
          dr[u][v] = Vec8<T>::load_raw(dU + (long long)j * C + 8 * grp);
        } else {
          xr[u][v] = Vec8<T>::zero_raw();
          dr[u][v] = Vec8<T>::zero_raw();
        }
      }
    }
  };
  request(r0 + wave);
  for (int jb = r0 + wave; jb < r1; jb += 4 * U) {
    float x[U][NV][8], du[U][NV][8];
    float s1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      s1[u] = 0.f;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        Vec8<T>::unpack(xr[u][v], x[u][v]);
        Vec8<T>::unpack(dr[u][v], du[u][v]);
      }
    }
    if (jb + 4 * U < r1) request(jb + 4 * U);
    float mean[U], rstd[U], m1[U], m2[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int i = 0; i < 8; ++i) s1[u] += x[u][v][i];
      mean[u] = wave_sum(s1[u]) * invC;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float s2 = 0.f;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const bool ok = lane + 64 * v < ngroups;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float d = ok ? x[u][v][i] - mean[u] : 0.f;
          x[u][v][i] = d;
          s2 += d * d;
        }
      }
      rstd[u] = rsqrtf(wave_sum(s2) * invC + eps);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float a1 = 0.f, a2 = 0.f;
#pragma unroll
      for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float xh = x[u][v][i] * rstd[u];
          const float g = du[u][v][i] * gam[v][i];
          x[u][v][i] = xh;
          a1 += g;
          a2 += g * xh;
          sg[v][i] += du[u][v][i] * xh;
          sb[v][i] += du[u][v][i];
        }
      m1[u] = wave_sum(a1) * invC;
      m2[u] = wave_sum(a2) * invC;
    }
    if (dX) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = jb + 4 * u;
        if (j < r1) {
          const long long orow = idx_out ? (long long)idx_out[j] : (long long)j;
#pragma unroll
          for (int v = 0; v < NV; ++v) {
            const int grp = lane + 64 * v;
            if (grp < ngroups) {
              float o[8];
#pragma unroll
              for (int i = 0; i < 8; ++i) o[i] = (du[u][v][i] * gam[v][i] - m1[u] - x[u][v][i] * m2[u]) * rstd[u];
              Vec8<T>::store(dX + orow * C + 8 * grp, o);
            }
          }
        }
      }
    }
  }
  if (!partial) return;
  // the block's partial sums: wavefronts added in the order 0, 1, 2, 3; first dgamma's, then dbeta's
#pragma unroll
  for (int which = 0; which < 2; ++which) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int grp = lane + 64 * v;
      if (grp < ngroups) {
#pragma unroll
        for (int i = 0; i < 8; ++i) red[wave * C + 8 * grp + i] = which == 0 ? sg[v][i] : sb[v][i];
      }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < C; c += PW_THREADS)
      partial[((long long)blockIdx.x * 2 + which) * C + c] = ((red[c] + red[C + c]) + red[2 * C + c]) + red[3 * C + c];
    __syncthreads();
  }
}

// Plain path, any C: one wavefront per row, the row read from memory in every pass; mean and rstd go to
// stats[K][2] for the column kernel.
template <typename T>
__global__ void __launch_bounds__(64) ln_bwd_plain_rows_kernel(const T* __restrict__ dU, const T* __restrict__ Xk,
                                                                const float* __restrict__ gamma, float eps,
                                                                const int32_t* __restrict__ idx_out, int K, int C,
                                                                T* __restrict__ dX, float* __restrict__ stats) {
  const int lane = threadIdx.x;
  for (int j = blockIdx.x; j < K; j += gridDim.x) {
    const T* x = Xk + (long long)j * C;
    const T* du = dU + (long long)j * C;
    float s = 0.f;
    for (int c = lane; c < C; c += 64) s += Vec8<T>::load1(x + c);
    const float mean = wave_sum(s) / (float)C;
    s = 0.f;
    for (int c = lane; c < C; c += 64) { const float d = Vec8<T>::load1(x + c) - mean; s += d * d; }
    const float rstd = rsqrtf(wave_sum(s) / (float)C + eps);
    float m1 = 0.f, m2 = 0.f;
    for (int c = lane; c < C; c += 64) {
      const float g = Vec8<T>::load1(du + c) * gamma[c];
      m1 += g;
      m2 += g * (Vec8<T>::load1(x + c) - mean) * rstd;
    }
    m1 = wave_sum(m1) / (float)C;
    m2 = wave_sum(m2) / (float)C;
    if (lane == 0) { stats[2 * j] = mean; stats[2 * j + 1] = rstd; }
    if (dX) {
      T* o = dX + (idx_out ? (long long)idx_out[j] : (long long)j) * C;
      for (int c = lane; c < C; c += 64) {
        const float xh = (Vec8<T>::load1(x + c) - mean) * rstd;
        Vec8<T>::store1(o + c, (Vec8<T>::load1(du + c) * gamma[c] - m1 - xh * m2) * rstd);
      }
    }
  }
}

// plain path: partial[slice][0/1][c] over the rows of a slice, a thread per column
template <typename T>
__global__ void __launch_bounds__(PW_THREADS) ln_bwd_plain_cols_kernel(const T* __restrict__ dU, const T* __restrict__ Xk,
                                                                        const float* __restrict__ stats, int K, int C,
                                                                        int rows_per_block, float* __restrict__ partial) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  const int r0 = blockIdx.y * rows_per_block, r1 = min(K, r0 + rows_per_block);
  float sg = 0.f, sb = 0.f;
  for (int j = r0; j < r1; ++j) {
    const float du = Vec8<T>::load1(dU + (long long)j * C + c);
    sg += du * (Vec8<T>::load1(Xk + (long long)j * C + c) - stats[2 * j]) * stats[2 * j + 1];
    sb += du;
  }
  partial[((long long)blockIdx.y * 2 + 0) * C + c] = sg;
  partial[((long long)blockIdx.y * 2 + 1) * C + c] = sb;
}

// out[o] = sum over the blocks b of partial[b * n_out + o] (o < split goes to out0[o], the rest to out1[o - split]).
// 32 lanes per output: lane q adds the partials q, q + 32, ... in order (eight loads in flight), then the 32 sums are
// added in a fixed order (inside 16 lanes by lane selects of the vector ALU, then the two halves).  Few lanes per
// output left most CUs without work: 768 outputs x 8 lanes were 24 workgroups walking 100 dependent loads each.
__global__ void __launch_bounds__(PW_THREADS) partials_reduce_kernel(const float* __restrict__ partial, int nblocks, int n_out,
                                                                      int split, float* __restrict__ out0, float* __restrict__ out1,
                                                                      int accumulate) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int o = t >> 5, q = t & 31;
  const bool live = o < n_out;
  float a = 0.f;
  if (live) {
    for (int b0 = q; b0 < nblocks; b0 += 256) {
      float p[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) p[u] = b0 + 32 * u < nblocks ? partial[(long long)(b0 + 32 * u) * n_out + o] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) a += p[u];
    }
  }
  a += dpp_lane<0xB1>(a);
  a += dpp_lane<0x4E>(a);
  a += dpp_lane<0x141>(a);
  a += dpp_lane<0x140>(a);
  a += __shfl_xor(a, 16, 64);
  float* out = o < split ? out0 : out1;
  const int c = o < split ? o : o - split;
  if (live && q == 0 && out) out[c] = (accumulate ? out[c] : 0.f) + a;
}

__global__ void __launch_bounds__(PW_THREADS) ln_fill_zero_kernel(float* __restrict__ p, int n) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) p[t] = 0.f;
}

static constexpr int kLnMaxBlocks = 512;
static constexpr int kLnMaxNV = 8;                       // fast path up to C = 64 * 8 * 8 = 4096

LnPlan plan_layernorm(int64_t M, int64_t K, int32_t C, int32_t, uint32_t flags) {
  LnPlan p{};
  p.fast = C % 8 == 0 && C <= 64 * 8 * kLnMaxNV;
  // a block walks at least 16 rows (four per wavefront); at most kLnMaxBlocks partial sums
  p.nblocks = (int)std::max<int64_t>(1, std::min<int64_t>(kLnMaxBlocks, ceil_div(K, 16)));
  size_t off = 0;
  p.off_partial = off;
  off += align_up((size_t)p.nblocks * 2 * C * sizeof(float), 256);
  p.off_stats = off;
  if (!p.fast) off += align_up((size_t)std::max<int64_t>(K, 1) * 2 * sizeof(float), 256);
  p.off_inv = off;
  if (!(flags & SBP_FLAG_DX_COMPACT)) off += align_up((size_t)M * sizeof(int32_t), 256);
  p.bytes = off;
  return p;
}

template <typename T, int NV>
static void launch_ln_fast(const LnPlan& p, const T* dU, const T* Xk, const float* gamma, float eps,
                           const int32_t* idx_out, int K, int C, int rpb, T* dX, float* partial, const int32_t* inv, int M,
                           hipStream_t s) {
  const size_t lds = (size_t)4 * C * sizeof(float);   // at most 64 KB (C <= 4096)
  // scattered output: zero-fill blocks ride in the same launch
  const int nz = (dX && idx_out && inv) ? (int)std::min<int64_t>(128, std::max<int64_t>(8, ceil_div(M, 256))) : 0;
  SBP_LAUNCH(SBP_PROF_OTHER, s, (ln_bwd_rows_kernel<T, NV>), dim3(p.nblocks + nz), dim3(PW_THREADS), lds, s, dU, Xk, gamma, eps,
             idx_out, K, C, rpb, dX, partial, p.nblocks, inv, M);
}

// returns true if the launch also zero-filled the dropped rows of a scattered dX
template <typename T>
static bool launch_ln_t(const LnPlan& p, const T* dU, const T* Xk, const float* gamma, float eps, const int32_t* idx_out,
                        int K, int C, T* dX, float* partial, float* stats, const int32_t* inv, int M, hipStream_t s) {
  const int rpb = (int)ceil_div(K, p.nblocks);
  const bool aligned = (uintptr_t)dU % 16 == 0 && (uintptr_t)Xk % 16 == 0 && (uintptr_t)dX % 16 == 0 && (uintptr_t)gamma % 16 == 0;
  if (p.fast && aligned) {
    const int nv = (int)ceil_div(C / 8, 64);
    switch (nv) {
      case 1: launch_ln_fast<T, 1>(p, dU, Xk, gamma, eps, idx_out, K, C, rpb, dX, partial, inv, M, s); break;
      case 2: launch_ln_fast<T, 2>(p, dU, Xk, gamma, eps, idx_out, K, C, rpb, dX, partial, inv, M, s); break;
      case 3: case 4: launch_ln_fast<T, 4>(p, dU, Xk, gamma, eps, idx_out, K, C, rpb, dX, partial, inv, M, s); break;
      default: launch_ln_fast<T, 8>(p, dU, Xk, gamma, eps, idx_out, K, C, rpb, dX, partial, inv, M, s); break;
    }
    return dX && idx_out && inv;
  } else {
    const unsigned rows_grid = (unsigned)std::min<int64_t>(K, 8192);
    SBP_LAUNCH(SBP_PROF_OTHER, s, (ln_bwd_plain_rows_kernel<T>), dim3(rows_grid), dim3(64), 0, s, dU, Xk, gamma, eps, idx_out, K,
               C, dX, stats);
    if (partial)
      SBP_LAUNCH(SBP_PROF_OTHER, s, (ln_bwd_plain_cols_kernel<T>), dim3((unsigned)ceil_div(C, PW_THREADS), p.nblocks),
                 dim3(PW_THREADS), 0, s, dU, Xk, stats, K, C, rpb, partial);
  }
  return false;
}

int32_t launch_backward_layernorm(const LnPlan& p, const void* dU, const void* Xk, const float* gamma, float eps,
                                  const int32_t* idx, const int32_t* inv_in, int64_t M, int64_t K, int32_t C,
                                  int32_t dtype, float* dgamma, float* dbeta, void* dX, void* ws, uint32_t flags,
                                  hipStream_t s) {
  const int eb = dtype == SBP_F32 ? 4 : 2;
  const bool dx_compact = flags & SBP_FLAG_DX_COMPACT;
  const int accumulate = (flags & SBP_FLAG_ACCUMULATE_DW) ? 1 : 0;
  float* partial = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_partial);
  float* stats = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_stats);
  int32_t* inv_ws = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + p.off_inv);
  const bool want_params = dgamma || dbeta;

  // the inverse map for the zero fill of a scattered dX (built here unless the caller brought the sampler's)
  const int32_t* inv = inv_in;
  if (dX && !dx_compact && !inv) {
    launch_build_inverse(idx, K, inv_ws, s);
    inv = inv_ws;
  }
  bool zero_filled = false;
  if (K == 0) {   // nothing kept: gradients are zero
    if (!accumulate && want_params) {
      if (dgamma) SBP_LAUNCH(SBP_PROF_OTHER, s, ln_fill_zero_kernel, dim3((unsigned)ceil_div(C, PW_THREADS)), dim3(PW_THREADS), 0, s, dgamma, C);
      if (dbeta) SBP_LAUNCH(SBP_PROF_OTHER, s, ln_fill_zero_kernel, dim3((unsigned)ceil_div(C, PW_THREADS)), dim3(PW_THREADS), 0, s, dbeta, C);
    }
  } else {
    const int32_t* idx_out = dx_compact ? nullptr : idx;
    if (dtype == SBP_F32)
      zero_filled = launch_ln_t<float>(p, (const float*)dU, (const float*)Xk, gamma, eps, idx_out, (int)K, C, (float*)dX,
                                       want_params ? partial : nullptr, stats, inv, (int)M, s);
    else
      zero_filled = launch_ln_t<uint16_t>(p, (const uint16_t*)dU, (const uint16_t*)Xk, gamma, eps, idx_out, (int)K, C,
                                          (uint16_t*)dX, want_params ? partial : nullptr, stats, inv, (int)M, s);
    if (want_params)
      SBP_LAUNCH(SBP_PROF_REDUCE, s, partials_reduce_kernel, dim3((unsigned)ceil_div(32 * 2 * (int64_t)C, PW_THREADS)), dim3(PW_THREADS), 0, s,
                 partial, p.nblocks, 2 * C, C, dgamma, dbeta, accumulate);
  }
  if (dX && !dx_compact && !zero_filled) launch_zero_dropped_rows(idx, inv, K, M, (int64_t)C * eb, dX, s);
  return check_launch("backward_layernorm");
}

// ---- per-channel layer scale U = gamma * Y on the kept rows ---------------------------------------------
// dY_k = dU_k * gamma, dgamma = sum_j dU_k[j] * Y_k[j].  A thread owns VEC (8 or 1) adjacent channels; the G threads
// that cover a row form a row lane, a block has RL row lanes (G * RL <= 256 threads) that walk the rows of the block's
// slab in turn, four rows in flight each; the lanes' sums are added through LDS in lane order, the block writes one
// partial of dgamma, a second launch adds the partials in block order (deterministic).
static constexpr int kLsMaxBlocks = 1024;

template <typename T, int VEC>
__global__ void __launch_bounds__(PW_THREADS) layerscale_bwd_kernel(const T* __restrict__ dU, const T* __restrict__ Y,
                                                                    const float* __restrict__ gamma, int K, int C,
                                                                    int rows_per_block, int G, int RL, T* __restrict__ dY,
                                                                    float* __restrict__ partial) {
  extern __shared__ float ls_red[];                              // [RL][G * VEC] (RL > 1 only)
  const int rr = threadIdx.x / G, gl = threadIdx.x - rr * G;
  const int c0 = (blockIdx.y * G + gl) * VEC;                   // first channel of this thread
  const bool live = c0 < C;
  const int r0 = blockIdx.x * rows_per_block, r1 = min(K, r0 + rows_per_block);
  float gam[VEC], acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { gam[e] = live ? gamma[c0 + e] : 0.f; acc[e] = 0.f; }
  if (live)
    for (int r = r0 + 4 * rr; r < r1; r += 4 * RL) {
      float u[4][VEC], y[4][VEC];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const long long o = (long long)min(r + q, r1 - 1) * C + c0;
        if (VEC == 8) { Vec8<T>::load(dU + o, reinterpret_cast<float(&)[8]>(u[q])); Vec8<T>::load(Y + o, reinterpret_cast<float(&)[8]>(y[q])); }
        else { u[q][0] = Vec8<T>::load1(dU + o); y[q][0] = Vec8<T>::load1(Y + o); }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (r + q >= r1) break;
        float o8[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) { acc[e] = fmaf(u[q][e], y[q][e], acc[e]); o8[e] = u[q][e] * gam[e]; }
        if (dY) {
          const long long o = (long long)(r + q) * C + c0;
          if (VEC == 8) Vec8<T>::store(dY + o, reinterpret_cast<float(&)[8]>(o8));
          else Vec8<T>::store1(dY + o, o8[0]);
        }
      }
    }
  if (!partial) return;
  if (RL > 1) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) ls_red[(rr * G + gl) * VEC + e] = acc[e];
    __syncthreads();
    if (rr == 0) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        float a = acc[e];
        for (int l = 1; l < RL; ++l) a += ls_red[(l * G + gl) * VEC + e];
        acc[e] = a;
      }
    }
  }
  if (rr == 0 && live) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) partial[(long long)blockIdx.x * C + c0 + e] = acc[e];
  }
}

int ls_blocks(int64_t K) { return (int)std::max<int64_t>(1, std::min<int64_t>(kLsMaxBlocks, ceil_div(K, 8))); }

int32_t launch_backward_layerscale(const void* dU, const void* Y, const float* gamma, int64_t K, int32_t C, int32_t dtype,
                                   float* dgamma, void* dY, float* partial, uint32_t flags, hipStream_t s) {
  const int accumulate = (flags & SBP_FLAG_ACCUMULATE_DW) ? 1 : 0;
  if (K == 0) {
    if (dgamma)   // no partials: writes zeros (or leaves dgamma as it is when accumulating)
      SBP_LAUNCH(SBP_PROF_REDUCE, s, partials_reduce_kernel, dim3((unsigned)ceil_div(32 * (int64_t)C, PW_THREADS)), dim3(PW_THREADS), 0, s,
                 partial, 0, C, C, dgamma, (float*)nullptr, accumulate);
    return check_launch("backward_layerscale (K = 0)");
  }
  const int eb = dtype == SBP_F32 ? 4 : 2;
  const bool vec = C % 8 == 0 && (uintptr_t)dU % 16 == 0 && (uintptr_t)Y % 16 == 0 && (uintptr_t)dY % 16 == 0 && ((size_t)C * eb) % 16 == 0;
  const int groups = vec ? C / 8 : C;
  const int G = std::min(groups, PW_THREADS);                    // threads along a row
  const int RL = std::max(1, PW_THREADS / G);                    // row lanes of a block
  const int nblocks = ls_blocks(K), rpb = (int)ceil_div(K, nblocks);
  const dim3 grid((unsigned)nblocks, (unsigned)ceil_div(groups, G));
  const size_t lds = RL > 1 ? (size_t)RL * G * (vec ? 8 : 1) * sizeof(float) : 0;
  float* part = dgamma ? partial : nullptr;
#define SBP_LS(T, V) SBP_LAUNCH(SBP_PROF_OTHER, s, (layerscale_bwd_kernel<T, V>), grid, dim3(G * RL), lds, s, (const T*)dU, (const T*)Y, gamma, \
                                (int)K, C, rpb, G, RL, (T*)dY, part)
  if (dtype == SBP_F32) { if (vec) SBP_LS(float, 8); else SBP_LS(float, 1); }
  else { if (vec) SBP_LS(uint16_t, 8); else SBP_LS(uint16_t, 1); }
#undef SBP_LS
  if (dgamma)
    SBP_LAUNCH(SBP_PROF_REDUCE, s, partials_reduce_kernel, dim3((unsigned)ceil_div(32 * (int64_t)C, PW_THREADS)), dim3(PW_THREADS), 0, s,
               partial, nblocks, C, C, dgamma, (float*)nullptr, accumulate);
  return check_launch("backward_layerscale");
}

}  // namespace sbp
