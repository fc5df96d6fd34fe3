// SBP backward of a linear / pointwise-conv layer on the kept rows only
// (paper, section "Calculation of Linear Layers", eq:backward_fc_sbp with the dropped terms removed):
//   dW[o,i] = sum_j dY[idx[j],o] X_k[j,i]      db[o] = sum_j dY[idx[j],o]
//   dX[idx[j],:] = dY[idx[j],:] W              every other row of dX = +0
// W is stored [Cout, Cin].
//
// bf16 path: both contractions run on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate).  The kept rows of dY are gathered by the tile loaders themselves, so dY_k is never
// materialised.  Operands whose contraction index is the slow axis in memory (dY and X_k for dW, W for
// dX) are transposed in registers on their way into LDS, so that every MFMA operand is one 16-byte LDS
// read.  dW is split along the kept rows into partial sums that a second kernel adds in a fixed order
// (deterministic, no floating-point atomics).
// fp32 and odd shapes take plain kernels.
#include "sbp_internal.h"

namespace sbp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

static constexpr int BK = 64;          // contraction elements per LDS stage
static constexpr int NTHREADS = 256;   // 4 wavefronts, arranged 2 x 2 over the block tile

// ------------------------------------------------------------------------------------------------
// LDS tile layout.  A tile holds ROWS rows of BK bf16 (128 bytes, eight 16-byte chunks).  Row m is
// stored at physical row prow(m) (bits 0 and 3 exchanged) and its chunk c at slot c ^ (m & 7).  With
// this, the 16-byte reads of an MFMA operand (32 consecutive rows, one chunk), the writes of the
// row-major loader (eight chunks of one row per 8 lanes) and the writes of the transposing loader
// (rows 8 apart across lane groups) all spread over the 64 banks.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int prow(int m) { return (m & ~9) | ((m & 1) << 3) | ((m >> 3) & 1); }
__device__ __forceinline__ int lds_off(int m, int c) { return prow(m) * 128 + ((c ^ (m & 7)) << 4); }

__device__ __forceinline__ uint32_t bf16_round(float f) {   // round-to-nearest-even, NaN kept quiet
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
// 16-bit halves `hi ? upper : lower` of two words, first word's half in the low 16 bits
__device__ __forceinline__ uint32_t pack_halves(uint32_t first, uint32_t second, int hi) {
  return hi ? ((first >> 16) | (second & 0xffff0000u)) : ((first & 0xffffu) | (second << 16));
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ------------------------------------------------------------------------------------------------
// Loader for an operand stored [rows][k] with k contiguous (dY as the left operand of dX).
// Rows may be gathered through idx.  Each thread owns chunk (t & 7) of physical rows (t>>3) + 32 i.
// ------------------------------------------------------------------------------------------------
template <int ROWS>
struct RowMajorLoader {
  static constexpr int NI = ROWS / 32;
  const uint16_t* ptr[NI];
  uint4 reg[NI];
  int soff[NI];
  int c;
  int kdim;

  __device__ __forceinline__ void init(const uint16_t* src, const int32_t* idx, long long ld, int row0, int nrows,
                                       int kdim_, int t) {
    c = t & 7;
    kdim = kdim_;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = (t >> 3) + 32 * i;        // physical row
      const int m = prow(q);                  // logical row (prow is its own inverse)
      const int r = row0 + m;
      soff[i] = q * 128 + ((c ^ (m & 7)) << 4);
      if (r < nrows) {
        const long long g = idx ? (long long)idx[r] : (long long)r;
        ptr[i] = src + g * ld + c * 8;
      } else {
        ptr[i] = nullptr;
      }
    }
  }
  __device__ __forceinline__ void load(int kt) {
    const int k = kt * BK + c * 8;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      if (ptr[i] && k < kdim) reg[i] = *reinterpret_cast<const uint4*>(ptr[i] + (long long)kt * BK);
      else reg[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(char* buf) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) *reinterpret_cast<uint4*>(buf + soff[i]) = reg[i];
  }
};

// ------------------------------------------------------------------------------------------------
// Loader for an operand stored [k][cols] with cols contiguous (contraction index on the slow axis).
// The k rows may be gathered through idx.  Thread (kg = t & 7, mg = t >> 3) loads the 8(k) x MW(col)
// block at k rows 8 kg .. 8 kg + 7 and columns MW mg .., transposes it in registers (v_perm) and
// writes MW rows of eight k each into the tile.
// ------------------------------------------------------------------------------------------------
template <int ROWS>
struct TransposingLoader {
  static constexpr int MW = ROWS / 32;          // 8 (16-byte loads), 4 (8-byte) or 2 (4-byte)
  static constexpr int ND = MW / 2;             // dwords per loaded row piece
  const uint16_t* src;
  const int32_t* idx;
  long long ld;
  int kdim, kg, col;                            // col: first column of this thread's block (absolute)
  bool col_ok;
  int soff[MW];
  uint32_t reg[8][ND];

  __device__ __forceinline__ void init(const uint16_t* src_, const int32_t* idx_, long long ld_, int col0,
                                       int ncols, int kdim_, int t) {
    src = src_; idx = idx_; ld = ld_; kdim = kdim_;
    kg = t & 7;
    const int mg = t >> 3;
    col = col0 + MW * mg;
    col_ok = col < ncols;
#pragma unroll
    for (int mm = 0; mm < MW; ++mm) soff[mm] = lds_off(MW * mg + mm, kg);
  }
  __device__ __forceinline__ void load(int kbase) {   // kbase: first contraction row of this stage
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = kbase + 8 * kg + i;
      if (col_ok && k < kdim) {
        const long long g = idx ? (long long)idx[k] : (long long)k;
        const uint16_t* p = src + g * ld + col;
        if constexpr (ND == 4) {
          uint4 v = *reinterpret_cast<const uint4*>(p);
          reg[i][0] = v.x; reg[i][1] = v.y; reg[i][2] = v.z; reg[i][3] = v.w;
        } else if constexpr (ND == 2) {
          uint2 v = *reinterpret_cast<const uint2*>(p);
          reg[i][0] = v.x; reg[i][1] = v.y;
        } else {
          reg[i][0] = *reinterpret_cast<const uint32_t*>(p);
        }
      } else {
#pragma unroll
        for (int d = 0; d < ND; ++d) reg[i][d] = 0;
      }
    }
  }
  __device__ __forceinline__ void store(char* buf) const {
#pragma unroll
    for (int mm = 0; mm < MW; ++mm) {
      uint4 v;   // element e of the 16-byte vector = contraction row 8 kg + e (compiles to v_perm_b32)
      v.x = pack_halves(reg[0][mm >> 1], reg[1][mm >> 1], mm & 1);
      v.y = pack_halves(reg[2][mm >> 1], reg[3][mm >> 1], mm & 1);
      v.z = pack_halves(reg[4][mm >> 1], reg[5][mm >> 1], mm & 1);
      v.w = pack_halves(reg[6][mm >> 1], reg[7][mm >> 1], mm & 1);
      *reinterpret_cast<uint4*>(buf + soff[mm]) = v;
    }
  }
};

// One LDS stage of MFMAs for a wavefront: FM x FN tiles of 32x32, contraction BK = 4 x 16.
// Lane l supplies row (l & 31), contraction elements 8 (l >> 5) .. + 7 of each 16-wide step.
template <int FM, int FN>
__device__ __forceinline__ void mma_stage(const char* tA, const char* tB, int a_off, int b_off, int lane_s,
                                          int lane_h, f32x16_t (&acc)[FM][FN]) {
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) {
    const int ch = ((2 * ks + lane_h) ^ lane_s) << 4;
    bf16x8_t a[FM], b[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) a[i] = *reinterpret_cast<const bf16x8_t*>(tA + a_off + i * 4096 + ch);
#pragma unroll
    for (int j = 0; j < FN; ++j) b[j] = *reinterpret_cast<const bf16x8_t*>(tB + b_off + j * 4096 + ch);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
}

// ------------------------------------------------------------------------------------------------
// dX tile kernel.  C[j, i] = sum_o dY[row(j), o] W[o, i] for a BM x BN tile of (kept row, input channel).
// ------------------------------------------------------------------------------------------------
template <int BM, int BN>
__global__ void __launch_bounds__(NTHREADS) dx_mfma_kernel(const uint16_t* __restrict__ dY,
                                                            const int32_t* __restrict__ idx_in,   // rows of dY (NULL: compact)
                                                            const int32_t* __restrict__ idx_out,  // rows of dX (NULL: compact)
                                                            const uint16_t* __restrict__ W, int K, int Cin, int Cout,
                                                            uint16_t* __restrict__ dX) {
  constexpr int FM = BM / 64, FN = BN / 64;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
  const int tiles_n = (Cin + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  RowMajorLoader<BM> la;
  TransposingLoader<BN> lb;
  la.init(dY, idx_in, Cout, m0, K, Cout, t);
  lb.init(W, nullptr, Cin, n0, Cin, Cout, t);

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int a_off = prow(wm + (lane & 31)) * 128, b_off = prow(wn + (lane & 31)) * 128;
  const int lane_s = lane & 7, lane_h = lane >> 5;
  const int nk = (Cout + BK - 1) / BK;

  la.load(0); lb.load(0);
  la.store(smem); lb.store(smem + A_BYTES);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * STAGE;
    char* nxt = smem + ((kt + 1) & 1) * STAGE;
    if (kt + 1 < nk) { la.load(kt + 1); lb.load((kt + 1) * BK); }
    mma_stage<FM, FN>(cur, cur + A_BYTES, a_off, b_off, lane_s, lane_h, acc);
    if (kt + 1 < nk) { la.store(nxt); lb.store(nxt + A_BYTES); }
    __syncthreads();
  }

  // epilogue: acc register v of lane l is C[row = 8 (v/4) + 4 (l>>5) + (v&3)][col = l & 31] of its 32x32 tile
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int j = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (j < K) {
        const long long orow = idx_out ? (long long)idx_out[j] : (long long)j;
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) {
          const int col = n0 + wn + 32 * jn + (lane & 31);
          if (col < Cin) dX[orow * Cin + col] = (uint16_t)bf16_round(acc[i][jn][v]);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// dW tile kernel.  partial[s][o, i] = sum over the kept rows j of split s of dY[row(j), o] X_k[j, i].
// ------------------------------------------------------------------------------------------------
template <int BM, int BN>
__global__ void __launch_bounds__(NTHREADS) dw_mfma_kernel(const uint16_t* __restrict__ dY,
                                                            const int32_t* __restrict__ idx,   // rows of dY (NULL: compact)
                                                            const uint16_t* __restrict__ Xk, int K, int Cin, int Cout,
                                                            int rows_per_split, float* __restrict__ partial) {
  constexpr int FM = BM / 64, FN = BN / 64;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
  const int tiles_n = (Cin + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int split = blockIdx.y;
  const int j0 = split * rows_per_split;
  const int j1 = min(K, j0 + rows_per_split);

  TransposingLoader<BM> la;
  TransposingLoader<BN> lb;
  la.init(dY, idx, Cout, m0, Cout, j1, t);
  lb.init(Xk, nullptr, Cin, n0, Cin, j1, t);

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int a_off = prow(wm + (lane & 31)) * 128, b_off = prow(wn + (lane & 31)) * 128;
  const int lane_s = lane & 7, lane_h = lane >> 5;
  const int nk = (j1 - j0 + BK - 1) / BK;

  if (nk > 0) {
    la.load(j0); lb.load(j0);
    la.store(smem); lb.store(smem + A_BYTES);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * STAGE;
    char* nxt = smem + ((kt + 1) & 1) * STAGE;
    if (kt + 1 < nk) { la.load(j0 + (kt + 1) * BK); lb.load(j0 + (kt + 1) * BK); }
    mma_stage<FM, FN>(cur, cur + A_BYTES, a_off, b_off, lane_s, lane_h, acc);
    if (kt + 1 < nk) { la.store(nxt); lb.store(nxt + A_BYTES); }
    __syncthreads();
  }

  float* out = partial + (long long)split * Cout * Cin;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int o = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (o < Cout) {
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) {
          const int col = n0 + wn + 32 * jn + (lane & 31);
          if (col < Cin) out[(long long)o * Cin + col] = acc[i][jn][v];
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Column sums of the kept rows of dY (bf16), in row splits: dbp[s][o] = sum_{j in split s} dY[row(j), o].
// Thread (x, y): 8 columns starting at 8 (32 blockIdx.x + x), rows y, y + 8, ... of the split.
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(NTHREADS) colsum_bf16_kernel(const uint16_t* __restrict__ dY,
                                                                const int32_t* __restrict__ idx, int K, int Cout,
                                                                int rows_per_split, float* __restrict__ dbp) {
  __shared__ float red[8][32][9];
  const int x = threadIdx.x & 31, y = threadIdx.x >> 5;
  const int col = 8 * (32 * blockIdx.x + x);
  const int j0 = blockIdx.y * rows_per_split, j1 = min(K, j0 + rows_per_split);
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col < Cout) {
    for (int j = j0 + y; j < j1; j += 8) {
      const long long g = idx ? (long long)idx[j] : (long long)j;
      const uint4 v = *reinterpret_cast<const uint4*>(dY + g * Cout + col);
      s[0] += bf16_lo(v.x); s[1] += bf16_hi(v.x); s[2] += bf16_lo(v.y); s[3] += bf16_hi(v.y);
      s[4] += bf16_lo(v.z); s[5] += bf16_hi(v.z); s[6] += bf16_lo(v.w); s[7] += bf16_hi(v.w);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[y][x][e] = s[e];
  __syncthreads();
  if (y == 0 && col < Cout) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float a = 0.f;
#pragma unroll
      for (int yy = 0; yy < 8; ++yy) a += red[yy][x][e];
      dbp[(long long)blockIdx.y * Cout + col + e] = a;
    }
  }
}

// dW = sum_s partial[s] (+ dW), db = sum_s dbp[s] (+ db): fixed summation order.
__global__ void __launch_bounds__(NTHREADS) reduce_splits_kernel(const float* __restrict__ partial, int nsplit_w,
                                                                  long long nW, float* __restrict__ dW,
                                                                  const float* __restrict__ dbp, int nsplit_b, int Cout,
                                                                  float* __restrict__ db, int accumulate) {
  const long long nW4 = dW ? nW / 4 : 0;
  const long long nB = db ? Cout : 0;
  const long long total = nW4 + nB;
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
       e += (long long)gridDim.x * blockDim.x) {
    if (e < nW4) {
      float4 a = accumulate ? reinterpret_cast<const float4*>(dW)[e] : make_float4(0, 0, 0, 0);
      for (int s = 0; s < nsplit_w; ++s) {
        const float4 p = reinterpret_cast<const float4*>(partial + (long long)s * nW)[e];
        a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
      }
      reinterpret_cast<float4*>(dW)[e] = a;
    } else {
      const long long o = e - nW4;
      float a = accumulate ? db[o] : 0.f;
      for (int s = 0; s < nsplit_b; ++s) a += dbp[(long long)s * Cout + o];
      db[o] = a;
    }
  }
}

// same, element by element, for weight matrices whose size is not a multiple of 4
__global__ void __launch_bounds__(NTHREADS) reduce_splits_scalar_kernel(const float* __restrict__ partial, int nsplit,
                                                                         long long nW, float* __restrict__ dW,
                                                                         const float* __restrict__ dbp, int Cout,
                                                                         float* __restrict__ db, int accumulate) {
  const long long nWe = dW ? nW : 0;
  const long long total = nWe + (db ? Cout : 0);
  for (long long e = blockIdx.x * (long long)blockDim.x + threadIdx.x; e < total;
       e += (long long)gridDim.x * blockDim.x) {
    if (e < nWe) {
      float a = accumulate ? dW[e] : 0.f;
      for (int s = 0; s < nsplit; ++s) a += partial[(long long)s * nW + e];
      dW[e] = a;
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
  static __device__ __forceinline__ void st(uint16_t* p, float v) { *p = (uint16_t)bf16_round(v); }
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

LinearPlan plan_linear(int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype, uint32_t flags) {
  LinearPlan p{};
  p.mfma = dtype == SBP_BF16 && Cin % 8 == 0 && Cout % 8 == 0;
  int splits = 1;
  if (K > 0) {
    if (p.mfma) {
      // enough blocks to cover the chip about twice, each split at least 4 stages long
      const int64_t tiles = ceil_div(Cout, 128) * ceil_div(Cin, 128);
      int64_t want = ceil_div(2 * kNumCU, tiles);
      int64_t max_by_len = std::max<int64_t>(1, K / (4 * BK));
      splits = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(want, max_by_len), 64));
    } else {
      splits = (int)std::max<int64_t>(1, std::min<int64_t>(ceil_div(K, 512), 64));
    }
  }
  int64_t rps = K > 0 ? ceil_div(K, splits) : 0;
  rps = ceil_div(rps, BK) * BK;
  if (rps > 0) splits = (int)ceil_div(K, rps);
  p.splits = splits;
  p.rows_per_split = (int)rps;
  size_t off = 0;
  p.off_partial = off;
  off += align_up((size_t)splits * ((size_t)Cout * Cin + (size_t)Cout) * sizeof(float), 256);
  p.off_inv = off;
  if (!(flags & SBP_FLAG_DX_COMPACT)) off += align_up((size_t)M * sizeof(int32_t), 256);
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

template <int BM, int BN>
static void launch_dx_mfma(const uint16_t* dY, const int32_t* idx_in, const int32_t* idx_out, const uint16_t* W,
                           int K, int Cin, int Cout, uint16_t* dX, hipStream_t s) {
  const int tiles = (int)(ceil_div(K, BM) * ceil_div(Cin, BN));
  const size_t lds = 2 * (size_t)(BM + BN) * 128;
  SBP_LAUNCH(SBP_PROF_DX_GEMM, s, (dx_mfma_kernel<BM, BN>), dim3(tiles), dim3(NTHREADS), lds, s, dY, idx_in, idx_out, W, K, Cin,
                     Cout, dX);
}

template <int BM, int BN>
static void launch_dw_mfma(const uint16_t* dY, const int32_t* idx, const uint16_t* Xk, int K, int Cin, int Cout,
                           int splits, int rps, float* part, hipStream_t s) {
  const int tiles = (int)(ceil_div(Cout, BM) * ceil_div(Cin, BN));
  const size_t lds = 2 * (size_t)(BM + BN) * 128;
  SBP_LAUNCH(SBP_PROF_DW_GEMM, s, (dw_mfma_kernel<BM, BN>), dim3(tiles, splits), dim3(NTHREADS), lds, s, dY, idx, Xk, K, Cin,
                     Cout, rps, part);
}

int32_t launch_backward_linear(const LinearPlan& p, const void* dY, const int32_t* idx, const void* Xk,
                               const void* W, int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype,
                               float* dW, float* db, void* dX, void* ws, uint32_t flags, hipStream_t s) {
  const int eb = dtype == SBP_F32 ? 4 : 2;
  const bool dy_compact = flags & SBP_FLAG_DY_COMPACT, dx_compact = flags & SBP_FLAG_DX_COMPACT;
  const int accumulate = (flags & SBP_FLAG_ACCUMULATE_DW) ? 1 : 0;
  const int32_t* idx_in = dy_compact ? nullptr : idx;
  const int32_t* idx_out = dx_compact ? nullptr : idx;
  float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + p.off_partial);
  float* dbp = part + (size_t)p.splits * Cout * Cin;
  int32_t* inv = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + p.off_inv);
  const long long nW = (long long)Cin * Cout;

  if (K == 0) {  // nothing kept: gradients are zero
    if (!accumulate) {
      if (dW) SBP_LAUNCH(SBP_PROF_OTHER, s, fill_zero_kernel, dim3(256), dim3(NTHREADS), 0, s, (uint32_t*)dW, nW);
      if (db) SBP_LAUNCH(SBP_PROF_OTHER, s, fill_zero_kernel, dim3(1), dim3(NTHREADS), 0, s, (uint32_t*)db, (long long)Cout);
    }
    if (dX && !dx_compact)
      SBP_LAUNCH(SBP_PROF_OTHER, s, fill_zero_kernel, dim3(1024), dim3(NTHREADS), 0, s, (uint32_t*)dX,
                         (long long)M * Cin * eb / 4);
    return check_launch("backward_linear (K = 0)");
  }

  const bool scatter = dX && !dx_compact;
  if (scatter)
    SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, mark_rows_kernel, dim3((unsigned)ceil_div(K, NTHREADS)), dim3(NTHREADS), 0, s, idx, (int)K, inv);

  const bool aligned = ((uintptr_t)dY % 16 == 0) && ((uintptr_t)Xk % 16 == 0) && ((uintptr_t)W % 16 == 0) &&
                       ((uintptr_t)dX % 16 == 0);
  if (p.mfma && aligned) {
    const uint16_t* dYh = static_cast<const uint16_t*>(dY);
    if (db) {
      dim3 grid((unsigned)ceil_div(Cout, 256), p.splits);
      SBP_LAUNCH(SBP_PROF_COLSUM, s, colsum_bf16_kernel, grid, dim3(NTHREADS), 0, s, dYh, idx_in, (int)K, Cout, p.rows_per_split,
                         dbp);
    }
    if (dW)
      launch_dw_mfma<128, 128>(dYh, idx_in, static_cast<const uint16_t*>(Xk), (int)K, Cin, Cout, p.splits,
                               p.rows_per_split, part, s);
    if (dX)
      launch_dx_mfma<128, 128>(dYh, idx_in, idx_out, static_cast<const uint16_t*>(W), (int)K, Cin, Cout,
                               static_cast<uint16_t*>(dX), s);
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
      unsigned blocks = (unsigned)std::min<long long>(ceil_div(total, NTHREADS), 4096);
      SBP_LAUNCH(SBP_PROF_REDUCE, s, reduce_splits_kernel, dim3(blocks), dim3(NTHREADS), 0, s, part, p.splits, nW, dW, dbp,
                         p.splits, Cout, db, accumulate);
    } else {
      const long long total = (dW ? nW : 0) + (db ? Cout : 0);
      unsigned blocks = (unsigned)std::min<long long>(ceil_div(total, NTHREADS), 4096);
      SBP_LAUNCH(SBP_PROF_REDUCE, s, reduce_splits_scalar_kernel, dim3(blocks), dim3(NTHREADS), 0, s, part, p.splits, nW, dW,
                         dbp, Cout, db, accumulate);
    }
  }

  if (scatter) {
    const long long row_bytes = (long long)Cin * eb;
    if (row_bytes % 16 == 0 && (uintptr_t)dX % 16 == 0) {
      const int ppr = (int)(row_bytes / 16);
      unsigned blocks = (unsigned)std::min<long long>(ceil_div(M * ppr, NTHREADS), 8192);
      SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, zero_dropped_rows_kernel, dim3(blocks), dim3(NTHREADS), 0, s, idx, inv, (int)K,
                         (long long)M, ppr, (uint4*)dX);
    } else if (eb == 4) {
      unsigned blocks = (unsigned)std::min<long long>(ceil_div(M * Cin, NTHREADS), 8192);
      SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, (zero_dropped_rows_elem_kernel<uint32_t>), dim3(blocks), dim3(NTHREADS), 0, s, idx, inv,
                         (int)K, (long long)M, Cin, (uint32_t*)dX);
    } else {
      unsigned blocks = (unsigned)std::min<long long>(ceil_div(M * Cin, NTHREADS), 8192);
      SBP_LAUNCH(SBP_PROF_ZERO_ROWS, s, (zero_dropped_rows_elem_kernel<uint16_t>), dim3(blocks), dim3(NTHREADS), 0, s, idx, inv,
                         (int)K, (long long)M, Cin, (uint16_t*)dX);
    }
  }
  return check_launch("backward_linear");
}

}  // namespace sbp
